"""Seeded synthetic workloads: shapes, spans, lazy masks and random Q/K/V tensors.

This module serves both the CPU oracle's tests and the HIP library's tests and
benchmark.  It holds none of the method's arithmetic: it only describes the
benchmark configurations and draws N(0,1) inputs (rounded once to the storage
type), so that both sides read identical bits.

Two input recipes.  "normal": every element i.i.d. N(0,1).  "peaked": the same draws with the queries
multiplied by Q_GAIN, which widens the scaled scores from about +-3 to about +-20, and with a few key
rows replaced by copies of (unscaled) query rows, which gives those query/key pairs a score of about
Q_GAIN*sqrt(head_dim), far above everything else in their row.  The planted keys sit late in the
visual span, behind it, and in a late part of the prompt for the query of decode step PEAK_STEP, so
that running maxima jump in late key tiles, chunk maxima lie far apart, and inherited rows carry
peaks as well.  Softmax attention is defined for any score range; the recipe only moves the inputs
into the range where a careless implementation of it breaks.

The shapes stand in for LLaVA-1.5 / LLaVA-NeXT / video prompts (576 visual
tokens per image tile or frame, 32 or 40 heads of width 128); real prompts,
images and weights are not used anywhere.
"""
from dataclasses import dataclass, field
from typing import List

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
SEED_BASE = 0x51C0
Q_GAIN = 6.0        # "peaked" recipe: factor on every query
PEAK_STEP = 1       # "peaked" recipe: the decode step whose queries have planted keys in the prompt


def block_lazy_mask(n_layers, block=3):
    """Blocks of one ordinary layer followed by block-1 lazy layers, between layer 2 and layer N-2.

    The first two layers and the last layer stay ordinary (the paper reports
    them as dissimilar to their neighbours); block=3 gives about 60 % lazy
    layers, block=2 about 45 %.
    """
    return [int(2 <= l <= n_layers - 2 and (l - 2) % block != 0) for l in range(n_layers)]


@dataclass
class Workload:
    name: str
    index: int
    n_layers: int
    n_heads: int
    head_dim: int
    dtype: str                      # "f32" | "bf16"
    vis_start: List[int]            # per sequence
    vis_len: List[int]
    seq_len: List[int]              # prompt lengths
    decode_steps: int
    lazy_mask: List[int]
    max_seq: int = 0
    max_vis: int = 0
    max_text: int = 0
    seed_tag: int = field(default=0)
    recipe: str = "normal"          # "normal" | "peaked" (see the module docstring)

    def __post_init__(self):
        if not self.max_seq:
            self.max_seq = max(self.seq_len) + self.decode_steps
        if not self.max_vis:
            self.max_vis = max(self.vis_len)
        if not self.max_text:
            self.max_text = max(l - v for l, v in zip(self.seq_len, self.vis_len)) + self.decode_steps

    @property
    def batch(self):
        return len(self.seq_len)

    @property
    def total_tokens(self):
        return sum(self.seq_len)

    @property
    def cu_seqlens(self):
        out = [0]
        for l in self.seq_len:
            out.append(out[-1] + l)
        return out

    @property
    def elem_bytes(self):
        return 2 if self.dtype == "bf16" else 4

    @property
    def n_lazy(self):
        return sum(self.lazy_mask)


def config(i, lazy_block=3):
    """The five benchmark configurations (0-based index)."""
    if i == 0:
        return Workload("cfg1_tiny_f32", 0, 4, 8, 64, "f32", [8], [144], [176], 16, [0, 0, 1, 1])
    if i == 1:
        return Workload("cfg2_llava15_7b_b1", 1, 32, 32, 128, "bf16", [32], [576], [640], 256,
                        block_lazy_mask(32, lazy_block))
    if i == 2:
        rng = np.random.default_rng(SEED_BASE + 2000)
        text = rng.integers(128, 513, size=32)
        lens = [int(576 + t) for t in text]
        return Workload("cfg3_llava15_7b_b32_decode", 2, 32, 32, 128, "bf16", [32] * 32, [576] * 32,
                        lens, 512, block_lazy_mask(32, lazy_block))
    if i == 3:
        return Workload("cfg4_llavanext_7b_b8_prefill", 3, 32, 32, 128, "bf16", [32] * 8, [2880] * 8,
                        [3008] * 8, 0, block_lazy_mask(32, lazy_block))
    if i == 4:
        return Workload("cfg5_video_13b_b4", 4, 40, 40, 128, "bf16", [32] * 4, [4608] * 4,
                        [4864] * 4, 1024, block_lazy_mask(40, lazy_block))
    raise ValueError("no such configuration")


def custom(name, n_layers, n_heads, head_dim, dtype, vis_start, vis_len, seq_len, decode_steps,
           lazy_mask, seed_tag=77, recipe="normal", **caps):
    return Workload(name, 9, n_layers, n_heads, head_dim, dtype, list(vis_start), list(vis_len),
                    list(seq_len), decode_steps, list(lazy_mask), seed_tag=seed_tag, recipe=recipe, **caps)


def _draw_f32(shape, seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def _draw(w, shape, seed, device):
    return _draw_f32(shape, seed, device).to(TORCH_DTYPE[w.dtype])


def planted_keys(w, layer, b):
    """"peaked" recipe: list of (key position, source) for sequence b of `layer`; source is
    ("prompt", query position, gain) or ("decode", layer whose PEAK_STEP query is copied, gain); the key
    row becomes gain times the unscaled query row.  The key aimed at a lazy layer's decode query from
    inside the span of its block's first layer is the stronger of that query's two planted keys."""
    s, vn, L = w.vis_start[b], w.vis_len[b], w.seq_len[b]
    out = []
    if vn >= 4:
        out.append((s + vn - 3, ("prompt", s + vn - 1, 1.0)))          # late in the span, for the last visual query
    if L - (s + vn) >= 6:
        out.append((L - 5, ("prompt", L - 1, 1.0)))                    # behind the span, for the last prompt query
    j = max(s + vn, L - 70)
    if j < L - 5:
        out.append((j, ("decode", layer, 0.75)))                        # a late chunk, for this layer's decode query
    if layer + 1 < w.n_layers and w.lazy_mask[layer + 1] and not w.lazy_mask[layer] and vn >= 8:
        out.append((s + vn // 2, ("decode", layer + 1, 1.0)))          # inside the span, for the next (lazy) layer's decode query
    return out


def _seed(w, layer, step):
    return SEED_BASE + 1000 * (w.index + 1) + 7919 * w.seed_tag + layer + 100000 * (step + 1)


def prefill_qkv(w, layer, device="cpu"):
    """Q, K, V of one layer for the packed prompts: three [total_tokens, H, D] tensors."""
    shape = (3, w.total_tokens, w.n_heads, w.head_dim)
    if w.recipe == "normal":
        x = _draw(w, shape, _seed(w, layer, -1), device)
        return x[0], x[1], x[2]
    assert w.recipe == "peaked"
    x = _draw_f32(shape, _seed(w, layer, -1), device)
    cu = w.cu_seqlens
    dec_shape = (3, w.batch, w.n_heads, w.head_dim)
    for b in range(w.batch):
        for j, (kind, src, gain) in planted_keys(w, layer, b):
            row = x[0, cu[b] + src] if kind == "prompt" else _draw_f32(dec_shape, _seed(w, src, PEAK_STEP), device)[0, b]
            x[1, cu[b] + j] = gain * row
    x[0] *= Q_GAIN
    x = x.to(TORCH_DTYPE[w.dtype])
    return x[0], x[1], x[2]


def decode_qkv(w, layer, step, device="cpu"):
    """q, k, v of one layer for decode step `step`: three [B, H, D] tensors."""
    x = _draw_f32((3, w.batch, w.n_heads, w.head_dim), _seed(w, layer, step), device)
    if w.recipe == "peaked":
        x[0] *= Q_GAIN
    x = x.to(TORCH_DTYPE[w.dtype])
    return x[0], x[1], x[2]


def to_f64(t):
    """Tensor (any device, f32 or bf16) -> numpy fp64 with the exact same values."""
    return t.detach().to("cpu", torch.float32).numpy().astype(np.float64)
