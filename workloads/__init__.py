"""Seeded synthetic workloads: shapes, spans, lazy masks and random Q/K/V tensors.

This module serves both the CPU oracle's tests and the HIP library's tests and
benchmark.  It holds none of the method's arithmetic: it only describes the
benchmark configurations and draws N(0,1) inputs (rounded once to the storage
type), so that both sides read identical bits.

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
           lazy_mask, seed_tag=77, **caps):
    return Workload(name, 9, n_layers, n_heads, head_dim, dtype, list(vis_start), list(vis_len),
                    list(seq_len), decode_steps, list(lazy_mask), seed_tag=seed_tag, **caps)


def _draw(w, shape, seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    return x.to(TORCH_DTYPE[w.dtype])


def _seed(w, layer, step):
    return SEED_BASE + 1000 * (w.index + 1) + 7919 * w.seed_tag + layer + 100000 * (step + 1)


def prefill_qkv(w, layer, device="cpu"):
    """Q, K, V of one layer for the packed prompts: three [total_tokens, H, D] tensors."""
    x = _draw(w, (3, w.total_tokens, w.n_heads, w.head_dim), _seed(w, layer, -1), device)
    return x[0], x[1], x[2]


def decode_qkv(w, layer, step, device="cpu"):
    """q, k, v of one layer for decode step `step`: three [B, H, D] tensors."""
    x = _draw(w, (3, w.batch, w.n_heads, w.head_dim), _seed(w, layer, step), device)
    return x[0], x[1], x[2]


def to_f64(t):
    """Tensor (any device, f32 or bf16) -> numpy fp64 with the exact same values."""
    return t.detach().to("cpu", torch.float32).numpy().astype(np.float64)
