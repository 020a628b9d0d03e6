"""GPU parity for Global Lazy Attention (Eq. 5 / Eq. 6): the HIP library in QC_GLA mode against the
separately written CPU oracle, same seeded inputs, through the C ABI.  Outputs are compared element
by element; the K/V arena, the Q Cache arena and the byte accounting are compared exactly."""
import numpy as np
import pytest
import torch

import paper_2602_01901_amd as P
from paper_2602_01901_amd import binding as B
import workloads
from stack_runner import TOL, run_full_parity

pytestmark = pytest.mark.gpu


def gla_session(w):
    return P.Session.for_workload(w, mode="gla")


def test_gla_cfg1_tiny_fp32_full_parity():
    w = workloads.config(0)
    ep, ed = run_full_parity(w, 8, gla_session(w))
    print("gla cfg1 max abs err prefill %.3g decode %.3g" % (ep, ed), flush=True)
    assert ep <= TOL["f32"] and ed <= TOL["f32"]


@pytest.mark.parametrize("mask", [[0, 1, 1, 0, 1], [0, 0, 1, 0, 0], [0, 1, 0, 1, 1], [0, 0, 0, 0, 0]])
def test_gla_block_structures_fp32(mask):
    """Several blocks, a block at the end of the stack, single lazy layers, no lazy layer at all."""
    w = workloads.custom("gla_blocks", 5, 4, 64, "f32", [3, 0], [20, 9], [75, 33], 3, mask, seed_tag=sum(mask))
    ep, ed = run_full_parity(w, 3, gla_session(w))
    assert ep <= TOL["f32"] and ed <= TOL["f32"]


@pytest.mark.parametrize("dtype,D", [("f32", 128), ("bf16", 64), ("bf16", 128)])
def test_gla_ragged_batch_small(dtype, D):
    """Three sequences of unequal length, several key tiles and a ragged tail each."""
    w = workloads.custom("gla_ragged", 5, 3, D, dtype, [5, 0, 17], [70, 33, 0], [131, 64, 45], 5, [0, 1, 1, 0, 1])
    ep, ed = run_full_parity(w, 5, gla_session(w))
    print("gla ragged %s D=%d: prefill %.3g decode %.3g" % (dtype, D, ep, ed), flush=True)
    assert ep <= TOL[dtype] and ed <= TOL[dtype]


def test_gla_lazy_layers_never_read_q_and_k():
    """Lazy layers are handed q and k tensors that are NaN everywhere."""
    w = workloads.custom("gla_poison", 4, 2, 128, "bf16", [3, 9], [150, 40], [200, 77], 2, [0, 1, 1, 1])
    ep, ed = run_full_parity(w, 2, gla_session(w), poison_span=True)
    assert ep <= TOL["bf16"] and ed <= TOL["bf16"]


def test_gla_several_query_tiles_and_decode_chunks_bf16():
    """One sequence long enough for several 128-row query tiles and a split key axis at decode."""
    w = workloads.custom("gla_long", 3, 2, 128, "bf16", [10], [600], [1100], 3, [0, 1, 1])
    ep, ed = run_full_parity(w, 3, gla_session(w))
    print("gla long: prefill %.3g decode %.3g" % (ep, ed), flush=True)
    assert ep <= TOL["bf16"] and ed <= TOL["bf16"]


def test_gla_cfg2_llava15_shape_full_parity():
    """32 layers, 32 heads, D=128, bf16, 640 tokens, 19 lazy layers; 3 decode steps."""
    w = workloads.config(1)
    s = gla_session(w)
    ep, ed = run_full_parity(w, 3, s)
    print("gla cfg2 max abs err prefill %.3g decode %.3g" % (ep, ed), flush=True)
    assert ep <= TOL["bf16"] and ed <= TOL["bf16"]
    st = s.stats()
    per_row = w.n_heads * w.head_dim * 2
    n_lazy = sum(w.lazy_mask)
    assert st["k_bytes"] == (w.n_layers - n_lazy) * 643 * per_row      # n/(2N) of the KV cache saved
    assert st["q_bytes"] == 643 * per_row                              # 1/(2N) of a standard KV cache


def test_gla_more_than_eight_sequences():
    """Per-sequence integers come from the metadata block instead of the kernel arguments."""
    n = 11
    w = workloads.custom("gla_many", 3, 2, 64, "bf16", [1] * n, [4] * n, [20 + 3 * i for i in range(n)], 2, [0, 1, 0])
    ep, ed = run_full_parity(w, 2, gla_session(w))
    assert ep <= TOL["bf16"] and ed <= TOL["bf16"]


def test_gla_order_error_when_the_q_cache_belongs_to_another_block():
    w = workloads.custom("gla_order", 4, 2, 64, "f32", [0], [4], [12], 1, [0, 1, 0, 1])
    s = gla_session(w)
    s.reset(w.vis_start, w.vis_len)
    for l in range(w.n_layers):
        q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, l))
        s.prefill(l, None if w.lazy_mask[l] else q, None if w.lazy_mask[l] else k, v, w.cu_seqlens)
    assert s.stats()["q_owner"] == 2
    q, k, v = (t.cuda() for t in workloads.decode_qkv(w, 0, 0))
    s.decode(0, q, k, v)
    assert s.stats()["q_owner"] == 0
    s.decode(1, None, None, v)
    with pytest.raises(P.QcError) as e:      # layer 2 must run before layer 3 can inherit from it
        s.decode(3, None, None, v)
    assert e.value.status == B.QC_EORDER
    torch.cuda.synchronize()


def test_gla_lazy_decode_reads_no_key_rows():
    """Between a block's first layer and its lazy layers the whole K region is overwritten with NaN
    bit patterns: the lazy layers must give the same bits as in an untouched twin session, because
    they reuse the block's scores and stream only their own V rows."""
    w = workloads.custom("gla_nokeys", 3, 2, 128, "bf16", [2], [100], [333], 2, [0, 1, 1])
    sessions = [gla_session(w), gla_session(w)]
    for s in sessions:
        s.reset(w.vis_start, w.vis_len)
        for l in range(w.n_layers):
            q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, l))
            s.prefill(l, None if w.lazy_mask[l] else q, None if w.lazy_mask[l] else k, v, w.cu_seqlens)
    k_region_bytes = B.qc_locate(sessions[0].kv, B.QC_V, 0, 0, 0, 0)[1]   # the V region starts where K ends
    for t in range(2):
        outs = []
        for i, s in enumerate(sessions):
            q, k, v = (x.cuda() for x in workloads.decode_qkv(w, 0, t))
            acc = [s.decode(0, q, k, v).clone()]
            saved = None
            if i == 1:
                saved = s.kv_arena[:k_region_bytes].clone()
                s.kv_arena[:k_region_bytes] = 0xFF
            for l in (1, 2):
                acc.append(s.decode(l, None, None, workloads.decode_qkv(w, l, t)[2].cuda()).clone())
            if saved is not None:
                s.kv_arena[:k_region_bytes] = saved
            outs.append(acc)
        for a, b in zip(*outs):
            assert torch.isfinite(a.float()).all() and torch.equal(a, b)
    torch.cuda.synchronize()
