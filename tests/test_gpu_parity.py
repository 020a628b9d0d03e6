"""GPU parity: the HIP library against the CPU oracle on identical seeded inputs, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2602_01901_amd as P
import workloads
from stack_runner import TOL, run_full_parity

pytestmark = pytest.mark.gpu


def session_for(w):
    return P.Session.for_workload(w)


def test_cfg1_tiny_fp32_full_parity():
    """4 layers, 8 heads, D=64, fp32, 144 visual + 32 text tokens, lazy {2,3}, 16 decode steps."""
    w = workloads.config(0)
    s = session_for(w)
    ep, ed = run_full_parity(w, 16, s)
    print("cfg1 max abs err prefill %.3g decode %.3g" % (ep, ed), flush=True)
    assert ep <= TOL["f32"] and ed <= TOL["f32"]


@pytest.mark.parametrize("s,vn,L", [(0, 144, 176), (32, 144, 176), (8, 0, 40), (8, 168, 176), (0, 176, 176)])
def test_fp32_span_placements(s, vn, L):
    """Span at the very start, no suffix text, no visual tokens, everything visual."""
    w = workloads.custom("span", 4, 8, 64, "f32", [s], [vn], [L], 3, [0, 0, 1, 1], seed_tag=s + vn)
    ep, ed = run_full_parity(w, 3, session_for(w))
    assert ep <= TOL["f32"] and ed <= TOL["f32"]


def test_fp32_one_based_mask_reading():
    """Lazy layers {1,2} (the 1-based reading of the tiny configuration's mask)."""
    w = workloads.custom("mask12", 4, 8, 64, "f32", [8], [144], [176], 2, [0, 1, 1, 0])
    ep, ed = run_full_parity(w, 2, session_for(w))
    assert ep <= TOL["f32"] and ed <= TOL["f32"]


@pytest.mark.parametrize("dtype,D", [("f32", 128), ("bf16", 64), ("bf16", 128)])
def test_ragged_batch_small(dtype, D):
    """Three sequences of unequal length and span, several key tiles and a ragged tail each."""
    w = workloads.custom("ragged", 5, 3, D, dtype, [5, 0, 17], [70, 33, 0], [131, 64, 45], 5, [0, 1, 1, 0, 1])
    ep, ed = run_full_parity(w, 5, session_for(w))
    print("ragged %s D=%d: prefill %.3g decode %.3g" % (dtype, D, ep, ed), flush=True)
    assert ep <= TOL[dtype] and ed <= TOL[dtype]


def test_lazy_layers_never_read_span_rows_of_q_and_k():
    w = workloads.custom("poison", 4, 2, 128, "bf16", [3, 9], [150, 40], [200, 77], 2, [0, 1, 1, 1])
    ep, ed = run_full_parity(w, 2, session_for(w), poison_span=True)
    assert ep <= TOL["bf16"] and ed <= TOL["bf16"]


def test_cfg2_llava15_shape_full_parity():
    """32 layers, 32 heads, D=128, bf16, 576 visual + 64 text, 19 lazy layers; 4 decode steps."""
    w = workloads.config(1)
    ep, ed = run_full_parity(w, 4, session_for(w))
    print("cfg2 max abs err prefill %.3g decode %.3g" % (ep, ed), flush=True)
    assert ep <= TOL["bf16"] and ed <= TOL["bf16"]


def test_cfg2_unaligned_span_and_second_mask():
    w = workloads.config(1, lazy_block=2)
    w.vis_start = [35]
    ep, ed = run_full_parity(w, 2, session_for(w))
    assert ep <= TOL["bf16"] and ed <= TOL["bf16"]


def test_results_are_bitwise_reproducible():
    """Split merges run in fixed order: two runs give identical bits (a cheap race detector)."""
    w = workloads.custom("repro", 3, 4, 128, "bf16", [4], [300], [700], 3, [0, 1, 1])
    outs = []
    for _ in range(2):
        s = session_for(w)
        s.reset(w.vis_start, w.vis_len)
        acc = []
        for l in range(w.n_layers):
            q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, l))
            acc.append(s.prefill(l, q, k, v, w.cu_seqlens).clone())
        for t in range(3):
            for l in range(w.n_layers):
                q, k, v = (x.cuda() for x in workloads.decode_qkv(w, l, t))
                acc.append(s.decode(l, q, k, v).clone())
        torch.cuda.synchronize()
        outs.append(acc)
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_capacity_and_order_errors_on_device_handles():
    w = workloads.custom("caps", 2, 2, 64, "f32", [2], [10], [20], 1, [0, 1])
    s = session_for(w)     # max_seq = 21
    s.reset(w.vis_start, w.vis_len)
    q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, 0))
    with pytest.raises(P.QcError) as e:
        s.decode(0, q[:1], k[:1], v[:1])
    assert e.value.status == P.binding.QC_EORDER
    s.prefill(0, q, k, v, w.cu_seqlens)
    s.prefill(1, q, k, v, w.cu_seqlens)
    dq, dk, dv = (t.cuda() for t in workloads.decode_qkv(w, 0, 0))
    for l in range(2):
        s.decode(l, dq, dk, dv)
    with pytest.raises(P.QcError) as e:
        s.decode(0, dq, dk, dv)          # would be position 22 > max_seq
    assert e.value.status == P.binding.QC_ECAPACITY
    assert s.stats()["tokens"] == 21
