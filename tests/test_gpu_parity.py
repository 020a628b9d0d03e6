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


def test_more_than_64_sequences():
    """Per-sequence metadata is uploaded 64 sequences per launch: 70 short sequences of mixed shape."""
    B = 70
    lens = [20 + (7 * b) % 50 for b in range(B)]
    vlen = [min(lens[b] - 3, (5 * b) % 30) for b in range(B)]
    vstart = [min(2, lens[b] - vlen[b]) for b in range(B)]
    w = workloads.custom("b70", 3, 2, 64, "f32", vstart, vlen, lens, 2, [0, 1, 1])
    ep, ed = run_full_parity(w, 2, session_for(w))
    assert ep <= TOL["f32"] and ed <= TOL["f32"]


def test_decode_many_chunks_merge():
    """Batch 1, 2 heads, 2100-token context: 33 split chunks, so the merge pass loops over several
    batches of partials; the lazy layer's three key segments each span many chunks."""
    w = workloads.custom("chunks", 3, 2, 128, "bf16", [300], [1500], [2100], 3, [0, 1, 0])
    ep, ed = run_full_parity(w, 3, session_for(w))
    print("many chunks: decode %.3g" % ed, flush=True)
    assert ep <= TOL["bf16"] and ed <= TOL["bf16"]


def test_strided_inputs_and_custom_scale():
    """Q/K/V as slices of one fused [tokens, 3, H, D'] projection output (token and head strides
    larger than the packed ones) and a caller-supplied softmax scale."""
    import numpy as np
    from stack_runner import new_oracles, max_abs_err
    w = workloads.custom("strided", 2, 4, 128, "bf16", [10, 0], [120, 64], [300, 130], 1, [0, 1])
    s = session_for(w)
    s.reset(w.vis_start, w.vis_len)
    scale = 0.05
    stacks = new_oracles(w)
    for st in stacks:
        st.scale = scale
    cu = w.cu_seqlens
    for l in range(w.n_layers):
        q, k, v = workloads.prefill_qkv(w, l)
        fused = torch.zeros(w.total_tokens, 3, w.n_heads, 160, dtype=torch.bfloat16, device="cuda")
        fused[:, 0, :, :128], fused[:, 1, :, :128], fused[:, 2, :, :128] = q.cuda(), k.cuda(), v.cuda()
        outbuf = torch.zeros_like(fused)
        qs, ks, vs, os_ = fused[:, 0, :, :128], fused[:, 1, :, :128], fused[:, 2, :, :128], outbuf[:, 0, :, :128]
        assert qs.stride() == (3 * w.n_heads * 160, 160, 1)
        s.prefill(l, qs, ks, vs, w.cu_seqlens, out=os_, softmax_scale=scale)
        q64, k64, v64 = (workloads.to_f64(t) for t in (q, k, v))
        for b in range(w.batch):
            ref = stacks[b].prefill(l, q64[cu[b]:cu[b + 1]], k64[cu[b]:cu[b + 1]], v64[cu[b]:cu[b + 1]])
            assert max_abs_err(os_[cu[b]:cu[b + 1]], ref) <= TOL["bf16"]
        assert float(outbuf[:, 1:].abs().max()) == 0.0 and float(outbuf[:, 0, :, 128:].abs().max()) == 0.0
    for l in range(w.n_layers):
        q, k, v = workloads.decode_qkv(w, l, 0)
        out = s.decode(l, q.cuda(), k.cuda(), v.cuda(), softmax_scale=scale)
        q64, k64, v64 = (workloads.to_f64(t) for t in (q, k, v))
        ref = np.stack([stacks[b].decode(l, q64[b], k64[b], v64[b]) for b in range(w.batch)])
        assert max_abs_err(out, ref) <= TOL["bf16"]


def test_kernel_timing_counts_launches():
    w = workloads.custom("timing", 2, 2, 128, "bf16", [4], [100], [200], 2, [0, 1])
    s = session_for(w)
    B = P.binding
    B.qc_timing_enable(s.kv, 1)
    s.reset(w.vis_start, w.vis_len)
    for l in range(2):
        q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, l))
        s.prefill(l, q, k, v, w.cu_seqlens)
    for t in range(2):
        for l in range(2):
            q, k, v = (x.cuda() for x in workloads.decode_qkv(w, l, t))
            s.decode(l, q, k, v)
    ms_p, n_p = B.qc_timing_read(s.kv, 0)
    ms_d, n_d = B.qc_timing_read(s.kv, 1)
    assert (n_p, n_d) == (2, 4) and ms_p > 0 and ms_d > 0
    assert B.qc_timing_read(s.kv, 1) == (0.0, 0)
    B.qc_timing_enable(s.kv, 0)


@pytest.mark.parametrize("mode", ["vla", "gla"])
@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128)])
def test_nothing_reads_memory_it_has_not_written(mode, dtype, D):
    """Arenas and workspace start as all-ones bytes (NaN in either element type) and are not cleared:
    every output must still be finite and within the bar, for ordinary calls and for graph replays."""
    import paper_2602_01901_amd as P2
    from test_gpu_graph import prefill_both, run_steps, step_buffers
    from stack_runner import new_oracles
    w = workloads.custom("poison", 5, 3, D, dtype, [4, 0, 9], [70, 0, 33], [150, 40, 65], 3, [0, 1, 0, 1, 1], seed_tag=51)
    s = P2.Session.for_workload(w, mode=mode)
    for t in (s.kv_arena, s.q_arena, s.workspace):
        t.fill_(0xFF)
    wp, wd = run_full_parity(w, 3, s, check_arena=False, zero_fill=False)
    assert max(wp, wd) <= TOL[dtype]
    s.close()
    s = P2.Session.for_workload(w, mode=mode)
    for t in (s.kv_arena, s.q_arena, s.workspace):
        t.fill_(0xFF)
    stacks = new_oracles(w, mode=mode)
    s.reset(w.vis_start, w.vis_len, zero_fill=False)
    for l in range(w.n_layers):
        q, k, v = workloads.prefill_qkv(w, l)
        from stack_runner import oracle_prefill_layer
        oracle_prefill_layer(w, stacks, l, q, k, v)
        no_qk = mode == "gla" and w.lazy_mask[l]
        s.prefill(l, None if no_qk else q.cuda(), None if no_qk else k.cuda(), v.cuda(), w.cu_seqlens)
    bufs = step_buffers(w, mode)
    g = s.decode_graph(*bufs)
    run_steps(w, s, stacks, mode, g, bufs, "ggg")
    s.close()
