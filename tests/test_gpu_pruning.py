"""GPU parity for token pruning on top of Lazy Attention against oracle.pruning.

Survivor selection and row gathering are integer / byte work: bit-exact.  The ranking is decided
from the fp32 scores the library itself produced (both sides look at the same fp32 numbers).  The
attention outputs of the pruned stack carry the usual bars (1e-4 fp32, 3e-2 bf16); cache images and
accounting are exact."""
import numpy as np
import pytest
import torch

import paper_2602_01901_amd as P
from paper_2602_01901_amd import binding as B
import workloads
from oracle import layout as olayout
from oracle import selection
from oracle.pruning import PrunedStackOracle, kept_visual_positions, packed_row_map
from stack_runner import TOL, max_abs_err, oracle_layout, reset_session

pytestmark = pytest.mark.gpu


def cu_of(lens):
    cu = [0]
    for n in lens:
        cu.append(cu[-1] + n)
    return cu


def select_on_gpu(scores, lens, vis_start, vis_len, keep):
    n_out = sum(l - v + k for l, v, k in zip(lens, vis_len, keep))
    row_map = torch.full((n_out + 8,), -7, dtype=torch.int32, device="cuda")
    B.qc_prune_select(scores, scores.stride(0), len(lens), cu_of(lens), vis_start, vis_len, keep, row_map)
    torch.cuda.synchronize()
    got = row_map.cpu().numpy()
    assert np.all(got[n_out:] == -7), "wrote past the end of the row map"
    return got[:n_out], row_map


@pytest.mark.parametrize("case", [
    dict(lens=[40, 17, 9], vs=[3, 0, 9], vl=[30, 17, 0], keep=[7, 17, 0], levels=4),
    dict(lens=[1500, 1100, 2200], vs=[5, 0, 100], vl=[1400, 1025, 2048], keep=[700, 1, 1024], levels=50),
    dict(lens=[9000, 4200], vs=[32, 7], vl=[8800, 4097], keep=[4400, 0], levels=0),
    dict(lens=[30 + (i % 11) for i in range(70)], vs=[i % 5 for i in range(70)], vl=[20 + (i % 6) for i in range(70)],
         keep=[(3 * i) % 20 for i in range(70)], levels=3),
])
def test_survivor_selection_matches_oracle(case):
    lens, vs, vl, keep = case["lens"], case["vs"], case["vl"], case["keep"]
    rng = np.random.default_rng(len(lens) * 1000 + lens[0])
    stride = max(lens) + 3
    sc = rng.random((len(lens), stride)).astype(np.float32)
    if case["levels"]:
        sc = np.floor(sc * case["levels"]).astype(np.float32) / case["levels"]     # many exact ties
    sc[0, vs[0]: vs[0] + min(vl[0], 2)] = -0.0                                     # signed zeros compare equal
    got, _ = select_on_gpu(torch.from_numpy(sc).cuda(), lens, vs, vl, keep)
    kept = [kept_visual_positions(sc[b], vs[b], vl[b], keep[b]) for b in range(len(lens))]
    want = packed_row_map(lens, vs, vl, kept)
    assert np.array_equal(got, want)


def adversarial_scores(kind, V, rng):
    """Finite score vectors that stress a selection: every key byte pattern the radix passes can meet."""
    if kind == "all_equal":
        return np.full(V, 0.25, dtype=np.float32)
    if kind == "two_values":
        return rng.choice(np.array([0.5, 0.5000001], dtype=np.float32), size=V)          # differ in the last key byte only
    if kind == "ascending":
        return np.arange(V, dtype=np.float32) * np.float32(1e-4)
    if kind == "descending":
        return (V - np.arange(V, dtype=np.float32)) * np.float32(1e-4)
    if kind == "softmax_like":                                                             # what the ranking really sees
        x = rng.standard_normal(V).astype(np.float32) * 4
        e = np.exp(x - x.max())
        return (e / e.sum()).astype(np.float32)
    if kind == "mixed_signs_and_denormals":
        x = rng.standard_normal(V).astype(np.float32)
        x[::7] = 0.0
        x[3::7] = -0.0
        x[5::11] = np.float32(1e-41)                                                       # denormal
        x[6::13] = -np.float32(3e38)
        return x
    if kind == "shared_prefix":                                                            # equal top three key bytes, random last byte
        base = np.float32(1.0).view(np.uint32)
        return (base + rng.integers(0, 256, size=V).astype(np.uint32)).view(np.float32)
    raise ValueError(kind)


@pytest.mark.parametrize("V", [576, 2880, 4608, 32000])
@pytest.mark.parametrize("kind", ["all_equal", "two_values", "ascending", "descending", "softmax_like",
                                  "mixed_signs_and_denormals", "shared_prefix"])
def test_survivor_selection_large_spans_and_adversarial_scores(V, kind):
    """The span sizes of the benchmark configurations (one image, five tiles, eight frames) and one far
    beyond them, with keep at both ends, in the middle and next to the ends."""
    rng = np.random.default_rng(V + len(kind))
    keeps = [0, 1, V // 2, V - 1, V, V // 3 + 1]
    lens = [V + 40 + 3 * i for i in range(len(keeps))]
    vs = [7 + i for i in range(len(keeps))]
    vl = [V] * len(keeps)
    stride = max(lens) + 5
    sc = rng.random((len(keeps), stride)).astype(np.float32)
    for b in range(len(keeps)):
        sc[b, vs[b]: vs[b] + V] = adversarial_scores(kind, V, rng)
    got, _ = select_on_gpu(torch.from_numpy(sc).cuda(), lens, vs, vl, keeps)
    kept = [kept_visual_positions(sc[b], vs[b], vl[b], keeps[b]) for b in range(len(keeps))]
    assert np.array_equal(got, packed_row_map(lens, vs, vl, kept))


def test_survivor_selection_stays_in_bounds_with_nan_scores():
    lens, vs, vl, keep = [50, 60], [4, 0], [40, 60], [10, 30]
    sc = np.random.default_rng(3).random((2, 64)).astype(np.float32)
    sc[0, 10:30] = np.nan
    sc[1, ::3] = -np.nan
    got, _ = select_on_gpu(torch.from_numpy(sc).cuda(), lens, vs, vl, keep)
    cu = cu_of(lens)
    out0 = 0
    for b in range(2):                      # which visual tokens survive is unspecified; the shape is not
        n = lens[b] - vl[b] + keep[b]
        rows = got[out0:out0 + n] - cu[b]
        assert np.all(np.diff(rows) > 0) and rows.min() >= 0 and rows.max() < lens[b]
        text = [p for p in range(lens[b]) if not vs[b] <= p < vs[b] + vl[b]]
        assert set(text) <= set(rows.tolist())
        out0 += n


@pytest.mark.parametrize("row_elems,dtype,pad", [(128, torch.bfloat16, 0), (4096, torch.bfloat16, 64), (8, torch.float32, 4),
                                                 (3 * 64, torch.float32, 0)])
def test_gather_rows_is_bit_exact(row_elems, dtype, pad):
    rng = np.random.default_rng(row_elems)
    n_src, n_out = 777, 501
    src = torch.randn(n_src, row_elems + pad, device="cuda").to(dtype)
    rows = np.sort(rng.choice(n_src, size=n_out, replace=False)).astype(np.int32)
    dst = torch.zeros(n_out, row_elems + 2 * pad, device="cuda", dtype=dtype)
    e = src.element_size()
    B.qc_gather_rows(src, src.stride(0) * e, torch.from_numpy(rows).cuda(), n_out, row_elems * e, dst, dst.stride(0) * e)
    torch.cuda.synchronize()
    want = src.cpu().view(torch.int16 if e == 2 else torch.int32).numpy()[rows][:, :row_elems]
    got = dst.cpu().view(torch.int16 if e == 2 else torch.int32).numpy()
    assert np.array_equal(got[:, :row_elems], want)
    assert np.all(got[:, row_elems:] == 0)              # padding of the destination rows untouched


def run_pruned_parity(w, first_late, keep, mode, decode_steps, caps=None, max_seq_late=0, use_graph=False, paged=False):
    """Early layers, ranking from the last early layer's last-row attention, pruning, late layers, decode."""
    s = (P.Session.for_workload(w, mode=mode, prune_before_layer=first_late, max_seq_late=max_seq_late) if max_seq_late
         else P.Session.for_workload(w, mode=mode))
    reset_session(s, w, caps, paged=paged)
    pools = None
    if paged:                                   # pages follow the unpruned lengths: one list serves every layer
        from stack_runner import oracle_page_pools
        pools = oracle_page_pools(w, mode)
        pools.prefill(range(w.batch), w.seq_len, w.vis_len)
    stacks = [PrunedStackOracle(w.n_layers, w.n_heads, w.head_dim, w.lazy_mask, w.vis_start[b], w.vis_len[b],
                                first_late, keep[b], mode=mode) for b in range(w.batch)]
    cu = w.cu_seqlens
    gla = mode == "gla"
    worst = 0.0
    row_map = row_map_host = None
    late_lens = [w.seq_len[b] - w.vis_len[b] + keep[b] for b in range(w.batch)]
    cu_late = cu_of(late_lens)
    # the ranking comes from the last early layer that holds all of its keys (a lazy layer does not)
    rank_layer = max(l for l in range(first_late) if not w.lazy_mask[l])
    for l in range(w.n_layers):
        q, k, v = workloads.prefill_qkv(w, l)
        qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
        q64, k64, v64 = (workloads.to_f64(t) for t in (q, k, v))
        if l >= first_late:                 # the caller drops the pruned rows of whatever it feeds the late layers
            n = len(row_map_host)
            eb = vg.element_size() * w.n_heads * w.head_dim
            dropped = []
            for t in (qg, kg, vg):
                d = torch.empty((n,) + tuple(t.shape[1:]), dtype=t.dtype, device="cuda")
                B.qc_gather_rows(t, eb, row_map, n, eb, d, eb)
                dropped.append(d)
            qg, kg, vg = dropped
            q64, k64, v64 = q64[row_map_host], k64[row_map_host], v64[row_map_host]
            cu_l = cu_late
        else:
            cu_l = cu
        ref = np.concatenate([stacks[b].prefill(l, q64[cu_l[b]:cu_l[b + 1]], k64[cu_l[b]:cu_l[b + 1]],
                                                v64[cu_l[b]:cu_l[b + 1]]) for b in range(w.batch)], axis=0)
        if gla and w.lazy_mask[l]:
            qg = kg = None
        out = s.prefill(l, qg, kg, vg, cu_l)
        err = max_abs_err(out, ref)
        assert np.isfinite(err)
        worst = max(worst, err)
        if l == rank_layer:
            # ranking: the last prompt token's attention in that layer, read in the middle of the pass
            q_last = torch.stack([q[cu[b + 1] - 1] for b in range(w.batch)]).contiguous().cuda()
            ws = torch.empty(B.qc_select_workspace_bytes(s.cfg), dtype=torch.uint8, device="cuda")
            stride = max(w.max_seq, max(w.seq_len)) + 5
            probs = torch.zeros((w.batch, stride), dtype=torch.float32, device="cuda")
            B.qc_last_row_attention(s.kv, l, q_last, probs, stride, 0.0, ws, ws.numel())
            torch.cuda.synchronize()
            p_host = probs.cpu().numpy()
            for b in range(w.batch):
                K = np.transpose(k64[cu[b]:cu[b + 1]], (1, 0, 2))
                want_p = selection.last_row_attention(q64[cu[b + 1] - 1], K, 1.0 / np.sqrt(w.head_dim))
                assert np.all(np.abs(p_host[b, :w.seq_len[b]] - want_p) <= 1e-5 + 1e-4 * want_p)
            kept = [kept_visual_positions(p_host[b], w.vis_start[b], w.vis_len[b], keep[b]) for b in range(w.batch)]
            row_map_host = packed_row_map(w.seq_len, w.vis_start, w.vis_len, kept)
            row_map = torch.empty(len(row_map_host), dtype=torch.int32, device="cuda")
            B.qc_prune_select(probs, stride, w.batch, cu, w.vis_start, w.vis_len, keep, row_map)
            torch.cuda.synchronize()
            assert np.array_equal(row_map.cpu().numpy(), row_map_host)
        if l == first_late - 1:
            s.prune(first_late, keep)
    graph = bufs = None
    if use_graph:                              # decode steps as replays of one graph recorded behind the boundary
        shape = (w.batch, w.n_heads, w.head_dim)
        mk = lambda: [torch.zeros(shape, dtype=workloads.TORCH_DTYPE[w.dtype], device="cuda") for _ in range(w.n_layers)]
        bufs = [mk(), mk(), mk(), mk()]
        if gla:
            for i in (0, 1):
                bufs[i] = [None if w.lazy_mask[l] else bufs[i][l] for l in range(w.n_layers)]
        graph = s.decode_graph(*bufs)
    for t in range(decode_steps):
        if paged:
            pools.decode_step(range(w.batch), [n + t for n in w.seq_len], w.vis_len)
        ins = [workloads.decode_qkv(w, l, t) for l in range(w.n_layers)]
        if use_graph:
            for l in range(w.n_layers):
                if bufs[0][l] is not None:
                    bufs[0][l].copy_(ins[l][0]); bufs[1][l].copy_(ins[l][1])
                bufs[2][l].copy_(ins[l][2])
            s.graph_launch(graph)
            torch.cuda.synchronize()
        for l in range(w.n_layers):
            q, k, v = ins[l]
            q64, k64, v64 = (workloads.to_f64(x) for x in (q, k, v))
            ref = np.stack([stacks[b].decode(l, q64[b], k64[b], v64[b]) for b in range(w.batch)], axis=0)
            if use_graph:
                out = bufs[3][l]
            else:
                qg, kg = q.cuda(), k.cuda()
                if gla and w.lazy_mask[l]:
                    qg = kg = None
                out = s.decode(l, qg, kg, v.cuda())
            err = max_abs_err(out, ref)
            assert np.isfinite(err)
            worst = max(worst, err)
    torch.cuda.synchronize()
    lay = oracle_layout(w, mode, caps, late=(first_late, max_seq_late) if max_seq_late else None,
                        paged=pools.tables() if paged else None)
    if paged:
        from stack_runner import check_page_lists
        check_page_lists(s, pools)
    assert np.array_equal(s.kv_arena[: lay.rows_bytes()].cpu().numpy(), olayout.kv_rows_image(lay, stacks)), "K/V rows differ"
    assert np.array_equal(s.q_arena.cpu().numpy()[: lay.q_arena_bytes()], olayout.q_arena_image(lay, stacks)), "Q arena differs"
    res = olayout.resident_bytes(lay, stacks)
    st = s.stats()
    for key in ("k_bytes", "v_bytes", "q_bytes", "tokens"):
        assert st[key] == res[key], key
    assert st["q_owner"] == stacks[0].q_owner
    # per-layer rows and key locations as the oracle's stacks hold them
    for l in range(w.n_layers):
        rk, rv = B.qc_layer_rows(s.kv, l)
        assert rk == sum(st_.Kc[l].shape[1] for st_ in stacks) and rv == sum(st_.Vc[l].shape[1] for st_ in stacks)
    print("pruned %s %s: worst |err| %.3g" % (mode, w.dtype, worst), flush=True)
    return worst


MASK6 = [0, 0, 1, 0, 1, 1]


@pytest.mark.parametrize("mode", ["vla", "gla"])
@pytest.mark.parametrize("use_graph", [False, True])
def test_pruned_stack_on_pages_matches_oracle(mode, use_graph):
    """Token pruning on a paged batch: the layers behind the boundary use the first rows of the same page
    lists (pages follow the unpruned lengths); decode steps cross a page boundary."""
    lens, vs, vl = [150, 97, 64], [5, 0, 20], [100, 80, 0]
    w = workloads.custom("pruned_paged", 6, 3, 128, "bf16", vs, vl, lens, 3, MASK6, seed_tag=21,
                         max_seq=192, max_vis=128, max_text=128)
    worst = run_pruned_parity(w, 3, [37, 80, 0], mode, 3, paged=True, use_graph=use_graph)
    assert worst <= TOL["bf16"]


@pytest.mark.parametrize("mode", ["vla", "gla"])
@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128)])
def test_pruned_stack_matches_oracle(mode, dtype, D):
    lens, vs, vl = [150, 97, 64], [5, 0, 20], [100, 80, 0]
    w = workloads.custom("pruned", 6, 3, D, dtype, vs, vl, lens, 3, MASK6, seed_tag=21)
    worst = run_pruned_parity(w, 3, [37, 80, 0], mode, 3)
    assert worst <= TOL[dtype]


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_pruned_stack_large_batch_and_boundary_after_first_layer(mode):
    """More than 8 sequences (per-sequence integers come from device memory) and a boundary after layer 0."""
    n = 11
    lens = [70 + 9 * i for i in range(n)]
    vl = [40 + 3 * i for i in range(n)]
    vs = [i % 4 for i in range(n)]
    keep = [(7 * i) % 40 for i in range(n)]
    w = workloads.custom("pruned_b11", 4, 2, 64, "bf16", vs, vl, lens, 2, [0, 0, 1, 1], seed_tag=22)
    assert run_pruned_parity(w, 1, keep, mode, 2) <= TOL["bf16"]


def test_prune_validation():
    w = workloads.custom("pruned_val", 4, 2, 64, "f32", [2], [10], [20], 2, [0, 0, 1, 0], seed_tag=23)
    s = P.Session.for_workload(w)
    s.reset(w.vis_start, w.vis_len)
    with pytest.raises(B.QcError) as e:
        B.qc_prune(s.kv, s.qc, [5])                       # no layer has run yet
    assert e.value.status == B.QC_EORDER
    qkv = [tuple(t.cuda() for t in workloads.prefill_qkv(w, l)) for l in range(4)]
    s.prefill(0, *qkv[0], w.cu_seqlens)
    with pytest.raises(B.QcError) as e:
        B.qc_prune(s.kv, s.qc, [11])                      # more than the span holds
    assert e.value.status == B.QC_EINVAL
    s.prefill(1, *qkv[1], w.cu_seqlens)
    with pytest.raises(B.QcError) as e:
        B.qc_prune(s.kv, s.qc, [5])                       # layer 2 is lazy
    assert e.value.status == B.QC_EINVAL
    s.prefill(2, *qkv[2], w.cu_seqlens)
    s.prune(3, [5])
    with pytest.raises(B.QcError) as e:
        B.qc_prune(s.kv, s.qc, [4])                       # one boundary per pass
    assert e.value.status == B.QC_EORDER
    with pytest.raises(B.QcError) as e:
        s.prefill(3, *qkv[3], w.cu_seqlens)               # still the unpruned prompt
    assert e.value.status == B.QC_EINVAL
    short = tuple(t[:15].contiguous() for t in qkv[3])
    with pytest.raises(B.QcError) as e:                   # span arrays must name the kept count
        B.qc_prefill(s.kv, s.qc, 3, 0, *short, torch.empty_like(short[2]), [0, 15], short[2].stride(0),
                     short[2].stride(1), w.vis_start, w.vis_len)
    assert e.value.status == B.QC_EINVAL
    s.prefill(3, *short, [0, 15])
    assert B.qc_seq_len(s.kv, 0) == 20
    assert B.qc_layer_rows(s.kv, 3) == (15, 15) and B.qc_layer_rows(s.kv, 0) == (20, 20)
    with pytest.raises(B.QcError) as e:
        B.qc_prune(s.kv, s.qc, [5])                       # the pass is over
    assert e.value.status == B.QC_EORDER
    s.reset(w.vis_start, w.vis_len)                       # a new batch starts unpruned
    s.prefill(0, *qkv[0], w.cu_seqlens)
    s.prefill(1, *qkv[1], w.cu_seqlens)
    s.prefill(2, *qkv[2], w.cu_seqlens)
    s.prefill(3, *qkv[3], w.cu_seqlens)
    assert B.qc_layer_rows(s.kv, 3) == (20, 20)


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_pruned_stack_with_smaller_late_layers(mode):
    """The boundary is known when the caches are sized: the layers behind it get regions for the
    shortened sequences only, and the whole arena still matches the oracle's image byte for byte."""
    lens, vs, vl, keep = [150, 97, 64], [5, 0, 20], [100, 80, 0], [37, 20, 0]
    steps = 3
    w = workloads.custom("pruned_late", 6, 3, 128, "bf16", vs, vl, lens, steps, MASK6, seed_tag=24)
    late_cap = max(L - v + k for L, v, k in zip(lens, vl, keep)) + steps
    assert late_cap < w.max_seq
    plain = P.make_config(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.batch, w.max_seq, w.max_vis, w.max_text, w.lazy_mask,
                          mode=mode)
    small = P.make_config(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.batch, w.max_seq, w.max_vis, w.max_text, w.lazy_mask,
                          mode=mode, prune_before_layer=3, max_seq_late=late_cap)
    assert B.qc_kv_arena_bytes(small) < B.qc_kv_arena_bytes(plain)
    assert run_pruned_parity(w, 3, keep, mode, steps, max_seq_late=late_cap) <= TOL["bf16"]


def test_smaller_late_layers_validation():
    w = workloads.custom("late_val", 4, 2, 64, "f32", [2], [10], [20], 2, [0, 0, 1, 0], seed_tag=25)
    mk = lambda **kw: P.make_config(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.batch, w.max_seq, w.max_vis, w.max_text,
                                    w.lazy_mask, **kw)
    assert B.qc_kv_arena_bytes(mk(prune_before_layer=2, max_seq_late=12)) == 0       # layer 2 is lazy
    assert B.qc_kv_arena_bytes(mk(prune_before_layer=0, max_seq_late=12)) == 0       # capacity without a boundary
    assert B.qc_kv_arena_bytes(mk(prune_before_layer=3, max_seq_late=0)) == 0
    assert B.qc_kv_arena_bytes(mk(prune_before_layer=3, max_seq_late=w.max_seq + 1)) == 0
    s = P.Session.for_workload(w, prune_before_layer=3, max_seq_late=17)
    s.reset(w.vis_start, w.vis_len)
    qkv = [tuple(t.cuda() for t in workloads.prefill_qkv(w, l)) for l in range(4)]
    s.prefill(0, *qkv[0], w.cu_seqlens)
    with pytest.raises(B.QcError) as e:
        B.qc_prune(s.kv, s.qc, [5])                       # the configuration expects the boundary before layer 3
    assert e.value.status == B.QC_EINVAL
    s.prefill(1, *qkv[1], w.cu_seqlens)
    s.prefill(2, *qkv[2], w.cu_seqlens)
    with pytest.raises(B.QcError) as e:
        s.prefill(3, *qkv[3], w.cu_seqlens)               # unpruned: 20 tokens do not fit the late layers' 17 rows
    assert e.value.status == B.QC_ECAPACITY
    s.prune(3, [5])
    short = tuple(t[:15].contiguous() for t in qkv[3])
    s.prefill(3, *short, [0, 15])
    ins = [t.cuda() for t in workloads.decode_qkv(w, 0, 0)]
    for t in range(2):
        for l in range(4):
            s.decode(l, *ins)
    with pytest.raises(B.QcError) as e:                   # 17 rows in the late layers: a third step does not fit
        s.decode(0, *ins)
    assert e.value.status == B.QC_ECAPACITY
    with pytest.raises(B.QcError) as e:
        B.qc_reset_ragged(s.kv, s.qc, 1, [2], [10], [24], [12], 0, torch.cuda.current_stream().cuda_stream)
    assert e.value.status == B.QC_EINVAL
    s.close()
