"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The whole tensors are too large for the fp64 oracle, so a few (sequence, head) pairs are run
through oracle instances of their own (heads are independent) and compared on sampled query
rows; the cache rows of those heads are compared bit for bit.
"""
import numpy as np
import pytest
import torch

import paper_2602_01901_amd as P
from paper_2602_01901_amd import binding as B
import workloads
from oracle.global_lazy_stack import GlobalLazyStackOracle
from oracle.lazy_stack import LazyStackOracle
from stack_runner import TOL

pytestmark = pytest.mark.gpu


def sample_rows(w, b, rng, extra=6):
    L, s, vn = w.seq_len[b], w.vis_start[b], w.vis_len[b]
    rows = {0, 1, L - 1, L - 2, max(s - 1, 0), s, min(s + 1, L - 1), s + vn - 1, min(s + vn, L - 1), 63, 64, 127, 128, 255, 256}
    rows |= set(int(x) for x in rng.integers(0, L, size=extra))
    return sorted(r for r in rows if 0 <= r < L)


def head_slice(t, w, b, h):
    cu = w.cu_seqlens
    return workloads.to_f64(t[cu[b]:cu[b + 1], h:h + 1, :])


def arena_rows(sess, which, layer, b, h, pos_list):
    """Cache rows as the library locates them, as raw int16/int32 words."""
    rowb = sess.head_dim * (2 if sess.dtype == "bf16" else 4)
    out = []
    for pos in pos_list:
        src, off = B.qc_locate(sess.kv, which, layer, b, h, pos)
        out.append(sess.kv_arena[off:off + rowb].clone())
    return torch.stack(out).cpu().numpy()


def run_sampled(w, n_layers, pairs, decode_steps=0, seed=0, mode="vla", paged=False):
    rng = np.random.default_rng(seed)
    gla = mode == "gla"
    sess = P.Session.for_workload(w, mode=mode)
    sess.reset(w.vis_start, w.vis_len, zero_fill=False, paged=paged)
    if gla:
        oracles = {p: GlobalLazyStackOracle(w.n_layers, 1, w.head_dim, w.lazy_mask) for p in pairs}
    else:
        oracles = {p: LazyStackOracle(w.n_layers, 1, w.head_dim, w.lazy_mask, w.vis_start[p[0]], w.vis_len[p[0]])
                   for p in pairs}
    rows = {p: sample_rows(w, p[0], rng) for p in pairs}
    worst = 0.0
    cu = w.cu_seqlens
    for l in range(n_layers):
        q, k, v = workloads.prefill_qkv(w, l, device="cuda")
        no_qk = gla and w.lazy_mask[l]
        out = sess.prefill(l, None if no_qk else q, None if no_qk else k, v, w.cu_seqlens)
        for (b, h) in pairs:
            ref = oracles[(b, h)].prefill(l, head_slice(q, w, b, h), head_slice(k, w, b, h), head_slice(v, w, b, h),
                                          rows=rows[(b, h)])
            got = workloads.to_f64(out[cu[b]:cu[b + 1], h, :][rows[(b, h)]])
            err = float(np.max(np.abs(got - ref[:, 0, :])))
            assert np.isfinite(err)
            worst = max(worst, err)
            # cache rows: bit-exact copies of the inputs, at the rows the library reports
            pos = rows[(b, h)]
            want_v = v[cu[b]:cu[b + 1], h, :][pos].contiguous().view(torch.uint8).cpu().numpy()
            assert np.array_equal(arena_rows(sess, B.QC_V, l, b, h, pos), want_v)
            st = oracles[(b, h)]
            if gla:   # every key of a lazy layer is the block's first layer's
                src_rows = [(st.first_layer_of_block(l) if w.lazy_mask[l] else l, p_) for p_ in pos]
            else:
                src_rows = [st.k_source(l, p_) for p_ in pos]
            got_k = arena_rows(sess, B.QC_K, l, b, h, pos)
            for n, (src, row) in enumerate(src_rows):
                want = st.Kc[src][0, row].astype(np.float32)
                gotf = torch.from_numpy(got_k[n].copy()).view(torch.bfloat16 if w.dtype == "bf16" else torch.float32)
                assert np.array_equal(gotf.float().numpy(), want), (l, b, h, pos[n])
        del q, k, v, out
    assert n_layers == w.n_layers or decode_steps == 0
    for t in range(decode_steps):
        for l in range(w.n_layers):
            q, k, v = workloads.decode_qkv(w, l, t, device="cuda")
            no_qk = gla and w.lazy_mask[l]
            out = sess.decode(l, None if no_qk else q, None if no_qk else k, v)
            for (b, h) in pairs:
                ref = oracles[(b, h)].decode(l, workloads.to_f64(q[b, h:h + 1]), workloads.to_f64(k[b, h:h + 1]),
                                             workloads.to_f64(v[b, h:h + 1]))
                err = float(np.max(np.abs(workloads.to_f64(out[b, h]) - ref[0])))
                assert np.isfinite(err)
                worst = max(worst, err)
    torch.cuda.synchronize()
    return worst, sess


def test_cfg4_highres_prefill_sampled():
    """Batch 8 x 3008 tokens (2880 visual), 32 heads: the 256-row prefill kernel, first 8 layers
    (two ordinary layers, then two blocks of one ordinary + two lazy layers)."""
    w = workloads.config(3)
    worst, sess = run_sampled(w, 8, [(0, 0), (1, 9), (3, 17), (4, 30), (6, 1), (7, 31)])
    print("cfg4 sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]
    rk, rv = B.qc_layer_rows(sess.kv, 3)
    assert rv == 8 * 3008 and rk == 8 * 128   # a lazy layer keeps text keys only


def test_cfg3_batched_decode_sampled():
    """Batch 32 with unequal lengths: full 32-layer prefill then 3 decode steps, sampled heads."""
    w = workloads.config(2)
    worst, sess = run_sampled(w, w.n_layers, [(0, 5), (7, 16), (13, 0), (20, 31), (26, 11), (31, 31)], decode_steps=3)
    print("cfg3 sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]
    st = sess.stats()
    want_k = sum((L + 3 - lz * 576) for L in w.seq_len for lz in w.lazy_mask) * 32 * 128 * 2
    assert st["k_bytes"] == want_k and st["tokens"] == sum(w.seq_len) + 3 * 32


def test_cfg3_batched_decode_sampled_on_pages():
    """The same on a paged batch, in the launch configuration the benchmark times; the page lists against
    the hand-out rule (three steps open no page at these lengths except where a length is a multiple of 64)."""
    import dataclasses
    from oracle.layout import PagePools
    w = workloads.config(2)
    w = dataclasses.replace(w, max_seq=-(-w.max_seq // 64) * 64, max_text=-(-w.max_text // 64) * 64)   # whole pages
    worst, sess = run_sampled(w, w.n_layers, [(0, 5), (7, 16), (13, 0), (20, 31), (26, 11), (31, 31)], decode_steps=3, paged=True)
    print("cfg3 paged sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]
    pools = PagePools(w.batch, w.max_seq, w.max_vis, w.max_text)
    pools.prefill(range(w.batch), w.seq_len, w.vis_len)
    for t in range(3):
        pools.decode_step(range(w.batch), [n + t for n in w.seq_len], w.vis_len)
    want = pools.tables()
    for pool, kind in enumerate(("seq", "text", "vis")):
        for b in range(w.batch):
            assert B.qc_seq_pages(sess.kv, b, pool) == want[kind][b], (kind, b)


def test_cfg4_highres_prefill_sampled_on_pages():
    w = workloads.config(3)
    worst, _ = run_sampled(w, 8, [(0, 0), (3, 17), (7, 31), (5, 8)], paged=True)
    print("cfg4 paged sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]


def test_cfg5_video_shape_sampled():
    """13B-shaped video workload: 40 heads, 4864-token prompts; first 5 layers of prefill."""
    w = workloads.config(4)
    worst, _ = run_sampled(w, 5, [(0, 39), (0, 0), (1, 20), (2, 33), (3, 7), (3, 39)])
    print("cfg5 sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]


def test_cfg5_video_shape_sampled_on_pages():
    """The same on a paged batch: 76 key tiles per prompt, 72 of them inside the span, so a lazy layer walks
    more than 64 pages of the first layer's keys."""
    w = workloads.config(4)
    assert w.max_seq % 64 == 0 and w.max_vis % 64 == 0 and w.max_text % 64 == 0
    worst, _ = run_sampled(w, 5, [(0, 39), (1, 0), (2, 20), (3, 39)], seed=9, paged=True)
    print("cfg5 paged sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]


def test_cfg5_decode_sampled():
    """13B-shaped video workload as bench.py times it: the full 40-layer prefill of 4 x 4864 tokens, then
    3 decode steps (8 key chunks per (sequence, head), merged), sampled heads including the last one."""
    w = workloads.config(4)
    pairs = [(0, 0), (0, 39), (1, 17), (2, 39), (3, 5), (3, 39)]
    worst, sess = run_sampled(w, w.n_layers, pairs, decode_steps=3, seed=5)
    print("cfg5 prefill + decode sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]
    st = sess.stats()
    per_row = 40 * 128 * 2
    assert st["tokens"] == 4 * (4864 + 3) and st["generated"] == 3
    assert st["k_bytes"] == sum((4864 + 3 - lz * 4608) for _ in range(4) for lz in w.lazy_mask) * per_row
    assert st["v_bytes"] == 40 * 4 * (4864 + 3) * per_row


def test_long_prompt_32k():
    """One 32768-token prompt (32000 visual), 8 heads: 256 query tiles per head and key walks of up to
    512 tiles; an ordinary layer then a lazy one, sampled rows."""
    w = workloads.custom("long", 2, 8, 128, "bf16", [256], [32000], [32768], 0, [0, 1])
    worst, sess = run_sampled(w, 2, [(0, 0), (0, 1), (0, 3), (0, 4), (0, 6), (0, 7)])
    print("long prompt sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]
    assert B.qc_layer_rows(sess.kv, 1) == (768, 32768)


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_long_prompt_32k_on_pages(mode):
    """The same prompt on a paged batch: 512 pages of positions, 500 of visual rows; the lazy layer walks the
    first layer's keys page by page through eight blocks of 64 pages."""
    w = workloads.custom("long_paged", 2, 8, 128, "bf16", [256], [32000], [32768], 0, [0, 1],
                         max_seq=32768, max_vis=32000, max_text=768)
    worst, sess = run_sampled(w, 2, [(0, 0), (0, 3), (0, 7)], seed=3, mode=mode, paged=True)
    print("long prompt on pages (%s) sampled max abs err %.3g" % (mode, worst), flush=True)
    assert worst <= TOL["bf16"]
    assert B.qc_seq_pages(sess.kv, 0, 0) == list(range(512))
    assert B.qc_pool_pages(sess.kv, 0) == (512, 0)


def test_gla_cfg4_highres_prefill_sampled():
    """Global Lazy Attention at batch 8 x 3008 tokens: every row of a lazy layer comes from the Q Cache and
    from the K cache of its block's first layer; first 8 layers."""
    w = workloads.config(3)
    worst, sess = run_sampled(w, 8, [(0, 0), (1, 9), (3, 17), (4, 30), (6, 1), (7, 31)], mode="gla")
    print("gla cfg4 sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]
    assert B.qc_layer_rows(sess.kv, 3) == (0, 8 * 3008)   # a lazy layer keeps no keys at all


def test_gla_cfg3_batched_decode_sampled():
    """Global Lazy Attention, batch 32 with unequal lengths: full prefill then 3 decode steps in which the
    lazy layers reuse their block's scores."""
    w = workloads.config(2)
    worst, sess = run_sampled(w, w.n_layers, [(0, 5), (7, 16), (13, 0), (20, 31), (26, 11), (31, 31)], decode_steps=3, mode="gla")
    print("gla cfg3 sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]
    st = sess.stats()
    per_row = 32 * 128 * 2
    tokens = sum(w.seq_len) + 3 * 32
    assert st["tokens"] == tokens
    assert st["k_bytes"] == (w.n_layers - w.n_lazy) * tokens * per_row and st["q_bytes"] == tokens * per_row


def test_cfg2_headline_decode_graph_sampled():
    """The headline configuration as bench.py times it: 32 layers, batch 1, 640-token prompt, decode steps
    replayed from the HIP graph (one replay per step), sampled heads against the oracle at every step."""
    w = workloads.config(1)
    pairs = [(0, 0), (0, 7), (0, 13), (0, 18), (0, 26), (0, 31)]
    sess = P.Session.for_workload(w)
    sess.reset(w.vis_start, w.vis_len, zero_fill=False)
    oracles = {p: LazyStackOracle(w.n_layers, 1, w.head_dim, w.lazy_mask, w.vis_start[0], w.vis_len[0]) for p in pairs}
    for l in range(w.n_layers):
        q, k, v = workloads.prefill_qkv(w, l, device="cuda")
        sess.prefill(l, q, k, v, w.cu_seqlens)
        for p in pairs:
            oracles[p].prefill(l, head_slice(q, w, 0, p[1]), head_slice(k, w, 0, p[1]), head_slice(v, w, 0, p[1]), rows=[0])
    shape = (1, w.n_heads, w.head_dim)
    mk = lambda: [torch.zeros(shape, dtype=torch.bfloat16, device="cuda") for _ in range(w.n_layers)]
    qb, kb, vb, ob = mk(), mk(), mk(), mk()
    g = sess.decode_graph(qb, kb, vb, ob)
    worst = 0.0
    steps = 24
    for t in range(steps):
        ins = [workloads.decode_qkv(w, l, t, device="cuda") for l in range(w.n_layers)]
        for l in range(w.n_layers):
            qb[l].copy_(ins[l][0]); kb[l].copy_(ins[l][1]); vb[l].copy_(ins[l][2])
        sess.graph_launch(g)
        torch.cuda.synchronize()
        for l in range(w.n_layers):
            q, k, v = ins[l]
            for (b, h) in pairs:
                ref = oracles[(b, h)].decode(l, workloads.to_f64(q[b, h:h + 1]), workloads.to_f64(k[b, h:h + 1]),
                                             workloads.to_f64(v[b, h:h + 1]))
                err = float(np.max(np.abs(workloads.to_f64(ob[l][b, h]) - ref[0])))
                assert np.isfinite(err) and err <= TOL["bf16"], (t, l, h, err)
                worst = max(worst, err)
    print("cfg2 graph replays sampled max abs err %.3g" % worst, flush=True)
    st = sess.stats()
    assert st["generated"] == steps and st["tokens"] == 640 + steps
    sess.close()


def test_cfg3_pruned_decode_sampled():
    """The pruning configuration bench.py times: cfg3 (batch 32), boundary before layer 2, half of every
    image kept by the last prompt token's attention in layer 1; 32-layer prefill and 2 decode steps."""
    from oracle.pruning import PrunedStackOracle, kept_visual_positions, packed_row_map
    w = workloads.config(2)
    first_late, rank_layer = 2, 1
    keep = [v // 2 for v in w.vis_len]
    pairs = [(0, 5), (7, 16), (13, 0), (20, 31), (26, 11), (31, 31)]
    rng = np.random.default_rng(4)
    sess = P.Session.for_workload(w)
    sess.reset(w.vis_start, w.vis_len, zero_fill=False)
    oracles = {p: PrunedStackOracle(w.n_layers, 1, w.head_dim, w.lazy_mask, w.vis_start[p[0]], w.vis_len[p[0]],
                                    first_late, keep[p[0]]) for p in pairs}
    cu = w.cu_seqlens
    late_len = [L - v + k for L, v, k in zip(w.seq_len, w.vis_len, keep)]
    cu_late = [0]
    for n in late_len:
        cu_late.append(cu_late[-1] + n)
    worst = 0.0
    row_map = row_map_host = None
    for l in range(w.n_layers):
        q, k, v = workloads.prefill_qkv(w, l, device="cuda")
        late = l >= first_late
        if late:
            eb = w.n_heads * w.head_dim * 2
            parts = []
            for t in (q, k, v):
                d = torch.empty((cu_late[-1],) + tuple(t.shape[1:]), dtype=t.dtype, device="cuda")
                B.qc_gather_rows(t, eb, row_map, cu_late[-1], eb, d, eb)
                parts.append(d)
            q, k, v = parts
        cu_l = cu_late if late else cu
        out = sess.prefill(l, q, k, v, cu_l)
        for (b, h) in pairs:
            Lb = cu_l[b + 1] - cu_l[b]
            rows = sorted(set([0, Lb - 1, Lb // 2] + [int(x) for x in rng.integers(0, Lb, size=4)]))
            sl = lambda t: workloads.to_f64(t[cu_l[b]:cu_l[b + 1], h:h + 1, :])
            ref = oracles[(b, h)].prefill(l, sl(q), sl(k), sl(v), rows=rows)
            got = workloads.to_f64(out[cu_l[b]:cu_l[b + 1], h, :][rows])
            err = float(np.max(np.abs(got - ref[:, 0, :])))
            assert np.isfinite(err)
            worst = max(worst, err)
        if l == rank_layer:
            q_last = torch.stack([q[cu[b + 1] - 1] for b in range(w.batch)]).contiguous()
            ws = torch.empty(B.qc_select_workspace_bytes(sess.cfg), dtype=torch.uint8, device="cuda")
            stride = w.max_seq
            probs = torch.zeros((w.batch, stride), dtype=torch.float32, device="cuda")
            B.qc_last_row_attention(sess.kv, l, q_last, probs, stride, 0.0, ws, ws.numel())
            row_map = torch.empty(cu_late[-1], dtype=torch.int32, device="cuda")
            B.qc_prune_select(probs, stride, w.batch, cu, w.vis_start, w.vis_len, keep, row_map)
            torch.cuda.synchronize()
            p_host = probs.cpu().numpy()
            kept = [kept_visual_positions(p_host[b], w.vis_start[b], w.vis_len[b], keep[b]) for b in range(w.batch)]
            row_map_host = packed_row_map(w.seq_len, w.vis_start, w.vis_len, kept)
            assert np.array_equal(row_map.cpu().numpy(), row_map_host)
        if l == first_late - 1:
            sess.prune(first_late, keep)
        del q, k, v, out
    for t in range(2):
        for l in range(w.n_layers):
            q, k, v = workloads.decode_qkv(w, l, t, device="cuda")
            out = sess.decode(l, q, k, v)
            for (b, h) in pairs:
                ref = oracles[(b, h)].decode(l, workloads.to_f64(q[b, h:h + 1]), workloads.to_f64(k[b, h:h + 1]),
                                             workloads.to_f64(v[b, h:h + 1]))
                err = float(np.max(np.abs(workloads.to_f64(out[b, h]) - ref[0])))
                assert np.isfinite(err)
                worst = max(worst, err)
    print("cfg3 pruned sampled max abs err %.3g" % worst, flush=True)
    assert worst <= TOL["bf16"]
    per_row = 32 * 128 * 2
    st = sess.stats()
    want_v = sum((2 * (L + 2) + 30 * (Ll + 2)) for L, Ll in zip(w.seq_len, late_len)) * per_row
    assert st["v_bytes"] == want_v
