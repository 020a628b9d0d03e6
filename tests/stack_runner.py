"""Drive the same seeded workload through the HIP library and through the CPU oracle."""
import numpy as np
import torch

import workloads
from oracle import layout as olayout
from oracle.global_lazy_stack import GlobalLazyStackOracle
from oracle.lazy_stack import LazyStackOracle

TOL = {"f32": 1e-4, "bf16": 3e-2}   # max-abs-error bars for outputs (fp32 / bf16 storage)


def oracle_layout(w, mode="vla", caps=None, late=None, paged=None):
    """caps: None, or (cap_seq, cap_text) per sequence (the Q arena is then split by vis_len).
    late: None, or (first late layer, max_seq_late) of a configuration with smaller late layers.
    paged: None, or the page lists per pool and slot (oracle.layout.PagePools.tables())."""
    ragged = None if caps is None else (caps[0], caps[1], w.vis_len)
    return olayout.ArenaLayout(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.batch, w.max_seq, w.max_vis,
                               w.max_text, w.lazy_mask, mode=mode, ragged=ragged, late=late, paged=paged)


def oracle_page_pools(w, mode="vla"):
    return olayout.PagePools(w.batch, w.max_seq, w.max_vis, w.max_text, mode=mode, any_lazy=any(w.lazy_mask))


def check_page_lists(session, pools):
    """The library hands out the pages the stated rule hands out."""
    from paper_2602_01901_amd import binding as B
    want = pools.tables()
    for pool, kind in enumerate(("seq", "text", "vis")):
        for b in range(len(want[kind])):
            assert B.qc_seq_pages(session.kv, b, pool) == want[kind][b], (kind, b)
        if kind in pools._kinds():
            held = sum(len(x) for x in want[kind])
            assert B.qc_pool_pages(session.kv, pool) == (held + len(pools.free[kind]), len(pools.free[kind])), kind
        else:
            assert B.qc_pool_pages(session.kv, pool) == (0, 0), kind


def reset_session(session, w, caps=None, zero_fill=True, paged=False):
    if paged:
        session.reset(w.vis_start, w.vis_len, zero_fill=zero_fill, paged=True)
    elif caps is None:
        session.reset(w.vis_start, w.vis_len, zero_fill=zero_fill)
    else:
        session.reset(w.vis_start, w.vis_len, zero_fill=zero_fill, cap_seq=caps[0], cap_text=caps[1])


def new_oracles(w, heads=None, mode="vla"):
    H = w.n_heads if heads is None else len(heads)
    if mode == "gla":
        return [GlobalLazyStackOracle(w.n_layers, H, w.head_dim, w.lazy_mask, vis_start=w.vis_start[b],
                                      vis_len=w.vis_len[b]) for b in range(w.batch)]
    return [LazyStackOracle(w.n_layers, H, w.head_dim, w.lazy_mask, w.vis_start[b], w.vis_len[b])
            for b in range(w.batch)]


def oracle_prefill_layer(w, stacks, layer, q, k, v):
    """q, k, v: torch tensors [tokens, H, D] (any device).  Returns fp64 [tokens, H, D]."""
    q64, k64, v64 = (workloads.to_f64(t) for t in (q, k, v))
    cu = w.cu_seqlens
    outs = [stacks[b].prefill(layer, q64[cu[b]:cu[b + 1]], k64[cu[b]:cu[b + 1]], v64[cu[b]:cu[b + 1]])
            for b in range(w.batch)]
    return np.concatenate(outs, axis=0)


def oracle_decode_layer(w, stacks, layer, q, k, v):
    q64, k64, v64 = (workloads.to_f64(t) for t in (q, k, v))
    return np.stack([stacks[b].decode(layer, q64[b], k64[b], v64[b]) for b in range(w.batch)], axis=0)


def check_kv_rows(session, lay, stacks):
    """The K and V row regions byte for byte against the oracle's image, and what the library keeps of
    each sequence beside them through its own queries (the oracle does not describe those bytes)."""
    want = olayout.kv_rows_image(lay, stacks)
    got = session.kv_arena[: lay.rows_bytes()].cpu().numpy()
    assert got.shape == want.shape
    assert np.array_equal(got, want), "K/V rows differ from the oracle's image"
    from paper_2602_01901_amd import binding as B
    for b, st in enumerate(stacks):
        late = getattr(st, "late", None)        # a stack pruned between two layers keeps its unpruned length in `early`
        want_len = (st.early.len if late is not None and hasattr(st, "early") else st.len)
        if want_len:
            assert B.qc_seq_len(session.kv, b) == want_len, b
    for l in range(lay.N):
        rk, rv = B.qc_layer_rows(session.kv, l)
        assert rk == sum(st.Kc[l].shape[1] for st in stacks), l
        assert rv == sum(st.Vc[l].shape[1] for st in stacks), l


def max_abs_err(gpu_tensor, ref64):
    return float(np.max(np.abs(workloads.to_f64(gpu_tensor) - ref64)))


def run_full_parity(w, decode_steps, session, poison_span=False, check_arena=True, caps=None, zero_fill=True,
                    paged=False):
    """Prefill every layer then `decode_steps` decode steps on both sides; returns worst errors.

    With poison_span the span rows of q and k handed to lazy layers hold NaN on the GPU side
    (the oracle gets the clean tensors): lazy layers must never read them.  A session in "gla"
    mode is checked against the Global Lazy Attention oracle; its lazy layers get no q and k at
    all (None), or, with poison_span, tensors that are NaN everywhere.
    """
    dev = session.device
    mode = session.mode
    gla = mode == "gla"
    stacks = new_oracles(w, mode=mode)
    reset_session(session, w, caps, zero_fill=zero_fill, paged=paged)
    pools = oracle_page_pools(w, mode) if paged else None
    if paged:
        pools.prefill(range(w.batch), w.seq_len, w.vis_len)
    worst_p = worst_d = 0.0
    for l in range(w.n_layers):
        q, k, v = workloads.prefill_qkv(w, l)
        ref = oracle_prefill_layer(w, stacks, l, q, k, v)
        qg, kg, vg = q.to(dev), k.to(dev), v.to(dev)
        if gla and w.lazy_mask[l]:
            qg, kg = (qg * float("nan"), kg * float("nan")) if poison_span else (None, None)
        elif poison_span and w.lazy_mask[l]:
            cu = w.cu_seqlens
            for b in range(w.batch):
                s, e = cu[b] + w.vis_start[b], cu[b] + w.vis_start[b] + w.vis_len[b]
                qg[s:e] = float("nan")
                kg[s:e] = float("nan")
        out = session.prefill(l, qg, kg, vg, w.cu_seqlens)
        err = max_abs_err(out, ref)
        assert np.isfinite(err), "layer %d produced non-finite output" % l
        worst_p = max(worst_p, err)
    for t in range(decode_steps):
        if paged:
            pools.decode_step(range(w.batch), [n + t for n in w.seq_len], w.vis_len)
        for l in range(w.n_layers):
            q, k, v = workloads.decode_qkv(w, l, t)
            ref = oracle_decode_layer(w, stacks, l, q, k, v)
            qg, kg = q.to(dev), k.to(dev)
            if gla and w.lazy_mask[l]:
                qg, kg = (qg * float("nan"), kg * float("nan")) if poison_span else (None, None)
            out = session.decode(l, qg, kg, v.to(dev))
            err = max_abs_err(out, ref)
            assert np.isfinite(err)
            worst_d = max(worst_d, err)
    torch.cuda.synchronize()
    if paged:
        check_page_lists(session, pools)
    if check_arena:
        lay = oracle_layout(w, mode, caps, paged=pools.tables() if paged else None)
        check_kv_rows(session, lay, stacks)
        want_q = olayout.q_arena_image(lay, stacks)
        got_q = session.q_arena.cpu().numpy()[: lay.q_arena_bytes()]
        assert np.array_equal(got_q, want_q), "Q Cache arena differs from the oracle's image"
        res = olayout.resident_bytes(lay, stacks)
        st = session.stats()
        for key in ("k_bytes", "v_bytes", "q_bytes", "tokens"):
            assert st[key] == res[key], key
        assert st["q_owner"] == stacks[0].q_owner
    return worst_p, worst_d
