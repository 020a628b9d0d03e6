"""GPU parity for decode steps replayed from a HIP graph (qc_decode_graph_*) against the CPU oracle.

Every replay is checked, with eager work (input copies, ordinary qc_decode steps) and
synchronisations between replays; the caches must end up byte for byte as the oracle's image."""
import numpy as np
import pytest
import torch

import paper_2602_01901_amd as P
from paper_2602_01901_amd import binding as B
import workloads
from oracle import layout as olayout
from stack_runner import (TOL, check_kv_rows, max_abs_err, new_oracles, oracle_decode_layer, oracle_layout, oracle_prefill_layer,
                          reset_session)

pytestmark = pytest.mark.gpu


def prefill_both(w, s, stacks, mode, caps=None):
    reset_session(s, w, caps)
    for l in range(w.n_layers):
        q, k, v = workloads.prefill_qkv(w, l)
        oracle_prefill_layer(w, stacks, l, q, k, v)
        qg, kg = q.cuda(), k.cuda()
        if mode == "gla" and w.lazy_mask[l]:
            qg = kg = None
        s.prefill(l, qg, kg, v.cuda(), w.cu_seqlens)


def step_buffers(w, mode):
    shape = (w.batch, w.n_heads, w.head_dim)
    dt = workloads.TORCH_DTYPE[w.dtype]
    mk = lambda: [torch.zeros(shape, dtype=dt, device="cuda") for _ in range(w.n_layers)]
    q, k, v, out = mk(), mk(), mk(), mk()
    if mode == "gla":
        q = [None if w.lazy_mask[l] else q[l] for l in range(w.n_layers)]
        k = [None if w.lazy_mask[l] else k[l] for l in range(w.n_layers)]
    return q, k, v, out


def run_steps(w, s, stacks, mode, graph, bufs, schedule, t0=0):
    """schedule: one letter per step, 'g' = graph replay, 'e' = ordinary qc_decode calls.  Returns the worst error."""
    q, k, v, out = bufs
    worst = 0.0
    for i, kind in enumerate(schedule):
        t = t0 + i
        ins = [workloads.decode_qkv(w, l, t) for l in range(w.n_layers)]
        refs = [oracle_decode_layer(w, stacks, l, *ins[l]) for l in range(w.n_layers)]
        if kind == "g":
            for l in range(w.n_layers):
                if q[l] is not None:
                    q[l].copy_(ins[l][0])
                    k[l].copy_(ins[l][1])
                v[l].copy_(ins[l][2])
                out[l].zero_()
            s.graph_launch(graph)
            torch.cuda.synchronize()
            got = out
        else:
            got = []
            for l in range(w.n_layers):
                skip = mode == "gla" and w.lazy_mask[l]
                got.append(s.decode(l, None if skip else ins[l][0].cuda(), None if skip else ins[l][1].cuda(), ins[l][2].cuda()))
            torch.cuda.synchronize()
        for l in range(w.n_layers):
            err = max_abs_err(got[l], refs[l])
            assert np.isfinite(err) and err <= TOL[w.dtype], (t, kind, l, err)
            worst = max(worst, err)
    return worst


def check_caches(w, s, stacks, mode, caps=None):
    lay = oracle_layout(w, mode, caps)
    check_kv_rows(s, lay, stacks)
    assert np.array_equal(s.q_arena.cpu().numpy()[: lay.q_arena_bytes()], olayout.q_arena_image(lay, stacks)), "Q arena differs"
    res = olayout.resident_bytes(lay, stacks)
    st = s.stats()
    for key in ("k_bytes", "v_bytes", "q_bytes", "tokens"):
        assert st[key] == res[key], key
    assert st["q_owner"] == stacks[0].q_owner


CASES = [
    # name, layers, heads, D, dtype, vis_start, vis_len, seq_len, mask
    ("split_f32", 4, 8, 64, "f32", [8], [144], [176], [0, 0, 1, 1]),                       # 3 key chunks per head, merged
    ("ragged_bf16", 5, 4, 128, "bf16", [3, 0, 10], [60, 0, 33], [130, 70, 65], [0, 1, 0, 1, 1]),
    ("batch11_bf16", 3, 2, 64, "bf16", [i % 3 for i in range(11)], [20 + i for i in range(11)], [40 + 5 * i for i in range(11)], [0, 1, 1]),
]


@pytest.mark.parametrize("mode", ["vla", "gla"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_graph_replays_match_oracle(case, mode):
    name, N, H, D, dtype, vs, vl, lens, mask = case
    w = workloads.custom(name, N, H, D, dtype, vs, vl, lens, 7, mask, seed_tag=31)
    s = P.Session.for_workload(w, mode=mode)
    stacks = new_oracles(w, mode=mode)
    prefill_both(w, s, stacks, mode)
    bufs = step_buffers(w, mode)
    g = s.decode_graph(*bufs)
    schedule = "ggeggeg"
    worst = run_steps(w, s, stacks, mode, g, bufs, schedule)
    check_caches(w, s, stacks, mode)
    print("graph %s %s: worst |err| %.3g" % (name, mode, worst), flush=True)
    # the sequences are full now: neither path may start another step
    with pytest.raises(B.QcError) as e:
        s.graph_launch(g)
    assert e.value.status == B.QC_ECAPACITY
    s.close()


def test_graph_serves_a_new_batch_of_the_same_size_and_refuses_another():
    w1 = workloads.custom("g1", 3, 2, 64, "bf16", [2, 0], [30, 10], [50, 90], 4, [0, 1, 0], seed_tag=32,
                          max_seq=128, max_vis=40, max_text=100)
    s = P.Session.for_workload(w1)
    stacks = new_oracles(w1)
    prefill_both(w1, s, stacks, "vla")
    bufs = step_buffers(w1, "vla")
    g = s.decode_graph(*bufs)
    run_steps(w1, s, stacks, "vla", g, bufs, "gg")
    # another batch of two sequences with other lengths and spans: same graph
    w2 = workloads.custom("g2", 3, 2, 64, "bf16", [0, 5], [25, 40], [100, 61], 4, [0, 1, 0], seed_tag=33,
                          max_seq=128, max_vis=40, max_text=100)
    stacks2 = new_oracles(w2)
    prefill_both(w2, s, stacks2, "vla")
    run_steps(w2, s, stacks2, "vla", g, bufs, "geg")
    check_caches(w2, s, stacks2, "vla")
    # one sequence only: the graph does not fit
    w3 = workloads.custom("g3", 3, 2, 64, "bf16", [0], [25], [100], 4, [0, 1, 0], seed_tag=34,
                          max_seq=128, max_vis=40, max_text=100)
    s.reset(w3.vis_start, w3.vis_len)
    for l in range(3):
        q, k, v = (t.cuda() for t in workloads.prefill_qkv(w3, l))
        s.prefill(l, q, k, v, w3.cu_seqlens)
    with pytest.raises(B.QcError) as e:
        s.graph_launch(g)
    assert e.value.status == B.QC_EORDER
    s.close()


def test_graph_create_needs_a_finished_prefill():
    w = workloads.custom("g4", 2, 2, 64, "f32", [0], [8], [16], 2, [0, 1], seed_tag=35)
    s = P.Session.for_workload(w)
    bufs = step_buffers(w, "vla")
    s.reset(w.vis_start, w.vis_len)
    with pytest.raises(B.QcError) as e:
        s.decode_graph(*bufs)
    assert e.value.status == B.QC_EORDER
    q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, 0))
    s.prefill(0, q, k, v, w.cu_seqlens)
    with pytest.raises(B.QcError) as e:
        s.decode_graph(*bufs)
    assert e.value.status == B.QC_EORDER
    s.close()


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_graph_replays_are_bitwise_equal_to_ordinary_calls_and_repeatable(mode):
    """Same kernels, same arithmetic, fixed merge order, and here the same split of the key axis (64 keys
    per workgroup in both): a replayed step must give the very bits the ordinary calls give, run after run."""
    w = workloads.custom("bits", 6, 4, 128, "bf16", [4, 0], [300, 40], [700, 90], 5, [0, 0, 1, 1, 0, 1], seed_tag=36)
    results = []
    for use_graph in (False, True, True):
        s = P.Session.for_workload(w, mode=mode)
        stacks = new_oracles(w, mode=mode)
        prefill_both(w, s, stacks, mode)
        bufs = step_buffers(w, mode)
        q, k, v, out = bufs
        g = s.decode_graph(*bufs) if use_graph else None
        outs = []
        for t in range(5):
            ins = [workloads.decode_qkv(w, l, t, device="cuda") for l in range(w.n_layers)]
            for l in range(w.n_layers):
                if q[l] is not None:
                    q[l].copy_(ins[l][0]); k[l].copy_(ins[l][1])
                v[l].copy_(ins[l][2])
            if use_graph:
                s.graph_launch(g)
            else:
                for l in range(w.n_layers):
                    s.decode(l, q[l], k[l], v[l], out=out[l])
            torch.cuda.synchronize()
            outs.append(torch.stack(out).view(torch.int16).cpu().numpy().copy())
        lay = oracle_layout(w, mode)
        kv = s.kv_arena.cpu().numpy()[: lay.rows_bytes()].copy()    # cache rows only: the library's step counter differs by design
        results.append((outs, kv))
        s.close()
    for outs, kv in results[1:]:
        for a, b in zip(results[0][0], outs):
            assert np.array_equal(a, b)
        assert np.array_equal(results[0][1], kv)


def test_everything_runs_on_the_callers_stream():
    """Prefill, ordinary decode calls and graph replays enqueued on a side stream only, with a long-running
    kernel ahead of them on that stream: results are right once that stream has drained, which they
    would not be if any launch had gone to another stream."""
    w = workloads.custom("side", 4, 2, 64, "bf16", [2, 0], [30, 12], [80, 50], 4, [0, 1, 0, 1], seed_tag=37)
    s = P.Session.for_workload(w)
    stacks = new_oracles(w)
    side = torch.cuda.Stream()
    big = torch.randn(4096, 4096, device="cuda")
    with torch.cuda.stream(side):
        for _ in range(20):
            big = big @ big * 1e-4                       # keeps the side stream busy for a while
        prefill_both(w, s, stacks, "vla")
        bufs = step_buffers(w, "vla")
        g = s.decode_graph(*bufs)
        q, k, v, out = bufs
        refs, gots = [], []
        for t, kind in enumerate("egge"):
            ins = [workloads.decode_qkv(w, l, t) for l in range(w.n_layers)]
            refs.append([oracle_decode_layer(w, stacks, l, *ins[l]) for l in range(w.n_layers)])
            for l in range(w.n_layers):
                q[l].copy_(ins[l][0].cuda(), non_blocking=True)
                k[l].copy_(ins[l][1].cuda(), non_blocking=True)
                v[l].copy_(ins[l][2].cuda(), non_blocking=True)
            if kind == "g":
                s.graph_launch(g)
            else:
                for l in range(w.n_layers):
                    s.decode(l, q[l], k[l], v[l], out=out[l])
            gots.append([o.clone() for o in out])
    side.synchronize()
    for t in range(4):
        for l in range(w.n_layers):
            assert max_abs_err(gots[t][l], refs[t][l]) <= TOL["bf16"], (t, l)
    s.close()
