"""Paged batches (qc_reset_paged) against the oracle: outputs element by element, the page lists against the
stated hand-out rule, the K/V rows and the Q Cache byte for byte against the paged layout, row locations."""
import numpy as np
import pytest
import torch

import workloads
from oracle import layout as olayout
import stack_runner as sr

pytestmark = pytest.mark.gpu


def _session(w, mode="vla"):
    import paper_2602_01901_amd as P
    return P.Session.for_workload(w, mode=mode)


def _f32_workload(decode_steps=70):
    # three sequences of unequal lengths; the first crosses a page boundary of both its pools while decoding
    # (120 + 70 positions; 120 - 70 + 70 text rows), the third starts exactly at one (64 positions)
    return workloads.custom("paged_f32", 4, 4, 64, "f32", [10, 0, 3], [70, 0, 40], [120, 33, 64], decode_steps,
                            [0, 1, 1, 0], max_seq=256, max_vis=128, max_text=128)


def _bf16_workload(decode_steps=6):
    # head_dim 128 in bf16: the matrix-core prefill kernel; spans that start and end inside key tiles, a
    # sequence shorter than one tile, several key tiles wholly inside the span (read from the first layer's
    # pages), a prompt that ends exactly on a page
    return workloads.custom("paged_bf16", 5, 4, 128, "bf16", [30, 5, 0, 64], [330, 20, 0, 128], [400, 40, 129, 256],
                            decode_steps, [0, 1, 1, 0, 1], max_seq=448, max_vis=384, max_text=192)


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_f32_stack_on_pages(mode):
    w = _f32_workload()
    s = _session(w, mode)
    worst_p, worst_d = sr.run_full_parity(w, w.decode_steps, s, paged=True)
    assert worst_p <= sr.TOL["f32"] and worst_d <= sr.TOL["f32"], (worst_p, worst_d)
    s.close()


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_bf16_stack_on_pages(mode):
    w = _bf16_workload()
    s = _session(w, mode)
    worst_p, worst_d = sr.run_full_parity(w, w.decode_steps, s, paged=True, poison_span=True)
    assert worst_p <= sr.TOL["bf16"] and worst_d <= sr.TOL["bf16"], (worst_p, worst_d)
    s.close()


def test_pages_give_the_same_outputs_as_runs_of_rows():
    """Where a row lives does not enter the arithmetic: the same stack with and without pages, bit for bit."""
    w = _bf16_workload(decode_steps=3)
    outs = []
    for paged in (False, True):
        s = _session(w)
        sr.reset_session(s, w, zero_fill=True, paged=paged)
        got = []
        for l in range(w.n_layers):
            q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, l))
            got.append(s.prefill(l, q, k, v, w.cu_seqlens).cpu())
        for t in range(w.decode_steps):
            for l in range(w.n_layers):
                q, k, v = (x.cuda() for x in workloads.decode_qkv(w, l, t))
                got.append(s.decode(l, q, k, v).cpu())
        torch.cuda.synchronize()
        outs.append(got)
        s.close()
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_locate_follows_the_page_lists():
    from paper_2602_01901_amd import binding as B
    w = _f32_workload(decode_steps=2)
    s = _session(w)
    sr.run_full_parity(w, w.decode_steps, s, paged=True, check_arena=False)
    pools = sr.oracle_page_pools(w)
    pools.prefill(range(w.batch), w.seq_len, w.vis_len)
    for t in range(w.decode_steps):
        pools.decode_step(range(w.batch), [n + t for n in w.seq_len], w.vis_len)
    lay = sr.oracle_layout(w, paged=pools.tables())
    for b in range(w.batch):
        n = w.seq_len[b] + w.decode_steps
        for l in range(w.n_layers):
            for h in (0, w.n_heads - 1):
                for pos in sorted({0, 1, 63, 64, 65, n - 1, w.vis_start[b], w.vis_start[b] + w.vis_len[b]} & set(range(n))):
                    assert B.qc_locate(s.kv, B.QC_V, l, b, h, pos) == lay.locate_v(l, b, h, pos)
                    assert B.qc_locate(s.kv, B.QC_K, l, b, h, pos) == lay.locate_k(l, b, h, pos, w.vis_start[b], w.vis_len[b])
        with pytest.raises(B.QcError):       # a position on a page the sequence does not hold
            B.qc_locate(s.kv, B.QC_V, 0, b, 0, ((n + 63) // 64) * 64)
    s.close()
