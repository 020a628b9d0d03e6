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


# ---- sequences leaving and joining a paged batch ---------------------------------------------------------
from test_gpu_join_leave import A, Bq, C, Dq, E, SEQ_LEN, VIS_LEN, VIS_START, Driver


def paged_population(dtype, D):
    return workloads.custom("paged_join_leave", 5, 3, D, dtype, VIS_START, VIS_LEN, SEQ_LEN, 6,
                            [0, 1, 1, 0, 1], seed_tag=311, max_seq=256, max_vis=192, max_text=128)


class PagedDriver(Driver):
    """The join/leave driver with pages instead of extents: the oracle side replays the hand-out rule."""

    def __init__(self, w, mode, slots):
        super().__init__(w, mode, slots)
        self.pools = olayout.PagePools(slots, w.max_seq, w.max_vis, w.max_text, mode=mode, any_lazy=True)

    def layout(self):
        w = self.w
        return olayout.ArenaLayout(w.n_layers, w.n_heads, w.head_dim, w.dtype, len(self.slots), w.max_seq, w.max_vis,
                                   w.max_text, w.lazy_mask, mode=self.mode, paged=self.pools.tables())

    def place(self, slot, i):
        self.slots[slot] = i
        self.stacks[slot] = self.new_stack(i)
        self.steps[i] = 0

    def reset(self, seqs):
        w = self.w
        for slot, i in enumerate(seqs):
            if i is not None:
                self.place(slot, i)
        vs = [0 if i is None else w.vis_start[i] for i in seqs]
        vl = [0 if i is None else w.vis_len[i] for i in seqs]
        self.session.reset(vs, vl, zero_fill=True, paged=True, present=[i is not None for i in seqs])
        self.prefill_pass([s for s, i in enumerate(seqs) if i is not None])

    def join(self, slot, i):
        self.place(slot, i)
        self.session.seq_join(slot, self.w.vis_start[i], self.w.vis_len[i])

    def leave(self, slot):
        self.session.seq_leave(slot)
        self.pools.leave(slot)
        self.slots[slot] = self.stacks[slot] = None

    def check_extents(self):
        pass

    def check_pages(self):
        sr.check_page_lists(self.session, self.pools)

    def prefill_pass(self, part):
        w = self.w
        self.pools.prefill(part, {s: w.seq_len[self.slots[s]] for s in part}, {s: w.vis_len[self.slots[s]] for s in part})
        super().prefill_pass(part)
        self.check_pages()

    def decode_step(self):
        w = self.w
        live = [s for s, i in enumerate(self.slots) if i is not None]
        self.pools.decode_step(live, {s: w.seq_len[self.slots[s]] + self.steps[self.slots[s]] for s in live},
                               {s: w.vis_len[self.slots[s]] for s in live})
        super().decode_step()
        self.check_pages()


@pytest.mark.parametrize("mode", ["vla", "gla"])
@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128)])
def test_join_leave_schedule_on_pages(mode, dtype, D):
    w = paged_population(dtype, D)
    d = PagedDriver(w, mode, slots=3)
    d.reset([A, Bq, None])
    d.decode_step()
    d.decode_step()
    d.check_state()
    d.leave(0)
    d.join(0, C)            # C takes the lowest pages A gave back
    d.join(2, Dq)
    d.prefill_pass([0, 2])
    d.decode_step()
    d.decode_step()
    d.check_state()
    d.leave(1)
    d.decode_step()
    d.join(1, E)            # E needs more pages than B gave back: it also gets pages behind everybody's
    d.prefill_pass([1])
    d.decode_step()
    d.check_state()
    assert d.worst <= sr.TOL[dtype]
    d.session.close()


def test_a_dry_pool_refuses_before_anything_changes():
    from paper_2602_01901_amd import binding as B
    # two slots, 128 positions each: 4 position pages in all; prompts of 100 and 160 tokens need 2 + 3
    # (a sequence may hold more than max_seq positions: the pool is what bounds it)
    w = workloads.custom("paged_dry", 2, 2, 64, "f32", [0, 0], [0, 0], [100, 160], 0, [0, 0],
                         max_seq=192, max_vis=64, max_text=192)
    import paper_2602_01901_amd as P
    s = P.Session(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.lazy_mask, 2, 128, 64, 128)
    s.reset([0, 0], [0, 0], paged=True)
    q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, 0))
    with pytest.raises(B.QcError) as e:
        s.prefill(0, q, k, v, w.cu_seqlens)
    assert e.value.status == B.QC_ECAPACITY
    assert B.qc_seq_pages(s.kv, 0, 0) == [] and B.qc_seq_pages(s.kv, 1, 0) == []
    # the same slots take prompts that fit: 100 and 128 tokens, 2 + 2 pages; then no page is left to decode into
    w2 = workloads.custom("paged_dry2", 2, 2, 64, "f32", [0, 0], [0, 0], [100, 128], 1, [0, 0],
                          max_seq=192, max_vis=64, max_text=192)
    for l in range(2):
        q, k, v = (t.cuda() for t in workloads.prefill_qkv(w2, l))
        s.prefill(l, q, k, v, w2.cu_seqlens)
    assert B.qc_seq_pages(s.kv, 0, 0) == [0, 1] and B.qc_seq_pages(s.kv, 1, 0) == [2, 3]
    q, k, v = (t.cuda() for t in workloads.decode_qkv(w2, 0, 0))
    with pytest.raises(B.QcError) as e:      # slot 1 would open a third page
        s.decode(0, q, k, v)
    assert e.value.status == B.QC_ECAPACITY
    assert B.qc_seq_len(s.kv, 1) == 128 and s.stats()["next_layer"] == 0
    # calls a paged batch does not offer
    for call in (lambda: B.qc_seq_grow(s.kv, s.qc, 0, 64, 0), lambda: B.qc_seq_extent(s.kv, 0), lambda: B.qc_prune(s.kv, s.qc, [0, 0])):
        with pytest.raises(B.QcError) as e:
            call()
        assert e.value.status == B.QC_EORDER
    s.close()


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_one_sequence_may_take_more_than_its_share(mode):
    """Three slots sized for 128 positions each; one sequence of 300 positions and a short one share them."""
    w = workloads.custom("paged_long", 3, 2, 64, "f32", [5, 2], [200, 10], [300, 20], 3, [0, 1, 0],
                         max_seq=128, max_vis=128, max_text=64)
    import paper_2602_01901_amd as P
    s = P.Session(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.lazy_mask, 3, 128, 128, 64, mode=mode)
    # the oracle's pools are those of the three-slot arena
    stacks = sr.new_oracles(w, mode=mode)
    pools = olayout.PagePools(3, 128, 128, 64, mode=mode)
    s.reset(w.vis_start + [0], w.vis_len + [0], zero_fill=True, paged=True, present=[1, 1, 0])
    pools.prefill([0, 1], w.seq_len, w.vis_len)
    cu = w.cu_seqlens + [w.cu_seqlens[-1]]
    worst = 0.0
    for l in range(w.n_layers):
        q, k, v = workloads.prefill_qkv(w, l)
        ref = sr.oracle_prefill_layer(w, stacks, l, q, k, v)
        no_qk = mode == "gla" and w.lazy_mask[l]
        out = s.prefill(l, None if no_qk else q.cuda(), None if no_qk else k.cuda(), v.cuda(), cu)
        worst = max(worst, sr.max_abs_err(out, ref))
    for t in range(w.decode_steps):
        pools.decode_step([0, 1], [n + t for n in w.seq_len], w.vis_len)
        for l in range(w.n_layers):
            q, k, v = workloads.decode_qkv(w, l, t)
            ref = sr.oracle_decode_layer(w, stacks, l, q, k, v)
            pad = lambda x: torch.cat([x, torch.zeros_like(x[:1])]).cuda()
            no_qk = mode == "gla" and w.lazy_mask[l]
            out = s.decode(l, None if no_qk else pad(q), None if no_qk else pad(k), pad(v))
            worst = max(worst, sr.max_abs_err(out[:2], ref))
    assert worst <= sr.TOL["f32"], worst
    sr.check_page_lists(s, pools)
    assert len(pools.tables()["seq"][0]) == 5      # 303 positions on five pages, more than 128 / 64 = 2
    lay = olayout.ArenaLayout(w.n_layers, w.n_heads, w.head_dim, w.dtype, 3, 128, 128, 64, w.lazy_mask, mode=mode,
                              paged=pools.tables())
    torch.cuda.synchronize()
    want = olayout.kv_rows_image(lay, stacks + [None])
    assert np.array_equal(s.kv_arena[: lay.rows_bytes()].cpu().numpy(), want)
    s.close()


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128)])
def test_last_row_attention_reads_keys_from_pages(dtype, D):
    """The selection statistic (Eq. 3) of an ordinary layer on a paged batch against the oracle."""
    from oracle import selection
    from paper_2602_01901_amd import binding as B
    lens = [131, 64, 45, 7, 300]
    w = workloads.custom("select_paged", 3, 3, D, dtype, [0] * 5, [0] * 5, lens, 0, [0, 0, 0], seed_tag=D,
                         max_seq=192, max_vis=64, max_text=128)      # 300 positions exceed the per-slot share
    s = _session(w)
    s.reset(w.vis_start, w.vis_len, paged=True)
    ws = torch.empty(B.qc_select_workspace_bytes(s.cfg), dtype=torch.uint8, device="cuda")
    cu, stride, scale = w.cu_seqlens, 304, 1.0 / np.sqrt(D)
    worst = 0.0
    for l in range(w.n_layers):
        q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, l))
        s.prefill(l, q, k, v, cu)
        probs = torch.full((w.batch, stride), -1.0, dtype=torch.float32, device="cuda")
        q_last = torch.stack([q[cu[b + 1] - 1] for b in range(w.batch)]).contiguous()
        B.qc_last_row_attention(s.kv, l, q_last, probs, stride, 0.0, ws, ws.numel())
        got = probs.cpu().numpy().astype(np.float64)
        for b in range(w.batch):
            K = np.transpose(workloads.to_f64(k[cu[b]:cu[b + 1]]), (1, 0, 2))
            want = selection.last_row_attention(workloads.to_f64(q[cu[b + 1] - 1]), K, scale)
            assert np.all(np.abs(got[b, :lens[b]] - want) <= 1e-5 + 1e-4 * want), (l, b)
            assert np.all(got[b, lens[b]:] == -1.0)
            worst = max(worst, float(np.max(np.abs(got[b, :lens[b]] - want))))
    print("paged last-row attention: worst abs err %.3g" % worst, flush=True)
    s.close()


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_decode_graph_replays_on_pages(mode):
    """Graph replays and ordinary steps alternate on a paged batch; replays open pages (host work ahead of
    the launch); every step is checked, then the lists and both arenas."""
    from test_gpu_graph import run_steps, step_buffers
    w = _bf16_workload(decode_steps=30)
    s = _session(w, mode)
    stacks = sr.new_oracles(w, mode=mode)
    pools = sr.oracle_page_pools(w, mode)
    sr.reset_session(s, w, zero_fill=True, paged=True)
    pools.prefill(range(w.batch), w.seq_len, w.vis_len)
    for l in range(w.n_layers):
        q, k, v = workloads.prefill_qkv(w, l)
        sr.oracle_prefill_layer(w, stacks, l, q, k, v)
        no_qk = mode == "gla" and w.lazy_mask[l]
        s.prefill(l, None if no_qk else q.cuda(), None if no_qk else k.cuda(), v.cuda(), w.cu_seqlens)
    bufs = step_buffers(w, mode)
    graph = s.decode_graph(*bufs)
    schedule = "gggeg" * 6          # sequence 3 opens a page at step 0, sequence 1 at step 24: both in replays
    worst = run_steps(w, s, stacks, mode, graph, bufs, schedule)
    for t in range(len(schedule)):
        pools.decode_step(range(w.batch), [n + t for n in w.seq_len], w.vis_len)
    assert worst <= sr.TOL["bf16"]
    sr.check_page_lists(s, pools)
    lay = sr.oracle_layout(w, mode, paged=pools.tables())
    sr.check_kv_rows(s, lay, stacks)
    assert np.array_equal(s.q_arena.cpu().numpy()[: lay.q_arena_bytes()], olayout.q_arena_image(lay, stacks))
    s.close()


@pytest.mark.parametrize("mode", ["vla", "gla"])
@pytest.mark.parametrize("which", ["f32", "bf16"])
def test_nothing_reads_a_page_row_it_has_not_written(mode, which):
    """Arenas and workspace start as all-ones bytes (NaN in either element type) and are not cleared: rows
    of a page behind a sequence's last position, and pages nobody holds, must never reach an output."""
    w = _f32_workload(decode_steps=5) if which == "f32" else _bf16_workload(decode_steps=5)
    s = _session(w, mode)
    for t in (s.kv_arena, s.q_arena, s.workspace):
        t.fill_(0xFF)
    wp, wd = sr.run_full_parity(w, w.decode_steps, s, check_arena=False, zero_fill=False, paged=True)
    assert max(wp, wd) <= sr.TOL[w.dtype]
    s.close()
