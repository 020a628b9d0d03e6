"""Sequences leaving and joining a running batch (qc_seq_leave / qc_seq_join) against per-sequence
stack oracles: outputs of every layer call, the extents chosen for the joined sequences, the row
images of both arenas, the library's queries.

Five sequences A..E of one seeded population share three slots:
  reset            slots [A, B, free]      prefill pass, 2 decode steps
  A leaves; C joins slot 0 (fits the hole A left), D joins slot 2
                   slots [C, B, D]         prefill pass over C and D only, 2 decode steps
  B leaves         slots [C, free, D]      1 decode step
  E joins slot 1 (too long for any hole: goes behind the last extent)
                   slots [C, E, D]         prefill pass over E only, 1 decode step
Each sequence sees its own step index whatever the batch has done before it joined."""
import numpy as np
import pytest
import torch

import workloads
from oracle import layout as olayout
from oracle.global_lazy_stack import GlobalLazyStackOracle
from oracle.lazy_stack import LazyStackOracle
from paper_2602_01901_amd import Session, binding as B
from stack_runner import TOL

pytestmark = pytest.mark.gpu

A, Bq, C, Dq, E = range(5)
#            A    B    C    D    E
VIS_START = [3,   0,   5,   2,   4]
VIS_LEN = [70,  90,  40,  0,   130]
SEQ_LEN = [131, 150, 77,  33,  210]
CAP_SEQ = [144, 160, 88,  40,  224]     # prompt + decode steps, multiples of 8
CAP_TEXT = [70,  66,  45,  40,  90]


def population(dtype, D):
    return workloads.custom("join_leave", 5, 3, D, dtype, VIS_START, VIS_LEN, SEQ_LEN, 6,
                            [0, 1, 1, 0, 1], seed_tag=311, max_seq=224, max_vis=130, max_text=90)


class Driver:
    def __init__(self, w, mode, slots):
        self.w, self.mode, self.dev = w, mode, "cuda:0"
        self.session = Session(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.lazy_mask, slots, w.max_seq, w.max_vis,
                               w.max_text, mode=mode)
        self.slots = [None] * slots          # sequence index per slot
        self.stacks = [None] * slots
        self.steps = {}                      # decode steps each sequence has taken
        self.caps = [[0] * slots, [0] * slots, [0] * slots]
        self.bases = [[0] * slots, [0] * slots, [0] * slots]
        self.kv_img = self.q_img = None
        self.worst = 0.0

    def new_stack(self, i):
        w = self.w
        if self.mode == "gla":
            return GlobalLazyStackOracle(w.n_layers, w.n_heads, w.head_dim, w.lazy_mask, vis_start=w.vis_start[i],
                                         vis_len=w.vis_len[i])
        return LazyStackOracle(w.n_layers, w.n_heads, w.head_dim, w.lazy_mask, w.vis_start[i], w.vis_len[i])

    def layout(self):
        w = self.w
        return olayout.ArenaLayout(w.n_layers, w.n_heads, w.head_dim, w.dtype, len(self.slots), w.max_seq, w.max_vis,
                                   w.max_text, w.lazy_mask, mode=self.mode, ragged=tuple(self.caps) + tuple(self.bases))

    def place(self, slot, i):
        """Oracle side of a join: first-fit extents among the sequences present."""
        w = self.w
        want = (CAP_SEQ[i], CAP_TEXT[i], w.vis_len[i])
        pools = (len(self.slots) * w.max_seq, len(self.slots) * w.max_text, len(self.slots) * w.max_vis)
        for kind in range(3):
            used = [(self.bases[kind][s], self.caps[kind][s]) for s in range(len(self.slots)) if self.slots[s] is not None]
            base = olayout.first_fit(used, want[kind], pools[kind])
            if self.mode == "gla" and kind > 0:
                base = 0          # those pools hold nothing under Global Lazy Attention
            assert base is not None
            self.bases[kind][slot], self.caps[kind][slot] = base, want[kind]
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
        self.session.reset(vs, vl, zero_fill=True, cap_seq=self.caps[0], cap_text=self.caps[1])
        self.check_extents()
        self.prefill_pass([s for s, i in enumerate(seqs) if i is not None])

    def join(self, slot, i):
        self.place(slot, i)
        self.session.seq_join(slot, self.w.vis_start[i], self.w.vis_len[i], CAP_SEQ[i], CAP_TEXT[i])

    def leave(self, slot):
        self.session.seq_leave(slot)
        self.slots[slot] = self.stacks[slot] = None
        for kind in range(3):
            self.caps[kind][slot] = self.bases[kind][slot] = 0

    def grow(self, slot, cap_seq, cap_text):
        """New capacities: a pool whose capacity changes gives the sequence a new first-fit extent beside all
        extents in use, its own old one included; the rows move, the old extent is free afterwards."""
        w = self.w
        want = (cap_seq, cap_text)
        pools = (len(self.slots) * w.max_seq, len(self.slots) * w.max_text)
        for kind in range(2):
            if want[kind] == self.caps[kind][slot] or (self.mode == "gla" and kind == 1):
                continue
            used = [(self.bases[kind][s], self.caps[kind][s]) for s in range(len(self.slots)) if self.slots[s] is not None]
            base = olayout.first_fit(used, want[kind], pools[kind])
            assert base is not None
            self.bases[kind][slot], self.caps[kind][slot] = base, want[kind]
        self.session.seq_grow(slot, cap_seq, cap_text)
        self.check_extents()

    def check_extents(self):
        for s, i in enumerate(self.slots):
            live, b_seq, b_text, b_vis = B.qc_seq_extent(self.session.kv, s)
            assert bool(live) == (i is not None), s
            if i is not None:
                want = (self.bases[0][s],) + ((0, 0) if self.mode == "gla" else (self.bases[1][s], self.bases[2][s]))
                assert (b_seq, b_text, b_vis) == want, (s, (b_seq, b_text, b_vis), want)

    def prefill_pass(self, part):
        """One prefill pass over the slots in `part`; the other slots have no tokens."""
        w, cu_all = self.w, self.w.cu_seqlens
        self.check_extents()
        lens = [w.seq_len[self.slots[s]] if s in part else 0 for s in range(len(self.slots))]
        cu = [0]
        for n in lens:
            cu.append(cu[-1] + n)
        gla = self.mode == "gla"
        for l in range(w.n_layers):
            qa, ka, va = workloads.prefill_qkv(w, l)
            rows = [slice(cu_all[self.slots[s]], cu_all[self.slots[s] + 1]) for s in part]
            q, k, v = (torch.cat([t[r] for r in rows], dim=0) for t in (qa, ka, va))
            ref = np.concatenate([self.stacks[s].prefill(l, *(workloads.to_f64(t[r]) for t in (qa, ka, va)))
                                  for s, r in zip(part, rows)], axis=0)
            qg, kg = (None, None) if (gla and w.lazy_mask[l]) else (q.to(self.dev), k.to(self.dev))
            out = self.session.prefill(l, qg, kg, v.to(self.dev), cu)
            err = float(np.max(np.abs(workloads.to_f64(out) - ref)))
            assert err <= TOL[w.dtype], ("prefill", l, err)
            self.worst = max(self.worst, err)

    def decode_step(self):
        w, n = self.w, len(self.slots)
        gla = self.mode == "gla"
        sentinel = 1024.0
        for l in range(w.n_layers):
            q = torch.zeros(n, w.n_heads, w.head_dim, dtype=workloads.TORCH_DTYPE[w.dtype])
            k, v = torch.zeros_like(q), torch.zeros_like(q)
            ref = {}
            for s, i in enumerate(self.slots):
                if i is None:
                    q[s] = k[s] = v[s] = float("nan")      # a free slot's rows must never be read into a result
                    continue
                qa, ka, va = workloads.decode_qkv(w, l, self.steps[i])
                q[s], k[s], v[s] = qa[i], ka[i], va[i]
                ref[s] = self.stacks[s].decode(l, *(workloads.to_f64(t[i]) for t in (qa, ka, va)))
            out = torch.full((n, w.n_heads, w.head_dim), sentinel, dtype=q.dtype, device=self.dev)
            qg, kg = (None, None) if (gla and w.lazy_mask[l]) else (q.to(self.dev), k.to(self.dev))
            self.session.decode(l, qg, kg, v.to(self.dev), out=out)
            got = workloads.to_f64(out)
            for s, i in enumerate(self.slots):
                if i is None:
                    assert np.all(got[s] == sentinel), ("free slot written", s, l)
                else:
                    err = float(np.max(np.abs(got[s] - ref[s])))
                    assert err <= TOL[w.dtype], ("decode", l, s, err)
                    self.worst = max(self.worst, err)
        for i in self.slots:
            if i is not None:
                self.steps[i] += 1

    def decode_step_graph(self):
        """The same step through one replay of a decode graph recorded once over fixed input and output buffers."""
        w, n = self.w, len(self.slots)
        gla = self.mode == "gla"
        dt = workloads.TORCH_DTYPE[w.dtype]
        if getattr(self, "graph", None) is None:
            mk = lambda: [torch.zeros(n, w.n_heads, w.head_dim, dtype=dt, device=self.dev) for _ in range(w.n_layers)]
            self.gq, self.gk, self.gv, self.go = mk(), mk(), mk(), mk()
            no_qk = [gla and w.lazy_mask[l] for l in range(w.n_layers)]
            self.graph = self.session.decode_graph([None if no_qk[l] else self.gq[l] for l in range(w.n_layers)],
                                                   [None if no_qk[l] else self.gk[l] for l in range(w.n_layers)],
                                                   self.gv, self.go)
        refs = []
        for l in range(w.n_layers):
            q = torch.full((n, w.n_heads, w.head_dim), float("nan"), dtype=dt)
            k, v = q.clone(), q.clone()
            ref = {}
            for s, i in enumerate(self.slots):
                if i is None:
                    continue
                qa, ka, va = workloads.decode_qkv(w, l, self.steps[i])
                q[s], k[s], v[s] = qa[i], ka[i], va[i]
                ref[s] = self.stacks[s].decode(l, *(workloads.to_f64(t[i]) for t in (qa, ka, va)))
            refs.append(ref)
            self.gq[l].copy_(q); self.gk[l].copy_(k); self.gv[l].copy_(v)
            self.go[l].fill_(1024.0)
        self.session.graph_launch(self.graph)
        torch.cuda.synchronize()
        for l in range(w.n_layers):
            got = workloads.to_f64(self.go[l])
            for s, i in enumerate(self.slots):
                if i is None:
                    assert np.all(got[s] == 1024.0), ("free slot written", s, l)
                else:
                    err = float(np.max(np.abs(got[s] - refs[l][s])))
                    assert err <= TOL[w.dtype], ("graph decode", l, s, err)
                    self.worst = max(self.worst, err)
        for i in self.slots:
            if i is not None:
                self.steps[i] += 1

    def check_state(self):
        """Arena images (rows of departed sequences stay behind), lengths, row counts, row locations."""
        torch.cuda.synchronize()
        lay = self.layout()
        self.kv_img = olayout.kv_rows_image(lay, self.stacks, onto=self.kv_img)
        self.q_img = olayout.q_arena_image(lay, self.stacks, onto=self.q_img)
        got = self.session.kv_arena[: lay.rows_bytes()].cpu().numpy()
        assert np.array_equal(got, self.kv_img), "K/V rows differ from the oracle's image"
        got_q = self.session.q_arena.cpu().numpy()[: lay.q_arena_bytes()]
        assert np.array_equal(got_q, self.q_img), "Q Cache arena differs from the oracle's image"
        w, kv = self.w, self.session.kv
        for s, i in enumerate(self.slots):
            want_len = 0 if i is None else w.seq_len[i] + self.steps[i]
            assert B.qc_seq_len(kv, s) == want_len, s
            if i is None:
                with pytest.raises(B.QcError):
                    B.qc_locate(kv, B.QC_K, 0, s, 0, 0)
                continue
            for l in (1, w.n_layers - 1):
                for pos in (0, w.vis_start[i] + w.vis_len[i] // 2, want_len - 1):
                    assert B.qc_locate(kv, B.QC_K, l, s, 1, pos) == \
                        lay.locate_k(l, s, 1, pos, w.vis_start[i], w.vis_len[i]), (s, l, pos)
                    assert B.qc_locate(kv, B.QC_V, l, s, 1, pos) == lay.locate_v(l, s, 1, pos)
        live = [st for st in self.stacks if st is not None]
        for l in range(w.n_layers):
            rk, rv = B.qc_layer_rows(kv, l)
            assert rk == sum(st.Kc[l].shape[1] for st in live), l
            assert rv == sum(st.Vc[l].shape[1] for st in live), l
        res = olayout.resident_bytes(lay, self.stacks)
        st = self.session.stats()
        for key in ("k_bytes", "v_bytes", "q_bytes", "tokens"):
            assert st[key] == res[key], key


@pytest.mark.parametrize("mode", ["vla", "gla"])
@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128)])
def test_join_leave_schedule(mode, dtype, D):
    w = population(dtype, D)
    d = Driver(w, mode, slots=3)
    d.reset([A, Bq, None])
    d.decode_step()
    d.decode_step()
    d.check_state()

    d.leave(0)
    d.join(0, C)
    d.join(2, Dq)
    # C fits where A was; D fits behind C inside the same hole (88 + 40 <= 144)
    assert d.bases[0][0] == 0 and d.bases[0][2] == 88 and d.bases[0][1] == 144
    with pytest.raises(B.QcError):          # a pass is pending: no decode, no leave
        d.session.seq_leave(1)
    d.prefill_pass([0, 2])
    d.decode_step()
    d.decode_step()
    d.check_state()

    # C (capacity 88 positions and 45 text rows, 79 and 39 in use) is given more room: 104 positions do not
    # fit the 16 free rows between D and B, so C moves behind B (144 + 160 = 304); 56 text rows do not fit
    # the 25 free rows before B's either and go behind D's (136 + 40 = 176)
    with pytest.raises(B.QcError):
        d.session.seq_grow(0, 72, 45)       # below the 79 positions it holds
    d.grow(0, 104, 56)
    assert (d.bases[0][0], d.bases[1][0]) == ((304, 176) if mode == "vla" else (304, 0))
    d.check_state()
    d.leave(1)
    d.decode_step()
    d.check_state()

    d.join(1, E)
    # positions: C sits at 304..408 now and D at 88..128: the first gap of 224 rows is behind C; text rows: the
    # 136 rows before D's are free; Q Cache rows: behind C's 40
    assert (d.bases[0][1], d.bases[1][1], d.bases[2][1]) == ((408, 0, 40) if mode == "vla" else (408, 0, 0))
    d.prefill_pass([1])
    d.decode_step()
    d.check_state()
    assert d.steps == {A: 2, Bq: 4, C: 4, Dq: 4, E: 1}
    # C alone runs on to 92 positions and 52 text rows, beyond the 88 and 45 it joined with
    d.leave(1)
    d.leave(2)
    for _ in range(11):
        d.decode_step()
    d.check_state()
    assert d.steps[C] == 15
    with pytest.raises(B.QcError):          # the new limits: 56 text rows (the fifth step from here), 104 positions under GLA
        for _ in range(20):
            d.decode_step()
    print("join/leave %s %s: worst error %.2e" % (mode, dtype, d.worst))
    d.session.close()


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_graph_replays_across_leave_join_and_growth(mode):
    """A decode graph recorded before any change of the batch keeps serving it: it reads every per-sequence
    integer, extent and the step count from device memory.  Replays alternate with ordinary steps."""
    w = population("bf16", 128)
    d = Driver(w, mode, slots=3)
    d.reset([A, Bq, None])
    d.decode_step_graph()
    d.decode_step()
    d.check_state()                      # the image is carried along: rows of departed sequences stay behind
    d.leave(0)
    d.join(0, C)
    d.join(2, Dq)
    d.prefill_pass([0, 2])
    d.decode_step_graph()
    d.decode_step_graph()
    d.check_state()
    d.grow(0, 104, 56)
    d.leave(1)
    d.decode_step_graph()
    d.decode_step()
    d.decode_step_graph()
    d.check_state()
    assert d.steps == {A: 2, Bq: 4, C: 5, Dq: 5}
    d.session.close()


def test_join_errors():
    w = population("f32", 64)
    d = Driver(w, "vla", slots=3)
    s = d.session
    d.reset([A, Bq, None])
    with pytest.raises(B.QcError):          # slot taken
        s.seq_join(0, 0, 0, 8, 8)
    with pytest.raises(B.QcError):          # no run of 3*224 - 144 - 160 + 8 free positions
        s.seq_join(2, 0, 0, 3 * 224 - 144 - 160 + 8, 8)
    with pytest.raises(B.QcError):          # capacity not a multiple of 8
        s.seq_join(2, 0, 0, 12, 8)
    with pytest.raises(B.QcError):          # free slot cannot leave
        s.seq_leave(2)
    s.seq_join(2, VIS_START[Dq], VIS_LEN[Dq], CAP_SEQ[Dq], CAP_TEXT[Dq])
    q, k, v = (t[:SEQ_LEN[Dq]].to("cuda:0") for t in workloads.prefill_qkv(w, 0))
    with pytest.raises(B.QcError):          # a decoding sequence given tokens in a pass it takes no part in
        s.prefill(0, q, k, v, [0, 5, 5, 5 + SEQ_LEN[Dq] - 5])
    s.close()
    # a batch with equal capacities has no slots to trade
    s2 = Session(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.lazy_mask, 2, w.max_seq, w.max_vis, w.max_text)
    s2.reset([0, 0], [0, 0])
    with pytest.raises(B.QcError):
        s2.seq_leave(0)
    s2.close()
