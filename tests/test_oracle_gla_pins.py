"""Pins for the Global Lazy Attention oracle (Eq. 5 / Eq. 6): every check compares it with
something that is not itself: scalar brute force written from the equations, a library softmax,
the separately written Visual Lazy Attention oracle in the case where the two methods coincide,
invariants the equations imply, and the paper's closed-form saving rates.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

from oracle import attention, layout
from oracle.global_lazy_stack import GlobalLazyStackOracle, OrderError
from oracle.lazy_stack import LazyStackOracle

RNG = np.random.default_rng(4321)


def rand(*shape):
    return RNG.standard_normal(shape)


def stack_inputs(N, L, H, D):
    return [(rand(L, H, D), rand(L, H, D), rand(L, H, D)) for _ in range(N)]


def brute_rows(Q, K, V, scale):
    """Causal attention of one head with Python scalars only: Q, K, V are [L, D] lists."""
    L, D = len(Q), len(Q[0])
    out = []
    for i in range(L):
        sc = [scale * sum(Q[i][d] * K[j][d] for d in range(D)) for j in range(i + 1)]
        mx = max(sc)
        w = [math.exp(x - mx) for x in sc]
        z = sum(w)
        out.append([sum(w[j] * V[j][d] for j in range(i + 1)) / z for d in range(D)])
    return out


# ---------------------------------------------------------------------------
# prefill (Eq. 5)
# ---------------------------------------------------------------------------
def test_lazy_layer_uses_first_layers_q_and_k_and_its_own_v_bruteforce():
    N, L, H, D = 4, 6, 2, 3
    mask = [0, 1, 1, 0]
    ins = stack_inputs(N, L, H, D)
    st = GlobalLazyStackOracle(N, H, D, mask)
    outs = [st.prefill(l, *ins[l]) for l in range(N)]
    scale = 1.0 / math.sqrt(D)
    for l in range(N):
        src = 0 if mask[l] else l          # whose Q and K the layer attends with
        for h in range(H):
            want = brute_rows(ins[src][0][:, h].tolist(), ins[src][1][:, h].tolist(), ins[l][2][:, h].tolist(), scale)
            np.testing.assert_allclose(outs[l][:, h], np.array(want), rtol=0, atol=1e-13)


def test_lazy_output_is_first_layers_attention_matrix_times_own_values():
    # A is computed by Q and K alone, so a lazy layer's output is A^{l_c} V^{l_i}: build A with a
    # library softmax over the masked scores and multiply.
    N, L, H, D = 3, 9, 2, 4
    ins = stack_inputs(N, L, H, D)
    st = GlobalLazyStackOracle(N, H, D, [0, 1, 1], scale=0.4)
    outs = [st.prefill(l, *ins[l]) for l in range(N)]
    Q0, K0 = ins[0][0], ins[0][1]
    for h in range(H):
        sc = 0.4 * Q0[:, h] @ K0[:, h].T
        sc[np.triu_indices(L, 1)] = -np.inf
        A = scipy.special.softmax(sc, axis=1)
        for l in (1, 2):
            np.testing.assert_allclose(outs[l][:, h], A @ ins[l][2][:, h], rtol=0, atol=1e-13)


def test_same_values_give_the_first_layers_output():
    N, L, H, D = 3, 7, 2, 4
    ins = stack_inputs(N, L, H, D)
    ins[1] = (ins[1][0], ins[1][1], ins[0][2])   # layer 1 gets layer 0's V
    st = GlobalLazyStackOracle(N, H, D, [0, 1, 0])
    outs = [st.prefill(l, *ins[l]) for l in range(N)]
    np.testing.assert_array_equal(outs[1], outs[0])
    assert np.max(np.abs(outs[2] - outs[0])) > 1e-3   # an ordinary layer does not inherit


def test_no_lazy_layers_is_standard_attention():
    N, L, H, D = 3, 8, 2, 4
    ins = stack_inputs(N, L, H, D)
    st = GlobalLazyStackOracle(N, H, D, [0, 0, 0])
    for l in range(N):
        got = st.prefill(l, *ins[l])
        want = attention.causal_attention(*(np.transpose(x, (1, 0, 2)) for x in ins[l]))
        np.testing.assert_array_equal(got, np.transpose(want, (1, 0, 2)))
    assert st.q_owner == -1 and st.resident_rows() == (N * L, N * L, 0)


@pytest.mark.parametrize("mask", [[0, 1, 1, 0, 1], [0, 0, 1, 0, 0], [0, 1, 0, 1, 1]])
def test_prefill_equals_visual_lazy_attention_when_every_token_is_visual(mask):
    # Eq. 7 with an empty text set is Eq. 5: the two oracles were written separately.
    N, L, H, D = len(mask), 10, 2, 4
    ins = stack_inputs(N, L, H, D)
    g = GlobalLazyStackOracle(N, H, D, mask)
    v = LazyStackOracle(N, H, D, mask, 0, L)
    for l in range(N):
        np.testing.assert_array_equal(g.prefill(l, *ins[l]), v.prefill(l, *ins[l]))
        assert g.k_rows(l) == v.k_rows(l) == (0 if mask[l] else L)
        assert g.q_owner == v.q_owner


def test_lazy_layer_never_reads_its_q_and_k_arguments():
    N, L, H, D = 3, 6, 2, 4
    ins = stack_inputs(N, L, H, D)
    a = GlobalLazyStackOracle(N, H, D, [0, 1, 1])
    b = GlobalLazyStackOracle(N, H, D, [0, 1, 1])
    nan = np.full((L, H, D), np.nan)
    for l in range(N):
        oa = a.prefill(l, *ins[l])
        ob = b.prefill(l, *(ins[l] if l == 0 else (None, nan, ins[l][2])))
        np.testing.assert_array_equal(oa, ob)
    q, k, vv = rand(H, D), rand(H, D), rand(H, D)
    for l in range(N):
        oa = a.decode(l, q, k, vv)
        ob = b.decode(l, *((q, k, vv) if l == 0 else (None, None, vv)))
        np.testing.assert_array_equal(oa, ob)


def test_rows_argument_matches_full_evaluation():
    N, L, H, D = 3, 9, 2, 4
    ins = stack_inputs(N, L, H, D)
    a = GlobalLazyStackOracle(N, H, D, [0, 1, 0])
    b = GlobalLazyStackOracle(N, H, D, [0, 1, 0])
    for l in range(N):
        full = a.prefill(l, *ins[l])
        part = b.prefill(l, *ins[l], rows=[0, 4, 8])
        np.testing.assert_allclose(part, full[[0, 4, 8]], rtol=0, atol=1e-14)


# ---------------------------------------------------------------------------
# decode (Eq. 6)
# ---------------------------------------------------------------------------
def test_decode_equals_last_row_of_a_longer_prefill():
    # Generating T tokens after a prompt of L must give what prefill over L + T tokens gives in
    # its last T rows, layer by layer (same projections, same sharing rule).
    N, L, T, H, D = 5, 6, 3, 2, 4
    mask = [0, 1, 1, 0, 1]
    ins = stack_inputs(N, L + T, H, D)
    whole = GlobalLazyStackOracle(N, H, D, mask)
    ref = [whole.prefill(l, *ins[l]) for l in range(N)]
    st = GlobalLazyStackOracle(N, H, D, mask)
    for l in range(N):
        np.testing.assert_allclose(st.prefill(l, *(x[:L] for x in ins[l])), ref[l][:L], rtol=0, atol=1e-13)
    for t in range(T):
        for l in range(N):
            q, k, v = (x[L + t] for x in ins[l])
            o = st.decode(l, None if mask[l] else q, None if mask[l] else k, v)
            np.testing.assert_allclose(o, ref[l][L + t], rtol=0, atol=1e-13)
    for l in range(N):
        np.testing.assert_array_equal(st.Vc[l], whole.Vc[l])
        np.testing.assert_array_equal(st.Kc[l], whole.Kc[l])
    np.testing.assert_array_equal(st.Qc, whole.Qc)
    assert st.len == L + T


def test_decode_lazy_layer_bruteforce_from_the_equation():
    N, L, H, D = 3, 5, 2, 3
    ins = stack_inputs(N, L, H, D)
    st = GlobalLazyStackOracle(N, H, D, [0, 1, 1], scale=0.3)
    for l in range(N):
        st.prefill(l, *ins[l])
    new = [(rand(H, D), rand(H, D), rand(H, D)) for _ in range(N)]
    outs = [st.decode(l, *new[l]) for l in range(N)]
    for l in range(N):
        for h in range(H):
            q = new[0][0][h]                                             # Q Cache = layer 0's query
            K = np.vstack([ins[0][1][:, h], new[0][1][h]])               # K cache of layer 0 plus its new key
            V = np.vstack([ins[l][2][:, h], new[l][2][h]])               # own values plus the new row
            sc = [0.3 * sum(q[d] * K[j][d] for d in range(D)) for j in range(L + 1)]
            w = [math.exp(x - max(sc)) for x in sc]
            want = [sum(w[j] * V[j][d] for j in range(L + 1)) / sum(w) for d in range(D)]
            np.testing.assert_allclose(outs[l][h], want, rtol=0, atol=1e-13)


def test_q_cache_follows_the_block_during_decode():
    N, L, H, D = 5, 4, 1, 2
    mask = [0, 1, 0, 1, 0]
    ins = stack_inputs(N, L, H, D)
    st = GlobalLazyStackOracle(N, H, D, mask)
    for l in range(N):
        st.prefill(l, *ins[l])
    assert st.q_owner == 2
    np.testing.assert_array_equal(st.Qc, np.transpose(ins[2][0], (1, 0, 2)))
    new = [(rand(H, D), rand(H, D), rand(H, D)) for _ in range(N)]
    st.decode(0, *new[0])
    assert st.q_owner == 0 and st.Qc.shape[1] == L + 1
    np.testing.assert_array_equal(st.Qc[:, L], new[0][0])
    np.testing.assert_array_equal(st.Qc[:, :L], np.transpose(ins[2][0], (1, 0, 2)))   # older rows stay
    st.decode(1, None, None, new[1][2])
    st.decode(2, *new[2])
    assert st.q_owner == 2
    np.testing.assert_array_equal(st.Qc[:, L], new[2][0])


def test_order_errors():
    N, L, H, D = 4, 3, 1, 2
    ins = stack_inputs(N, L, H, D)
    st = GlobalLazyStackOracle(N, H, D, [0, 1, 0, 1])
    st.prefill(0, *ins[0])
    with pytest.raises(OrderError):
        st.prefill(2, *ins[2])
    with pytest.raises(OrderError):
        st.decode(0, rand(H, D), rand(H, D), rand(H, D))
    st.prefill(1, *ins[1])
    st.prefill(2, *ins[2])
    st.q_owner = 0                      # pretend the cache was not refreshed by layer 2
    with pytest.raises(OrderError):
        st.prefill(3, *ins[3])
    with pytest.raises(ValueError):
        GlobalLazyStackOracle(2, 1, 2, [1, 0])


# ---------------------------------------------------------------------------
# accounting and layout
# ---------------------------------------------------------------------------
def read_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "gla_saving_closed_form.txt")
    rows = []
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            N, n, save, share = line.split()
            rows.append((int(N), int(n), Fraction(save), Fraction(share)))
    return rows


@pytest.mark.parametrize("N,n,save,share", read_golden())
def test_saving_and_q_cache_share_match_the_papers_closed_forms(N, n, save, share):
    L, H, D = 5, 1, 2
    mask = [0] + [1 if i < n else 0 for i in range(N - 1)]
    st = GlobalLazyStackOracle(N, H, D, mask)
    z = np.zeros((L, H, D))
    for l in range(N):
        st.prefill(l, z, z, z, rows=[0])
    rk, rv, rq = st.resident_rows()
    standard = 2 * N * L
    assert Fraction(standard - (rk + rv), standard) == save == layout.gla_kv_saving_closed_form(N, n)
    assert Fraction(rq, standard) == share == layout.q_cache_share_closed_form(N)


def test_gla_layout_sizes_and_row_map():
    lay = layout.ArenaLayout(4, 2, 64, "bf16", 3, 20, 12, 9, [0, 1, 1, 0], mode="gla")
    row = 64 * 2
    assert [lay.cap_k(l) for l in range(4)] == [20, 0, 0, 20]
    assert lay.off_k(4) == 2 * 3 * 2 * 20 * row                  # two ordinary layers only
    assert lay.off_v(1) - lay.off_v(0) == 3 * 2 * 20 * row
    assert lay.q_arena_bytes() == 3 * 2 * 20 * row               # every position, not only the span
    assert lay.rows_bytes() == lay.off_k(4) + 4 * 3 * 2 * 20 * row  # K rows of two layers, V rows of all four
    for pos in (0, 7, 19):
        assert lay.locate_k(2, 1, 1, pos, 3, 5) == (0, lay.k_offset(0, 1, 1, pos))
        assert lay.locate_k(3, 1, 1, pos, 3, 5) == (3, lay.k_offset(3, 1, 1, pos))
    vla = layout.ArenaLayout(4, 2, 64, "bf16", 3, 20, 12, 9, [0, 1, 1, 0])
    assert vla.rows_bytes() - lay.rows_bytes() == 2 * 3 * 2 * 9 * row


def test_arena_images_hold_the_oracles_rows():
    N, L, H, D = 3, 4, 2, 64
    mask = [0, 1, 0]
    lay = layout.ArenaLayout(N, H, D, "f32", 2, 6, 3, 4, mask, mode="gla")
    sts = []
    for b in range(2):
        st = GlobalLazyStackOracle(N, H, D, mask, vis_start=1, vis_len=2)
        ins = [tuple(np.float32(rand(L - b, H, D)).astype(np.float64) for _ in range(3)) for _ in range(N)]
        for l in range(N):
            st.prefill(l, *ins[l])
        sts.append((st, ins))
    img = layout.kv_rows_image(lay, [s for s, _ in sts])
    qimg = layout.q_arena_image(lay, [s for s, _ in sts])
    st, ins = sts[1]
    o = lay.v_offset(1, 1, 1, 2)
    np.testing.assert_array_equal(img[o:o + D * 4].view(np.float32), np.float32(ins[1][2][2, 1]))
    o = lay.q_offset(1, 0, 2)
    np.testing.assert_array_equal(qimg[o:o + D * 4].view(np.float32), np.float32(ins[0][0][2, 0]))
    assert lay.off_k(2) == lay.off_k(1)                           # the lazy layer owns no K bytes
