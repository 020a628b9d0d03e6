"""Pins for the CPU oracle: every check here compares the oracle with something
that is not the oracle (scalar brute force, a library routine, closed forms,
invariants the paper's definitions imply, the paper's closed-form saving rate).
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import attention, layout
from oracle.lazy_stack import LazyStackOracle, OrderError

RNG = np.random.default_rng(1234)


def rand(*shape):
    return RNG.standard_normal(shape)


# ---------------------------------------------------------------------------
# attention.py against brute force, a library routine and closed forms
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("L,D", [(1, 1), (2, 3), (7, 4), (16, 8)])
def test_causal_attention_vs_scalar_bruteforce(L, D):
    Q, K, V = rand(L, D), rand(L, D), rand(L, D)
    scale = 1.0 / math.sqrt(D)
    want = np.array(attention.attention_scalar(Q.tolist(), K.tolist(), V.tolist(), scale, True))
    got = attention.causal_attention(Q, K, V)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("L,D", [(1, 2), (5, 3), (13, 8)])
def test_decode_attention_vs_scalar_bruteforce(L, D):
    q, K, V = rand(D), rand(L, D), rand(L, D)
    scale = 0.37
    want = np.array(attention.attention_scalar([q.tolist()], K.tolist(), V.tolist(), scale, False))[0]
    got = attention.decode_attention(q, K, V, scale)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("H,L,D", [(2, 9, 4), (3, 33, 16), (1, 64, 64)])
def test_causal_attention_vs_library_sdpa(H, L, D):
    """Eq. 1 reduces to the library's causal scaled-dot-product attention (default scale 1/sqrt(D))."""
    Q, K, V = rand(H, L, D), rand(H, L, D), rand(H, L, D)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), is_causal=True).numpy()
    got = attention.causal_attention(Q, K, V)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_decode_attention_vs_library_sdpa():
    H, L, D = 4, 37, 32
    q, K, V = rand(H, D), rand(H, L, D), rand(H, L, D)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q[:, None, :]), torch.from_numpy(K), torch.from_numpy(V)).numpy()[:, 0, :]
    np.testing.assert_allclose(attention.decode_attention(q, K, V), want, rtol=0, atol=1e-12)


def test_zero_queries_give_running_mean_of_values():
    """Closed form: all scores equal => causal attention is the prefix mean of V."""
    L, D = 11, 5
    V = rand(L, D)
    got = attention.causal_attention(np.zeros((L, D)), rand(L, D), V)
    want = np.cumsum(V, axis=0) / np.arange(1, L + 1)[:, None]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)


def test_one_dominant_key_selects_its_value():
    """Closed form: a key aligned with the query by a huge margin receives all the weight."""
    L, D = 6, 4
    K = np.zeros((L, D))
    K[2, 0] = 1.0
    q = np.array([4000.0, 0, 0, 0])
    V = rand(L, D)
    got = attention.decode_attention(q, K, V, scale=1.0)
    np.testing.assert_allclose(got, V[2], rtol=0, atol=1e-300)


def test_softmax_rows_sum_to_one_and_output_in_value_hull():
    H, L, D = 2, 19, 8
    Q, K, V = rand(H, L, D) * 3, rand(H, L, D) * 3, rand(H, L, D)
    S = attention.causal_scores(Q, K, 1 / math.sqrt(D))
    A = attention.softmax_lastaxis(S)
    np.testing.assert_allclose(A.sum(-1), 1.0, rtol=0, atol=1e-14)
    assert np.all(np.triu(A, k=1) == 0.0), "A must be lower triangular (Eq. 1)"
    O = attention.causal_attention(Q, K, V)
    for i in range(L):
        lo, hi = V[:, : i + 1].min(axis=1), V[:, : i + 1].max(axis=1)
        assert np.all(O[:, i] >= lo - 1e-12) and np.all(O[:, i] <= hi + 1e-12)


def test_decode_invariant_to_joint_permutation_of_keys_and_values():
    L, D = 23, 8
    q, K, V = rand(D), rand(L, D), rand(L, D)
    perm = RNG.permutation(L)
    a = attention.decode_attention(q, K, V)
    b = attention.decode_attention(q, K[perm], V[perm])
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)


def test_transposed_operand_would_be_caught():
    """Scores are q_i . k_j, not k_i . q_j: an asymmetric example with a known answer."""
    Q = np.array([[0.0, 0.0], [1.0, 0.0]])
    K = np.array([[50.0, 0.0], [0.0, 0.0]])
    V = np.array([[1.0], [0.0]])
    O = attention.causal_attention(Q, K, V, scale=1.0)
    # row 1: scores (50, 0) -> weight on key 0 is 1/(1+e^-50)
    assert abs(O[1, 0] - 1.0 / (1.0 + math.exp(-50.0))) < 1e-15
    assert O[0, 0] == 1.0


# ---------------------------------------------------------------------------
# lazy_stack.py
# ---------------------------------------------------------------------------
def make_stack_inputs(N, L, H, D):
    return [(rand(L, H, D), rand(L, H, D), rand(L, H, D)) for _ in range(N)]


def bruteforce_vla_prefill(N, H, D, lazy, s, Vn, inputs):
    """Eq. 7 restated with Python lists and the scalar attention: per head, per layer."""
    scale = 1.0 / math.sqrt(D)
    outs = []
    anchor_q = anchor_k = None
    for l in range(N):
        Q, K, V = inputs[l]
        layer_out = np.zeros_like(Q)
        if not lazy[l]:
            anchor_q, anchor_k = Q, K
        for h in range(H):
            q_rows, k_rows = [], []
            for p in range(Q.shape[0]):
                visual = s <= p < s + Vn
                if lazy[l] and visual:
                    q_rows.append(anchor_q[p, h].tolist())
                    k_rows.append(anchor_k[p, h].tolist())
                else:
                    q_rows.append(Q[p, h].tolist())
                    k_rows.append(K[p, h].tolist())
            o = attention.attention_scalar(q_rows, k_rows, V[:, h].tolist(), scale, True)
            layer_out[:, h, :] = np.array(o)
        outs.append(layer_out)
    return outs


@pytest.mark.parametrize("span", [(0, 0), (0, 5), (2, 4), (3, 6), (0, 9)])
def test_vla_prefill_vs_bruteforce_all_masks(span):
    N, H, D, L = 4, 2, 3, 9
    s, Vn = span
    inputs = make_stack_inputs(N, L, H, D)
    for bits in itertools.product([0, 1], repeat=N - 1):
        lazy = [0] + list(bits)
        st = LazyStackOracle(N, H, D, lazy, s, Vn)
        want = bruteforce_vla_prefill(N, H, D, lazy, s, Vn, inputs)
        for l in range(N):
            got = st.prefill(l, *inputs[l])
            np.testing.assert_allclose(got, want[l], rtol=0, atol=1e-13)


def test_no_lazy_layers_is_standard_causal_attention_library():
    N, H, D, L = 3, 2, 8, 21
    inputs = make_stack_inputs(N, L, H, D)
    st = LazyStackOracle(N, H, D, [0, 0, 0], 4, 9)
    for l in range(N):
        Q, K, V = (torch.from_numpy(np.transpose(x, (1, 0, 2)).copy()) for x in inputs[l])
        want = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)
        got = st.prefill(l, *inputs[l])
        np.testing.assert_allclose(got, want.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)
        assert st.k_rows(l) == L and st.v_rows(l) == L


def test_empty_visual_span_is_standard_attention_for_any_mask():
    N, H, D, L = 4, 2, 4, 10
    inputs = make_stack_inputs(N, L, H, D)
    st = LazyStackOracle(N, H, D, [0, 1, 0, 1], 3, 0)
    for l in range(N):
        got = st.prefill(l, *inputs[l])
        Q, K, V = (np.transpose(x, (1, 0, 2)) for x in inputs[l])
        want = np.transpose(attention.causal_attention(Q, K, V), (1, 0, 2))
        np.testing.assert_array_equal(got, want)
    o = st.decode(0, rand(H, D), rand(H, D), rand(H, D))
    assert o.shape == (H, D)


def test_lazy_layer_fed_anchor_qk_equals_standard_attention_with_own_v():
    """If a lazy layer's own Q, K equal the anchor's, substitution changes nothing (own V is used)."""
    N, H, D, L, s, Vn = 3, 2, 4, 12, 2, 7
    inputs = make_stack_inputs(N, L, H, D)
    inputs[2] = (inputs[1][0], inputs[1][1], inputs[2][2])
    st = LazyStackOracle(N, H, D, [0, 0, 1], s, Vn)
    for l in range(2):
        st.prefill(l, *inputs[l])
    got = st.prefill(2, *inputs[2])
    Q, K, V = (torch.from_numpy(np.transpose(x, (1, 0, 2)).copy()) for x in inputs[2])
    want = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)
    np.testing.assert_allclose(got, want.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


def test_visual_block_of_scores_is_inherited_exactly():
    """Fig. 3 caption / Q Cache definition: inside the span a lazy layer uses the block's first
    layer's queries and keys, so that block of pre-softmax scores is bitwise the anchor's; text
    rows/columns use the layer's own projections and differ."""
    N, H, D, L, s, Vn = 4, 2, 4, 14, 3, 6
    inputs = make_stack_inputs(N, L, H, D)
    st = LazyStackOracle(N, H, D, [0, 0, 1, 1], s, Vn)
    scores = []
    for l in range(N):
        _, S = st.prefill(l, *inputs[l], return_scores=True)
        scores.append(S)
    e = s + Vn
    for l in (2, 3):
        blk = scores[l][:, s:e, s:e]
        ref = scores[1][:, s:e, s:e]
        tri = np.tril(np.ones((Vn, Vn), dtype=bool))
        assert np.array_equal(blk[:, tri], ref[:, tri])
        assert not np.allclose(scores[l][:, e:, :s], scores[1][:, e:, :s])
        # text query row against visual keys: own q, anchor k
        Qown = np.transpose(inputs[l][0], (1, 0, 2))
        Kanc = np.transpose(inputs[1][1], (1, 0, 2))
        want = np.einsum("hd,hjd->hj", Qown[:, e, :], Kanc[:, s:e, :]) / math.sqrt(D)
        np.testing.assert_allclose(scores[l][:, e, s:e], want, rtol=0, atol=1e-14)


def test_span_rows_of_lazy_layer_inputs_are_never_read():
    """Eq. 7 projects only text tokens in a lazy layer: poison the span rows of its Q and K."""
    N, H, D, L, s, Vn = 3, 2, 4, 11, 2, 5
    inputs = make_stack_inputs(N, L, H, D)
    clean = LazyStackOracle(N, H, D, [0, 1, 1], s, Vn)
    dirty = LazyStackOracle(N, H, D, [0, 1, 1], s, Vn)
    for l in range(N):
        Q, K, V = inputs[l]
        a = clean.prefill(l, Q, K, V)
        if l > 0:
            Q, K = Q.copy(), K.copy()
            Q[s:s + Vn] = np.nan
            K[s:s + Vn] = np.nan
        b = dirty.prefill(l, Q, K, V)
        assert np.array_equal(a, b)
    for l in range(N):
        assert np.array_equal(clean.Kc[l], dirty.Kc[l])


def test_chain_inheritance_equals_anchor_inheritance():
    """Inheriting from the immediately preceding (lazy) layer is inheriting from the block's first
    layer: replace each lazy layer's span rows by the previous layer's *effective* rows."""
    N, H, D, L, s, Vn = 4, 1, 4, 10, 1, 6
    inputs = make_stack_inputs(N, L, H, D)
    lazy = [0, 1, 1, 1]
    st = LazyStackOracle(N, H, D, lazy, s, Vn)
    outs = [st.prefill(l, *inputs[l]) for l in range(N)]
    prevQ, prevK = inputs[0][0], inputs[0][1]
    for l in range(1, N):
        Q, K, V = (x.copy() for x in inputs[l])
        Q[s:s + Vn], K[s:s + Vn] = prevQ[s:s + Vn], prevK[s:s + Vn]
        want = attention.causal_attention(*(np.transpose(x, (1, 0, 2)) for x in (Q, K, V)))
        np.testing.assert_allclose(outs[l], np.transpose(want, (1, 0, 2)), rtol=0, atol=1e-14)
        prevQ, prevK = Q, K


@pytest.mark.parametrize("lazy,s,Vn", [([0, 0, 1, 1], 2, 5), ([0, 1, 0, 1], 0, 4), ([0, 1, 1, 0], 3, 6),
                                       ([0, 0, 0, 0], 1, 3)])
def test_decode_step_equals_last_row_of_longer_prefill(lazy, s, Vn):
    """Eq. 8 is Eq. 7 restricted to one new text query row: decoding t tokens after a prompt
    equals the last row of a prefill over prompt + generated tokens (generated = suffix text)."""
    N, H, D, L, steps = 4, 2, 4, 10, 3
    prompt = make_stack_inputs(N, L, H, D)
    gen = [[(rand(H, D), rand(H, D), rand(H, D)) for _ in range(N)] for _ in range(steps)]
    st = LazyStackOracle(N, H, D, lazy, s, Vn)
    for l in range(N):
        st.prefill(l, *prompt[l])
    for t in range(steps):
        outs = [st.decode(l, *gen[t][l]) for l in range(N)]
        ref = LazyStackOracle(N, H, D, lazy, s, Vn)
        for l in range(N):
            ext = [np.concatenate([prompt[l][c]] + [gen[u][l][c][None] for u in range(t + 1)], axis=0)
                   for c in range(3)]
            want = ref.prefill(l, *ext)[-1]
            np.testing.assert_allclose(outs[l], want, rtol=0, atol=1e-13)
        assert st.len == L + t + 1


def test_decode_vs_scalar_bruteforce_with_explicit_key_assembly():
    """Eq. 8 by hand: keys = own text prefix, anchor's visual rows, own text suffix, generated."""
    N, H, D, L, s, Vn = 3, 1, 3, 8, 2, 4
    prompt = make_stack_inputs(N, L, H, D)
    st = LazyStackOracle(N, H, D, [0, 1, 1], s, Vn)
    for l in range(N):
        st.prefill(l, *prompt[l])
    q, k, v = rand(N, H, D), rand(N, H, D), rand(N, H, D)
    for l in range(N):
        o = st.decode(l, q[l], k[l], v[l])
        Kp, Vp = prompt[l][1][:, 0], prompt[l][2][:, 0]
        if l == 0:
            keys = Kp.tolist()
        else:
            keys = Kp[:s].tolist() + prompt[0][1][s:s + Vn, 0].tolist() + Kp[s + Vn:].tolist()
        keys.append(k[l, 0].tolist())
        vals = Vp.tolist() + [v[l, 0].tolist()]
        want = attention.attention_scalar([q[l, 0].tolist()], keys, vals, 1 / math.sqrt(D), False)[0]
        np.testing.assert_allclose(o[0], np.array(want), rtol=0, atol=1e-13)


def test_cache_rows_and_row_map():
    """A lazy layer keeps text keys only; visual positions resolve to the block's first layer."""
    N, H, D, L, s, Vn = 5, 1, 2, 12, 3, 5
    lazy = [0, 1, 1, 0, 1]
    st = LazyStackOracle(N, H, D, lazy, s, Vn)
    inputs = make_stack_inputs(N, L, H, D)
    for l in range(N):
        st.prefill(l, *inputs[l])
    for l in range(N):
        assert st.v_rows(l) == L
        assert st.k_rows(l) == L - lazy[l] * Vn
    assert st.anchor(1) == 0 and st.anchor(2) == 0 and st.anchor(4) == 3
    assert st.k_source(2, 2) == (2, 2)
    assert st.k_source(2, 3) == (0, 3)
    assert st.k_source(2, 7) == (0, 7)
    assert st.k_source(2, 8) == (2, 3)
    assert st.k_source(4, 5) == (3, 5)
    assert st.k_source(3, 5) == (3, 5)
    # the rows a lazy layer kept are its own text keys in order
    K2 = np.transpose(inputs[2][1], (1, 0, 2))
    assert np.array_equal(st.Kc[2][:, :s], K2[:, :s])
    assert np.array_equal(st.Kc[2][:, s:], K2[:, s + Vn:])
    # the Q Cache belongs to the last block's first layer and holds its visual queries
    assert st.q_owner == 3
    assert np.array_equal(st.Qc, np.transpose(inputs[3][0], (1, 0, 2))[:, s:s + Vn])
    for l in range(N):
        st.decode(l, rand(H, D), rand(H, D), rand(H, D))
    assert [st.k_rows(l) for l in range(N)] == [L + 1 - lazy[l] * Vn for l in range(N)]
    assert st.q_owner == 3, "decode never touches the Q Cache"


def test_order_errors():
    st = LazyStackOracle(3, 1, 2, [0, 1, 0], 0, 2)
    x = make_stack_inputs(3, 4, 1, 2)
    with pytest.raises(OrderError):
        st.prefill(1, *x[1])
    with pytest.raises(OrderError):
        st.decode(0, rand(1, 2), rand(1, 2), rand(1, 2))
    st.prefill(0, *x[0])
    with pytest.raises(OrderError):
        st.prefill(0, *x[0])
    with pytest.raises(ValueError):
        LazyStackOracle(2, 1, 2, [1, 0], 0, 1)


# ---------------------------------------------------------------------------
# layout.py: closed-form saving rate from the paper, offsets by brute-force enumeration
# ---------------------------------------------------------------------------
def read_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "kv_saving_closed_form.txt")
    rows = []
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            N, n, V, T, frac = line.split()
            rows.append((int(N), int(n), int(V), int(T), Fraction(frac)))
    return rows


@pytest.mark.parametrize("N,n,V,T,want", read_golden())
def test_kv_saving_matches_paper_closed_form(N, n, V, T, want):
    """Count resident rows in the oracle after prefill; the saving must equal |V|/(|V|+|T|)*n/(2N)."""
    lazy = [0] * N
    for l in range(N - n, N):
        lazy[l] = 1
    H, D = 1, 2
    st = LazyStackOracle(N, H, D, lazy, min(1, T), V)
    z = np.zeros((V + T, H, D))
    for l in range(N):
        st.prefill(l, z, z, z, rows=[0])
    lay = layout.ArenaLayout(N, H, D, "bf16", 1, V + T, max(V, 1), max(T, 1), lazy)
    res = layout.resident_bytes(lay, [st])
    std = layout.standard_kv_bytes(lay, [V + T])
    saving = Fraction(std - res["k_bytes"] - res["v_bytes"], std)
    assert saving == want
    assert layout.vla_kv_saving_closed_form(N, n, V, T) == want
    # Q Cache share of the standard KV cache: visual rows of one layer = V/(V+T) * 1/(2N) <= 1/(2N)
    assert Fraction(res["q_bytes"], std) == Fraction(V, V + T) * Fraction(1, 2 * N)


def test_layout_offsets_are_a_dense_non_overlapping_tiling():
    """Enumerate every element slot of a small arena: K rows and V rows tile [0, rows_bytes) exactly once."""
    lay = layout.ArenaLayout(3, 2, 4, "bf16", 2, 6, 3, 4, [0, 1, 0])
    seen = np.zeros(lay.rows_bytes(), dtype=np.int32)
    rowb = lay.D * lay.e
    for l in range(3):
        for b in range(2):
            for h in range(2):
                for r in range(lay.cap_k(l)):
                    o = lay.k_offset(l, b, h, r)
                    seen[o:o + rowb] += 1
                for r in range(lay.max_seq):
                    o = lay.v_offset(l, b, h, r)
                    seen[o:o + rowb] += 1
    assert lay.rows_bytes() == lay.off_v(3)
    assert np.all(seen == 1)
    assert lay.cap_k(1) == 4 and lay.cap_k(0) == 6
    # lazy layers allocate fewer bytes, not just fewer resident rows
    assert lay.k_layer_bytes(1) * 6 == lay.k_layer_bytes(0) * 4


def test_arena_image_places_rows_where_locate_says():
    N, H, D, L, s, Vn = 3, 2, 4, 7, 1, 3
    lazy = [0, 1, 1]
    lay = layout.ArenaLayout(N, H, D, "f32", 2, 9, 3, 6, lazy)
    stacks = []
    inputs = []
    for b in range(2):
        st = LazyStackOracle(N, H, D, lazy, s, Vn)
        x = [tuple(a.astype(np.float32).astype(np.float64) for a in t) for t in make_stack_inputs(N, L, H, D)]
        for l in range(N):
            st.prefill(l, *x[l])
        stacks.append(st)
        inputs.append(x)
    img = layout.kv_rows_image(lay, stacks)
    assert img.shape == (lay.rows_bytes(),)
    for b in range(2):
        for l in range(N):
            for h in range(H):
                for pos in range(L):
                    src, off = lay.locate_k(l, b, h, pos, s, Vn)
                    got = img[off:off + D * 4].view(np.float32)
                    want = inputs[b][src][1][pos, h].astype(np.float32)
                    assert np.array_equal(got, want), (b, l, h, pos)
                    assert (src, (off - lay.k_offset(src, b, h, 0)) // (D * 4)) == stacks[b].k_source(l, pos)
                    _, off = lay.locate_v(l, b, h, pos)
                    assert np.array_equal(img[off:off + D * 4].view(np.float32),
                                          inputs[b][l][2][pos, h].astype(np.float32))


def test_encode_rows_bf16_is_exact_or_refuses():
    x = torch.randn(5, 8).to(torch.bfloat16)
    raw = layout.encode_rows(x.float().numpy().astype(np.float64), "bf16")
    assert np.array_equal(raw.view(np.uint16).reshape(5, 8), x.view(torch.int16).numpy().view(np.uint16))
    with pytest.raises(ValueError):
        layout.encode_rows(np.array([[1.0 + 2.0 ** -12]]), "bf16")
