"""Pins for the lazy-block selection oracle (Eq. 3 / Eq. 4) against things that are not itself:
a library Jensen-Shannon routine, closed forms, the attention oracle's full matrix, brute force."""
import itertools
import math

import numpy as np
import pytest
import scipy.spatial.distance
import scipy.stats

from oracle import attention, selection

RNG = np.random.default_rng(77)


def rand_dist(n, zeros=0):
    p = RNG.random(n)
    if zeros:
        p[RNG.choice(n, zeros, replace=False)] = 0.0
    return p / p.sum()


@pytest.mark.parametrize("n,zeros", [(2, 0), (7, 0), (64, 5), (300, 100)])
def test_js_matches_library_routine(n, zeros):
    p, q = rand_dist(n, zeros), rand_dist(n, zeros)
    want = scipy.spatial.distance.jensenshannon(p, q) ** 2      # natural logarithm; the library returns the square root
    assert abs(selection.js_divergence(p, q) - want) < 1e-12
    m = (p + q) / 2
    want2 = 0.5 * (scipy.stats.entropy(p, m) + scipy.stats.entropy(q, m))
    assert abs(selection.js_divergence(p, q) - want2) < 1e-12


def test_js_closed_forms_symmetry_and_bounds():
    p = rand_dist(40, 7)
    q = rand_dist(40, 3)
    assert selection.js_divergence(p, p) == 0.0
    assert selection.js_divergence(p, q) == selection.js_divergence(q, p)
    assert 0.0 < selection.js_divergence(p, q) < math.log(2)
    a = np.array([0.5, 0.5, 0.0, 0.0])
    b = np.array([0.0, 0.0, 0.25, 0.75])
    assert abs(selection.js_divergence(a, b) - math.log(2)) < 1e-15    # disjoint supports: exactly ln 2, the upper bound
    # two-point closed form: JS((1,0),(t,1-t)) = 1/2 [ -ln((1+t)/2) + t ln(2t/(1+t)) + (1-t) ln 2 ]
    t = 0.3
    want = 0.5 * (-math.log((1 + t) / 2) + t * math.log(2 * t / (1 + t)) + (1 - t) * math.log(2))
    assert abs(selection.js_divergence([1.0, 0.0], [t, 1 - t]) - want) < 1e-15
    # entropy form: JS = H(m) - (H(p) + H(q)) / 2
    H = lambda x: scipy.stats.entropy(x)
    assert abs(selection.js_divergence(p, q) - (H((p + q) / 2) - 0.5 * (H(p) + H(q)))) < 1e-12


def test_similarity_is_the_mean_over_samples():
    ps = [rand_dist(n) for n in (5, 9, 17)]
    qs = [rand_dist(n) for n in (5, 9, 17)]
    want = sum(scipy.spatial.distance.jensenshannon(p, q) ** 2 for p, q in zip(ps, qs)) / 3
    assert abs(selection.similarity(ps, qs) - want) < 1e-12
    with pytest.raises(ValueError):
        selection.similarity(ps, qs[:2])


def test_last_row_attention_is_the_last_row_of_the_full_matrix_averaged_over_heads():
    H, L, D = 3, 11, 4
    Q, K = RNG.standard_normal((H, L, D)), RNG.standard_normal((H, L, D))
    scale = 0.5
    sc = attention.causal_scores(Q, K, scale)                          # [H, L, L], -inf above the diagonal
    full = np.exp(sc - sc.max(axis=-1, keepdims=True))
    full /= full.sum(axis=-1, keepdims=True)
    want = full[:, -1, :].mean(axis=0)
    got = selection.last_row_attention(Q[:, -1, :], K, scale)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-15)
    assert abs(got.sum() - 1.0) < 1e-14
    # scalar brute force for one entry
    j = 4
    per_head = []
    for h in range(H):
        s = [scale * sum(Q[h, -1, d] * K[h, i, d] for d in range(D)) for i in range(L)]
        z = sum(math.exp(x - max(s)) for x in s)
        per_head.append(math.exp(s[j] - max(s)) / z)
    assert abs(got[j] - sum(per_head) / H) < 1e-15


def brute_force_mask(adjacent, eps):
    """All ways to cut the layer sequence into runs; keep those whose inner pairs are all < eps and
    pick the one with the fewest runs (maximal runs); layers that do not start a run are lazy."""
    n = len(adjacent) + 1
    best = None
    for cuts in itertools.product([0, 1], repeat=n - 1):               # cuts[i] = 1: a run starts at layer i + 1
        ok = all(cuts[i] or adjacent[i] < eps for i in range(n - 1))
        if ok and (best is None or sum(cuts) < sum(best)):
            best = cuts
    return [0] + [0 if c else 1 for c in best]


def test_grouping_matches_brute_force_over_all_partitions():
    for trial in range(40):
        n = int(RNG.integers(2, 9))
        adj = RNG.random(n - 1)
        eps = float(RNG.uniform(0.2, 0.8))
        assert selection.lazy_mask_from_similarity(adj, eps) == brute_force_mask(adj, eps)


def test_grouping_examples_and_edges():
    adj = [0.9, 0.1, 0.2, 0.7, 0.05, 0.6]
    mask = selection.lazy_mask_from_similarity(adj, 0.5)
    assert mask == [0, 0, 1, 1, 0, 1, 0]
    assert selection.blocks_of(mask) == [(1, 3), (4, 5)]
    assert selection.lazy_mask_from_similarity([0.5], 0.5) == [0, 0]   # strict inequality
    assert selection.lazy_mask_from_similarity([0.1, 0.1, 0.1], 1.0) == [0, 1, 1, 1]
    assert selection.lazy_mask_from_similarity([], 0.3) == [0]
    for bad in (0.0, 1.5, -0.1):
        with pytest.raises(ValueError):
            selection.lazy_mask_from_similarity(adj, bad)
