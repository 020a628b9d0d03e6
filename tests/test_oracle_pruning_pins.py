"""Pins for oracle.pruning: nothing here calls the function under test to produce its own expectation.

* the ranking against an exhaustive search over subsets, and its nesting property;
* the pruned stack against the unpruned stack oracles: keeping everything changes nothing, and
  dropping a token equals giving its key a weight of exactly zero in the full-length computation
  (a score so low that exp() underflows to 0 in fp64);
* the resident rows against a count written out by hand.
"""
import itertools

import numpy as np
import pytest

from oracle.global_lazy_stack import GlobalLazyStackOracle
from oracle.lazy_stack import LazyStackOracle
from oracle.pruning import (PrunedStackOracle, kept_visual_positions, packed_row_map, surviving_positions)


def exhaustive_best_subset(span_scores, keep):
    """Highest total score; among equal totals the lexicographically smallest positions."""
    best = None
    for combo in itertools.combinations(range(len(span_scores)), keep):
        key = (-sum(float(span_scores[i]) for i in combo), combo)
        if best is None or key < best:
            best = key
    return list(best[1])


@pytest.mark.parametrize("seed", range(6))
def test_ranking_matches_exhaustive_search(seed):
    rng = np.random.default_rng(seed)
    vis_start, vis_len, length = 3, 7, 13
    # small integers: sums are exact, ties are frequent
    scores = rng.integers(0, 4, size=length).astype(np.float32)
    for keep in range(vis_len + 1):
        want = [vis_start + i for i in exhaustive_best_subset(scores[vis_start:vis_start + vis_len], keep)]
        got = kept_visual_positions(scores, vis_start, vis_len, keep)
        assert got.tolist() == want


def test_ranking_is_nested_and_bounded():
    rng = np.random.default_rng(11)
    scores = rng.random(64).astype(np.float32)
    prev = set()
    for keep in range(41):
        got = kept_visual_positions(scores, 10, 40, keep)
        assert len(got) == keep and np.all(np.diff(got) > 0)
        assert got.size == 0 or (got.min() >= 10 and got.max() < 50)
        assert prev <= set(got.tolist())
        prev = set(got.tolist())
    assert kept_visual_positions(scores, 10, 40, 40).tolist() == list(range(10, 50))
    with pytest.raises(ValueError):
        kept_visual_positions(scores, 10, 40, 41)


def test_ranking_ignores_scores_outside_the_span():
    scores = np.array([9, 9, 1, 3, 2, 9, 9], dtype=np.float32)
    assert kept_visual_positions(scores, 2, 3, 2).tolist() == [3, 4]
    assert kept_visual_positions(scores, 2, 3, 1).tolist() == [3]


def test_surviving_positions_and_row_map():
    pos = surviving_positions(10, 2, 5, [3, 6])
    assert pos.tolist() == [0, 1, 3, 6, 7, 8, 9]
    rm = packed_row_map([10, 4], [2, 1], [5, 2], [[3, 6], []])
    assert rm.tolist() == [0, 1, 3, 6, 7, 8, 9, 10, 13]


def make_inputs(rng, n_layers, L, H, D):
    return [tuple(rng.standard_normal((L, H, D)) for _ in range(3)) for _ in range(n_layers)]


MASKS = [([0, 0, 0, 0, 0], 2), ([0, 0, 1, 0, 1], 3), ([0, 1, 1, 0, 1, 1], 3), ([0, 1, 0, 0], 2)]


@pytest.mark.parametrize("mode", ["vla", "gla"])
@pytest.mark.parametrize("mask,first_late", MASKS)
def test_keeping_every_token_changes_nothing(mode, mask, first_late):
    rng = np.random.default_rng(5)
    N, H, D, L, s, Vn, steps = len(mask), 2, 8, 14, 3, 6, 3
    pr = PrunedStackOracle(N, H, D, mask, s, Vn, first_late, Vn, mode=mode)
    if mode == "gla":
        plain = GlobalLazyStackOracle(N, H, D, mask, vis_start=s, vis_len=Vn)
    else:
        plain = LazyStackOracle(N, H, D, mask, s, Vn)
    for l, (Q, K, V) in enumerate(make_inputs(rng, N, L, H, D)):
        assert np.array_equal(pr.prefill(l, Q, K, V), plain.prefill(l, Q, K, V))
    for _ in range(steps):
        for l in range(N):
            q, k, v = (rng.standard_normal((H, D)) for _ in range(3))
            assert np.array_equal(pr.decode(l, q, k, v), plain.decode(l, q, k, v))
    assert pr.resident_rows() == plain.resident_rows()
    assert pr.q_owner == plain.q_owner


@pytest.mark.parametrize("mode", ["vla", "gla"])
@pytest.mark.parametrize("mask,first_late", MASKS)
def test_dropping_equals_zero_weight_in_the_full_computation(mode, mask, first_late):
    """Late layers at full length with a flag coordinate: every query carries 1 there, surviving keys 0,
    dropped keys -1e7, so a dropped key's softmax weight is exactly 0.  The unpruned stack oracle on
    those inputs must agree with the pruned one on the gathered inputs at every surviving row."""
    rng = np.random.default_rng(9)
    N, H, D, L, s, Vn, steps = len(mask), 2, 8, 15, 4, 7, 3
    kept = np.array([5, 6, 9])
    surv = surviving_positions(L, s, Vn, kept)
    dropped = np.setdiff1d(np.arange(L), surv)
    full = make_inputs(rng, N, L, H, D)
    for l in range(first_late, N):
        Q, K, V = full[l]
        Q[:, :, 0] = 1.0
        K[:, :, 0] = 0.0
        K[dropped, :, 0] = -1e7
    pr = PrunedStackOracle(N, H, D, mask, s, Vn, first_late, len(kept), mode=mode)
    if mode == "gla":
        plain = GlobalLazyStackOracle(N, H, D, mask, vis_start=s, vis_len=Vn)
    else:
        plain = LazyStackOracle(N, H, D, mask, s, Vn)
    for l in range(N):
        Q, K, V = full[l]
        want = plain.prefill(l, Q, K, V)
        if l < first_late:
            got = pr.prefill(l, Q, K, V)
        else:
            got = pr.prefill(l, Q[surv], K[surv], V[surv])
            want = want[surv]
        assert np.max(np.abs(got - want)) < 1e-12
    for _ in range(steps):
        for l in range(N):
            q, k, v = (rng.standard_normal((H, D)) for _ in range(3))
            if l >= first_late:
                q[:, 0] = 1.0
                k[:, 0] = 0.0
            assert np.max(np.abs(pr.decode(l, q, k, v) - plain.decode(l, q, k, v))) < 1e-12


@pytest.mark.parametrize("mode", ["vla", "gla"])
def test_resident_rows_written_out(mode):
    mask, first_late = [0, 1, 1, 0, 1, 0], 3
    N, H, D, L, s, Vn, keep, steps = len(mask), 1, 4, 20, 2, 11, 4, 2
    rng = np.random.default_rng(1)
    pr = PrunedStackOracle(N, H, D, mask, s, Vn, first_late, keep, mode=mode)
    Lp = L - (Vn - keep)
    for l in range(N):
        n = L if l < first_late else Lp
        pr.prefill(l, *(rng.standard_normal((n, H, D)) for _ in range(3)))
    for _ in range(steps):
        for l in range(N):
            pr.decode(l, *(rng.standard_normal((H, D)) for _ in range(3)))
    Le, Ll = L + steps, Lp + steps
    # layers 0 (ordinary), 1, 2 (lazy) see Le positions; 3 (ordinary), 4 (lazy), 5 (ordinary) see Ll
    if mode == "vla":
        k_rows = Le + 2 * (Le - Vn) + Ll + (Ll - keep) + Ll
        q_rows = keep                       # written last by layer 3
    else:
        k_rows = Le + 0 + 0 + Ll + 0 + Ll
        q_rows = Ll
    assert pr.resident_rows() == (k_rows, 3 * Le + 3 * Ll, q_rows)
    assert pr.q_owner == 3


def test_boundary_inside_a_block_is_refused():
    with pytest.raises(ValueError):
        PrunedStackOracle(4, 1, 4, [0, 0, 1, 0], 0, 4, 2, 2)
    with pytest.raises(ValueError):
        PrunedStackOracle(4, 1, 4, [0, 0, 1, 0], 0, 4, 0, 2)
    with pytest.raises(ValueError):
        PrunedStackOracle(4, 1, 4, [0, 0, 1, 0], 0, 4, 1, 5)
