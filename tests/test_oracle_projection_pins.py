"""Pins for the projection + rotary-embedding oracle against things that are not itself: scalar
brute force, the complex-number form of the rotation, its algebraic invariants, the paper's
closed-form share of omitted projector work."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import projection

RNG = np.random.default_rng(99)


def test_frequencies_closed_form():
    ang = projection.rope_angles([0, 1, 7], 4, 10000.0)
    np.testing.assert_allclose(ang, [[0, 0], [1, 0.01], [7, 0.07]], rtol=0, atol=1e-15)
    ang = projection.rope_angles([3], 8, 16.0)      # theta^(-2d/D) = 16^(-d/4) = 1, 1/2, 1/4, 1/8
    np.testing.assert_allclose(ang, [[3, 1.5, 0.75, 0.375]], rtol=0, atol=1e-15)


def test_rope_is_complex_multiplication_of_the_half_pairs():
    rows, H, D, theta = 5, 2, 8, 10000.0
    x = RNG.standard_normal((rows, H, D))
    pos = [0, 1, 2, 50, 4095]
    got = projection.apply_rope(x, pos, theta)
    z = x[..., :D // 2] + 1j * x[..., D // 2:]
    w = np.exp(1j * np.array(pos)[:, None, None] * theta ** (-2.0 * np.arange(D // 2) / D)[None, None, :])
    want = z * w
    np.testing.assert_allclose(got[..., :D // 2], want.real, rtol=0, atol=1e-12)
    np.testing.assert_allclose(got[..., D // 2:], want.imag, rtol=0, atol=1e-12)


def test_rope_invariants():
    rows, H, D, theta = 6, 3, 16, 500.0
    q, k = RNG.standard_normal((rows, H, D)), RNG.standard_normal((rows, H, D))
    pos = np.array([0, 3, 9, 10, 200, 1000])
    rq, rk = projection.apply_rope(q, pos, theta), projection.apply_rope(k, pos, theta)
    np.testing.assert_array_equal(rq[0], q[0])                                      # position 0: identity
    half = D // 2
    np.testing.assert_allclose(rq[..., :half] ** 2 + rq[..., half:] ** 2,          # pair norms are kept
                               q[..., :half] ** 2 + q[..., half:] ** 2, rtol=1e-12)
    # scores depend on the position difference only
    for (m, n) in [(1, 2), (4, 1), (5, 3)]:
        a = np.einsum("hd,hd->h", rq[m], rk[n])
        shifted_q = projection.apply_rope(q[m:m + 1], [pos[m] - pos[n]], theta)[0]
        b = np.einsum("hd,hd->h", shifted_q, k[n])
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-10)
    np.testing.assert_array_equal(projection.apply_rope(q, pos, 0.0), q)             # theta 0: no rotation


def test_projection_scalar_brute_force():
    T, dm, H, D = 4, 6, 2, 4
    X = RNG.standard_normal((T, dm))
    Wq, Wk = RNG.standard_normal((H * D, dm)), RNG.standard_normal((H * D, dm))
    rows, pos, theta = [0, 2, 3], [5, 7, 8], 100.0
    Q, K = projection.project_qk(X, Wq, Wk, H, D, rows, pos, theta)
    for W, got in ((Wq, Q), (Wk, K)):
        for r, (t, p) in enumerate(zip(rows, pos)):
            for h in range(H):
                y = [sum(X[t][c] * W[h * D + d][c] for c in range(dm)) for d in range(D)]
                for d in range(D // 2):
                    ang = p * theta ** (-2.0 * d / D)
                    lo = y[d] * math.cos(ang) - y[d + D // 2] * math.sin(ang)
                    hi = y[d + D // 2] * math.cos(ang) + y[d] * math.sin(ang)
                    assert abs(got[r, h, d] - lo) < 1e-12 and abs(got[r, h, d + D // 2] - hi) < 1e-12


def test_text_rows_and_the_papers_share_of_omitted_work():
    assert projection.text_rows(10, 3, 4) == [0, 1, 2, 7, 8, 9]
    assert projection.text_rows(5, 0, 5) == []
    assert projection.text_rows(5, 2, 0) == [0, 1, 2, 3, 4]
    # n lazy layers, both projectors each: omitted work / (one projector over all tokens) = |V|/(|V|+|T|) * 2n
    import os
    golden = []
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "projection_saving_closed_form.txt")):
        if line.strip() and not line.startswith("#"):
            N, n, V, T, frac = line.split()
            golden.append((int(N), int(n), int(V), int(T), Fraction(frac)))
    assert len(golden) == 3
    for (N, n, V, T, want) in golden:
        L, dm, H, D = V + T, 64, 2, 8
        full = projection.projector_flops(L, dm, H, D)
        done_lazy = 2 * projection.projector_flops(len(projection.text_rows(L, 5, V)), dm, H, D)
        omitted = n * (2 * full - done_lazy)
        assert Fraction(omitted, full) == want == projection.vla_projection_saving(n, V, T)
