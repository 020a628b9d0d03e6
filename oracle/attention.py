"""Softmax attention in fp64, written out from its definition (test infrastructure).

Eq. 1 of the paper (prefill):  A = Softmax((Q K^T + M) / sqrt(D)),  O = A V,
with M the causal mask (A is lower triangular).
Eq. 2 of the paper (decode):   one query row against all cached keys plus the
new one, no mask.

Nothing here is blocked, fused or reordered: scores, softmax, weighted sum.
`attention_scalar` is a second, independent formulation (Python scalars and
math.exp only) used to pin the vectorised functions on tiny inputs.
"""
import math

import numpy as np


def softmax_lastaxis(scores):
    """Softmax over the last axis in fp64; -inf entries get weight 0.

    Every row must hold at least one finite entry (true for causal attention,
    where the diagonal is never masked).
    """
    scores = np.asarray(scores, dtype=np.float64)
    top = np.max(scores, axis=-1, keepdims=True)
    weights = np.exp(scores - top)
    return weights / np.sum(weights, axis=-1, keepdims=True)


def causal_scores(Q, K, scale):
    """(Q K^T + M) * scale with M = 0 on and below the diagonal, -inf above (Eq. 1).

    Q: [..., Lq, D], K: [..., Lk, D] with Lq == Lk (prefill: query i sits at
    position i).  Returns [..., Lq, Lk].
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    L = Q.shape[-2]
    if K.shape[-2] != L:
        raise ValueError("prefill attention needs as many keys as queries")
    S = np.matmul(Q, np.swapaxes(K, -1, -2)) * scale
    above = np.triu(np.ones((L, L), dtype=bool), k=1)
    return np.where(above, -np.inf, S)


def causal_attention(Q, K, V, scale=None):
    """Eq. 1: O = Softmax(causal scores) V.  Shapes [..., L, D]; returns fp64 [..., L, D]."""
    Q = np.asarray(Q, dtype=np.float64)
    if scale is None:
        scale = 1.0 / math.sqrt(Q.shape[-1])
    A = softmax_lastaxis(causal_scores(Q, K, scale))
    return np.matmul(A, np.asarray(V, dtype=np.float64))


def decode_attention(q, K, V, scale=None):
    """Eq. 2: one query row q [..., D] against K, V [..., L, D] (new token's row included)."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    if scale is None:
        scale = 1.0 / math.sqrt(q.shape[-1])
    s = np.einsum("...d,...jd->...j", q, K) * scale
    a = softmax_lastaxis(s)
    return np.einsum("...j,...jd->...d", a, V)


def attention_row(q_row, K, V, scale):
    """Output of a single query row that may attend to every row of K, V given ([n, D])."""
    return decode_attention(q_row, K, V, scale)


def attention_scalar(Q, K, V, scale, causal):
    """Independent brute force: nested Python loops over (i, j, d), math.exp, lists.

    Q: Lq x D, K: Lk x D, V: Lk x Dv as nested lists or arrays.  With `causal`
    query i attends keys j <= i + (Lk - Lq) (so a single decode row, Lq == 1,
    sees every key).  Only for tiny sizes.
    """
    Lq, Lk = len(Q), len(K)
    D, Dv = len(Q[0]), len(V[0])
    shift = Lk - Lq
    out = []
    for i in range(Lq):
        last = i + shift if causal else Lk - 1
        s = []
        for j in range(last + 1):
            acc = 0.0
            for d in range(D):
                acc += float(Q[i][d]) * float(K[j][d])
            s.append(acc * scale)
        top = max(s)
        e = [math.exp(x - top) for x in s]
        z = sum(e)
        row = []
        for d in range(Dv):
            acc = 0.0
            for j in range(last + 1):
                acc += e[j] / z * float(V[j][d])
            row.append(acc)
        out.append(row)
    return out
