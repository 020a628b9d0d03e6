"""Lazy-block selection from layer-wise attention similarity (test infrastructure).

Follows the paper's "Lazy Attention" subsection:

* The last row a^l of a layer's attention matrix A^l stands for the layer's attention pattern.
* Eq. 3: S(l_m, l_n) = (1/N) sum_i JS(a_i^{l_m}, a_i^{l_n}) over N input samples, with
  JS(p, q) = (KL(p || m) + KL(q || m)) / 2 and m = (p + q) / 2.
* Eq. 4: a lazy block is a run of adjacent layers l_c .. l_c+n in which every adjacent pair has
  S(l_i, l_i+1) < epsilon, 0 < epsilon <= 1; its first layer stays an ordinary layer, the others
  become lazy layers.

Readings taken where the paper is silent (also listed in the design notes): the averaging over
attention heads that the paragraph before Eq. 3 mentions is applied to the attention rows (a^l is
the mean over heads of the per-head last rows, as in the token-pruning work the paper cites for the
last-row idea); logarithms are natural, so that JS <= ln 2 (the appendix on similarity inside the
language model plots ln 2 - S, which fixes the unit; the stated range 0 < epsilon <= 1 is then a
loose bound); terms with zero probability contribute zero; blocks are maximal runs.

All arithmetic is fp64.
"""
import numpy as np

from . import attention


def last_row_attention(q_last, K, scale):
    """a^l for one sample: q_last [H, D] (query of the last token), K [H, L, D] -> [L] (sums to 1)."""
    q_last = np.asarray(q_last, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    scores = np.einsum("hd,hld->hl", q_last, K) * scale      # the last row sees every key
    return attention.softmax_lastaxis(scores).mean(axis=0)


def kl_divergence(p, m):
    """KL(p || m) in nats; entries with p = 0 contribute nothing."""
    p = np.asarray(p, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    nz = p > 0
    return float(np.sum(p[nz] * (np.log(p[nz]) - np.log(m[nz]))))


def js_divergence(p, q):
    """Eq. 3, second line."""
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    m = (p + q) / 2.0
    return 0.5 * (kl_divergence(p, m) + kl_divergence(q, m))


def similarity(rows_m, rows_n):
    """Eq. 3, first line: rows_m[i], rows_n[i] are a_i^{l_m}, a_i^{l_n} of sample i (lengths may differ per i)."""
    if len(rows_m) != len(rows_n) or not rows_m:
        raise ValueError("need the same, non-zero number of samples for both layers")
    return sum(js_divergence(p, q) for p, q in zip(rows_m, rows_n)) / len(rows_m)


def lazy_mask_from_similarity(adjacent, eps):
    """Eq. 4.  adjacent[i] = S(l_i, l_i+1) for i = 0 .. N-2.  Returns N flags (1 = lazy layer)."""
    if not (0.0 < eps <= 1.0):
        raise ValueError("epsilon must lie in (0, 1]")
    n_layers = len(adjacent) + 1
    mask = [0] * n_layers
    start = 0                                   # first layer of the run being grown
    for i in range(1, n_layers):
        if adjacent[i - 1] < eps:
            mask[i] = 1                         # layer i joins the run that starts at `start`
        else:
            start = i                           # the run ends; layer i may start the next one
    assert mask[0] == 0 and start >= 0
    return mask


def blocks_of(mask):
    """The lazy blocks of a mask as (first layer, last layer) pairs, single ordinary layers left out."""
    out, c = [], None
    for i, f in enumerate(list(mask) + [0]):
        if i < len(mask) and f:
            continue
        if c is not None and i - 1 > c:
            out.append((c, i - 1))
        c = i
    return out
