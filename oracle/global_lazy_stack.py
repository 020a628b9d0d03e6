"""Global Lazy Attention over a decoder stack, one sequence at a time (test infrastructure).

Follows the paper's "Q Cache" subsection, GLA mode:

* Eq. 5 (GLA prefill): a lazy layer l_i of a block attends with the Q Cache (the queries of
  the block's first layer l_c, every token) and with the K cache of l_c (every token); its
  values are its own.
* Eq. 6 (GLA decode): the same for the token being generated: the query is the Q Cache, the
  keys are the K cache of l_c (which by then includes the new token's key, appended when
  l_c ran earlier in the same step), the values are the layer's own cache plus the new row.
* The sentence after Eq. 6 and "Efficiency Analysis", KV Cache paragraph: a lazy layer
  computes no query or key and stores no K rows at all; the Q Cache is one layer's worth of
  queries, 1/(2N) of a standard KV cache.

Readings taken where the paper is silent (listed in the design notes as well): heads are
independent and head h inherits from head h; layer 0 cannot be lazy; the Q Cache is written
by an ordinary layer exactly when the next layer is lazy; it is indexed by token position,
so during decode the first layer of a block stores the new token's query at row `len` and
the lazy layers of the block read that row; rows written by an earlier block stay until
overwritten.

All arithmetic is fp64; inputs are [L, H, D] (prefill) or [H, D] (decode) and are taken as
given.  A lazy layer's q and k arguments are never looked at and may be None.
"""
import math

import numpy as np

from . import attention


class OrderError(RuntimeError):
    """A layer was called out of sequence, or the Q Cache belongs to another block."""


def _heads_first(X, H, D):
    X = np.asarray(X, dtype=np.float64)
    if X.ndim != 3 or X.shape[1] != H or X.shape[2] != D:
        raise ValueError("expected [L, H, D]")
    return np.transpose(X, (1, 0, 2))


class GlobalLazyStackOracle:
    def __init__(self, n_layers, n_heads, head_dim, lazy_mask, scale=None, vis_start=0, vis_len=0):
        lazy_mask = [int(bool(x)) for x in lazy_mask]
        if len(lazy_mask) != n_layers:
            raise ValueError("lazy_mask needs one flag per layer")
        if n_layers > 0 and lazy_mask[0]:
            raise ValueError("layer 0 has no preceding layer to inherit from")
        self.N, self.H, self.D = n_layers, n_heads, head_dim
        self.lazy = lazy_mask
        self.scale = (1.0 / math.sqrt(head_dim)) if scale is None else float(scale)
        self.s, self.Vn = int(vis_start), int(vis_len)   # recorded for the arena's metadata only: GLA ignores the span
        self.Kc = [np.zeros((n_heads, 0, head_dim)) for _ in range(n_layers)]   # lazy layers stay empty
        self.Vc = [np.zeros((n_heads, 0, head_dim)) for _ in range(n_layers)]
        self.Qc = np.zeros((n_heads, 0, head_dim))   # row p = query of position p, from layer q_owner
        self.q_owner = -1
        self.len = 0
        self.prefill_len = 0
        self._next_prefill = 0
        self._next_decode = None

    def first_layer_of_block(self, l):
        """l_c of the block lazy layer l belongs to: the nearest preceding ordinary layer."""
        if not self.lazy[l]:
            raise ValueError("layer %d is not lazy" % l)
        c = l
        while self.lazy[c]:
            c -= 1
        return c

    def _writes_q(self, l):
        return (not self.lazy[l]) and l + 1 < self.N and bool(self.lazy[l + 1])

    def _block_start_checked(self, l):
        c = self.first_layer_of_block(l)
        if self.q_owner != c:
            raise OrderError("Q Cache holds layer %d, block of layer %d starts at %d" % (self.q_owner, l, c))
        return c

    # ----- prefill (Eq. 1 for an ordinary layer, Eq. 5 for a lazy one) ----------------------
    def prefill(self, l, Q, K, V, rows=None):
        """Returns O as [L, H, D], or [len(rows), H, D] when only some query rows are wanted."""
        if self._next_decode is not None or l != self._next_prefill:
            raise OrderError("prefill expected layer %d, got %d" % (self._next_prefill, l))
        Vh = _heads_first(V, self.H, self.D)
        L = Vh.shape[1]
        if l == 0:
            self.prefill_len = L
        elif L != self.prefill_len:
            raise ValueError("prompt length changed between layers")
        if self.lazy[l]:
            c = self._block_start_checked(l)
            Qh = self.Qc           # Q^{l_i} = Q Cache
            Kh = self.Kc[c]        # K^{l_i} = K cache of l_c
        else:
            Qh = _heads_first(Q, self.H, self.D)
            Kh = _heads_first(K, self.H, self.D)
            self.Kc[l] = Kh.copy()
            if self._writes_q(l):
                self.Qc = Qh.copy()
                self.q_owner = l
        self.Vc[l] = Vh.copy()
        self._next_prefill = l + 1
        if l + 1 == self.N:
            self.len = L
            self._next_decode = 0
        if rows is None:
            return np.transpose(attention.causal_attention(Qh, Kh, Vh, self.scale), (1, 0, 2))
        out = np.empty((len(rows), self.H, self.D))
        for n, i in enumerate(rows):
            out[n] = attention.attention_row(Qh[:, i, :], Kh[:, : i + 1, :], Vh[:, : i + 1, :], self.scale)
        return out

    # ----- decode (Eq. 2 for an ordinary layer, Eq. 6 for a lazy one) -----------------------
    def decode(self, l, q, k, v):
        """One generated token through layer l.  q, k, v: [H, D] (q, k unused if lazy).  Returns [H, D]."""
        if self._next_decode is None or l != self._next_decode:
            raise OrderError("decode expected layer %s, got %d" % (self._next_decode, l))
        v = np.asarray(v, dtype=np.float64).reshape(self.H, 1, self.D)
        self.Vc[l] = np.concatenate([self.Vc[l], v], axis=1)
        if self.lazy[l]:
            c = self._block_start_checked(l)
            if self.Qc.shape[1] != self.len + 1 or self.Kc[c].shape[1] != self.len + 1:
                raise OrderError("the block's first layer has not run in this step")
            q_eff = self.Qc[:, self.len, :]
            keys = self.Kc[c]
        else:
            q_eff = np.asarray(q, dtype=np.float64).reshape(self.H, self.D)
            k = np.asarray(k, dtype=np.float64).reshape(self.H, 1, self.D)
            self.Kc[l] = np.concatenate([self.Kc[l], k], axis=1)
            keys = self.Kc[l]
            if self._writes_q(l):
                self.Qc = np.concatenate([self.Qc[:, : self.len, :], q_eff[:, None, :]], axis=1)
                self.q_owner = l
        o = attention.decode_attention(q_eff, keys, self.Vc[l], self.scale)
        self._next_decode = l + 1
        if l + 1 == self.N:
            self.len += 1
            self._next_decode = 0
        return o

    # ----- accounting ("Efficiency Analysis", KV Cache paragraph) ---------------------------
    def k_rows(self, l):
        return self.Kc[l].shape[1]

    def v_rows(self, l):
        return self.Vc[l].shape[1]

    def resident_rows(self):
        """(K rows, V rows, Q Cache rows) summed over layers, per head."""
        return (sum(self.k_rows(l) for l in range(self.N)),
                sum(self.v_rows(l) for l in range(self.N)),
                self.Qc.shape[1] if self.q_owner >= 0 else 0)
