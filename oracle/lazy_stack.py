"""Visual Lazy Attention over a decoder stack, one sequence at a time (test infrastructure).

State and rules follow the paper's "Lazy Attention" and "Q Cache" subsections:

* A lazy block is a run of adjacent layers l_c, l_c+1, ..., l_c+n.  Its first
  layer l_c computes ordinary attention; the others are lazy layers.
* Q Cache definition: the cache holds the queries of l_c and is overwritten
  when the next block starts.  Visual Lazy Attention uses its visual rows only.
* Eq. 7 (VLA prefill): in a lazy layer the query and key rows of the visual
  tokens are the Q Cache rows and the K-cache rows of l_c; text rows use the
  layer's own projections; V is the layer's own for every token.
* Eq. 8 (VLA decode): the query is the new text token's own; keys are the
  layer's own text keys, the visual keys of l_c, and the new token's key;
  values are the layer's own.
* "Efficiency Analysis", KV Cache paragraph: a lazy layer keeps no visual K rows.

Readings taken where the paper is silent (each also listed in the design notes):
tokens keep their true positions and the visual tokens are one contiguous span
[vis_start, vis_start + vis_len); the causal mask uses true positions; heads
are independent and head h inherits from head h; generated tokens are text;
layer 0 cannot be lazy; the Q Cache is written during prefill by a normal
layer exactly when the next layer is lazy, and is never touched by decode.

All arithmetic is fp64.  Inputs are token-major [L, H, D] arrays whose values
are taken as given (bf16 inputs arrive already rounded).  Heads are carried as
a leading axis internally; sequences of a batch are separate instances.
"""
import math

import numpy as np

from . import attention


class OrderError(RuntimeError):
    """A layer was called out of sequence, or the Q Cache belongs to another block."""


class LazyStackOracle:
    def __init__(self, n_layers, n_heads, head_dim, lazy_mask, vis_start, vis_len, scale=None):
        lazy_mask = [int(bool(x)) for x in lazy_mask]
        if len(lazy_mask) != n_layers:
            raise ValueError("lazy_mask needs one flag per layer")
        if n_layers > 0 and lazy_mask[0]:
            raise ValueError("layer 0 has no preceding layer to inherit from")
        if vis_start < 0 or vis_len < 0:
            raise ValueError("bad visual span")
        self.N, self.H, self.D = n_layers, n_heads, head_dim
        self.lazy = lazy_mask
        self.s, self.Vn = int(vis_start), int(vis_len)
        self.scale = (1.0 / math.sqrt(head_dim)) if scale is None else float(scale)
        # caches: per layer, [H, rows, D] fp64
        self.Kc = [np.zeros((n_heads, 0, head_dim)) for _ in range(n_layers)]
        self.Vc = [np.zeros((n_heads, 0, head_dim)) for _ in range(n_layers)]
        self.Qc = np.zeros((n_heads, self.Vn, head_dim))
        self.q_owner = -1
        self.len = 0                 # tokens whose K/V are resident in every layer
        self.prefill_len = 0
        self._next_prefill = 0
        self._next_decode = None     # None until prefill has finished

    # ----- structure ---------------------------------------------------------
    def anchor(self, l):
        """First layer l_c of the block that lazy layer l belongs to."""
        if not self.lazy[l]:
            raise ValueError("layer %d is not lazy" % l)
        a = l - 1
        while self.lazy[a]:
            a -= 1
        return a

    def k_source(self, l, pos):
        """(layer, row) holding the key of position `pos` as seen by layer l (Eq. 8)."""
        s, Vn = self.s, self.Vn
        if not self.lazy[l]:
            return (l, pos)
        if pos < s:
            return (l, pos)
        if pos < s + Vn:
            return (self.anchor(l), pos)
        return (l, pos - Vn)

    def k_rows(self, l):
        return self.Kc[l].shape[1]

    def v_rows(self, l):
        return self.Vc[l].shape[1]

    # ----- prefill -----------------------------------------------------------
    @staticmethod
    def _heads_first(X, H, D):
        X = np.asarray(X, dtype=np.float64)
        if X.ndim != 3 or X.shape[1] != H or X.shape[2] != D:
            raise ValueError("expected [L, H, D]")
        return np.transpose(X, (1, 0, 2))

    def effective_qk(self, l, Q, K):
        """Eq. 7: the query and key matrices layer l actually attends with ([H, L, D])."""
        Qh = self._heads_first(Q, self.H, self.D).copy()
        Kh = self._heads_first(K, self.H, self.D).copy()
        if self.lazy[l] and self.Vn > 0:
            a = self.anchor(l)
            if self.q_owner != a:
                raise OrderError("Q Cache holds layer %d, block of layer %d starts at %d"
                                 % (self.q_owner, l, a))
            s, e = self.s, self.s + self.Vn
            Qh[:, s:e, :] = self.Qc
            Kh[:, s:e, :] = self.Kc[a][:, s:e, :]
        return Qh, Kh

    def prefill(self, l, Q, K, V, rows=None, return_scores=False):
        """Layer l over the whole prompt.  Returns O as [L, H, D] (or [len(rows), H, D]).

        `rows` limits which query rows are evaluated (caches are always
        updated in full).  In a lazy layer the span rows of Q and K are never
        read.  With return_scores the pre-softmax score matrix [H, L, L] is
        returned as well (full evaluation only).
        """
        if self._next_decode is not None or l != self._next_prefill:
            raise OrderError("prefill expected layer %d, got %d" % (self._next_prefill, l))
        L = np.asarray(Q).shape[0]
        if l == 0:
            if self.s + self.Vn > L:
                raise ValueError("visual span exceeds the prompt")
            self.prefill_len = L
        elif L != self.prefill_len:
            raise ValueError("prompt length changed between layers")
        Qeff, Keff = self.effective_qk(l, Q, K)
        Vh = self._heads_first(V, self.H, self.D)
        s, e = self.s, self.s + self.Vn
        if not self.lazy[l]:
            self.Kc[l] = Keff.copy()
            if l + 1 < self.N and self.lazy[l + 1]:
                self.Qc = Qeff[:, s:e, :].copy()
                self.q_owner = l
        else:
            Kown = self._heads_first(K, self.H, self.D)
            self.Kc[l] = np.concatenate([Kown[:, :s, :], Kown[:, e:, :]], axis=1)
        self.Vc[l] = Vh.copy()
        self._next_prefill = l + 1
        if l + 1 == self.N:
            self.len = L
            self._next_decode = 0
        if rows is None:
            O = attention.causal_attention(Qeff, Keff, Vh, self.scale)
            O = np.transpose(O, (1, 0, 2))
            if return_scores:
                return O, attention.causal_scores(Qeff, Keff, self.scale)
            return O
        out = np.empty((len(rows), self.H, self.D))
        for n, i in enumerate(rows):
            out[n] = attention.attention_row(Qeff[:, i, :], Keff[:, : i + 1, :], Vh[:, : i + 1, :],
                                             self.scale)
        return out

    # ----- decode ------------------------------------------------------------
    def decode_keys(self, l):
        """Eq. 8: key matrix [H, rows, D] in position order as layer l sees it (cached rows only)."""
        if not self.lazy[l] or self.Vn == 0:
            return self.Kc[l]
        a = self.anchor(l)
        s, e = self.s, self.s + self.Vn
        return np.concatenate([self.Kc[l][:, :s, :], self.Kc[a][:, s:e, :], self.Kc[l][:, s:, :]], axis=1)

    def decode(self, l, q, k, v):
        """One generated token through layer l.  q, k, v: [H, D].  Returns o [H, D]."""
        if self._next_decode is None or l != self._next_decode:
            raise OrderError("decode expected layer %s, got %d" % (self._next_decode, l))
        q = np.asarray(q, dtype=np.float64).reshape(self.H, self.D)
        k = np.asarray(k, dtype=np.float64).reshape(self.H, 1, self.D)
        v = np.asarray(v, dtype=np.float64).reshape(self.H, 1, self.D)
        self.Kc[l] = np.concatenate([self.Kc[l], k], axis=1)
        self.Vc[l] = np.concatenate([self.Vc[l], v], axis=1)
        Kall = self.decode_keys(l)
        o = attention.decode_attention(q, Kall, self.Vc[l], self.scale)
        self._next_decode = l + 1
        if l + 1 == self.N:
            self.len += 1
            self._next_decode = 0
        return o

    # ----- accounting ("Efficiency Analysis", KV Cache paragraph) ------------
    def resident_rows(self):
        """(K rows, V rows, Q Cache rows) summed over layers, per head."""
        return (sum(self.k_rows(l) for l in range(self.N)),
                sum(self.v_rows(l) for l in range(self.N)),
                self.Vn if self.q_owner >= 0 else 0)
