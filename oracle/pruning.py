"""Token-wise pruning on top of Lazy Attention (test infrastructure).

The paper's "Compatibility" paragraph and its table (VLA with FastV) state that a token pruning
method can be applied to a model that already runs Lazy Attention, and give no further detail.
This module restates what such a combination computes, in the simplest form that statement
allows:

* Pruning happens once, between two layers.  Layers before the boundary ("early") see the whole
  prompt; layers from the boundary on ("late") see every text token and a subset of the visual
  tokens, as FastV-style methods do (they rank the visual tokens by the attention they receive in
  the last early layer and keep the best ones).  Nothing else about a late layer changes: it is a
  decoder layer over a shorter sequence, so its cache rows, its visual span and its lazy blocks
  are those of the shorter sequence.
* A lazy block cannot contain the boundary: a lazy layer takes rows of its block's first layer by
  position, which is only defined when both index the same sequence.  The first late layer must be
  an ordinary layer.
* Which tokens survive: the `keep` visual tokens with the highest score, a tie going to the lower
  position; the survivors keep their order.

`PrunedStackOracle` is therefore nothing but two independent stack oracles, one per side of the
boundary, with the layer indices and the cache views stitched together.
"""
import numpy as np

from .global_lazy_stack import GlobalLazyStackOracle
from .lazy_stack import LazyStackOracle


def kept_visual_positions(scores, vis_start, vis_len, keep):
    """Positions (ascending) of the `keep` best visual tokens of one sequence.

    `scores[p]` ranks position p (only the span is looked at).  The comparison is done in the
    precision the scores arrive in.
    """
    if not 0 <= keep <= vis_len:
        raise ValueError("keep must lie in [0, vis_len]")
    span = np.asarray(scores)[vis_start:vis_start + vis_len]
    order = np.argsort(-span, kind="stable")          # descending; equal scores stay in position order
    return np.sort(vis_start + order[:keep]).astype(np.int64)


def surviving_positions(length, vis_start, vis_len, kept):
    """Positions of the shortened sequence in order: text before the span, kept visual tokens, the rest."""
    kept = np.asarray(kept, dtype=np.int64)
    return np.concatenate([np.arange(vis_start, dtype=np.int64), kept,
                           np.arange(vis_start + vis_len, length, dtype=np.int64)])


def packed_row_map(seq_len, vis_start, vis_len, kept_per_seq):
    """Row index into the packed prompts of every surviving token of a batch, sequence after sequence."""
    out, start = [], 0
    for L, s, n, kept in zip(seq_len, vis_start, vis_len, kept_per_seq):
        out.append(start + surviving_positions(L, s, n, kept))
        start += L
    return np.concatenate(out) if out else np.zeros(0, dtype=np.int64)


class PrunedStackOracle:
    """A decoder stack whose layers >= first_late see vis_len - keep fewer visual tokens.

    Layer indices are those of the whole stack.  Inputs of an early layer are [L, H, D], of a late
    layer [L - (vis_len - keep), H, D] (the caller has dropped the rows).  `mode` picks Visual or
    Global Lazy Attention for both sides.
    """

    def __init__(self, n_layers, n_heads, head_dim, lazy_mask, vis_start, vis_len, first_late, keep,
                 mode="vla", scale=None):
        lazy_mask = [int(bool(x)) for x in lazy_mask]
        if not 1 <= first_late < n_layers:
            raise ValueError("the boundary must have layers on both sides")
        if lazy_mask[first_late]:
            raise ValueError("the boundary falls inside a lazy block")
        if not 0 <= keep <= vis_len:
            raise ValueError("keep must lie in [0, vis_len]")
        self.N, self.H, self.D = n_layers, n_heads, head_dim
        self.lazy = lazy_mask
        self.P = first_late
        self.dropped = vis_len - keep
        self.mode = mode

        def make(mask, vn):
            if mode == "gla":
                return GlobalLazyStackOracle(len(mask), n_heads, head_dim, mask, scale=scale,
                                             vis_start=vis_start, vis_len=vn)
            return LazyStackOracle(len(mask), n_heads, head_dim, mask, vis_start, vn, scale=scale)

        self.early = make(lazy_mask[:first_late], vis_len)
        self.late = make(lazy_mask[first_late:], keep)

    def _side(self, l):
        return (self.early, l) if l < self.P else (self.late, l - self.P)

    def prefill(self, l, Q, K, V, rows=None):
        st, i = self._side(l)
        if st is self.late and i == 0:
            if self.early._next_decode is None:
                raise RuntimeError("late layers start after the early layers have run")
            if np.asarray(V).shape[0] != self.early.prefill_len - self.dropped:
                raise ValueError("a late layer takes the prompt without the dropped rows")
        return st.prefill(i, Q, K, V, rows=rows)

    def decode(self, l, q, k, v):
        st, i = self._side(l)
        return st.decode(i, q, k, v)

    # ---- views the layout and accounting code reads ------------------------------------------
    @property
    def Kc(self):
        return list(self.early.Kc) + list(self.late.Kc)

    @property
    def Vc(self):
        return list(self.early.Vc) + list(self.late.Vc)

    @property
    def q_owner(self):
        return self.late.q_owner + self.P if self.late.q_owner >= 0 else self.early.q_owner

    @property
    def Qc(self):
        """Rows of the Q Cache as memory holds them: what the early side wrote, overwritten from
        row 0 by what the late side wrote since."""
        img = np.array(self.early.Qc, copy=True)
        if self.late.q_owner >= 0:
            n = self.late.Qc.shape[1]
            if n > img.shape[1]:
                img = np.concatenate([img, np.zeros((self.H, n - img.shape[1], self.D))], axis=1)
            img[:, :n, :] = self.late.Qc
        return img

    @property
    def s(self):
        return self.early.s

    @property
    def Vn(self):
        return self.early.Vn

    @property
    def prefill_len(self):
        return self.early.prefill_len

    @property
    def len(self):
        return self.early.len

    def resident_rows(self):
        """(K rows, V rows, Q Cache rows): both sides' caches; the Q Cache counts for its current owner."""
        ek, ev, eq = self.early.resident_rows()
        lk, lv, lq = self.late.resident_rows()
        return ek + lk, ev + lv, (lq if self.late.q_owner >= 0 else eq)
