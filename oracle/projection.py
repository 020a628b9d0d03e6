"""Query/key projection feeding the attention path, text rows only in a lazy layer (test infrastructure).

What the paper fixes: Eq. 7 — in a lazy layer under Visual Lazy Attention only the text tokens
are projected (X_[T] W_Q, X_[T] W_K), the visual rows of Q and K being inherited — and the
"FLOPs and Latency" paragraph of "Efficiency Analysis": of the two projectors of a lazy layer
the share |V|/(|V|+|T|) of the work is omitted (all of it under Global Lazy Attention).

What the paper does not describe is the rotary position embedding its LLaMA-family models apply
to Q and K between the projection and the attention.  It is taken from its published
definition (RoFormer; rotate-half convention of the LLaMA implementations): within each head,
element d < D/2 is paired with element d + D/2 and the pair is rotated by the angle
pos * theta^(-2d/D), pos being the token's true position.  theta = 0 switches it off.

All arithmetic is fp64.  X: [tokens, d_model]; W_Q, W_K: [H*D, d_model] (row = output feature).
"""
import numpy as np


def rope_angles(positions, head_dim, theta):
    """[len(positions), D/2] rotation angles."""
    positions = np.asarray(positions, dtype=np.float64)
    half = head_dim // 2
    inv_freq = np.power(float(theta), -2.0 * np.arange(half, dtype=np.float64) / head_dim)
    return positions[:, None] * inv_freq[None, :]


def apply_rope(x, positions, theta):
    """x: [rows, H, D] -> rotated copy; row r uses positions[r]."""
    x = np.asarray(x, dtype=np.float64)
    if not theta:
        return x.copy()
    D = x.shape[-1]
    half = D // 2
    ang = rope_angles(positions, D, theta)
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * cos - hi * sin, hi * cos + lo * sin], axis=-1)


def text_rows(seq_len, vis_start, vis_len):
    """Positions of one sequence that are projected in a lazy layer: everything outside the span."""
    return [p for p in range(seq_len) if not (vis_start <= p < vis_start + vis_len)]


def project_qk(X, Wq, Wk, n_heads, head_dim, rows, positions, theta):
    """Rows `rows` of X (token indices) projected with both matrices and rotated at `positions`
    (one per row).  Returns (Q, K), each [len(rows), H, D]."""
    X = np.asarray(X, dtype=np.float64)
    Xr = X[list(rows)]
    outs = []
    for W in (Wq, Wk):
        W = np.asarray(W, dtype=np.float64)
        if W.shape != (n_heads * head_dim, X.shape[1]):
            raise ValueError("weight must be [H*D, d_model]")
        Y = (Xr @ W.T).reshape(len(Xr), n_heads, head_dim)
        outs.append(apply_rope(Y, positions, theta))
    return outs[0], outs[1]


def projector_flops(n_rows, d_model, n_heads, head_dim):
    """Multiply-adds counted as 2 flops, one projector."""
    return 2 * n_rows * d_model * n_heads * head_dim


def vla_projection_saving(n_lazy, vis_len, text_len):
    """"FLOPs and Latency" paragraph, in units of one projector's work over all tokens:
    |V|/(|V|+|T|) * 2n (the paper multiplies by beta, that projector's share of the model)."""
    from fractions import Fraction
    return Fraction(vis_len, vis_len + text_len) * 2 * n_lazy
