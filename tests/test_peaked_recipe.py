"""The "peaked" input recipe: that it has the score structure the GPU parity tests rely on, and
that the oracle is right on it (closed form: a score far above the rest of its row selects one value)."""
import math

import numpy as np

import workloads
from oracle.global_lazy_stack import GlobalLazyStackOracle
from oracle.lazy_stack import LazyStackOracle

LAZY = [0, 0, 1, 1, 0]


def small(dtype="bf16", D=128):
    return workloads.custom("peaked_small", 5, 2, D, dtype, [40, 7], [300, 200], [450, 330], 3, LAZY, recipe="peaked")


def log2_scores(w, layer, b, h):
    q, k, _ = workloads.prefill_qkv(w, layer)
    cu = w.cu_seqlens
    q64, k64 = workloads.to_f64(q[cu[b]:cu[b + 1], h]), workloads.to_f64(k[cu[b]:cu[b + 1], h])
    s = q64 @ k64.T / math.sqrt(w.head_dim) * math.log2(math.e)
    s[np.triu_indices(s.shape[0], 1)] = -np.inf
    return s


def test_normal_recipe_is_untouched_by_the_peaked_one():
    a = workloads.custom("x", 2, 2, 64, "f32", [4], [16], [40], 2, [0, 1])
    b = workloads.custom("x", 2, 2, 64, "f32", [4], [16], [40], 2, [0, 1], recipe="peaked")
    qa, ka, va = workloads.prefill_qkv(a, 0)
    qb, kb, vb = workloads.prefill_qkv(b, 0)
    assert np.array_equal(va.numpy(), vb.numpy())
    assert np.array_equal((qa * workloads.Q_GAIN).numpy(), qb.numpy())
    planted = {j for j, _ in workloads.planted_keys(b, 0, 0)}
    assert planted
    for j in range(40):
        assert np.array_equal(ka[j].numpy(), kb[j].numpy()) == (j not in planted)


def test_running_maximum_jumps_late_and_only_for_some_rows_of_a_wave():
    """In 64-key tiles, the way a flash-style kernel walks a row: some query rows see their running
    maximum grow by far more than 2^8 in a tile that is not their first, while other rows of the same
    group of 32 consecutive queries never do; and rows exist where it grows by a moderate amount."""
    w = small()
    s = log2_scores(w, 1, 0, 0)
    L = s.shape[0]
    big = {}
    moderate = 0
    for i in range(L):
        m = -np.inf
        for t in range(0, i + 1, 64):
            mt = s[i, t:t + 64].max()
            if np.isfinite(m) and mt - m > 8:
                big.setdefault(i, []).append((t // 64, mt - m))
            if np.isfinite(m) and 1 < mt - m <= 8:
                moderate += 1
            m = max(m, mt)
    assert any(t >= 2 and jump > 50 for v in big.values() for t, jump in v)
    groups_with = {i // 32 for i in big}
    assert any(any((g * 32 + r) not in big for r in range(32)) for g in groups_with)
    assert moderate > 20


def test_decode_chunk_maxima_lie_far_apart_at_the_peak_step():
    """At decode step PEAK_STEP the query of every layer has one planted key late in the prompt: the
    maximum of that key's 64-position chunk is far above the maxima of all other chunks."""
    w = small()
    for layer in (0, 1, 4):
        q = workloads.to_f64(workloads.decode_qkv(w, layer, workloads.PEAK_STEP)[0])
        k = workloads.to_f64(workloads.prefill_qkv(w, layer)[1])
        for b in range(w.batch):
            cu = w.cu_seqlens
            s = k[cu[b]:cu[b + 1], 0] @ q[b, 0] / math.sqrt(w.head_dim) * math.log2(math.e)
            chunk_max = [s[c:c + 64].max() for c in range(0, len(s), 64)]
            top = int(np.argmax(chunk_max))
            assert top >= 2
            others = [m for i, m in enumerate(chunk_max) if i != top]
            assert chunk_max[top] - max(others) > 30
    # and the key planted inside the span of an anchor layer is aimed at the next (lazy) layer's query
    q2 = workloads.to_f64(workloads.decode_qkv(w, 2, workloads.PEAK_STEP)[0])
    k1 = workloads.to_f64(workloads.prefill_qkv(w, 1)[1])
    s = k1[: w.seq_len[0], 1] @ q2[0, 1] / math.sqrt(w.head_dim)
    assert int(np.argmax(s)) == w.vis_start[0] + w.vis_len[0] // 2 and w.lazy_mask[2]


def dominant_bound(scores_row, j, vmax):
    """|softmax(scores) V - V[j]| <= 2 vmax sum_{i != j} exp(s_i - s_j)."""
    rest = np.delete(scores_row, j)
    return 2 * vmax * float(np.sum(np.exp(rest[np.isfinite(rest)] - scores_row[j])))


def test_oracle_on_peaked_inputs_selects_the_planted_value():
    """Closed form: where one score exceeds the rest of its row by a wide margin, the attention output
    is that key's value row up to the stated bound, in ordinary and lazy layers, prefill and decode."""
    w = small()
    for Oracle in (LazyStackOracle, GlobalLazyStackOracle):
        gla = Oracle is GlobalLazyStackOracle
        b = 0
        s0, vn, L = w.vis_start[b], w.vis_len[b], w.seq_len[b]
        st = Oracle(w.n_layers, w.n_heads, w.head_dim, w.lazy_mask, vis_start=s0, vis_len=vn)
        vs, ks, qs = [], [], []
        for l in range(w.n_layers):
            q, k, v = (workloads.to_f64(t[:L]) for t in workloads.prefill_qkv(w, l))
            out = st.prefill(l, q, k, v)
            vs.append(v); ks.append(k); qs.append(q)
            # effective query/key rows of this layer
            a = l
            while w.lazy_mask[a]:
                a -= 1
            if w.lazy_mask[l] and gla:
                qe, ke = qs[a], ks[a]
            elif w.lazy_mask[l]:
                qe, ke = q.copy(), k.copy()
                qe[s0:s0 + vn], ke[s0:s0 + vn] = qs[a][s0:s0 + vn], ks[a][s0:s0 + vn]
            else:
                qe, ke = q, k
            checked = 0
            for i in (s0 + vn - 1, L - 1):
                for h in range(w.n_heads):
                    row = ke[: i + 1, h] @ qe[i, h] / math.sqrt(w.head_dim)
                    j = int(np.argmax(row))
                    bound = dominant_bound(row, j, float(np.abs(v[:, h]).max()))
                    if bound < 1e-9:
                        assert np.max(np.abs(out[i, h] - v[j, h])) <= bound + 1e-12
                        checked += 1
            assert checked >= 2, (l, checked)
        # decode at the peak step: the planted prompt key wins in ordinary layers; a lazy layer under
        # Visual Lazy Attention finds its peak among the anchor's span keys
        for t in range(workloads.PEAK_STEP + 1):
            for l in range(w.n_layers):
                q, k, v = (workloads.to_f64(x[b]) for x in workloads.decode_qkv(w, l, t))
                o = st.decode(l, q, k, v)
                if t != workloads.PEAK_STEP:
                    continue
                a = l
                while w.lazy_mask[a]:
                    a -= 1
                pos = L + t
                if w.lazy_mask[l] and gla:
                    qe = workloads.to_f64(workloads.decode_qkv(w, a, t)[0][b])
                    keys = st.Kc[a][:, : pos + 1]
                elif w.lazy_mask[l]:
                    qe = q
                    own = st.Kc[l]                                   # text rows only, compacted
                    keys = np.concatenate([own[:, :s0], st.Kc[a][:, s0:s0 + vn], own[:, s0:]], axis=1)
                else:
                    qe, keys = q, st.Kc[l][:, : pos + 1]
                for h in range(w.n_heads):
                    row = keys[h] @ qe[h] / math.sqrt(w.head_dim)
                    j = int(np.argmax(row))
                    bound = dominant_bound(row, j, float(np.abs(st.Vc[l][h]).max()))
                    assert bound < 1e-4, (l, h, bound)
                    assert np.max(np.abs(o[h] - st.Vc[l][h, j])) <= bound + 1e-12
