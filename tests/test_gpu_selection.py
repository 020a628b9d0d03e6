"""GPU parity for the lazy-block selection statistics (Eq. 3 / Eq. 4) against the CPU oracle.

Tolerances (fp32 kernels against fp64): a probability is exp2 of a 64..128-term fp32 dot product
divided by a sum of such terms, so its relative error is a few 1e-6 times the score magnitude;
the bar is |err| <= 1e-5 + 1e-4*|p|.  JS and S are sums of p*ln terms bounded by ln 2: bar 1e-4.
The block decision of Eq. 4 is taken from the same fp32 similarities on both sides."""
import numpy as np
import pytest
import torch

import paper_2602_01901_amd as P
from paper_2602_01901_amd import binding as B
import workloads
from oracle import selection

pytestmark = pytest.mark.gpu


def prefilled_session(w):
    s = P.Session.for_workload(w)
    s.reset(w.vis_start, w.vis_len)
    qs, ks = [], []
    for l in range(w.n_layers):
        q, k, v = (t.cuda() for t in workloads.prefill_qkv(w, l))
        s.prefill(l, q, k, v, w.cu_seqlens)
        qs.append(q)
        ks.append(k)
    return s, qs, ks


def last_queries(w, q):
    """[batch][H][D]: the last prompt row of each sequence."""
    cu = w.cu_seqlens
    return torch.stack([q[cu[b + 1] - 1] for b in range(w.batch)]).contiguous()


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128), ("bf16", 64), ("f32", 128)])
def test_last_row_attention_and_similarity_match_oracle(dtype, D):
    lens = [131, 64, 45, 7, 300]
    w = workloads.custom("select", 4, 3, D, dtype, [0] * 5, [0] * 5, lens, 0, [0, 0, 0, 0], seed_tag=D)
    s, qs, ks = prefilled_session(w)
    cfg = s.cfg
    ws = torch.empty(B.qc_select_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    stride = 304
    probs = [torch.full((w.batch, stride), -1.0, dtype=torch.float32, device="cuda") for _ in range(w.n_layers)]
    scale = 1.0 / np.sqrt(D)
    cu = w.cu_seqlens
    want_rows = []
    for l in range(w.n_layers):
        B.qc_last_row_attention(s.kv, l, last_queries(w, qs[l]), probs[l], stride, 0.0, ws, ws.numel())
        rows = []
        for b in range(w.batch):
            K = np.transpose(workloads.to_f64(ks[l][cu[b]:cu[b + 1]]), (1, 0, 2))
            rows.append(selection.last_row_attention(workloads.to_f64(qs[l][cu[b + 1] - 1]), K, scale))
        want_rows.append(rows)
    torch.cuda.synchronize()
    worst_p = 0.0
    for l in range(w.n_layers):
        got = probs[l].cpu().numpy().astype(np.float64)
        for b in range(w.batch):
            err = np.abs(got[b, :lens[b]] - want_rows[l][b])
            assert np.all(err <= 1e-5 + 1e-4 * want_rows[l][b]), (l, b, err.max())
            worst_p = max(worst_p, float(err.max()))
            assert np.all(got[b, lens[b]:] == -1.0)            # nothing written past the row
            assert abs(got[b, :lens[b]].sum() - 1.0) < 1e-4
    js = torch.empty(w.batch, dtype=torch.float32, device="cuda")
    sim = torch.empty(1, dtype=torch.float32, device="cuda")
    adjacent = []
    worst_js = 0.0
    for l in range(w.n_layers - 1):
        B.qc_attention_similarity(probs[l], probs[l + 1], stride, w.batch, lens, js, sim)
        torch.cuda.synchronize()
        want_js = [selection.js_divergence(p, q) for p, q in zip(want_rows[l], want_rows[l + 1])]
        np.testing.assert_allclose(js.cpu().numpy(), want_js, rtol=0, atol=1e-4)
        worst_js = max(worst_js, float(np.max(np.abs(js.cpu().numpy() - np.array(want_js)))))
        want_s = selection.similarity(want_rows[l], want_rows[l + 1])
        assert abs(float(sim.item()) - want_s) <= 1e-4
        adjacent.append(float(sim.item()))
    print("selection %s D=%d: max |dp| %.3g, max |dJS| %.3g" % (dtype, D, worst_p, worst_js), flush=True)
    eps = float(np.float32(np.median(adjacent)))
    eps = min(max(eps, 1e-3), 1.0)
    assert B.qc_lazy_mask_from_similarity(adjacent, eps) == selection.lazy_mask_from_similarity(adjacent, eps)


def test_similarity_special_cases_and_many_samples():
    """Identical rows give 0, disjoint supports give exactly 1 bit; 130 samples span three launches."""
    n, stride = 130, 96
    rng = np.random.default_rng(3)
    lens = [int(x) for x in rng.integers(1, stride + 1, size=n)]
    p = np.zeros((n, stride), dtype=np.float32)
    q = np.zeros((n, stride), dtype=np.float32)
    for i, L in enumerate(lens):
        a, b = rng.random(L), rng.random(L)
        if i % 3 == 0 and L > 1:
            a[L // 2:] = 0
            b[:L // 2] = 0                       # disjoint supports
        if i % 3 == 1:
            b = a.copy()                         # identical
        p[i, :L] = a / a.sum()
        q[i, :L] = b / b.sum()
    pd, qd = torch.from_numpy(p).cuda(), torch.from_numpy(q).cuda()
    js = torch.empty(n, dtype=torch.float32, device="cuda")
    sim = torch.empty(1, dtype=torch.float32, device="cuda")
    B.qc_attention_similarity(pd, qd, stride, n, lens, js, sim)
    torch.cuda.synchronize()
    got = js.cpu().numpy()
    want = np.array([selection.js_divergence(p[i, :L].astype(np.float64), q[i, :L].astype(np.float64))
                     for i, L in enumerate(lens)])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-4)
    for i, L in enumerate(lens):
        if i % 3 == 1:
            assert got[i] == 0.0
        if i % 3 == 0 and L > 1:
            assert abs(got[i] - np.log(2.0)) < 1e-5       # disjoint supports: the upper bound ln 2
    assert abs(float(sim.item()) - want.mean()) <= 1e-4


def test_selection_pipeline_at_the_7b_shape_finds_planted_blocks():
    """32 layers x 32 heads x D=128, 8 samples of 640 tokens.  Blocks are planted by giving the layers of a
    block the same Q and K (similarity exactly 0) and independent draws elsewhere (similarity near the
    value for unrelated rows); the recovered mask must equal the planted one."""
    w = workloads.custom("select7b", 32, 32, 128, "bf16", [32] * 8, [576] * 8, [640] * 8, 0, [0] * 32)
    planted = workloads.block_lazy_mask(32, 3)
    s = P.Session.for_workload(w)
    s.reset(w.vis_start, w.vis_len)
    ws = torch.empty(B.qc_select_workspace_bytes(s.cfg), dtype=torch.uint8, device="cuda")
    stride = 640
    probs = torch.zeros((32, 8, stride), dtype=torch.float32, device="cuda")
    src = 0
    for l in range(32):
        if not planted[l]:
            src = l
        q, k, _ = (t.cuda() for t in workloads.prefill_qkv(w, src))
        v = workloads.prefill_qkv(w, l)[2].cuda()
        s.prefill(l, q, k, v, w.cu_seqlens)
    for l in range(32):
        src = l
        while planted[src]:
            src -= 1
        q = workloads.prefill_qkv(w, src)[0].cuda()
        B.qc_last_row_attention(s.kv, l, last_queries(w, q), probs[l], stride, 0.0, ws, ws.numel())
    js = torch.empty(8, dtype=torch.float32, device="cuda")
    sim = torch.empty(1, dtype=torch.float32, device="cuda")
    adjacent = []
    for l in range(31):
        B.qc_attention_similarity(probs[l], probs[l + 1], stride, 8, [640] * 8, js, sim)
        adjacent.append(float(sim.item()))
    inside = [a for a, f in zip(adjacent, planted[1:]) if f]
    across = [a for a, f in zip(adjacent, planted[1:]) if not f]
    print("similarity inside blocks max %.3g, across blocks min %.3g" % (max(inside), min(across)), flush=True)
    assert max(inside) == 0.0 and min(across) > 0.007     # head averaging flattens unrelated rows: about 0.012 nats
    assert B.qc_lazy_mask_from_similarity(adjacent, 0.005) == planted
