#!/usr/bin/env python3
"""Benchmark of the Lazy Attention / Q Cache attention stack on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: reset the caches,
prefill every layer of the stack (ordinary and lazy layers in order), then run the workload's
decode steps, each of which visits every layer.  Inputs are seeded N(0,1) tensors resident in
HBM before the timed region starts; every call goes through the C ABI (qc_prefill / qc_decode).

The headline line is measured on the largest single-GPU configuration, the 13B-shaped video workload
(40 layers x 40 heads, batch 4, 4864-token prompts of which 4608 visual, 1024 generated tokens).  The
other configurations (batch-1 7B shape, batched decode, high-resolution prefill) and the widened
entry points are timed in the same run and reported under "workloads".

Prints ONE JSON line on stdout; progress goes to stderr.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(key, field="bytes_per_launch"):
    """HBM bytes per launch from committed rocprofv3 --pmc runs (profiles/hbm_traffic.json), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(key, {}).get(field)
    except (OSError, ValueError):
        return None


def prefill_flops_per_layer(w):
    """4*D flops per attended (query, key) pair: sum_b H * 4*D * L_b(L_b+1)/2."""
    return sum(w.n_heads * 4 * w.head_dim * L * (L + 1) // 2 for L in w.seq_len)


def decode_bytes_per_layer(w, generated):
    """K and V rows streamed once plus q,k,v in, o out, k,v appended: sum_b (2*(L_b+1)+6)*H*D*e."""
    return sum((2 * (L + generated + 1) + 6) * w.n_heads * w.head_dim * w.elem_bytes for L in w.seq_len)


class Runner:
    """Holds resident inputs for one workload and drives the library."""

    def __init__(self, w, decode_steps, distinct_decode_inputs=8, mode="vla", graph=False):
        import torch
        import paper_2602_01901_amd as P
        import workloads
        self.torch, self.w = torch, w
        self.decode_steps = decode_steps
        self.sess = P.Session.for_workload(w, mode=mode)
        # Global Lazy Attention: a lazy layer has no q and k of its own
        self.no_qk = [mode == "gla" and bool(f) for f in w.lazy_mask]
        dev = self.sess.device
        self.pre = [workloads.prefill_qkv(w, l, device=dev) for l in range(w.n_layers)]
        self.out_pre = torch.empty_like(self.pre[0][0])
        nd = max(1, min(distinct_decode_inputs, decode_steps))
        self.dec = [[workloads.decode_qkv(w, l, t, device=dev) for l in range(w.n_layers)] for t in range(nd)]
        self.out_dec = torch.empty_like(self.dec[0][0][0])
        # graph=True: a decode step is one replay of a HIP graph recorded once (after the first prefill)
        # over the first set of decode inputs, which then stand for the buffers a model's projections
        # would refill in place before every step
        self.use_graph, self.graph = graph, None
        torch.cuda.synchronize()

    def prefill_stack(self):
        w, s = self.w, self.sess
        s.reset(w.vis_start, w.vis_len, zero_fill=False)
        for l in range(w.n_layers):
            q, k, v = self.pre[l]
            if self.no_qk[l]:
                q = k = None
            s.prefill(l, q, k, v, w.cu_seqlens, out=self.out_pre)

    def decode_steps_run(self, steps, time_every=0, timed_steps=None):
        """time_every > 0: the library's per-kernel HIP events are switched on for one decode step in
        every `time_every` (ordinary calls only); the index of each such step (= tokens generated
        before it) is appended to timed_steps."""
        w, s = self.w, self.sess
        stream = self.torch.cuda.current_stream(s.device).cuda_stream
        if time_every and not self.use_graph:
            from paper_2602_01901_amd import binding as B
            g0 = s.stats()["generated"]
            for t in range(steps):
                on = t % time_every == time_every // 2
                if on:
                    B.qc_timing_enable(s.kv, 1)
                    timed_steps.append(g0 + t)
                row = self.dec[t % len(self.dec)]
                for l in range(w.n_layers):
                    q, k, v = row[l]
                    if self.no_qk[l]:
                        q = k = None
                    s.decode(l, q, k, v, out=self.out_dec, stream=stream)
                if on:
                    B.qc_timing_enable(s.kv, 0)
            return
        if self.use_graph:
            if self.graph is None:
                row = self.dec[0]
                self.graph = s.decode_graph([None if self.no_qk[l] else row[l][0] for l in range(w.n_layers)],
                                            [None if self.no_qk[l] else row[l][1] for l in range(w.n_layers)],
                                            [row[l][2] for l in range(w.n_layers)], [self.out_dec] * w.n_layers)
            for t in range(steps):
                s.graph_launch(self.graph, stream)
            return
        for t in range(steps):
            row = self.dec[t % len(self.dec)]
            for l in range(w.n_layers):
                q, k, v = row[l]
                if self.no_qk[l]:
                    q = k = None
                s.decode(l, q, k, v, out=self.out_dec, stream=stream)

    def step(self):
        self.prefill_stack()
        self.decode_steps_run(self.decode_steps)

    def kernel_times(self, fn):
        """Run fn with the library's per-kernel HIP-event timing on; returns
        {"prefill": (avg_us, launches), "decode": (avg_us, launches)} for its dominant kernels."""
        from paper_2602_01901_amd import binding as B
        B.qc_timing_enable(self.sess.kv, 1)
        B.qc_timing_read(self.sess.kv, 0)
        B.qc_timing_read(self.sess.kv, 1)
        B.qc_timing_read(self.sess.kv, 2)
        graph, self.use_graph = self.use_graph, False      # events sit between individual launches: ordinary calls
        fn()
        self.use_graph = graph
        self.torch.cuda.synchronize()
        out = {}
        for name, which in (("prefill", 0), ("decode", 1), ("decode_shared", 2)):
            ms, n = B.qc_timing_read(self.sess.kv, which)
            out[name] = (ms * 1e3 / n if n else 0.0, n)
        B.qc_timing_enable(self.sess.kv, 0)
        return out


def timed(torch, fn, reps):
    """Wall-clock seconds per repetition, synchronised on both sides, plus HIP-event time."""
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / reps
    return wall, e0.elapsed_time(e1) * 1e-3 / reps


def bench_cfg2(args):
    """Batch-1 7B shape (640-token prompt, 256 decode steps): launch- and latency-bound on a 256-CU part;
    decode steps are replayed from one HIP graph."""
    import torch
    import workloads
    w = workloads.config(1)
    r = Runner(w, w.decode_steps, graph=not args.no_graph)
    r.step()
    torch.cuda.synchronize()
    # whole steps
    wall, _ = timed(torch, r.step, 3)
    # split of the same step into its two phases (extra passes, not part of `value`)
    pre_wall, pre_ev = timed(torch, r.prefill_stack, max(args.steps, 3))
    r.prefill_stack()
    dec_wall, dec_ev = timed(torch, lambda: r.decode_steps_run(w.decode_steps), 1)
    stats = r.sess.stats()
    # per-launch duration of the dominant kernels: HIP events recorded by the library on the launch
    # stream around the kernel itself, over one more whole step
    stats_prefill = {}

    def one_step():
        r.prefill_stack()
        stats_prefill.update(r.sess.stats())
        r.decode_steps_run(w.decode_steps)
    kt = r.kernel_times(one_step)
    dec_us, dec_n = kt["decode"]
    pre_us, pre_n = kt["prefill"]
    mean_bytes = sum(decode_bytes_per_layer(w, g) for g in range(w.decode_steps)) / w.decode_steps
    achieved = mean_bytes / (dec_us * 1e-6) / 1e9
    pf = prefill_flops_per_layer(w) * w.n_layers
    res = {
        "workload": w.name, "batch": w.batch,
        "decode_launch": "ordinary qc_decode calls" if args.no_graph else "one replay of a HIP graph of the 32 layer calls per decode step",
        "ms_per_step": wall * 1e3,
        "decode_tokens_per_s": w.batch * w.decode_steps / dec_ev,
        "decode_ms_per_token_step": dec_ev / w.decode_steps * 1e3,
        "prefill_ms": pre_ev * 1e3,
        "prefill_tflops": pf / pre_ev / 1e12,
        "k_cache_bytes_per_token": stats["k_bytes"] / stats["tokens"],
        "k_cache_bytes_per_token_standard": w.n_layers * w.n_heads * w.head_dim * w.elem_bytes,
        "k_cache_bytes_per_token_after_prefill": stats_prefill["k_bytes"] / stats_prefill["tokens"],
        # kernels of a few microseconds: an event pair also brackets the dispatch gap, so the figure that
        # fits inside the step is the whole replayed decode phase (all bytes of a step over its duration)
        "roofline": {"bound": "hbm", "kernel": "decode_split_kernel<bf16,128> + decode_merge_kernel (whole replayed decode phase)",
                     "achieved": mean_bytes * w.n_layers * w.decode_steps / dec_ev / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": mean_bytes * w.n_layers * w.decode_steps / dec_ev / 1e9 / HBM_PEAK_GBS,
                     "traffic": measured_traffic("decode_cfg2"),
                     "avg_launch_us": dec_ev / (w.n_layers * w.decode_steps) * 1e6,
                     "launches_timed": w.n_layers * w.decode_steps, "algorithmic_bytes_per_launch": mean_bytes,
                     "event_pair_around_split_kernel_us": dec_us, "event_pair_GBps": achieved,
                     "note": "latency-bound shape: 12.6 MB per layer call would take 1.6 us at the HBM peak"},
        "prefill_kernel": {"kernel": "prefill_mfma_kernel", "avg_launch_us": pre_us, "launches_timed": pre_n,
                           "tflops": prefill_flops_per_layer(w) / (pre_us * 1e-6) / 1e12 if pre_us else None},
    }
    del r
    torch.cuda.empty_cache()
    return res


def bench_decode_batched(args, w=None, traffic_key="decode_cfg3"):
    """Batch-32 decode (HBM-bound): caches filled by an untimed prefill, then timed decode steps.  Also used
    (as a profiling aid) for the decode phase of the headline workload alone."""
    import torch
    import workloads
    w = w or workloads.config(2)
    steps = args.decode_batched_steps
    r = Runner(w, steps, distinct_decode_inputs=4)
    r.prefill_stack()
    r.decode_steps_run(2)
    torch.cuda.synchronize()
    g0 = r.sess.stats()["generated"]
    _, ev_s = timed(torch, lambda: r.decode_steps_run(steps), 1)
    g1 = r.sess.stats()["generated"]
    kt = r.kernel_times(lambda: r.decode_steps_run(4))
    call_us, call_n = kt["decode"]
    bytes_call = sum(decode_bytes_per_layer(w, g1 + t) for t in range(4)) / 4
    bytes_step = sum(decode_bytes_per_layer(w, g0 + t) for t in range(steps)) / steps * w.n_layers
    stats = r.sess.stats()
    # duration of a layer call = timed decode phase / layer calls (launch gaps charged to the kernel); the
    # event pairs the library records around the kernel alone are given beside it
    calls = steps * w.n_layers
    call_phase_us = ev_s / calls * 1e6
    bytes_mean = bytes_step / w.n_layers
    achieved = bytes_mean / (call_phase_us * 1e-6) / 1e9
    res = {
        "workload": w.name, "batch": w.batch, "decode_steps_timed": steps,
        "decode_tokens_per_s": w.batch * steps / ev_s,
        "decode_ms_per_step": ev_s / steps * 1e3,
        "stack_GBps": bytes_step / (ev_s / steps) / 1e9,
        "k_cache_bytes_per_token": stats["k_bytes"] / stats["tokens"],
        "roofline": {"bound": "hbm", "kernel": "decode_split_kernel<bf16,128> (no split at this batch: one launch per layer call; "
                     "duration = decode phase / layer calls)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(traffic_key), "avg_launch_us": call_phase_us, "launches_timed": calls,
                     "algorithmic_bytes_per_launch": bytes_mean,
                     "event_pairs_around_kernel": {"avg_us": call_us, "launches": call_n, "algorithmic_bytes_per_launch": bytes_call,
                                                   "GBps": bytes_call / (call_us * 1e-6) / 1e9}},
    }
    del r
    torch.cuda.empty_cache()
    return res


def gla_shared_decode_bytes_per_layer(w, generated):
    """Lazy layer under Global Lazy Attention: V rows and one fp32 score per position streamed once,
    v in, o out, v appended: sum_b ((L_b+1+3)*D*e + (L_b+1)*4) * H."""
    return sum(((L + generated + 4) * w.head_dim * w.elem_bytes + (L + generated + 1) * 4) * w.n_heads
               for L in w.seq_len)


def bench_gla_decode_batched(args):
    """The batched-decode configuration under Global Lazy Attention: lazy layers reuse the scores of
    their block's first layer and stream only their V cache."""
    import torch
    import workloads
    w = workloads.config(2)
    steps = args.decode_batched_steps
    r = Runner(w, steps, distinct_decode_inputs=4, mode="gla")
    r.prefill_stack()
    r.decode_steps_run(2)
    torch.cuda.synchronize()
    g0 = r.sess.stats()["generated"]
    _, ev_s = timed(torch, lambda: r.decode_steps_run(steps), 1)
    g1 = r.sess.stats()["generated"]
    kt = r.kernel_times(lambda: r.decode_steps_run(4))
    sh_us, sh_n = kt["decode_shared"]
    od_us, od_n = kt["decode"]
    sh_bytes = sum(gla_shared_decode_bytes_per_layer(w, g1 + t) for t in range(4)) / 4
    od_bytes = sum(decode_bytes_per_layer(w, g1 + t) for t in range(4)) / 4
    n_lazy = w.n_lazy
    step_bytes = sum((w.n_layers - n_lazy) * decode_bytes_per_layer(w, g0 + t) +
                     n_lazy * gla_shared_decode_bytes_per_layer(w, g0 + t) for t in range(steps)) / steps
    stats = r.sess.stats()
    calls = steps * w.n_layers
    call_phase_us = ev_s / calls * 1e6
    achieved = step_bytes / w.n_layers / (call_phase_us * 1e-6) / 1e9
    res = {
        "workload": w.name + " (GLA)", "batch": w.batch, "decode_steps_timed": steps,
        "decode_tokens_per_s": w.batch * steps / ev_s,
        "decode_ms_per_step": ev_s / steps * 1e3,
        "stack_GBps": step_bytes / (ev_s / steps) / 1e9,
        "k_cache_bytes_per_token": stats["k_bytes"] / stats["tokens"],
        "q_cache_bytes_per_token": stats["q_bytes"] / stats["tokens"],
        "ordinary_layer_kernel": {"avg_launch_us": od_us, "launches_timed": od_n,
                                  "GBps": od_bytes / (od_us * 1e-6) / 1e9 if od_us else None},
        "roofline": {"bound": "hbm", "kernel": "decode_split_kernel<bf16,128> in its two forms (13 layer calls that stream K and V, "
                     "19 score-sharing ones that stream V only); duration = decode phase / layer calls",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic("gla_decode_cfg3"), "avg_launch_us": call_phase_us, "launches_timed": calls,
                     "algorithmic_bytes_per_launch": step_bytes / w.n_layers,
                     "event_pairs_around_score_sharing_kernel": {"avg_us": sh_us, "launches": sh_n, "algorithmic_bytes_per_launch": sh_bytes,
                                                                 "GBps": sh_bytes / (sh_us * 1e-6) / 1e9}},
    }
    del r
    torch.cuda.empty_cache()
    return res


def bench_projection(args):
    """Q/K projection + rotary embedding at the high-resolution prompt shape (d_model 4096, 32 x 128): an
    ordinary layer projects all 8 x 3008 tokens, a lazy layer only the 8 x 128 text tokens (Eq. 7)."""
    import torch
    import workloads
    from paper_2602_01901_amd import binding as B
    w = workloads.config(3)
    d_model, H, D = 4096, w.n_heads, w.head_dim
    tokens = sum(w.seq_len)
    g = torch.Generator().manual_seed(0x51C0 + 77)
    pad = int(os.environ.get("QC_BENCH_ROW_PAD", "0"))   # elements between rows of x and of the weights (no measurable effect)
    ld = d_model + pad

    def rows_of(t):
        buf = torch.zeros(t.shape[0], ld, dtype=torch.bfloat16, device="cuda")
        buf[:, :d_model] = t.cuda()
        return buf
    x = rows_of(torch.randn(tokens, d_model, generator=g).to(torch.bfloat16))
    wq = rows_of((torch.randn(H * D, d_model, generator=g) / d_model ** 0.5).to(torch.bfloat16))
    wk = rows_of((torch.randn(H * D, d_model, generator=g) / d_model ** 0.5).to(torch.bfloat16))
    q = torch.empty(tokens, H, D, dtype=torch.bfloat16, device="cuda")
    k = torch.empty_like(q)

    def run(skip):
        B.qc_project_qk(x, ld, wq, wk, ld, q, k, H * D, D, d_model, H, D, w.batch, w.cu_seqlens, None,
                        w.vis_start, w.vis_len, skip, 10000.0)
    out = {"workload": w.name, "d_model": d_model, "heads": H, "head_dim": D, "row_stride_elements": ld}
    for name, skip, rows in (("ordinary_layer", 0, tokens), ("lazy_layer_text_rows", 1, tokens - sum(w.vis_len))):
        run(skip)
        _, ev_s = timed(torch, lambda: run(skip), 5)
        flops = 2 * 2 * rows * d_model * H * D
        out[name] = {"rows": rows, "us": ev_s * 1e6, "tflops": flops / ev_s / 1e12,
                     "roofline": {"bound": "mfma", "kernel": "project_qk_kernel<128> (W_Q and W_K in one launch)",
                                  "achieved": flops / ev_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                  "frac": flops / ev_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                  "traffic": measured_traffic("projection_ordinary" if not skip else "projection_lazy"),
                                  "avg_launch_us": ev_s * 1e6, "algorithmic_flops_per_launch": flops}}
    out["time_saved_per_lazy_layer_us"] = out["ordinary_layer"]["us"] - out["lazy_layer_text_rows"]["us"]
    # decode: one token per sequence (batch 32): weight streaming, 2 x 33.5 MB per layer
    wd = workloads.config(2)
    cu = list(range(wd.batch + 1))
    pos0 = list(wd.seq_len)

    def run_dec():
        B.qc_project_qk(x, ld, wq, wk, ld, q, k, H * D, D, d_model, H, D, wd.batch, cu, pos0, None, None, 0, 10000.0)
    run_dec()
    _, ev_s = timed(torch, run_dec, 10)
    dec_bytes = 2 * H * D * d_model * 2 + wd.batch * d_model * 2 + 2 * wd.batch * H * D * 2   # weights, x rows, q and k rows
    out["decode_batch32"] = {"us": ev_s * 1e6,
                             "roofline": {"bound": "hbm", "kernel": "project_qk_skinny_kernel<128>",
                                          "achieved": dec_bytes / ev_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                          "frac": dec_bytes / ev_s / 1e9 / HBM_PEAK_GBS,
                                          "traffic": measured_traffic("projection_decode"),
                                          "avg_launch_us": ev_s * 1e6, "algorithmic_bytes_per_launch": dec_bytes}}
    del x, wq, wk, q, k
    torch.cuda.empty_cache()
    return out


def bench_selection(args):
    """Lazy-block selection statistics (Eq. 3) at the batched 7B shape with every layer ordinary: the
    head-averaged last-row attention of all 32 layers, then the 31 adjacent-layer similarities."""
    import torch
    import workloads
    from paper_2602_01901_amd import binding as B
    base = workloads.config(2)
    w = workloads.custom("extra_selection_b32", base.n_layers, base.n_heads, base.head_dim, "bf16", base.vis_start,
                         base.vis_len, base.seq_len, 0, [0] * base.n_layers)
    r = Runner(w, 0)
    r.prefill_stack()
    s = r.sess
    ws = torch.empty(B.qc_select_workspace_bytes(s.cfg), dtype=torch.uint8, device=s.device)
    stride = max(w.seq_len)
    probs = torch.zeros((w.n_layers, w.batch, stride), dtype=torch.float32, device=s.device)
    cu = w.cu_seqlens
    q_last = [torch.stack([r.pre[l][0][cu[b + 1] - 1] for b in range(w.batch)]).contiguous() for l in range(w.n_layers)]
    js = torch.empty(w.batch, dtype=torch.float32, device=s.device)
    sim = torch.empty(w.n_layers - 1, dtype=torch.float32, device=s.device)

    def rows():
        for l in range(w.n_layers):
            B.qc_last_row_attention(s.kv, l, q_last[l], probs[l], stride, 0.0, ws, ws.numel())

    def sims():
        for l in range(w.n_layers - 1):
            B.qc_attention_similarity(probs[l], probs[l + 1], stride, w.batch, w.seq_len, js, sim[l:l + 1])
    rows()
    sims()
    _, rows_s = timed(torch, rows, 3)
    _, sims_s = timed(torch, sims, 3)
    k_bytes = sum(w.seq_len) * w.n_heads * w.head_dim * w.elem_bytes          # per layer: every key row once
    score_bytes = 2 * sum(w.seq_len) * w.n_heads * 4                          # scores written, then read back
    adjacent = [float(x) for x in sim.cpu()]
    res = {
        "workload": w.name, "batch": w.batch, "layers": w.n_layers,
        "last_row_attention_us_per_layer": rows_s / w.n_layers * 1e6,
        "last_row_attention_GBps": (k_bytes + score_bytes) / (rows_s / w.n_layers) / 1e9,
        "similarity_us_per_layer_pair": sims_s / (w.n_layers - 1) * 1e6,
        "similarity_min": min(adjacent), "similarity_max": max(adjacent),
        "note": "independent random layers: every adjacent pair is equally dissimilar; offline analysis, two tiny "
                "launches per layer, latency-bound",
    }
    del r
    torch.cuda.empty_cache()
    return res


def bench_prefill_highres(args, w=None, traffic_key="prefill_cfg4", layers=None, mode="vla"):
    """Batch-8, 3008-token prefill (MFMA-bound); also used for the other prefill shapes."""
    import torch
    import workloads
    w = w or workloads.config(3)
    r = Runner(w, 0, mode=mode)
    r.prefill_stack()
    torch.cuda.synchronize()
    reps = args.prefill_reps
    _, ev_s = timed(torch, r.prefill_stack, reps)
    kt = r.kernel_times(r.prefill_stack)
    call_us, call_n = kt["prefill"]
    flops_layer = prefill_flops_per_layer(w)
    stats = r.sess.stats()
    achieved = flops_layer / (call_us * 1e-6) / 1e12
    res = {
        "workload": w.name + (" (GLA)" if mode == "gla" else ""), "batch": w.batch, "seq_len": w.seq_len[0],
        "prefill_ms": ev_s * 1e3, "prefill_tflops": flops_layer * w.n_layers / ev_s / 1e12,
        "k_cache_bytes_per_token": stats["k_bytes"] / stats["tokens"],
        "roofline": {"bound": "mfma", "kernel": "prefill_mfma_kernel (attention + fused cache writes: whole layer call)",
                     "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": measured_traffic(traffic_key),
                     "avg_launch_us": call_us, "launches_timed": call_n, "algorithmic_flops_per_launch": flops_layer},
    }
    del r
    torch.cuda.empty_cache()
    return res


class PrunedRunner(Runner):
    """Runner with a token-pruning boundary: layers >= first_late see `keep_frac` of each span.

    The prefill pass ranks the visual tokens by the last prompt token's attention in the last ordinary
    early layer, selects the survivors, drops the pruned rows of one hidden-state-sized tensor
    ([tokens][d_model] bf16, what a model would carry across the boundary) and moves the boundary into
    the cache state; all of that is inside the timed pass.  The late layers' q/k/v inputs are gathered
    once at construction with the same row map (the ranking is deterministic)."""

    def __init__(self, w, decode_steps, first_late, keep_frac, d_model=4096, **kw):
        super().__init__(w, decode_steps, **kw)
        from paper_2602_01901_amd import binding as B
        torch = self.torch
        self.B, self.first_late = B, first_late
        self.keep = [int(v * keep_frac) for v in w.vis_len]
        self.rank_layer = max(l for l in range(first_late) if not w.lazy_mask[l])
        self.late_len = [L - v + k for L, v, k in zip(w.seq_len, w.vis_len, self.keep)]
        self.cu_late = [0]
        for n in self.late_len:
            self.cu_late.append(self.cu_late[-1] + n)
        dev = self.sess.device
        cu = w.cu_seqlens
        self.q_last = torch.stack([self.pre[self.rank_layer][0][cu[b + 1] - 1] for b in range(w.batch)]).contiguous()
        self.sel_ws = torch.empty(B.qc_select_workspace_bytes(self.sess.cfg), dtype=torch.uint8, device=dev)
        self.stride = w.max_seq
        self.probs = torch.zeros((w.batch, self.stride), dtype=torch.float32, device=dev)
        self.row_map = torch.zeros(self.cu_late[-1], dtype=torch.int32, device=dev)
        self.hidden = torch.randn(w.total_tokens, d_model, device=dev).to(torch.bfloat16)
        self.hidden_late = torch.empty(self.cu_late[-1], d_model, dtype=torch.bfloat16, device=dev)
        self.row_bytes = d_model * 2
        self.out_late = None
        self.prefill_stack()                 # first pass: fixes the row map; late layers still read full-length inputs' heads
        torch.cuda.synchronize()
        rows = self.row_map.long()
        for l in range(first_late, w.n_layers):
            self.pre[l] = tuple(t.index_select(0, rows).contiguous() for t in self.pre[l])
        self.out_late = torch.empty_like(self.pre[first_late][2])

    def prefill_stack(self):
        w, s, B = self.w, self.sess, self.B
        s.reset(w.vis_start, w.vis_len, zero_fill=False)
        for l in range(w.n_layers):
            q, k, v = self.pre[l]
            late = l >= self.first_late
            if late and self.out_late is None:          # construction pass: any rows of the right count will do
                q, k, v = (t[: self.cu_late[-1]] for t in (q, k, v))
            if self.no_qk[l]:
                q = k = None
            out = self.out_pre[: v.shape[0]] if (not late or self.out_late is None) else self.out_late
            s.prefill(l, q, k, v, self.cu_late if late else w.cu_seqlens, out=out)
            if l == self.rank_layer:
                B.qc_last_row_attention(s.kv, l, self.q_last, self.probs, self.stride, 0.0, self.sel_ws,
                                        self.sel_ws.numel())
                B.qc_prune_select(self.probs, self.stride, w.batch, w.cu_seqlens, w.vis_start, w.vis_len, self.keep,
                                  self.row_map)
                B.qc_gather_rows(self.hidden, self.row_bytes, self.row_map, self.cu_late[-1], self.row_bytes,
                                 self.hidden_late, self.row_bytes)
            if l == self.first_late - 1:
                s.prune(self.first_late, self.keep)

    def decode_bytes_per_step(self, generated):
        """Algorithmic decode bytes of one step over all layers (late layers stream the shortened sequences)."""
        w = self.w
        e = w.n_heads * w.head_dim * w.elem_bytes
        early = sum((2 * (L + generated + 1) + 6) * e for L in w.seq_len)
        late = sum((2 * (L + generated + 1) + 6) * e for L in self.late_len)
        return self.first_late * early + (w.n_layers - self.first_late) * late


def bench_pruning(args):
    """Token pruning on top of Visual Lazy Attention ("Compatibility" paragraph): the batched-decode
    configuration with a boundary after layer 1 that keeps half of every image's tokens, beside the same
    configuration without pruning, timed in the same run; then the cost of the boundary itself."""
    import torch
    import workloads
    from paper_2602_01901_amd import binding as B
    w = workloads.config(2)
    steps = args.decode_batched_steps
    first_late, keep_frac = 2, 0.5
    out = {"workload": w.name + " + pruning", "boundary_before_layer": first_late, "kept_fraction_of_visual_tokens": keep_frac}
    for name in ("unpruned", "pruned"):
        r = (PrunedRunner(w, steps, first_late, keep_frac, distinct_decode_inputs=4) if name == "pruned"
             else Runner(w, steps, distinct_decode_inputs=4))
        r.prefill_stack()
        _, pre_s = timed(torch, r.prefill_stack, 3)
        r.decode_steps_run(2)
        torch.cuda.synchronize()
        g0 = r.sess.stats()["generated"]
        _, ev_s = timed(torch, lambda: r.decode_steps_run(steps), 1)
        g1 = r.sess.stats()["generated"]
        kt = r.kernel_times(lambda: r.decode_steps_run(4))
        call_us, call_n = kt["decode"]
        if name == "pruned":
            bytes_call = sum(r.decode_bytes_per_step(g1 + t) for t in range(4)) / 4 / w.n_layers
        else:
            bytes_call = sum(decode_bytes_per_layer(w, g1 + t) for t in range(4)) / 4
        stats = r.sess.stats()
        achieved = bytes_call / (call_us * 1e-6) / 1e9
        out[name] = {
            "prefill_ms": pre_s * 1e3,
            "decode_tokens_per_s": w.batch * steps / ev_s, "decode_ms_per_step": ev_s / steps * 1e3,
            "kv_cache_bytes_per_token": (stats["k_bytes"] + stats["v_bytes"]) / stats["tokens"],
            "roofline": {"bound": "hbm", "kernel": "decode_split_kernel<bf16,128> (mean over the layers of a step)",
                         "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                         "traffic": None, "avg_launch_us": call_us, "launches_timed": call_n,
                         "algorithmic_bytes_per_launch": bytes_call},
        }
        if name == "pruned":
            def boundary_select():
                B.qc_prune_select(r.probs, r.stride, w.batch, w.cu_seqlens, w.vis_start, w.vis_len, r.keep, r.row_map)

            def boundary_gather():
                B.qc_gather_rows(r.hidden, r.row_bytes, r.row_map, r.cu_late[-1], r.row_bytes, r.hidden_late, r.row_bytes)
            _, sel_s = timed(torch, boundary_select, 20)
            _, gat_s = timed(torch, boundary_gather, 20)
            moved = 2 * r.cu_late[-1] * r.row_bytes + 4 * r.cu_late[-1]
            out["boundary"] = {"select_us": sel_s * 1e6, "gather_us": gat_s * 1e6,
                               "gather_rows": r.cu_late[-1], "gather_row_bytes": r.row_bytes,
                               "gather_roofline": {"bound": "hbm", "kernel": "gather_rows_kernel", "achieved": moved / gat_s / 1e9,
                                                   "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": moved / gat_s / 1e9 / HBM_PEAK_GBS,
                                                   "traffic": measured_traffic("pruning_gather"), "avg_launch_us": gat_s * 1e6,
                                                   "algorithmic_bytes_per_launch": moved}}
        del r
        torch.cuda.empty_cache()
    out["decode_speedup"] = out["pruned"]["decode_tokens_per_s"] / out["unpruned"]["decode_tokens_per_s"]
    # survivor selection alone at the spans of the other configurations (half of every span kept): one
    # workgroup per sequence, O(span) work, latency-bound
    sizes = {}
    for name, cfg_i in (("cfg2_576x1", 1), ("cfg4_2880x8", 3), ("cfg5_4608x4", 4)):
        wc = workloads.config(cfg_i)
        stride = max(wc.seq_len)
        g = torch.Generator(device="cuda").manual_seed(0x51C0 + 99)
        sc = torch.rand((wc.batch, stride), generator=g, device="cuda", dtype=torch.float32)
        keep = [v // 2 for v in wc.vis_len]
        rm = torch.zeros(sum(L - v + k for L, v, k in zip(wc.seq_len, wc.vis_len, keep)), dtype=torch.int32, device="cuda")
        run = lambda: B.qc_prune_select(sc, stride, wc.batch, wc.cu_seqlens, wc.vis_start, wc.vis_len, keep, rm)
        run()
        _, sel_s = timed(torch, run, 20)
        sizes[name] = {"visual_tokens": wc.vis_len[0], "batch": wc.batch, "select_us": sel_s * 1e6}
    out["select_by_span"] = sizes
    return out


def bench_capacity(args):
    """The maximum-batch comparison of the "Efficiency Evaluation" paragraph, re-run here: 7B shape, 2048
    positions per sequence, and the memory that holds exactly 21 such sequences without lazy layers.
    qc_plan_max_batch gives the batch each variant fits into that memory (22 lazy layers: the count
    whose Global-Lazy-Attention saving n/2N is closest to the 35 % the paper reports); each variant then
    decodes at its own maximum batch."""
    import torch
    import workloads
    import paper_2602_01901_amd as P
    from paper_2602_01901_amd import binding as B
    N, H, D, steps = 32, 32, 128, args.decode_batched_steps
    L0, vis, vs = 2048 - steps - 2, 1728, 32
    lazy22 = [int(2 <= l <= 30 and ((l - 2) % 4 != 0 or l == 30)) for l in range(N)]
    assert sum(lazy22) == 22 and not lazy22[0]
    plain_cfg = lambda b: P.make_config(N, H, D, "bf16", b, 2048, vis, 2048 - vis, [0] * N)
    budget = B.qc_kv_arena_bytes(plain_cfg(21)) + 4096
    out = {"positions_per_sequence": 2048, "visual_tokens": vis, "lazy_layers": 22, "budget_bytes": budget,
           "pruned_variants": "boundary before layer 2, half of the visual tokens kept, later layers sized for the shortened sequences",
           "variants": {}}
    keep = vis // 2                       # token pruning: half of the visual tokens survive a boundary before layer 2
    late = dict(prune_before_layer=2, max_seq_late=2048 - (vis - keep))
    for name, mask, mode, prune in (("plain", [0] * N, "vla", False), ("vla", lazy22, "vla", False),
                                    ("gla", lazy22, "gla", False), ("vla_pruned", lazy22, "vla", True),
                                    ("gla_pruned", lazy22, "gla", True)):
        extra = late if prune else {}
        cfg1 = P.make_config(N, H, D, "bf16", 1, 2048, vis, 2048 - vis, mask, mode=mode, **extra)
        batch = B.qc_plan_max_batch(cfg1, budget, B.QC_PLAN_KV)
        batch_all = B.qc_plan_max_batch(cfg1, budget, B.QC_PLAN_KV | B.QC_PLAN_Q | B.QC_PLAN_WORKSPACE)
        w = workloads.custom("capacity_" + name, N, H, D, "bf16", [vs] * batch, [vis] * batch, [L0] * batch, steps + 2,
                             mask, max_seq=2048, max_vis=vis, max_text=2048 - vis)
        s = P.Session.for_workload(w, mode=mode, **extra)
        q, k, v = workloads.prefill_qkv(w, 0, device=s.device)      # one set of inputs serves every layer
        o = torch.empty_like(v)
        s.reset(w.vis_start, w.vis_len, zero_fill=False)
        L1 = L0 - (vis - keep)
        cu_late = [b * L1 for b in range(batch + 1)]
        for l in range(N):
            no_qk = mode == "gla" and mask[l]
            if prune and l == 2:
                s.prune(2, [keep] * batch)
            if prune and l >= 2:                # the shortened prompts: any rows of the right count will do here
                n = cu_late[-1]
                s.prefill(l, None if no_qk else q[:n], None if no_qk else k[:n], v[:n], cu_late, out=o[:n])
            else:
                s.prefill(l, None if no_qk else q, None if no_qk else k, v, w.cu_seqlens, out=o)
        dq, dk, dv = workloads.decode_qkv(w, 0, 0, device=s.device)
        do = torch.empty_like(dv)

        def run(n):
            for _ in range(n):
                for l in range(N):
                    no_qk = mode == "gla" and mask[l]
                    s.decode(l, None if no_qk else dq, None if no_qk else dk, dv, out=do)
        run(2)
        _, ev_s = timed(torch, lambda: run(steps), 1)
        st = s.stats()
        out["variants"][name] = {"max_batch": batch, "max_batch_counting_q_cache_and_workspace": batch_all,
                                 "kv_arena_bytes": s.kv_bytes, "q_arena_bytes": s.q_bytes,
                                 "decode_tokens_per_s": batch * steps / ev_s, "decode_ms_per_step": ev_s / steps * 1e3,
                                 "kv_cache_bytes_per_token": (st["k_bytes"] + st["v_bytes"]) / st["tokens"]}
        log("capacity %s: batch %d, %.0f tok/s" % (name, batch, batch * steps / ev_s))
        s.close()
        del s, q, k, v, o
        torch.cuda.empty_cache()
    out["ragged_batch"] = bench_ragged_arena(args)
    p = out["variants"]["plain"]
    for name in ("vla", "gla", "vla_pruned", "gla_pruned"):
        out["variants"][name]["batch_vs_plain"] = out["variants"][name]["max_batch"] / p["max_batch"]
        out["variants"][name]["attention_throughput_vs_plain"] = out["variants"][name]["decode_tokens_per_s"] / p["decode_tokens_per_s"]
    out["note"] = ("attention only: streaming a sequence's caches costs the same at any batch, so the larger batch "
                   "raises throughput here only where the bytes per token drop (score sharing under GLA); the "
                   "weight-streaming part of a decode step, which a larger batch amortises, lies outside this path")
    return out


def bench_ragged_arena(args):
    """The batched-decode configuration (32 prompts of 704..1088 tokens, 512 generated) in an arena with one
    capacity for all (sized by the longest sequence) and in one with per-sequence capacities (sized by the
    sum): bytes allocated and decode throughput of the same batch."""
    import torch
    import workloads
    import paper_2602_01901_amd as P
    base = workloads.config(2)
    steps = args.decode_batched_steps
    cap_seq = [(L + base.decode_steps + 7) // 8 * 8 for L in base.seq_len]
    cap_text = [L - v + base.decode_steps for L, v in zip(base.seq_len, base.vis_len)]
    n = base.batch
    per = lambda total: -(-total // n)
    ragged = workloads.custom("cfg3_ragged_arena", base.n_layers, base.n_heads, base.head_dim, "bf16", base.vis_start,
                              base.vis_len, base.seq_len, base.decode_steps, base.lazy_mask, seed_tag=0,
                              max_seq=per(sum(cap_seq)), max_vis=base.max_vis, max_text=per(sum(cap_text)))
    res = {}
    for name, w, caps in (("one_capacity_for_all", base, None), ("per_sequence_capacities", ragged, (cap_seq, cap_text))):
        s = P.Session.for_workload(w)
        q, k, v = workloads.prefill_qkv(w, 0, device=s.device)
        o = torch.empty_like(v)
        if caps:
            s.reset(w.vis_start, w.vis_len, zero_fill=False, cap_seq=caps[0], cap_text=caps[1])
        else:
            s.reset(w.vis_start, w.vis_len, zero_fill=False)
        for l in range(w.n_layers):
            s.prefill(l, q, k, v, w.cu_seqlens, out=o)
        dq, dk, dv = workloads.decode_qkv(w, 0, 0, device=s.device)
        do = torch.empty_like(dv)

        def run(nsteps):
            for _ in range(nsteps):
                for l in range(w.n_layers):
                    s.decode(l, dq, dk, dv, out=do)
        run(2)
        _, ev_s = timed(torch, lambda: run(steps), 1)
        res[name] = {"kv_arena_bytes": s.kv_bytes, "q_arena_bytes": s.q_bytes, "max_seq": w.max_seq, "max_text": w.max_text,
                     "decode_tokens_per_s": w.batch * steps / ev_s}
        if caps:
            # Four pairs of neighbouring slots leave and come back, the second of each pair first (qc_seq_leave /
            # qc_seq_join): first-fit then fills each pair's hole in the other order, so slot order and row
            # order differ (the arena has no spare rows, so this is the reordering that is sure to fit).
            # Prefill pass over the eight, then the same timed decode steps for the whole batch.
            pairs = [(b, b + 1) for b in range(2, w.batch - 1, 8)]
            movers = sorted(b for pr in pairs for b in pr)
            B = P.binding
            for b in movers:
                s.seq_leave(b)
            for lo, hi in pairs:
                for b in (hi, lo):
                    s.seq_join(b, w.vis_start[b], w.vis_len[b], caps[0][b], caps[1][b])
            moved = sum(B.qc_seq_extent(s.kv, b)[1] != sum(caps[0][:b]) for b in movers)
            cu = [0]
            for b in range(w.batch):
                cu.append(cu[-1] + (w.seq_len[b] if b in movers else 0))
            rows = torch.cat([torch.arange(w.cu_seqlens[b], w.cu_seqlens[b + 1], device=s.device) for b in movers])
            qj, kj, vj = q[rows], k[rows], v[rows]
            oj = torch.empty_like(vj)
            for l in range(w.n_layers):
                s.prefill(l, qj, kj, vj, cu, out=oj)
            run(2)
            _, ev_j = timed(torch, lambda: run(steps), 1)
            res["after_leave_and_join"] = {"sequences_moved": len(movers), "extents_at_new_rows": int(moved),
                                           "decode_tokens_per_s": w.batch * steps / ev_j}
            del qj, kj, vj, oj
        s.close()
        del s, q, k, v, o
        torch.cuda.empty_cache()
    res["arena_bytes_ratio"] = res["per_sequence_capacities"]["kv_arena_bytes"] / res["one_capacity_for_all"]["kv_arena_bytes"]
    res["decode_rate_vs_one_capacity"] = {k: res[k]["decode_tokens_per_s"] / res["one_capacity_for_all"]["decode_tokens_per_s"]
                                          for k in ("per_sequence_capacities", "after_leave_and_join")}
    return res


def bench_paged(args):
    """Pages against runs of rows: the batched-decode configuration (32 prompts of 704..1088 tokens, capacities
    rounded up to whole pages) decoded from both layouts in the same run, again after a quarter of the batch
    has left and other sequences have taken the freed pages, and the high-resolution prefill on pages."""
    import dataclasses
    import torch
    import workloads
    import paper_2602_01901_amd as P
    base = workloads.config(2)
    up = lambda x: -(-x // 64) * 64
    w = dataclasses.replace(base, max_seq=up(base.max_seq), max_text=up(base.max_text))
    steps = args.decode_batched_steps
    res = {"workload": w.name + " (capacities in whole pages)", "page_rows": 64}
    for name, paged in (("rows_in_runs", False), ("pages", True)):
        s = P.Session.for_workload(w)
        q, k, v = workloads.prefill_qkv(w, 0, device=s.device)
        o = torch.empty_like(v)
        s.reset(w.vis_start, w.vis_len, zero_fill=False, paged=paged)

        def prefill_all(qq, kk, vv, cu, oo):
            for l in range(w.n_layers):
                s.prefill(l, qq, kk, vv, cu, out=oo)
        prefill_all(q, k, v, w.cu_seqlens, o)
        torch.cuda.synchronize()
        s.reset(w.vis_start, w.vis_len, zero_fill=False, paged=paged)
        _, ev_p = timed(torch, lambda: prefill_all(q, k, v, w.cu_seqlens, o), 1)
        dq, dk, dv = workloads.decode_qkv(w, 0, 0, device=s.device)
        do = torch.empty_like(dv)

        def run(nsteps):
            for _ in range(nsteps):
                for l in range(w.n_layers):
                    s.decode(l, dq, dk, dv, out=do)
        run(2)
        _, ev_s = timed(torch, lambda: run(steps), 1)
        res[name] = {"prefill_stack_ms": ev_p * 1e3, "decode_tokens_per_s": w.batch * steps / ev_s}
        if paged:
            # what the pools hold now, and what the batch would hold with every sequence decoded to the end:
            # the admission arithmetic a serving loop does with qc_pages_needed and qc_pool_pages
            pools = [P.binding.qc_pool_pages(s.kv, pool) for pool in range(3)]
            at_end = [sum(x) for x in zip(*[P.binding.qc_pages_needed(s.cfg, w.seq_len[b] + w.decode_steps, w.vis_len[b])
                                            for b in range(w.batch)])]
            res[name]["pool_pages"] = {"total": [t for t, _ in pools], "held_now": [t - f for t, f in pools],
                                       "held_after_%d_decode_steps" % w.decode_steps: at_end}
            # every fourth sequence leaves; the freed pages go, lowest first, to the same prompts joining in
            # the reverse order, so a sequence's pages are scattered over the pools
            movers = list(range(1, w.batch, 4))
            for b in movers:
                s.seq_leave(b)
            for b in reversed(movers):
                s.seq_join(b, w.vis_start[b], w.vis_len[b])
            cu = [0]
            for b in range(w.batch):
                cu.append(cu[-1] + (w.seq_len[b] if b in movers else 0))
            rows = torch.cat([torch.arange(w.cu_seqlens[b], w.cu_seqlens[b + 1], device=s.device) for b in movers])
            qj, kj, vj = q[rows], k[rows], v[rows]
            prefill_all(qj, kj, vj, cu, torch.empty_like(vj))
            run(2)
            _, ev_j = timed(torch, lambda: run(steps), 1)
            B = P.binding
            lists = [B.qc_seq_pages(s.kv, b, 0) for b in movers]
            res["pages_after_leave_and_join"] = {
                "sequences_moved": len(movers),
                "page_lists_not_consecutive": sum(any(y != x + 1 for x, y in zip(l, l[1:])) for l in lists),
                "decode_tokens_per_s": w.batch * steps / ev_j}
            del qj, kj, vj
        s.close()
        del s, q, k, v, o
        torch.cuda.empty_cache()
    res["decode_rate_pages_vs_runs"] = res["pages"]["decode_tokens_per_s"] / res["rows_in_runs"]["decode_tokens_per_s"]
    res["decode_rate_scattered_pages_vs_runs"] = (res["pages_after_leave_and_join"]["decode_tokens_per_s"] /
                                                  res["rows_in_runs"]["decode_tokens_per_s"])
    # prefill at the high-resolution shape (8 x 3008 tokens): the matrix-core kernel in both layouts
    w4 = workloads.config(3)
    flops = prefill_flops_per_layer(w4)
    layers = [l for l in range(w4.n_layers)][:8]
    for name, paged in (("rows_in_runs", False), ("pages", True)):
        s = P.Session.for_workload(w4)
        pre = [workloads.prefill_qkv(w4, l, device=s.device) for l in layers]
        o = torch.empty_like(pre[0][2])

        def run_pre():
            s.reset(w4.vis_start, w4.vis_len, zero_fill=False, paged=paged)
            for l in layers:
                s.prefill(l, *pre[l], w4.cu_seqlens, out=o)
        run_pre()
        _, ev = timed(torch, run_pre, args.prefill_reps)
        res[name]["prefill_highres_tflops"] = flops * len(layers) / ev / 1e12
        s.close()
        del s, pre, o
        torch.cuda.empty_cache()
    res["prefill_rate_pages_vs_runs"] = res["pages"]["prefill_highres_tflops"] / res["rows_in_runs"]["prefill_highres_tflops"]
    return res


def bench_headline(args):
    """13B-shaped video workload (cfg5): the line's headline.  A step = reset + 40-layer prefill of
    4 x 4864 tokens + 1024 decode steps x 40 layers, through ordinary qc_prefill / qc_decode calls
    (65 us kernels: replaying a graph gains nothing here).  Inside the timed region HIP events on the
    launch stream mark the two phases of every step; the library's own event pairs around the dominant
    kernels are on for every prefill launch and for one decode step in every 32 (1280 of 40960 decode
    launches per step), so that they do not slow the step they measure."""
    import torch
    import workloads
    w = workloads.config(4)
    r = Runner(w, w.decode_steps, distinct_decode_inputs=4)
    from paper_2602_01901_amd import binding as B
    kv = r.sess.kv
    for i in range(args.warmup):
        r.step()
        log("headline: warmup step %d done" % (i + 1))
    torch.cuda.synchronize()
    for which in (0, 1, 2):
        B.qc_timing_read(kv, which)
    timed_steps, phases = [], []
    stats_prefill = {}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record()
        B.qc_timing_enable(kv, 1)
        r.prefill_stack()
        B.qc_timing_enable(kv, 0)
        ev[1].record()
        if i == 0:
            stats_prefill.update(r.sess.stats())
        r.decode_steps_run(w.decode_steps, time_every=32, timed_steps=timed_steps)
        ev[2].record()
        phases.append(ev)
        if (i + 1) % 4 == 0:
            log("headline: timed step %d enqueued" % (i + 1))
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / args.steps
    pre_s = sum(e[0].elapsed_time(e[1]) for e in phases) * 1e-3 / args.steps
    dec_s = sum(e[1].elapsed_time(e[2]) for e in phases) * 1e-3 / args.steps
    pre_ms, pre_n = B.qc_timing_read(kv, 0)
    dec_ms, dec_n = B.qc_timing_read(kv, 1)
    assert dec_n == len(timed_steps) * w.n_layers, (dec_n, len(timed_steps))
    pre_us, dec_us = pre_ms * 1e3 / pre_n, dec_ms * 1e3 / dec_n
    stats = r.sess.stats()
    flops_layer = prefill_flops_per_layer(w)
    bytes_call = sum(decode_bytes_per_layer(w, g) for g in timed_steps) / len(timed_steps)
    bytes_phase = sum(decode_bytes_per_layer(w, g) for g in range(w.decode_steps)) * w.n_layers
    launches_per_step = w.decode_steps * w.n_layers
    # Dominant kernel: the streaming decode kernel, launched once per layer call.  Its duration is taken
    # as the decode phase's HIP-event time divided by the number of layer calls: that charges the small
    # merge pass and every launch gap to it (a lower bound on its bandwidth) and by construction fits
    # inside the step.  The event pairs the library records around the kernel alone, on sampled steps,
    # are given beside it; a pair also brackets the dispatch of the kernel it surrounds.
    call_us = dec_s / launches_per_step * 1e6
    bytes_mean = bytes_phase / launches_per_step
    achieved = bytes_mean / (call_us * 1e-6) / 1e9
    res = {
        "ms_per_step": wall * 1e3,
        "decode_tokens_per_s": w.batch * w.decode_steps / dec_s,
        "tokens_per_s_whole_step": w.batch * w.decode_steps / wall,
        "decode_ms_per_token_step": dec_s / w.decode_steps * 1e3,
        "decode_phase_ms": dec_s * 1e3,
        "prefill_ms": pre_s * 1e3,
        "prefill_tflops": flops_layer * w.n_layers / pre_s / 1e12,
        "k_cache_bytes_per_token": stats["k_bytes"] / stats["tokens"],
        "k_cache_bytes_per_token_after_prefill": stats_prefill["k_bytes"] / stats_prefill["tokens"],
        "k_cache_bytes_per_token_standard": w.n_layers * w.n_heads * w.head_dim * w.elem_bytes,
        "roofline": {"bound": "hbm", "kernel": "decode_split_kernel<bf16,128> (8 key chunks per (sequence, head): 5 workgroups per compute unit; duration = decode "
                     "phase / layer calls, so the merge pass and the launch gaps are charged to it)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic("decode_cfg5"),
                     "traffic_measured_at": "the first 22 decode steps (lengths 4865..4886: 399.7 MB algorithmic per launch there; "
                                            "the timed region's mean over 1024 steps is algorithmic_bytes_per_launch)",
                     "avg_launch_us": call_us, "launches_timed": launches_per_step * args.steps,
                     "algorithmic_bytes_per_launch": bytes_mean, "launches_per_step": launches_per_step,
                     "event_pairs_around_kernel": {"avg_us": dec_us, "launches": dec_n, "algorithmic_bytes_per_launch": bytes_call,
                                                   "GBps": bytes_call / (dec_us * 1e-6) / 1e9}},
        "prefill_kernel": {"bound": "mfma", "kernel": "prefill_mfma_kernel (attention + fused cache writes: whole layer call)",
                           "achieved": flops_layer / (pre_us * 1e-6) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": flops_layer / (pre_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                           "traffic": measured_traffic("prefill_cfg5"), "avg_launch_us": pre_us, "launches_timed": pre_n,
                           "algorithmic_flops_per_launch": flops_layer},
    }
    del r
    torch.cuda.empty_cache()
    return w, res


def bench_prefill_long(args):
    """One 32768-token prompt (32000 visual tokens), 7B head shape, 4 layers with one lazy block: the
    prefill kernel's steady state, where per-workgroup fixed costs are amortised over 257 key tiles."""
    import workloads
    w = workloads.custom("extra_long_prompt_32k_b1", 4, 32, 128, "bf16", [256], [32000], [32768], 0, [0, 0, 1, 1])
    return bench_prefill_highres(args, w=w, traffic_key="prefill_long")


def host_threads():
    """Threads the oracle's numpy routines actually use (its matrix products run in the BLAS pool)."""
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads", 0) for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return max(n)
    except Exception:
        pass
    return os.cpu_count() or 1


def cpu_baseline_sample(w, heads, seq=0):
    """The fp64 oracle as it stands, on the host cores, on a bounded sample of workload `w`: sequence
    `seq`, the first `heads` heads (sequences and heads are independent instances of the method), fed
    the very inputs the GPU run uses.  Timed: ONE prefill layer (layer 0, every query row) and ONE decode
    step (all layers, caches filled by an untimed pass that stores every layer's rows).  Rates are what
    was run divided by its time; the decode rate is expressed in the metric's unit by the share of the
    batch's (sequence, head) pairs the sample covers.  Nothing is extrapolated across layers."""
    import workloads
    from oracle.lazy_stack import LazyStackOracle
    cu = w.cu_seqlens
    L = w.seq_len[seq]
    st = LazyStackOracle(w.n_layers, heads, w.head_dim, w.lazy_mask, w.vis_start[seq], w.vis_len[seq])

    def sample(t):
        return workloads.to_f64(t[cu[seq]:cu[seq + 1], :heads])
    q, k, v = (sample(t) for t in workloads.prefill_qkv(w, 0, device="cuda"))
    t0 = time.perf_counter()
    st.prefill(0, q, k, v)
    t_pre = time.perf_counter() - t0
    for l in range(1, w.n_layers):
        q, k, v = (sample(t) for t in workloads.prefill_qkv(w, l, device="cuda"))
        st.prefill(l, q, k, v, rows=[0])
    ins = [[workloads.to_f64(t[seq, :heads]) for t in workloads.decode_qkv(w, l, 0, device="cuda")] for l in range(w.n_layers)]
    t1 = time.perf_counter()
    for l in range(w.n_layers):
        st.decode(l, *ins[l])
    t_dec = time.perf_counter() - t1
    flops = heads * 4 * w.head_dim * L * (L + 1) // 2
    share = heads / (w.batch * w.n_heads)           # of the batch's (sequence, head) pairs
    return {"value": w.batch * share / t_dec, "unit": "tokens/s", "cores": host_threads(), "kind": "oracle",
            "sample": "%s, sequence %d (%d tokens), heads 0..%d of %d: one prefill layer in full (%.2f s) and one decode "
                      "step over all %d layers (%.3f s); tokens/s = batch x (sample's share of the batch's (sequence, head) "
                      "pairs) / decode-step time" % (w.name, seq, L, heads - 1, w.n_heads, t_pre, w.n_layers, t_dec),
            "prefill_tflops_fp64": flops / t_pre / 1e12, "prefill_layer_s": t_pre, "decode_step_s": t_dec,
            "pairs_share": share}


def cpu_baseline_cfg2(budget_s=8.0):
    """The batch-1 7B shape is small enough for the oracle to run whole: the full 32-layer prefill, then
    as many 32-layer decode steps as fit the budget."""
    import workloads
    from oracle.lazy_stack import LazyStackOracle
    w = workloads.config(1)
    st = LazyStackOracle(w.n_layers, w.n_heads, w.head_dim, w.lazy_mask, w.vis_start[0], w.vis_len[0])
    inputs = [[workloads.to_f64(t) for t in workloads.prefill_qkv(w, l, device="cuda")] for l in range(w.n_layers)]
    t0 = time.perf_counter()
    for l in range(w.n_layers):
        st.prefill(l, *inputs[l])
    t_pre = time.perf_counter() - t0
    del inputs
    steps = 0
    t1 = time.perf_counter()
    while steps < w.decode_steps and (time.perf_counter() - t1) < budget_s:
        for l in range(w.n_layers):
            st.decode(l, *[workloads.to_f64(t[0]) for t in workloads.decode_qkv(w, l, steps, device="cuda")])
        steps += 1
    t_dec = time.perf_counter() - t1
    return {"value": w.batch * steps / t_dec, "unit": "tokens/s", "cores": host_threads(), "kind": "oracle",
            "sample": "%s: full 32-layer prefill (%.2f s) then %d decode steps of 32 layers (%.2f s)" % (w.name, t_pre, steps, t_dec),
            "prefill_tflops_fp64": prefill_flops_per_layer(w) * w.n_layers / t_pre / 1e12}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--decode-batched-steps", type=int, default=16)
    ap.add_argument("--prefill-reps", type=int, default=3)
    ap.add_argument("--skip-extra", action="store_true", help="headline workload only")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="batch-1 workload: ordinary qc_decode calls instead of one HIP-graph replay per decode step")
    ap.add_argument("--only", choices=["headline", "cfg2", "decode_batched", "prefill_highres", "gla_decode_batched", "selection",
                                      "projection", "pruning", "capacity", "paged", "prefill_long", "prefill_cfg5", "decode_cfg5"],
                    help="profiling aid: run just this workload and print its object")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="profiling aid: run plain 1 GiB device copies (known HBM traffic) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (nothing in the attention path needs a collective); "
                 "use --gpus 1")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the library has no CPU path")
    import paper_2602_01901_amd as P
    import workloads
    P.load_library()

    if args.copy_calibration:
        # 1 GiB read + 1 GiB written per launch: the yardstick for the FETCH_SIZE / WRITE_SIZE counters
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_launch": 1 << 30, "bytes_written_per_launch": 1 << 30,
                                               "launches": 5}}))
        return
    if args.only:
        fn = {"headline": lambda a: bench_headline(a)[1], "cfg2": bench_cfg2,
              "decode_batched": bench_decode_batched, "prefill_highres": bench_prefill_highres,
              "gla_decode_batched": bench_gla_decode_batched, "selection": bench_selection,
              "projection": bench_projection, "pruning": bench_pruning, "capacity": bench_capacity,
              "prefill_long": bench_prefill_long, "paged": bench_paged,
              "prefill_cfg5": lambda a: bench_prefill_highres(a, w=workloads.config(4), traffic_key="prefill_cfg5"),
              "decode_cfg5": lambda a: bench_decode_batched(a, w=workloads.config(4), traffic_key="decode_cfg5")}[args.only]
        print(json.dumps({args.only: fn(args)}))
        return

    w, r = bench_headline(args)
    log("cfg5 done: %.1f tok/s decode (%.0f GB/s in the streaming kernel), prefill %.1f TFLOP/s"
        % (r["decode_tokens_per_s"], r["roofline"]["achieved"], r["prefill_tflops"]))
    extra = {}
    if not args.skip_extra:
        extra["llava15_7b_b1"] = bench_cfg2(args)
        log("cfg2 done: %.1f tok/s decode, prefill %.2f TFLOP/s" % (extra["llava15_7b_b1"]["decode_tokens_per_s"],
                                                                   extra["llava15_7b_b1"]["prefill_tflops"]))
        extra["decode_batched"] = bench_decode_batched(args)
        log("cfg3 done: %.1f tok/s, %.0f GB/s" % (extra["decode_batched"]["decode_tokens_per_s"],
                                                 extra["decode_batched"]["roofline"]["achieved"]))
        extra["prefill_highres"] = bench_prefill_highres(args)
        log("cfg4 done: %.1f TFLOP/s" % extra["prefill_highres"]["prefill_tflops"])
        extra["prefill_long_32k"] = bench_prefill_long(args)
        log("32k prompt done: %.1f TFLOP/s" % extra["prefill_long_32k"]["prefill_tflops"])
        extra["gla_decode_batched"] = bench_gla_decode_batched(args)
        log("GLA cfg3 done: %.1f tok/s, lazy layers %.0f GB/s" % (extra["gla_decode_batched"]["decode_tokens_per_s"],
                                                                 extra["gla_decode_batched"]["roofline"]["achieved"]))
        extra["gla_prefill_highres"] = bench_prefill_highres(args, traffic_key="gla_prefill_cfg4", mode="gla")
        log("GLA cfg4 done: %.1f TFLOP/s" % extra["gla_prefill_highres"]["prefill_tflops"])
        extra["projection"] = bench_projection(args)
        log("projection done: ordinary %.1f TFLOP/s, lazy layer %.1f us" % (extra["projection"]["ordinary_layer"]["tflops"],
                                                                        extra["projection"]["lazy_layer_text_rows"]["us"]))
        extra["selection"] = bench_selection(args)
        log("selection done: %.1f us per layer" % extra["selection"]["last_row_attention_us_per_layer"])
        extra["pruning"] = bench_pruning(args)
        log("pruning done: %.1f -> %.1f tok/s" % (extra["pruning"]["unpruned"]["decode_tokens_per_s"],
                                                extra["pruning"]["pruned"]["decode_tokens_per_s"]))
        extra["capacity"] = bench_capacity(args)
        extra["paged"] = bench_paged(args)
        log("pages done: decode %.3f x, scattered %.3f x, prefill %.3f x the rate with rows in runs"
            % (extra["paged"]["decode_rate_pages_vs_runs"], extra["paged"]["decode_rate_scattered_pages_vs_runs"],
               extra["paged"]["prefill_rate_pages_vs_runs"]))
    cpu = None
    if not args.skip_cpu:
        cpu = cpu_baseline_sample(w, heads=8)
        log("oracle on cfg5 sample: %.3f tok/s, prefill %.4f TFLOP/s fp64" % (cpu["value"], cpu["prefill_tflops_fp64"]))
        if not args.skip_extra:
            extra["llava15_7b_b1"]["cpu_baseline"] = cpu_baseline_cfg2()
            extra["decode_batched"]["cpu_baseline"] = cpu_baseline_sample(workloads.config(2), heads=8)
            extra["prefill_highres"]["cpu_baseline"] = cpu_baseline_sample(workloads.config(3), heads=8)
            log("oracle on cfg2/cfg3/cfg4 samples done")
    line = {
        "metric": "decode_tokens_per_s", "value": r["decode_tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "layers": w.n_layers, "heads": w.n_heads, "head_dim": w.head_dim,
                   "batch": w.batch, "visual_tokens": w.vis_len[0], "text_tokens": w.seq_len[0] - w.vis_len[0],
                   "decode_steps": w.decode_steps, "lazy_layers": w.n_lazy,
                   "step": "reset + 40-layer prefill of 4 x 4864 tokens + 1024 decode steps x 40 layers",
                   "value_is": "tokens generated / time of the decode phases inside the timed steps (HIP events on the launch stream)",
                   "decode_launch": "ordinary qc_decode calls"},
        "tokens_per_s_whole_step": r["tokens_per_s_whole_step"],
        "prefill_tflops": r["prefill_tflops"], "prefill_ms": r["prefill_ms"],
        "decode_phase_ms": r["decode_phase_ms"],
        "decode_ms_per_token_step": r["decode_ms_per_token_step"],
        "k_cache_bytes_per_token": r["k_cache_bytes_per_token"],
        "k_cache_bytes_per_token_after_prefill": r["k_cache_bytes_per_token_after_prefill"],
        "k_cache_bytes_per_token_standard": r["k_cache_bytes_per_token_standard"],
        "roofline": r["roofline"],
        "prefill_kernel": r["prefill_kernel"],
        "cpu_baseline": cpu,
        # what the paper itself reports, as context (another machine, whole model): not a target of this run
        "paper_context": {"hardware": "one 80 GB A100, LLaVA-NeXT-7B, input length 2048",
                          "kv_cache_saving": "35 % (GLA and VLA)", "max_batch": "21 -> 32",
                          "decode_throughput": "1.6x (GLA), 1.5x (VLA) over the unmodified model",
                          "efficiency_table_with_FastV": "prefill 30.88 -> 18.49 TFLOPs, 142.60 -> 67.21 ms, KV cache 1.01 -> 0.36 GB (VLA)"},
        # every workload timed in this run with a roofline figure of its own (details under "workloads")
        "roofline_summary": {k: {"bound": v["roofline"]["bound"], "frac": v["roofline"]["frac"],
                                 "achieved": v["roofline"]["achieved"], "unit": v["roofline"]["unit"]}
                             for k, v in extra.items() if isinstance(v, dict) and "roofline" in v},
        "workloads": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
