"""CPU checks of the byte/flop accounting that bench.py reports: the formulas of the scope table
evaluated on the benchmark configurations, and the K-cache bytes per token the layout predicts."""
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench
import workloads
from oracle import layout
from oracle.lazy_stack import LazyStackOracle


def k_bytes_per_token_after_prefill(w):
    """Resident K bytes / tokens, from row counts only: sum_b sum_l (L_b - lazy[l]*Vn_b) * H * D * e."""
    rows = sum(L - lz * v for L, v in zip(w.seq_len, w.vis_len) for lz in w.lazy_mask)
    return rows * w.n_heads * w.head_dim * w.elem_bytes / sum(w.seq_len)


def test_k_cache_bytes_per_token_predictions():
    want = {0: 851968 / 176, 1: 122060.8, 3: 113119.319, 4: 176774.737}
    for i, val in want.items():
        got = k_bytes_per_token_after_prefill(workloads.config(i))
        assert abs(got - val) < 1e-2, (i, got)
    w = workloads.config(1)
    assert w.n_layers * w.n_heads * w.head_dim * w.elem_bytes == 262144


def test_row_count_formula_matches_oracle_state():
    w = workloads.custom("acc", 5, 2, 4, "bf16", [3, 0], [6, 4], [15, 9], 0, [0, 1, 1, 0, 1])
    stacks = [LazyStackOracle(w.n_layers, w.n_heads, w.head_dim, w.lazy_mask, w.vis_start[b], w.vis_len[b])
              for b in range(w.batch)]
    for b, st in enumerate(stacks):
        z = np.zeros((w.seq_len[b], w.n_heads, w.head_dim))
        for l in range(w.n_layers):
            st.prefill(l, z, z, z, rows=[0])
    lay = layout.ArenaLayout(w.n_layers, w.n_heads, w.head_dim, w.dtype, w.batch, w.max_seq, w.max_vis,
                             w.max_text, w.lazy_mask)
    res = layout.resident_bytes(lay, stacks)
    assert res["k_bytes"] / res["tokens"] == k_bytes_per_token_after_prefill(w)


def test_prefill_flops_and_decode_bytes_of_the_benchmark_shapes():
    assert bench.prefill_flops_per_layer(workloads.config(1)) == 32 * 4 * 128 * 640 * 641 // 2        # 3.36 GFLOP
    assert round(bench.prefill_flops_per_layer(workloads.config(3)) / 1e9, 1) == 593.2
    w5 = workloads.config(4)
    assert bench.prefill_flops_per_layer(w5) == sum(40 * 512 * L * (L + 1) // 2 for L in w5.seq_len)
    w = workloads.config(1)
    assert bench.decode_bytes_per_layer(w, 0) == (2 * 641 + 6) * 32 * 128 * 2                         # 10.6 MB
    # a lazy layer reads as many bytes as an ordinary one (its visual keys come from another buffer)
    assert bench.decode_bytes_per_layer(workloads.config(2), 5) == sum(
        (2 * (L + 6) + 6) * 32 * 128 * 2 for L in workloads.config(2).seq_len)


def test_max_batch_figures_of_the_paper_follow_from_the_cache_layout():
    """The paper reports a KV-cache saving of 35 % and a maximum batch growing from 21 to 32 at fixed memory.
    With N = 32 the saving n/(2N) closest to 35 % is n = 22 lazy layers; a K/V arena sized for exactly 21
    sequences without lazy layers then holds exactly 32 sequences under Global Lazy Attention
    (21 * 64 / 42 = 32): the layout's byte counts reproduce the printed pair."""
    N_, pct, b0, b1 = [int(x) for x in open(os.path.join(ROOT, "tests", "golden", "max_batch_fig5.txt")).read().split("\n")[-2].split()]
    n = min(range(N_), key=lambda k: abs(k / (2 * N_) - pct / 100))
    assert n == 22
    H, D, L = 32, 128, 2048
    mask = [0] * (N_ - n) + [1] * n
    mask = [0] + mask[1:] if mask[0] else mask          # layer 0 stays ordinary
    per_seq = lambda m, mode: (layout.ArenaLayout(N_, H, D, "bf16", 1, L, L, L, m, mode=mode).rows_bytes())
    budget = b0 * per_seq([0] * N_, "vla")
    assert budget // per_seq(mask, "gla") == b1
    assert (b0 + 1) * per_seq([0] * N_, "vla") > budget   # 22 plain sequences do not fit
    assert layout.gla_kv_saving_closed_form(N_, n) == pytest.approx(pct / 100, abs=0.01)


def test_bench_refuses_more_than_one_gpu_and_needs_no_gpu_to_say_so():
    """bench.py --gpus N with N > 1 exits with a message: nothing in this path uses a second GPU."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
    assert res.stdout.strip() == ""
