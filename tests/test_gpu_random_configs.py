"""Seeded random small configurations through every path of the library against the oracle:
Visual and Global Lazy Attention, fp32 and bf16, head_dim 64 and 128, batches on both sides of the
inline-metadata limit, empty spans, spans at either end of the prompt, optional pruning boundary,
decode by ordinary calls or by graph replays.  Outputs within the usual bars; arenas and accounting
exact."""
import numpy as np
import pytest
import torch

import paper_2602_01901_amd as P
import workloads
from stack_runner import TOL, run_full_parity
from test_gpu_graph import check_caches, prefill_both, run_steps, step_buffers
from test_gpu_pruning import run_pruned_parity
from stack_runner import new_oracles

pytestmark = pytest.mark.gpu


def random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    N = int(rng.integers(2, 7))
    H = int(rng.integers(1, 4))
    D = int(rng.choice([64, 128]))
    dtype = str(rng.choice(["f32", "bf16"]))
    batch = int(rng.choice([1, 2, 3, 9, 10]))
    mask = [0] + [int(rng.random() < 0.5) for _ in range(N - 1)]
    lens, vs, vl = [], [], []
    for _ in range(batch):
        L = int(rng.integers(2, 150))
        kind = rng.integers(0, 5)
        if kind == 0:
            s, v = 0, 0                                  # no visual tokens
        elif kind == 1:
            s, v = 0, int(rng.integers(1, L + 1))        # span at the start (possibly the whole prompt)
        elif kind == 2:
            v = int(rng.integers(1, L + 1))
            s = L - v                                    # span at the end
        else:
            s = int(rng.integers(0, L))
            v = int(rng.integers(0, L - s + 1))
        lens.append(L); vs.append(s); vl.append(v)
    steps = int(rng.integers(1, 5))
    w = workloads.custom("rand%d" % seed, N, H, D, dtype, vs, vl, lens, steps, mask, seed_tag=100 + seed)
    return w, rng


@pytest.mark.parametrize("seed", range(36))
def test_random_configuration(seed):
    w, rng = random_case(seed)
    mode = "gla" if seed % 2 else "vla"
    flavour = seed % 3
    if flavour == 0:                                     # ordinary calls, whole-arena comparison
        s = P.Session.for_workload(w, mode=mode)
        wp, wd = run_full_parity(w, w.decode_steps, s, poison_span=bool(seed % 4 == 0))
        assert max(wp, wd) <= TOL[w.dtype]
        s.close()
    elif flavour == 1:                                   # decode by graph replays mixed with ordinary steps
        s = P.Session.for_workload(w, mode=mode)
        stacks = new_oracles(w, mode=mode)
        prefill_both(w, s, stacks, mode)
        bufs = step_buffers(w, mode)
        g = s.decode_graph(*bufs)
        schedule = "".join(str(rng.choice(["g", "e"])) for _ in range(w.decode_steps))
        run_steps(w, s, stacks, mode, g, bufs, schedule)
        last_g = max([i for i, c in enumerate(schedule) if c == "g"], default=-1)
        check_caches(w, s, stacks, mode)
        s.close()
    else:                                                # pruning boundary before a random ordinary layer
        candidates = [l for l in range(1, w.n_layers) if not w.lazy_mask[l]]
        if not candidates:
            pytest.skip("no ordinary layer after layer 0 in this mask")
        first_late = int(rng.choice(candidates))
        keep = [int(rng.integers(0, v + 1)) for v in w.vis_len]
        keep = [max(k, 1 if L == v else 0) for k, L, v in zip(keep, w.seq_len, w.vis_len)]   # every sequence keeps a token
        assert run_pruned_parity(w, first_late, keep, mode, w.decode_steps, use_graph=bool(seed % 2)) <= TOL[w.dtype]


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration_on_pages(seed):
    """The same population on paged batches (capacities rounded up to whole pages): ordinary calls with the
    arenas and page lists compared, or a pruning boundary with or without graph replays."""
    import dataclasses
    w, rng = random_case(seed)
    up = lambda x: -(-x // 64) * 64
    w = dataclasses.replace(w, max_seq=up(w.max_seq), max_vis=up(w.max_vis), max_text=up(w.max_text))
    mode = "gla" if seed % 2 else "vla"
    if seed % 3 != 2:
        s = P.Session.for_workload(w, mode=mode)
        wp, wd = run_full_parity(w, w.decode_steps, s, poison_span=bool(seed % 4 == 0), paged=True)
        assert max(wp, wd) <= TOL[w.dtype]
        s.close()
    else:
        candidates = [l for l in range(1, w.n_layers) if not w.lazy_mask[l]]
        if not candidates:
            pytest.skip("no ordinary layer after layer 0 in this mask")
        first_late = int(rng.choice(candidates))
        keep = [int(rng.integers(0, v + 1)) for v in w.vis_len]
        keep = [max(k, 1 if L == v else 0) for k, L, v in zip(keep, w.seq_len, w.vis_len)]
        assert run_pruned_parity(w, first_late, keep, mode, w.decode_steps, use_graph=bool(seed % 2), paged=True) <= TOL[w.dtype]
