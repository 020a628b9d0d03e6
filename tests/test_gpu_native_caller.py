"""The library driven by a program that uses nothing but the HIP runtime and include/qcache.h
(tests/c_abi_gpu_probe.cpp, built by the package's build step): no Python and no tensor library on the
product side.  The test regenerates the program's inputs with the shared counter-based generator, runs the
oracle and compares every layer call's output and the byte accounting."""
import os
import subprocess

import numpy as np
import pytest

from oracle.lazy_stack import LazyStackOracle
from workloads.counter_inputs import counter_values
from stack_runner import TOL

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
N, H, D, B, STEPS = 3, 2, 128, 2, 2
MASK = [0, 1, 0]
LENS, VIS_START, VIS_LEN = [150, 70], [20, 0], [100, 33]


def bf16_file_to_f64(raw):
    bits = np.frombuffer(raw, dtype=np.uint16).astype(np.uint32) << 16
    return bits.view(np.float32).astype(np.float64)


def test_program_without_python_matches_oracle(tmp_path):
    exe = os.path.join(HERE, "c_abi_gpu_probe")
    if not os.path.exists(exe):
        pytest.fail("tests/c_abi_gpu_probe is missing: build it with __graft_entry__.build()")
    out_path = str(tmp_path / "outputs.bf16")
    res = subprocess.run([exe, out_path], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    stats = dict((k, int(v)) for k, v in (line.split() for line in res.stdout.strip().splitlines()))
    got = bf16_file_to_f64(open(out_path, "rb").read())
    tokens = sum(LENS)
    assert got.size == N * tokens * H * D + STEPS * N * B * H * D

    stacks = [LazyStackOracle(N, H, D, MASK, VIS_START[b], VIS_LEN[b]) for b in range(B)]
    cu = [0, LENS[0], tokens]
    worst, at = 0.0, 0
    for l in range(N):
        q, k, v = (counter_values(3 * l + j, tokens * H * D).reshape(tokens, H, D) for j in range(3))
        ref = np.concatenate([stacks[b].prefill(l, q[cu[b]:cu[b + 1]], k[cu[b]:cu[b + 1]], v[cu[b]:cu[b + 1]])
                              for b in range(B)], axis=0)
        out = got[at:at + ref.size].reshape(ref.shape)
        at += ref.size
        worst = max(worst, float(np.max(np.abs(out - ref))))
    for t in range(STEPS):
        for l in range(N):
            tag = 100 + 3 * (t * N + l)
            q, k, v = (counter_values(tag + j, B * H * D).reshape(B, H, D) for j in range(3))
            ref = np.stack([stacks[b].decode(l, q[b], k[b], v[b]) for b in range(B)])
            out = got[at:at + ref.size].reshape(ref.shape)
            at += ref.size
            worst = max(worst, float(np.max(np.abs(out - ref))))
    print("program without Python: worst abs err %.3g" % worst, flush=True)
    assert np.isfinite(worst) and worst <= TOL["bf16"]
    row = H * D * 2
    final = [n + STEPS for n in LENS]
    assert stats["tokens"] == sum(final)
    assert stats["v_bytes"] == N * sum(final) * row
    assert stats["k_bytes"] == sum((n - lz * vl) * row for n, vl in zip(final, VIS_LEN) for lz in MASK)
    assert stats["q_bytes"] == sum(VIS_LEN) * row
