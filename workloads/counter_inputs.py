"""Counter-based input generator shared with tests/c_abi_gpu_probe.cpp (which writes it out again in C++):
element i of stream `tag` is a multiple of 1/32 in [-2, 2], exactly representable in bf16.  Input
generation only; none of the method's arithmetic lives here."""
import numpy as np


def counter_values(tag, count):
    """fp64 array of `count` elements of stream `tag`."""
    i = np.arange(count, dtype=np.uint64)
    m = np.uint64(0xFFFFFFFF)
    u = (i * np.uint64(2654435761) + np.uint64(tag) * np.uint64(40503) + np.uint64(12345)) & m
    u ^= u >> np.uint64(15)
    u = (u * np.uint64(2246822519)) & m
    u ^= u >> np.uint64(13)
    return ((u % np.uint64(129)).astype(np.int64) - 64) / 32.0
