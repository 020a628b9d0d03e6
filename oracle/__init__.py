"""CPU oracle for Lazy Attention with the layer-shared Q Cache (test infrastructure).

This package is a slow, plain fp64 restatement of what the paper's attention
path computes.  It exists only so that tests, the smoke check and the
benchmark's cpu_baseline leg can compare the HIP library against it.  The
product package never imports it, and it never imports the product package.

Modules
-------
attention   softmax attention exactly as Eq. 1 (prefill, causal) and Eq. 2
            (decode) define it, plus an independent scalar brute force.
lazy_stack  the per-layer state machine of Visual Lazy Attention: Q Cache,
            text/visual K partitions, V cache (Eq. 7, Eq. 8, the Q Cache
            definition in the "Lazy Attention" subsection, and the KV-cache
            paragraph of "Efficiency Analysis").
layout      byte layout of the caches in device memory and the resident-byte
            accounting ("Efficiency Analysis", KV Cache paragraph).
"""
