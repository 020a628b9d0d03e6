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
            accounting ("Efficiency Analysis", KV Cache paragraph); per-sequence
            capacities, separately sized layers behind a pruning boundary, and
            the maximum-batch search ("Efficiency Evaluation" paragraph).
global_lazy_stack  the same state machine for Global Lazy Attention (Eq. 5, Eq. 6).
selection   layer-wise attention similarity and lazy-block grouping (Eq. 3, Eq. 4).
projection  query/key projection of the text rows with rotary embedding (Eq. 7)
            and the projector-FLOP saving ("Efficiency Analysis", FLOPs).
pruning     token pruning between two layers on top of Lazy Attention
            ("Compatibility" paragraph): survivor ranking and the pruned stack.
"""
