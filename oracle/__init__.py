"""CPU oracle for the speculative-decoding hot path (TEST INFRASTRUCTURE ONLY).

This package is the slow, plain, obviously-correct reference that the HIP
library is checked against.  It is test infrastructure: only the test-suite,
the smoke check and the benchmark's CPU-baseline leg may import it.  The
product (the HIP kernels, the C-ABI library and its Python binding) never
imports, links or calls anything in here, and nothing in here imports the
product.

Arithmetic is numpy float64 unless a function says otherwise (the decisions
of the speculative sampler are taken in float32 / integers because those are
what the method's accept test and sampler are defined on; see
``spec_sampling``).

Modules
-------
decoder        LLaMA-style decoder forward with a KV cache (target and draft).
spec_sampling  softmax, accept test, residual distribution, fixed-point
               inverse-CDF sampler, one speculative block, whole generation
               loops (speculative and plain autoregressive).
metrics        block efficiency and memory-bound speed-up.
"""
