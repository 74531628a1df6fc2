"""CPU checker for the decode-time MoE block of AdapMoE (arXiv 2408.10284).

TEST INFRASTRUCTURE, NOT PRODUCT.  Plain, slow, float64 NumPy written from the
paper's definitions so that it can be checked against the paper by eye.  It
shares no code with the HIP library, imports nothing from it, and nothing in
the product path may import it: only the test-suite, the smoke check and the
benchmark's CPU-baseline leg call into this package.

Modules (each function cites the passage it follows):
  gate     - router, softmax, top-2, adaptive test (Eq.1, Eq.3-4, Eq.8), predictor (Sec.4.3)
  expert   - SwiGLU expert, weighted combine (Eq.2-4), int4 storage decode
  cache    - per-layer LRU expert cache with demand + prefetch policy (Sec.4.4, Alg.1)
  planner  - on-demand-load cost model and knapsack DP (Eq.10-19)
  stack    - multi-layer residual stack used by the multi-layer workloads (not in the paper)

Pin status: every function here is pinned by tests that do not re-use it
(hand-worked values under tests/golden/, closed forms, brute force on tiny
inputs, exhaustive enumeration, a textbook LRU reference string).  The one
exception is `stack.run_stack`, whose residual/normalisation wiring is this
build's own choice and not defined by the paper: parity unpinned for the
wiring itself (its parts are pinned).
"""
