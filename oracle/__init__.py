"""CPU oracle for the paged-attention decode + KV swapping path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, float64 statement of
what the path computes.  Only the test-suite, the smoke check and the
benchmark's `cpu_baseline` leg may import it; the product (the HIP library and
its Python binding) never does, and this package imports nothing of the
product.

Pinned by (see tests/test_oracle_*.py):
  attention.paged_attention_decode  - brute-force dense softmax attention on
      tiny inputs, closed forms (ctx = 1, constant V, equal keys, peaked
      softmax, key-shift invariance), GQA == MHA with repeated heads, a library
      cross-check, residency independence.
  pool_model.PoolModel              - conservation invariants, byte-identical
      swap round trips, brute-force dictionary bookkeeping.
  expansion.*                       - the worked example's printed 1.28 (= 9/7),
      the buffered form on the same example, the 800 KB-per-token figure.
  controller_sim.AdaptiveExpansion  - the closed-form fixed point of the
      transparency condition, the worked example's m = 4, start-at-zero,
      shrink-after-slowdown, spike tolerance, plateau.
  layer_fifo.simulate               - the worked example's four-layer trace,
      queue length and residence time, the tight swap constraint, the largest
      number of CPU layers its timing hides.
  layout.element_index              - bijection, vector contents, hand-worked
      positions.
  chunk_book.ChunkBook              - the worked example's 9/7 per layer with two
      of nine layers away, growth visible exactly when the second has left, a
      refused and a granted shrink, conservation under random histories.
  serving_sim.simulate              - a hand-worked three-request stream
      (tests/test_serving_host.py); closed forms (equal requests run in waves,
      a one-request budget serialises the stream, idle gaps are skipped) and
      invariants recomputed from the trace under random streams
      (tests/test_oracle_serving_sim.py).  The scheduling rules themselves are
      this build's reading of an engine the paper inherits.
Absolute throughput numbers: parity unpinned (the paper prints none for this path).
"""
