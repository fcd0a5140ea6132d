"""CPU oracle for latent-KV attention (FDC, arXiv 2408.04107).

TEST INFRASTRUCTURE ONLY. This package is a plain, slow, float64 / integer
reference of what the GPU library computes. It exists so that tests, the smoke
check and the benchmark's CPU-baseline leg can compare the HIP path against
something written independently from the paper. The product path never imports
it, and it imports nothing from the product package.

Modules
  factors    truncated-SVD factors W ~= A.B              (Section 2, low-rank KV paragraph)
  attention  latent projection, query absorption, decode / causal-prefill
             attention on latent K/V, output absorption  (Section 2; Section 5 overview, steps 4-7)
  layout     ragged per-head cache offsets
  planner    decode LPT list scheduling, prefill row-block rescaling and
             last-round redistribution                   (Section 5.3)
  rank_select  per-head compression rate from the singular-value removal rate (Eq. 1)
  rope, gqa    post-RoPE rotation (Sections 3, 5.1) and grouped queries (Section 5.1)
  fp8, fp4     quantised storage of the latent rows: E4M3 and E2M1 codes (a reading of Section 6.2)

Pin status: every function is pinned by the CPU tests (full-rank equals
standard attention, exact-rank equals uncompressed attention, closed forms,
brute force, scheduling invariants and the paper's worked scheduling example).
The KV-chunk splitting of the decode planner, the softmax weight and the
causal-cost mode of the prefill planner extend the paper (it prints no numbers
for them): besides the invariants (coverage, load sums, list-scheduling bounds)
each of their decisions -- the fit rule and its tie, the order of equal-cost
chunks, the cost formulas, the hand-out order -- is pinned by schedules worked
out by hand from the stated reading (tests/test_oracle_planner.py).
"""
