"""CPU oracle for the ReaLB hot path (one EP rank's precision-adaptive MoE layer).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain NumPy/FP64 statement
of what the path computes, written from the paper before any GPU code.  It is
imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline
leg, and by nothing else: the product (paper_2604_19503_amd) never routes
through it and shares no code, table or helper with it.

Modules (each function cites the passage of the paper it follows):
  bf16     bfloat16 bit patterns <-> float64, nearest-even rounding
  router   top-k gating + renormalised gate weights; per-expert / per-rank counts
  policy   LB gate, hotspot set, vision-ratio test, AIMD threshold update
  mxfp4    BF16 -> MXFP4 (E2M1 codes + one E8M0 scale per 32) and back
  permute  canonical group-by-expert permutation of the rank's assignments
  ffn      SwiGLU expert FFN (BF16 and FP4 operand variants), weighted combine
  layer    the steps above chained for one rank

Parity pins (tests/test_oracle_*.py, all CPU): every function above is pinned
to something other than itself -- exhaustive exact-rational FP4 rounding,
closed forms of the AIMD recurrence, conservation invariants, brute-force loops
on tiny inputs, reductions to library routines (scipy softmax, dense matmul).
No function here is "parity unpinned".
"""
