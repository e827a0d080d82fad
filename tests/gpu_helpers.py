"""Helpers shared by the GPU parity tests: progress lines, tolerances, and the row-wise and
element-wise comparisons used next to the relative Frobenius norm.

Tolerances (one place):
  * integer / byte / index results: bit-exact;
  * gate weights: 1e-6 relative;
  * BF16 path GEMM / combine outputs: relative Frobenius <= 1e-2;
  * FP4 path, stage-isolated (the oracle's GEMM run on the very operand codes the GPU consumed):
    relative Frobenius <= 2e-3;
  * FP4 path end to end (the oracle's own intermediate h codes instead of the GPU's): <= 4e-3.
    The GPU accumulates h in FP32 and the oracle in FP64, so a few h values land on the other side
    of a BF16 or E2M1 rounding boundary; one flipped code changes that element by a whole code
    step (up to 40 % of its value), which the end-to-end figure carries and the staged figure,
    by construction, does not.  The staged figure is the BF16 rounding of the output and nothing
    else: round-to-nearest of values with 8 significant bits has a relative rms error of about
    2^-7/sqrt(12) x 0.74 = 1.66e-3, which is what every staged comparison measures (1.66-1.69e-3).
    Flips at the allowed rate of 1e-4 of the codes add about 2.7e-3 in quadrature, hence 4e-3;
    measured end to end: 1.67-1.78e-3 (flip rates of 0 to 5e-6).
  * per row (staged FP4 rows, BF16 rows, combined tokens): relative error of the row <= 4e-3
    (ROW_TOL).  The worst case of the output rounding alone is 2^-8 = 3.9e-3 (every element half
    an ulp off at the bottom of its binade); rows of 256 to 2048 elements measure 1.8e-3 to 2.6e-3.
    A wrong 16-column strip of a 2048-wide row would read about 9e-2.
  * element-wise, wherever the two sides consume identical operands (staged FP4, BF16 down and
    combine): |got - want| <= 2^-7 |want| + 2^-7 rms(want row).  The first term is two BF16 output
    roundings (2^-8 each: one on the GPU, one where the comparison value was itself rounded), the
    second covers FP32 accumulation and the rounding of values near zero.
"""
import os
import sys

import numpy as np

FP4_TOL = 2e-3          # stage-isolated
FP4_E2E_TOL = 4e-3      # end to end
BF16_TOL = 1e-2
ROW_TOL = 4e-3          # one row's relative error (output rounding only)
GATE_W_RTOL = 1e-6
MAX_FLIP_FRACTION = 1e-3


def say(tag, msg):
    print(f"[{tag}] {msg}", flush=True)
    sys.stdout.flush()
    out_dir = os.environ.get("REALB_TEST_LOG_DIR", "")     # optional: also append the progress lines to a file there
    if out_dir and os.path.isdir(out_dir):
        with open(os.path.join(out_dir, "parity_metrics.log"), "a") as f:
            f.write(f"[{tag}] {msg}\n")


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def same(a, b):
    """Bit-exact comparison that reports briefly (count and first mismatch) on failure."""
    a, b = np.asarray(a), np.asarray(b)
    if a.shape != b.shape:
        print(f"shape mismatch {a.shape} vs {b.shape}", flush=True)
        return False
    bad = np.nonzero(a.reshape(-1) != b.reshape(-1))[0]
    if bad.size:
        i = int(bad[0])
        print(f"{bad.size} of {a.size} elements differ; first at flat index {i}: got {a.reshape(-1)[i]} want {b.reshape(-1)[i]}", flush=True)
        return False
    return True


def row_report(got, want):
    """(worst per-row relative error, number of elements outside the element-wise bound, worst
    excess over the bound in units of the bound) for two [rows, cols] float64 arrays."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0, 0, 0.0
    diff = np.abs(got - want)
    rms = np.sqrt(np.mean(want * want, axis=1, keepdims=True))
    bound = 2.0 ** -7 * np.abs(want) + 2.0 ** -7 * rms
    den = np.linalg.norm(want, axis=1)
    num = np.linalg.norm(got - want, axis=1)
    per_row = np.where(den > 0, num / np.where(den > 0, den, 1.0), num)
    bad = diff > bound
    worst = float((diff / np.where(bound > 0, bound, 1.0)).max()) if bound.size else 0.0
    return float(per_row.max()), int(bad.sum()), worst
