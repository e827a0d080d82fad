"""bfloat16 helpers for the oracle.  BF16 tensors are numpy uint16 bit patterns.

The paper fixes BF16 as the standard precision of weights and activations
(Sec. "Setup": W16A16 baseline); where the path rounds an intermediate to BF16
the rounding is IEEE nearest, ties to even.
"""
import numpy as np


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of each bf16 pattern as float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def round_f64_to_bf16_value(v: np.ndarray) -> np.ndarray:
    """Round float64 to the nearest bf16-representable value (ties to even),
    in one rounding step (no detour through float32).  Returns float64.

    bf16 has 8 significand bits: a value with binary exponent e (|v| in
    [2^e, 2^(e+1))) is a multiple of 2^(e-7); below 2^-126 the spacing stays
    2^-133 (subnormals)."""
    v = np.asarray(v, dtype=np.float64)
    _, ex = np.frexp(v)                      # |v| = m * 2^ex, m in [0.5, 1)
    e = np.maximum(ex - 1, -126)
    q = np.ldexp(1.0, e - 7)                 # spacing of bf16 at this magnitude
    r = np.rint(v / q) * q                   # rint = nearest, ties to even; v/q is exact
    r = np.where(np.abs(r) >= 2.0 ** 128, np.copysign(np.inf, v), r)
    return np.where(v == 0, v, r)


def f64_to_bits(v: np.ndarray) -> np.ndarray:
    """Nearest-even bf16 bit pattern of each float64 (finite inputs)."""
    r = round_f64_to_bf16_value(v).astype(np.float32)    # exact: r is bf16-representable
    return (r.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
