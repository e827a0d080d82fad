"""NVFP4-faithful variant of the BF16 -> FP4 encoder (paper Appendix "Implementation
Details", paragraph "Quantization Details"): E2M1 elements, groups of 16, an FP8
E4M3 scale per group derived from the group's absolute maximum divided by 6.0 and
a global (per-tensor) scale, the scale rounded into FP8 and clamped to its range,
each value divided by the scale and mapped to the nearest FP4 value.

It exists beside oracle/mxfp4.py only to measure what the mapping onto MXFP4 costs
in accuracy; no GEMM consumes it (gfx950's block-scaled matrix instructions take
power-of-two scales).

Where floating point decides an integer, the decision is DEFINED to be taken in IEEE
binary32 (the paper fixes no precision for it; binary32 is what a runtime encoder of
BF16 data would naturally use), each step rounded once, in this order:

    amax    = max |x| over the group            (exact: a BF16 value)
    s_local = fl32(amax / 6)
    r       = fl32(s_local / g)                 g = the tensor's global scale (> 0, FP32)
    byte    = E4M3 value nearest to r, ties to the even mantissa, clamped to 448
    s_eff   = fl32(E4M3(byte) * g)
    q_i     = fl32(|x_i| / s_eff)               (s_eff == 0: magnitude code 0)
    code_i  = sign bit of x_i | E2M1 value nearest to q_i, ties to the even code, saturating at 6

Readings where the paper is silent or cut off:
  * the sentence defining the dynamic range is cut off; read as max |x| of the group;
  * the global scale is the tensor's max |x| divided by (6 * 448), so that the largest
    group scale lands on the top of the E4M3 range (the paper takes it from offline
    calibration, which needs its models and data); an all-zero tensor uses g = 1;
  * E4M3 is the OCP FP8 E4M3 format (bias 7, subnormals, largest finite value 448, no
    infinities); scales are non-negative, a group whose r rounds to 0 gets byte 0 and
    all-zero magnitudes;
  * sign of a value that rounds to zero, packing and non-finite inputs: as in mxfp4.py.
"""
import numpy as np
from .bf16 import bits_to_f64
from .mxfp4 import E2M1_VALUES, pack, unpack  # noqa: F401  (same element format and packing)

GROUP = 16
E4M3_MAX = 448.0


def e4m3_values() -> np.ndarray:
    """The 127 non-negative finite E4M3 values, index = byte 0x00..0x7E:
    exponent field e = byte >> 3, mantissa m = byte & 7;
    e == 0: m * 2^-9 (subnormal);  else (1 + m/8) * 2^(e - 7)."""
    b = np.arange(0x7F)
    e, m = b >> 3, b & 7
    return np.where(e == 0, m * 2.0 ** -9, (1 + m / 8.0) * np.ldexp(1.0, e - 7))


def e4m3_round(r: np.ndarray) -> np.ndarray:
    """Byte of the E4M3 value nearest to r >= 0 (float32), ties to the even byte, clamped to 448."""
    r = np.asarray(r, dtype=np.float32).astype(np.float64)
    vals = e4m3_values()
    mids = (vals[:-1] + vals[1:]) / 2                     # exactly representable
    lo = np.searchsorted(mids, r, side="left")            # number of midpoints strictly below r
    hi = np.searchsorted(mids, r, side="right")           # number of midpoints <= r
    byte = np.where(lo == hi, lo, np.where(lo % 2 == 0, lo, hi))   # on a midpoint: lo and lo+1 are the neighbours
    return np.minimum(byte, 0x7E).astype(np.uint8)


def e2m1_round_mag_f32(q: np.ndarray) -> np.ndarray:
    """Magnitude code 0..7 of the E2M1 value nearest to q >= 0 (float32); half-way points go to
    the even code; above 6 saturates (same intervals as mxfp4.e2m1_round_mag)."""
    q = np.asarray(q, dtype=np.float32)
    c = np.zeros(q.shape, dtype=np.uint8)
    for thr, strict in ((0.25, True), (0.75, False), (1.25, True), (1.75, False), (2.5, True), (3.5, False), (5.0, True)):
        c += ((q > np.float32(thr)) if strict else (q >= np.float32(thr))).astype(np.uint8)
    return c


def global_scale(bits: np.ndarray) -> np.float32:
    """g = fl32(max |x| of the tensor / (6 * 448)); 1 for an all-zero tensor."""
    amax = np.float32(np.abs(bits_to_f64(np.asarray(bits, dtype=np.uint16))).max())
    return np.float32(1.0) if amax == 0 else np.float32(amax / np.float32(6.0 * 448.0))


def quantize(bits: np.ndarray, g):
    """bf16 patterns [..., K] (K % 16 == 0), global scale g -> (codes uint8 [..., K] one 4-bit
    code per element, scales uint8 [..., K/16] E4M3 bytes)."""
    bits = np.asarray(bits, dtype=np.uint16)
    K = bits.shape[-1]
    assert K % GROUP == 0
    g = np.float32(g)
    assert g > 0
    v = bits_to_f64(bits)
    assert np.isfinite(v).all()
    vb = np.abs(v).astype(np.float32).reshape(bits.shape[:-1] + (K // GROUP, GROUP))    # BF16 values are exact in FP32
    amax = vb.max(axis=-1)
    s_local = (amax / np.float32(6.0)).astype(np.float32)
    with np.errstate(over="ignore"):                       # an overflowing quotient is +inf: clamps to 448 / saturates to 6
        r = (s_local / g).astype(np.float32)
    byte = e4m3_round(r)
    s_eff = (e4m3_values()[byte].astype(np.float32) * g).astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        q = (vb / s_eff[..., None]).astype(np.float32)
    mag = np.where(s_eff[..., None] == 0, np.uint8(0), e2m1_round_mag_f32(np.where(s_eff[..., None] == 0, 0, q)))
    sign = ((bits >> np.uint16(15)) & np.uint16(1)).astype(np.uint8).reshape(vb.shape)
    codes = (sign << np.uint8(3)) | mag.astype(np.uint8)
    return codes.reshape(bits.shape), byte


def dequantize(codes: np.ndarray, scales: np.ndarray, g) -> np.ndarray:
    """float64 values: (-1)^sign * E2M1 value * (E4M3 value * g), the scale product rounded to FP32 as
    the encoder used it."""
    codes = np.asarray(codes, dtype=np.uint8)
    K = codes.shape[-1]
    mag = E2M1_VALUES[codes & np.uint8(7)]
    sgn = np.where((codes >> np.uint8(3)) & np.uint8(1), -1.0, 1.0)
    s_eff = (e4m3_values()[np.asarray(scales)].astype(np.float32) * np.float32(g)).astype(np.float32).astype(np.float64)
    val = (sgn * mag).reshape(codes.shape[:-1] + (K // GROUP, GROUP)) * s_eff[..., None]
    return val.reshape(codes.shape)
