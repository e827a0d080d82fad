"""On-the-fly precision transformation BF16 -> FP4 (paper Sec. "Overhead-Aware
Pipeline Orchestration", paragraph "Overlapping Pipeline"; format in Appendix
"Implementation Details", paragraph "Quantization Details").

The paper's format is NVFP4: E2M1 elements (largest magnitude 6.0), groups of
16, an FP8-E4M3 scale per group derived from the group's absolute maximum
divided by 6.0, times a calibrated global scale; each value divided by the scale
and mapped to the nearest FP4 value.  (The sentence that defines the dynamic
range is cut off in the paper; it is read as the group's max |x|.)

This build runs on the block-scaled FP4 matrix instructions of gfx950, whose
native scale type is E8M0, so the encoding is OCP Microscaling MXFP4:

  paper (NVFP4)                         here (MXFP4)
  ----------------------------------    ------------------------------------
  E2M1 element, max 6.0                 same: magnitudes 0,.5,1,1.5,2,3,4,6
  group of 16                           block of 32 along the contraction dim
  E4M3 scale = amax/6 * global          E8M0 scale 2^se, se = floor(log2 amax)-2
  calibrated FP32 global scale          none
  amax maps to 6.0                      amax lands in [4,8)*2^se; (6,8) saturates
  nearest FP4 value                     nearest, ties to the even code, saturating

Readings where neither text decides:
  * an all-zero block gets scale byte 127 (2^0);
  * se is clamped to [-127, 127] (byte 0..254; 255 is NaN in E8M0, never made);
  * the sign bit of the input is kept even when the magnitude rounds to zero;
  * non-finite inputs are outside the contract (asserted);
  * packing: element 2i in the low nibble, 2i+1 in the high nibble of byte i.
"""
import numpy as np
from .bf16 import bits_to_f64

BLOCK = 32
E2M1_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def e2m1_round_mag(s: np.ndarray) -> np.ndarray:
    """Magnitude code 0..7 of the E2M1 value nearest to s >= 0; a value exactly
    half-way between two neighbours goes to the even code; above 6 saturates.
    Written as the eight intervals, so it can be read against the value table:
      code 0: s <= .25        code 1: .25 < s < .75     code 2: .75 <= s <= 1.25
      code 3: 1.25 < s < 1.75 code 4: 1.75 <= s <= 2.5  code 5: 2.5 < s < 3.5
      code 6: 3.5 <= s <= 5   code 7: s > 5"""
    s = np.asarray(s, dtype=np.float64)
    c = np.zeros(s.shape, dtype=np.uint8)
    c[(s > 0.25) & (s < 0.75)] = 1
    c[(s >= 0.75) & (s <= 1.25)] = 2
    c[(s > 1.25) & (s < 1.75)] = 3
    c[(s >= 1.75) & (s <= 2.5)] = 4
    c[(s > 2.5) & (s < 3.5)] = 5
    c[(s >= 3.5) & (s <= 5.0)] = 6
    c[s > 5.0] = 7
    return c


def block_scale_exponent(amax: np.ndarray) -> np.ndarray:
    """se per block: 0 for an all-zero block, else clamp(floor(log2 amax) - 2, -127, 127)."""
    amax = np.asarray(amax, dtype=np.float64)
    _, ex = np.frexp(amax)                     # amax = m*2^ex, m in [0.5,1)  =>  floor(log2) = ex-1
    se = np.clip(ex.astype(np.int64) - 1 - 2, -127, 127)
    return np.where(amax == 0, 0, se)


def quantize(bits: np.ndarray):
    """bf16 patterns [..., K] (K % 32 == 0) -> (codes uint8 [..., K] one 4-bit code
    per element: bit 3 sign, bits 2..0 magnitude code; scales uint8 [..., K/32])."""
    bits = np.asarray(bits, dtype=np.uint16)
    K = bits.shape[-1]
    assert K % BLOCK == 0
    v = bits_to_f64(bits)
    assert np.isfinite(v).all()
    vb = v.reshape(bits.shape[:-1] + (K // BLOCK, BLOCK))
    amax = np.abs(vb).max(axis=-1)
    se = block_scale_exponent(amax)
    scaled = np.abs(vb) / np.ldexp(1.0, se)[..., None]          # exact: power-of-two divisor
    mag = e2m1_round_mag(scaled)
    sign = ((bits >> np.uint16(15)) & np.uint16(1)).astype(np.uint8).reshape(vb.shape)
    codes = (sign << np.uint8(3)) | mag
    return codes.reshape(bits.shape), (se + 127).astype(np.uint8)


def pack(codes: np.ndarray) -> np.ndarray:
    """[..., K] 4-bit codes -> [..., K/2] bytes, even element in the low nibble."""
    c = np.asarray(codes, dtype=np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << np.uint8(4))).astype(np.uint8)


def unpack(packed: np.ndarray) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = p & np.uint8(0xF)
    out[..., 1::2] = p >> np.uint8(4)
    return out


def dequantize(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """float64 values: (-1)^sign * E2M1_VALUES[mag] * 2^(scale byte - 127)."""
    codes = np.asarray(codes, dtype=np.uint8)
    K = codes.shape[-1]
    mag = E2M1_VALUES[codes & np.uint8(7)]
    sgn = np.where((codes >> np.uint8(3)) & np.uint8(1), -1.0, 1.0)
    sc = np.ldexp(1.0, np.asarray(scales).astype(np.int64) - 127)
    val = (sgn * mag).reshape(codes.shape[:-1] + (K // BLOCK, BLOCK)) * sc[..., None]
    return val.reshape(codes.shape)


def quantize_packed(bits: np.ndarray):
    codes, scales = quantize(bits)
    return pack(codes), scales
