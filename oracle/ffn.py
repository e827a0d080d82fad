"""Balanced MoE execution for one rank (paper Sec. "System Overview", stage 4:
each rank runs its experts' GEMMs in the planned precision, W16A16 or W4A4)
and the local part of the result combination (Sec. "MoE Load Balancing
Systems", Communication: dispatch + result combination).

The paper says only "GEMM"/"MoE computation"; the expert is the SwiGLU FFN of
both evaluated models:  y = W2 . ( silu(Wg x) * (Wu x) ),  silu(g) = g/(1+e^-g).
W13 stacks the gate rows [0, I) and the up rows [I, 2I).

Rounding points (the paper gives none; these are part of the definition used
here): products and sums in float64; the intermediate h is rounded once to
BF16; on the FP4 path that BF16 h is then encoded to MXFP4 along I (W4A4: the
second GEMM's activations are FP4 too) and the operands of both GEMMs are the
*dequantized* FP4 values; each output row is rounded once to BF16; the gate
weight multiplies the expert output at combine time, accumulated in float64
and rounded once to BF16.
"""
import numpy as np
from .bf16 import bits_to_f64, round_f64_to_bf16_value, f64_to_bits
from . import mxfp4


def _silu_mul(g: np.ndarray, u: np.ndarray) -> np.ndarray:
    return g / (1.0 + np.exp(-g)) * u


def _segments(expert_offsets):
    off = [int(v) for v in np.asarray(expert_offsets).reshape(-1)]
    return [(e, off[e], off[e + 1]) for e in range(len(off) - 1) if off[e + 1] > off[e]]


def gate_up(x: np.ndarray, w13: np.ndarray, expert_offsets) -> np.ndarray:
    """h[r, i] = silu(sum_h x[r,h] w13[e, i, h]) * (sum_h x[r,h] w13[e, I+i, h]) for
    the rows r of expert e.  x [R,H], w13 [n,2I,H] float64 -> float64 [R,I]."""
    I = w13.shape[1] // 2
    h = np.zeros((x.shape[0], I))
    for e, lo, hi in _segments(expert_offsets):
        gu = x[lo:hi] @ w13[e].T
        h[lo:hi] = _silu_mul(gu[:, :I], gu[:, I:])
    return h


def down(h: np.ndarray, w2: np.ndarray, expert_offsets) -> np.ndarray:
    """y[r, :] = w2[e] @ h[r, :] for the rows of expert e.  h [R,I], w2 [n,H,I] -> [R,H]."""
    y = np.zeros((h.shape[0], w2.shape[1]))
    for e, lo, hi in _segments(expert_offsets):
        y[lo:hi] = h[lo:hi] @ w2[e].T
    return y


def ffn_bf16(xperm_bits, w13_bits, w2_bits, expert_offsets):
    """W16A16 path.  Returns (h_bits uint16 [R,I], y float64 [R,H] unrounded)."""
    h = gate_up(bits_to_f64(xperm_bits), bits_to_f64(w13_bits), expert_offsets)
    h_bits = f64_to_bits(h)
    y = down(bits_to_f64(h_bits), bits_to_f64(w2_bits), expert_offsets)
    return h_bits, y


def ffn_fp4(xq, xs, w13q, w13s, w2q, w2s, expert_offsets):
    """W4A4 path on unpacked codes + scale bytes.  Returns (hq codes [R,I], hs
    [R,I/32], y float64 [R,H] unrounded)."""
    h = gate_up(mxfp4.dequantize(xq, xs), mxfp4.dequantize(w13q, w13s), expert_offsets)
    hq, hs = mxfp4.quantize(f64_to_bits(h))
    y = down(mxfp4.dequantize(hq, hs), mxfp4.dequantize(w2q, w2s), expert_offsets)
    return hq, hs, y


def down_fp4(hq, hs, w2q, w2s, expert_offsets):
    """Second GEMM alone on given FP4 intermediates (stage-isolated check)."""
    return down(mxfp4.dequantize(hq, hs), mxfp4.dequantize(w2q, w2s), expert_offsets)


def combine(yrows_bits, assign_to_row, topk_w, T: int, k: int) -> np.ndarray:
    """out[t] = sum over the token's assignments that are local (row >= 0) of
    w[t,j] * Yrows[row], float64; tokens with no local expert give exactly 0.
    Yrows are the BF16 rows the FFN stored.  Returns float64 [T,H] (unrounded)."""
    y = bits_to_f64(yrows_bits)
    a2r = np.asarray(assign_to_row, dtype=np.int64).reshape(T, k)
    w = np.asarray(topk_w, dtype=np.float64).reshape(T, k)
    out = np.zeros((T, y.shape[1]))
    for j in range(k):
        ok = a2r[:, j] >= 0
        out[ok] += w[ok, j][:, None] * y[a2r[ok, j]]
    return out


def to_bf16_bits(v: np.ndarray) -> np.ndarray:
    return f64_to_bits(v)


def to_bf16_value(v: np.ndarray) -> np.ndarray:
    return round_f64_to_bf16_value(v)
