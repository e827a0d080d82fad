"""Pins of the NVFP4-faithful encoder variant of the oracle (paper Appendix "Implementation Details",
Quantization Details) against things other than itself: the format's value table, torch's own FP8
conversion, exact-rational nearest search, the already pinned MXFP4 encoder on inputs where the two
formats coincide, the error bound of the definition, and a float64 re-derivation away from rounding
boundaries."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import nvfp4, mxfp4, bf16

GOLD = os.path.join(os.path.dirname(__file__), "golden", "e4m3_values.txt")


def _bf16_bits(a):
    import workloads as W
    return W.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_e4m3_table_matches_the_format_fixture_and_torch():
    vals = nvfp4.e4m3_values()
    assert vals.shape == (127,) and np.all(np.diff(vals) > 0) and vals[-1] == 448.0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        b, v = line.split()
        assert vals[int(b, 16)] == float(v)
    t = torch.arange(127, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    assert np.array_equal(t.astype(np.float64), vals)


def test_e4m3_rounding_is_nearest_even_by_exact_search():
    vals = [Fraction(float(v)) for v in nvfp4.e4m3_values()]
    rng = np.random.default_rng(5)
    r = np.concatenate([rng.uniform(0, 500, 4000), rng.uniform(0, 0.05, 2000), rng.uniform(0, 2, 2000)]).astype(np.float32)
    mids = np.array([(float(a) + float(b)) / 2 for a, b in zip(vals[:-1], vals[1:])], dtype=np.float32)
    r = np.concatenate([r, mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9)),
                        np.array([0, 448, 464, 465, 1e6, 2.0 ** -10, 2.0 ** -11], dtype=np.float32)])
    got = nvfp4.e4m3_round(r)
    for x, b in zip(r, got):
        fx = Fraction(float(x))
        d = [abs(fx - v) for v in vals]
        m = min(d)
        cands = [i for i, di in enumerate(d) if di == m]
        want = cands[0] if len(cands) == 1 else [i for i in cands if i % 2 == 0][0]
        assert int(b) == want, (float(x), int(b), want)


def test_e4m3_rounding_agrees_with_torch_inside_the_range():
    rng = np.random.default_rng(6)
    r = rng.uniform(0, 448, 20000).astype(np.float32)
    t = torch.from_numpy(r).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(nvfp4.e4m3_round(r), t)


def test_e2m1_f32_rounding_matches_the_tie_fixture():
    ties = os.path.join(os.path.dirname(__file__), "golden", "e2m1_ties.txt")
    for line in open(ties):
        if line.startswith("#") or not line.strip():
            continue
        s, want = map(float, line.split())
        c = nvfp4.e2m1_round_mag_f32(np.array([s], dtype=np.float32))[0]
        assert nvfp4.E2M1_VALUES[c] == want
    x = np.linspace(0, 8, 4001).astype(np.float32)
    assert np.array_equal(nvfp4.e2m1_round_mag_f32(x), mxfp4.e2m1_round_mag(x.astype(np.float64)))


def test_coincides_with_mxfp4_where_both_scales_are_the_same_power_of_two():
    """Groups whose maximum is 6 * 2^m and a power-of-two global scale: amax/6 = 2^m is an exact E4M3
    value, the MX block scale is floor(log2 amax) - 2 = m, so both encoders divide by 2^m."""
    rng = np.random.default_rng(7)
    for m, gexp in ((0, -3), (-4, -6), (3, 0), (-7, -9)):
        x = rng.uniform(-6, 6, (64, 32)) * 2.0 ** m
        x[:, 0] = 6.0 * 2.0 ** m
        x[:, 16] = -6.0 * 2.0 ** m
        bits = _bf16_bits(x)
        x_r = bf16.bits_to_f64(bits)
        assert np.all(np.abs(x_r).reshape(64, 2, 16).max(-1) == 6.0 * 2.0 ** m)
        cn, sn = nvfp4.quantize(bits, np.float32(2.0 ** gexp))
        cm, sm = mxfp4.quantize(bits)
        assert np.array_equal(cn, cm)
        assert np.all(nvfp4.e4m3_values()[sn] * 2.0 ** gexp == 2.0 ** m) and np.all(sm.astype(int) - 127 == m)
        assert np.array_equal(nvfp4.dequantize(cn, sn, 2.0 ** gexp), mxfp4.dequantize(cm, sm))


def test_error_bound_sign_zero_groups_and_packing():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((200, 64)) * rng.choice([1e-3, 0.02, 1.0, 30.0], size=(200, 1))
    x[3, :16] = 0.0
    x[4, 16:32] = -0.0
    bits = _bf16_bits(x)
    v = bf16.bits_to_f64(bits)
    g = nvfp4.global_scale(bits)
    assert g == np.float32(np.float32(np.abs(v).max()) / np.float32(6 * 448))
    codes, sc = nvfp4.quantize(bits, g)
    assert codes.shape == bits.shape and sc.shape == (200, 4)
    assert sc[3, 0] == 0 and np.all(codes[3, :16] == 0) and np.all(codes[4, 16:32] == 8)    # sign bit kept on zeros
    assert np.array_equal(codes >> 3, (bits >> 15).astype(np.uint8))
    d = nvfp4.dequantize(codes, sc, g)
    s_eff = (nvfp4.e4m3_values()[sc].astype(np.float32) * g).astype(np.float64)
    q = np.abs(v).reshape(200, 4, 16) / np.where(s_eff == 0, 1, s_eff)[..., None]
    step = np.where(q < 2, 0.5, np.where(q < 4, 1.0, 2.0))
    bound = np.maximum(step / 2, q - 6.0) * s_eff[..., None] * (1 + 1e-6)
    err = np.abs(v - d).reshape(200, 4, 16)
    assert np.all(err[s_eff > 0] <= bound[s_eff > 0])
    assert np.all(q.max(-1)[sc >= 8] <= 6.0 * (1 + 1 / 16) + 1e-3)            # a normal E4M3 scale is rounded down by at most 1/17
    assert np.any(sc < 8) and np.any(sc >= 8)                                # the subnormal scale range is exercised too
    assert np.array_equal(nvfp4.unpack(nvfp4.pack(codes)), codes)


def test_float64_rederivation_away_from_rounding_boundaries():
    """The same definition evaluated in float64 with a literal nearest search must give the same
    bytes and codes wherever the float64 quantities are not within 1e-5 (relative) of a boundary."""
    rng = np.random.default_rng(9)
    bits = _bf16_bits(rng.standard_normal((300, 32)) * 0.7)
    v = bf16.bits_to_f64(bits)
    g = float(nvfp4.global_scale(bits))
    codes, sc = nvfp4.quantize(bits, g)
    vals = nvfp4.e4m3_values()
    e2 = nvfp4.E2M1_VALUES
    checked = 0
    for i in range(300):
        for grp in range(2):
            blk = np.abs(v[i, grp * 16:(grp + 1) * 16])
            r = blk.max() / 6.0 / g
            d = np.abs(vals - r)
            order = np.argsort(d)
            if d[order[1]] - d[order[0]] < 1e-5 * r:
                continue
            assert sc[i, grp] == order[0]
            s_eff = vals[order[0]] * g
            for j, xj in enumerate(blk):
                qq = xj / s_eff
                dd = np.abs(e2 - min(qq, 6.0))
                oo = np.argsort(dd)
                if dd[oo[1]] - dd[oo[0]] < 1e-5 * max(qq, 1e-9):
                    continue
                assert (codes[i, grp * 16 + j] & 7) == oo[0]
                checked += 1
    assert checked > 8000
