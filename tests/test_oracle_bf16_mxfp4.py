"""Pins for oracle.bf16 and oracle.mxfp4 (CPU only).

Every check compares the oracle with something that is not the oracle: exact
rational arithmetic (fractions.Fraction) with a brute-force nearest search, the
printed value/tie tables under tests/golden/, torch's own float32->bfloat16
conversion, and invariants of the encoding.
"""
from fractions import Fraction
import os

import numpy as np
import pytest
import torch

from oracle import bf16, mxfp4


def _load_table(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(tuple(line.split()))
    return rows


def _frac_of_bf16(p: int) -> Fraction:
    """Exact value of a finite bf16 pattern, from the IEEE field definition."""
    s, e, m = p >> 15, (p >> 7) & 0xFF, p & 0x7F
    assert e != 0xFF
    mag = Fraction(m, 128) * Fraction(2) ** (-126) if e == 0 else (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)
    return -mag if s else mag


def _floor_log2(q: Fraction) -> int:
    e = q.numerator.bit_length() - q.denominator.bit_length()
    if Fraction(2) ** e > q:
        e -= 1
    assert Fraction(2) ** e <= q < Fraction(2) ** (e + 1)
    return e


def _nearest_code(s: Fraction, values) -> int:
    """Brute force: the code whose value is nearest to s; on an exact tie the even code."""
    best = None
    for c, v in enumerate(values):
        d = abs(s - v)
        if best is None or d < best[0] or (d == best[0] and c % 2 == 0 and best[1] % 2 == 1):
            best = (d, c)
    return best[1]


ALL_FINITE = np.array([p for p in range(65536) if ((p >> 7) & 0xFF) != 0xFF], dtype=np.uint16)


# ------------------------------------------------------------------ bf16
def test_bf16_bits_roundtrip_all_patterns():
    v = bf16.bits_to_f64(ALL_FINITE)
    assert np.array_equal(bf16.f64_to_bits(v), ALL_FINITE)


def test_bf16_value_matches_field_definition():
    idx = np.random.default_rng(0).choice(ALL_FINITE.size, 2000, replace=False)
    for p in ALL_FINITE[idx]:
        assert Fraction(float(bf16.bits_to_f64(np.array([p]))[0])) == _frac_of_bf16(int(p))


def test_bf16_rounding_matches_torch_on_float32_inputs():
    rng = np.random.default_rng(1)
    a = (rng.standard_normal(200000) * np.exp(rng.uniform(-30, 30, 200000))).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bf16.f64_to_bits(a.astype(np.float64)), want)


def test_bf16_rounding_ties_and_single_step():
    # exact midpoints between consecutive bf16 values go to the even pattern;
    # a float64 just off the midpoint goes to the nearer side (no double rounding)
    rng = np.random.default_rng(2)
    pats = rng.integers(0x0001, 0x7F00, 3000).astype(np.uint16)
    lo = bf16.bits_to_f64(pats)
    hi = bf16.bits_to_f64(pats + np.uint16(1))
    mid = (lo + hi) / 2
    even = np.where(pats % 2 == 0, pats, pats + 1).astype(np.uint16)
    assert np.array_equal(bf16.f64_to_bits(mid), even)
    assert np.array_equal(bf16.f64_to_bits(np.nextafter(mid, np.inf)), pats + np.uint16(1))
    assert np.array_equal(bf16.f64_to_bits(np.nextafter(mid, -np.inf)), pats)
    assert np.array_equal(bf16.f64_to_bits(-mid), even | np.uint16(0x8000))


# ------------------------------------------------------------------ E2M1 tables
def test_e2m1_value_table_is_the_printed_one(golden_dir):
    rows = _load_table(os.path.join(golden_dir, "e2m1_values.txt"))
    assert [int(c) for c, _ in rows] == list(range(8))
    assert [float(v) for _, v in rows] == list(mxfp4.E2M1_VALUES)
    assert mxfp4.E2M1_VALUES.max() == 6.0           # paper: maximum representable FP4 value


def test_e2m1_tie_table(golden_dir):
    for s, want in _load_table(os.path.join(golden_dir, "e2m1_ties.txt")):
        code = mxfp4.e2m1_round_mag(np.array([float(s)]))[0]
        assert mxfp4.E2M1_VALUES[code] == float(want), (s, want)


def test_e2m1_rounding_brute_force_exact_rational(golden_dir):
    """Every non-negative finite bf16 pattern x every power-of-two divisor that
    leaves the quotient in (2^-6, 16]: the oracle's code equals the brute-force
    nearest E2M1 value in exact rational arithmetic (ties -> even code)."""
    values = [Fraction(v) for _, v in _load_table(os.path.join(golden_dir, "e2m1_values.txt"))]
    pos = [int(p) for p in ALL_FINITE if p < 0x8000]
    checked = 0
    for p in pos:
        v = _frac_of_bf16(p)
        if v == 0:
            assert mxfp4.e2m1_round_mag(np.array([0.0]))[0] == 0
            continue
        e = _floor_log2(v)
        for se in range(e - 4, e + 7):              # quotient in [2^-6.., 2^5)
            if se < -127 or se > 127:
                continue
            s = v / Fraction(2) ** se
            want = _nearest_code(s, values)
            got = int(mxfp4.e2m1_round_mag(np.array([float(s)]))[0])
            assert got == want, (hex(p), se, s)
            checked += 1
    assert checked > 300000


# ------------------------------------------------------------------ block quantizer
def _brute_force_block(bits_block, values):
    """Reference for one block of 32 patterns, all in Fractions."""
    vals = [_frac_of_bf16(int(p)) for p in bits_block]
    amax = max(abs(v) for v in vals)
    if amax == 0:
        se = 0
    else:
        se = min(127, max(-127, _floor_log2(amax) - 2))
    codes = []
    for p, v in zip(bits_block, vals):
        mag = _nearest_code(abs(v) / Fraction(2) ** se, values)
        codes.append(((int(p) >> 15) << 3) | mag)
    return codes, se + 127


def test_quantize_blocks_brute_force(golden_dir):
    values = [Fraction(v) for _, v in _load_table(os.path.join(golden_dir, "e2m1_values.txt"))]
    rng = np.random.default_rng(3)
    blocks = []
    # random finite patterns (wide exponent spread), gaussian-like data, specials
    blocks.append(ALL_FINITE[rng.integers(0, ALL_FINITE.size, (150, 32))])
    g = (rng.standard_normal((150, 32)) * 0.02).astype(np.float32)
    blocks.append((g.view(np.uint32) >> 16).astype(np.uint16))
    narrow = (rng.integers(0x3F00, 0x4100, (150, 32)) | (rng.integers(0, 2, (150, 32)) << 15)).astype(np.uint16)
    blocks.append(narrow)
    sub = rng.integers(0, 0x0100, (50, 32)).astype(np.uint16)         # subnormals and tiny normals
    blocks.append(sub)
    big = rng.integers(0x7E00, 0x7F80, (50, 32)).astype(np.uint16)    # near the largest finite bf16
    blocks.append(big)
    special = np.zeros((4, 32), dtype=np.uint16)
    special[1, :] = 0x8000                                            # all -0.0
    special[2, 5] = 0x0001                                            # one smallest subnormal
    special[3, :] = 0x7F7F                                            # all max finite
    blocks.append(special)
    bits = np.concatenate(blocks, axis=0)
    codes, scales = mxfp4.quantize(bits)
    for b in range(bits.shape[0]):
        want_codes, want_scale = _brute_force_block(bits[b], values)
        assert int(scales[b, 0]) == want_scale, b
        assert list(map(int, codes[b])) == want_codes, b


def test_quantize_special_cases():
    z = np.zeros((1, 32), dtype=np.uint16)
    c, s = mxfp4.quantize(z)
    assert s[0, 0] == 127 and not c.any()                              # zero block -> scale 2^0
    z[0, 3] = 0x8000
    c, s = mxfp4.quantize(z)
    assert c[0, 3] == 0x8 and s[0, 0] == 127                           # sign of -0.0 kept
    # tiny negative next to a large value rounds to magnitude 0 but keeps its sign
    b = np.zeros((1, 32), dtype=np.uint16)
    b[0, 0] = 0x4080          # 4.0
    b[0, 1] = 0xBC00          # -2^-7
    c, s = mxfp4.quantize(b)
    assert s[0, 0] == 127 and c[0, 0] == 6 and c[0, 1] == 0x8
    # values in (6,8)*2^se saturate to 6
    b[0, 0] = 0x40E0          # 7.0
    c, s = mxfp4.quantize(b)
    assert s[0, 0] == 127 and c[0, 0] == 7
    # clamp: amax with exponent field 1 or subnormal -> byte 0
    for amax in (0x0080, 0x007F, 0x0001):
        b = np.zeros((1, 32), dtype=np.uint16)
        b[0, 7] = amax
        c, s = mxfp4.quantize(b)
        assert s[0, 0] == 0
    # 2^-126 / 2^-127 = 2 -> code 4 ; 2^-133 / 2^-127 = 2^-6 -> 0
    b = np.zeros((1, 32), dtype=np.uint16); b[0, 0] = 0x0080; b[0, 1] = 0x0001
    c, s = mxfp4.quantize(b)
    assert c[0, 0] == 4 and c[0, 1] == 0


def test_scale_byte_is_exponent_field_minus_two():
    rng = np.random.default_rng(4)
    bits = rng.integers(0x0100, 0x7F80, (2000, 32)).astype(np.uint16)   # normal, exponent field >= 2
    bits |= (rng.integers(0, 2, bits.shape) << 15).astype(np.uint16)
    _, scales = mxfp4.quantize(bits)
    ef_max = ((bits & 0x7FFF) >> 7).max(axis=1)
    assert np.array_equal(scales[:, 0], ef_max - 2)


def test_pack_nibble_order():
    codes = np.arange(32, dtype=np.uint8)[None, :] % 16
    p = mxfp4.pack(codes)
    assert p.shape == (1, 16)
    assert p[0, 0] == (0 | (1 << 4)) and p[0, 1] == (2 | (3 << 4))
    assert np.array_equal(mxfp4.unpack(p), codes)


def _rand_bits(rng, shape, std=1.0):
    v = (rng.standard_normal(shape) * std).astype(np.float32)
    return bf16.f64_to_bits(v.astype(np.float64))


def test_idempotence_and_exact_representability():
    rng = np.random.default_rng(5)
    for std in (1.0, 0.02, 300.0):
        bits = _rand_bits(rng, (64, 256), std)
        c1, s1 = mxfp4.quantize(bits)
        d = mxfp4.dequantize(c1, s1)
        db = bf16.f64_to_bits(d)
        assert np.array_equal(bf16.bits_to_f64(db), d)                  # D(Q(x)) is exact in bf16
        c2, s2 = mxfp4.quantize(db)
        assert np.array_equal(s1, s2)
        # codes equal, except that a dequantised -0 keeps its sign as well
        assert np.array_equal(c1, c2)


def test_error_bound_and_sign():
    rng = np.random.default_rng(6)
    bits = _rand_bits(rng, (256, 128), 1.0)
    x = bf16.bits_to_f64(bits)
    c, s = mxfp4.quantize(bits)
    d = mxfp4.dequantize(c, s)
    sc = np.repeat(np.ldexp(1.0, s.astype(np.int64) - 127), 32, axis=1)
    q = np.abs(d) / sc
    step = np.where(q < 2, 0.5, np.where(q < 4, 1.0, 2.0))
    sat = np.abs(x) / sc > 6
    err = np.abs(x - d) / sc
    assert (err[~sat] <= step[~sat] / 2 + 1e-12).all()
    assert (err[sat] <= 2.0).all() and sat.any()
    assert (np.sign(d) * np.sign(x) >= 0).all()
    # the block maximum always lands on magnitude 4 or 6 (codes 6, 7)
    top = (c & 7).reshape(256, 4, 32).max(axis=2)
    assert np.isin(top, (6, 7)).all()


def test_planted_mistakes_are_caught(golden_dir):
    """The brute-force pin is sharp: a wrong tie direction or a wrong scale offset
    in a copy of the oracle's formula disagrees with the exact search."""
    values = [Fraction(v) for _, v in _load_table(os.path.join(golden_dir, "e2m1_values.txt"))]
    assert _nearest_code(Fraction(5, 4), values) == 2 and _nearest_code(Fraction(5), values) == 6
    assert _nearest_code(Fraction(7, 4), values) == 4 and _nearest_code(Fraction(1, 4), values) == 0
    wrong_up = lambda s: int(np.searchsorted([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0], s, side="right"))
    assert wrong_up(1.25) != _nearest_code(Fraction(5, 4), values)
