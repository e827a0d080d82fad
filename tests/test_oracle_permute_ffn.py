"""Pins for oracle.permute, oracle.ffn and oracle.layer (CPU only)."""
import math

import numpy as np
import pytest

import workloads as W
from oracle import bf16, mxfp4, router, permute, ffn, layer, policy


# ------------------------------------------------------------------ permutation
def _perm_loops(ids, rank, n_local):
    T, k = ids.shape
    rows = []
    for e in range(rank * n_local, (rank + 1) * n_local):
        for a in range(T * k):
            if ids[a // k, a % k] == e:
                rows.append(a)
    return rows


def test_permutation_brute_force_and_invariants():
    rng = np.random.default_rng(0)
    ids = np.stack([rng.permutation(12)[:3] for _ in range(150)]).astype(np.int32)
    for rank in range(4):
        off, r2a, a2r = permute.permute_indices(ids, rank, 3)
        want = _perm_loops(ids, rank, 3)
        assert list(r2a) == want
        assert off[0] == 0 and off[-1] == len(want)
        flat = ids.reshape(-1)
        for e in range(3):
            seg = r2a[off[e]:off[e + 1]]
            assert (flat[seg] == rank * 3 + e).all()
            assert (np.diff(seg) > 0).all()                       # stable: ascending assignment index
            assert len(set(seg // 3)) == len(seg)                 # a token at most once per expert
        assert np.array_equal(a2r[r2a], np.arange(len(r2a)))
        local = (flat // 3) == rank
        assert ((a2r >= 0) == local).all()
    # numpy's stable argsort on the expert id reproduces the order
    off, r2a, _ = permute.permute_indices(ids, 0, 12)
    assert np.array_equal(r2a, np.argsort(ids.reshape(-1), kind="stable"))


def test_permutation_empty_expert_and_empty_rank():
    ids = np.array([[0, 2], [2, 0], [0, 2]], dtype=np.int32)
    off, r2a, a2r = permute.permute_indices(ids, 0, 3)
    assert list(off) == [0, 3, 3, 6] and list(r2a) == [0, 3, 4, 1, 2, 5]
    off, r2a, a2r = permute.permute_indices(ids, 1, 3)
    assert list(off) == [0, 0, 0, 0] and r2a.size == 0 and (a2r == -1).all()


def test_gather_rows():
    x = np.arange(5 * 4, dtype=np.uint16).reshape(5, 4)
    r2a = np.array([9, 0, 4, 5], dtype=np.int32)
    assert np.array_equal(permute.gather_rows(x, r2a, 2), x[[4, 0, 2, 2]])


# ------------------------------------------------------------------ FFN
def _bits(rng, shape, std):
    return W.f32_to_bf16_bits((rng.standard_normal(shape) * std).astype(np.float32))


def test_ffn_single_expert_is_dense_chain():
    rng = np.random.default_rng(1)
    R, H, I = 37, 64, 96
    x, w13, w2 = _bits(rng, (R, H), 1.0), _bits(rng, (1, 2 * I, H), 0.1), _bits(rng, (1, H, I), 0.1)
    h_bits, y = ffn.ffn_bf16(x, w13, w2, [0, R])
    xf, w13f, w2f = (bf16.bits_to_f64(a) for a in (x, w13, w2))
    g = xf @ w13f[0, :I].T
    u = xf @ w13f[0, I:].T
    h = g * (1 / (1 + np.exp(-g))) * u
    assert np.allclose(bf16.bits_to_f64(h_bits), h, rtol=2 ** -8, atol=1e-30)
    assert np.allclose(y, bf16.bits_to_f64(h_bits) @ w2f[0].T, rtol=1e-12, atol=1e-14)


def test_ffn_pure_python_triple_loop_on_a_few_rows():
    rng = np.random.default_rng(2)
    H, I = 32, 32
    offs = [0, 2, 2, 5]
    x, w13, w2 = _bits(rng, (5, H), 1.0), _bits(rng, (3, 2 * I, H), 0.2), _bits(rng, (3, H, I), 0.2)
    _, y = ffn.ffn_bf16(x, w13, w2, offs)
    xf, w13f, w2f = (bf16.bits_to_f64(a).tolist() for a in (x, w13, w2))
    for r, e in ((0, 0), (1, 0), (2, 2), (4, 2)):
        hrow = []
        for i in range(I):
            g = sum(xf[r][c] * w13f[e][i][c] for c in range(H))
            u = sum(xf[r][c] * w13f[e][I + i][c] for c in range(H))
            hv = g / (1.0 + math.exp(-g)) * u
            hrow.append(float(bf16.round_f64_to_bf16_value(np.array([hv]))[0]))
        for c in range(H):
            want = sum(hrow[i] * w2f[e][c][i] for i in range(I))
            assert y[r, c] == pytest.approx(want, rel=1e-11, abs=1e-15)


def test_fp4_path_equals_bf16_path_on_fp4_representable_inputs():
    """Inputs that are already E2M1 values times one power of two per block, with a
    block maximum of 4 or 6, encode losslessly, so both paths give the same h."""
    rng = np.random.default_rng(3)
    R, H, I = 24, 64, 64

    def fp4_exact(shape, exp):
        mags = mxfp4.E2M1_VALUES[rng.integers(0, 8, shape)]
        mags[..., ::32] = 4.0
        return bf16.f64_to_bits(mags * rng.choice([-1.0, 1.0], shape) * 2.0 ** exp)

    x, w13, w2 = fp4_exact((R, H), 0), fp4_exact((2, 2 * I, H), -6), fp4_exact((2, H, I), -5)
    offs = [0, 10, R]
    xq, xs = mxfp4.quantize(x)
    assert np.array_equal(mxfp4.dequantize(xq, xs), bf16.bits_to_f64(x))
    w13q, w13s = mxfp4.quantize(w13)
    w2q, w2s = mxfp4.quantize(w2)
    h_bits, y16 = ffn.ffn_bf16(x, w13, w2, offs)
    hq, hs, y4 = ffn.ffn_fp4(xq, xs, w13q, w13s, w2q, w2s, offs)
    hq_want, hs_want = mxfp4.quantize(h_bits)                      # same h before its FP4 encoding
    assert np.array_equal(hq, hq_want) and np.array_equal(hs, hs_want)
    assert np.allclose(y4, ffn.down_fp4(hq, hs, w2q, w2s, offs), rtol=0, atol=0)
    # and the FP4 result differs from BF16 only by the encoding error of h
    rel = np.linalg.norm(y4 - y16) / np.linalg.norm(y16)
    assert 0 < rel < 0.2


def test_down_is_linear_in_w2_and_respects_segments():
    rng = np.random.default_rng(4)
    h = rng.standard_normal((9, 32))
    wa, wb = rng.standard_normal((2, 16, 32)), rng.standard_normal((2, 16, 32))
    offs = [0, 4, 9]
    assert np.allclose(ffn.down(h, wa + 2 * wb, offs), ffn.down(h, wa, offs) + 2 * ffn.down(h, wb, offs))
    y = ffn.down(h, wa, offs)
    assert np.allclose(y[:4], h[:4] @ wa[0].T) and np.allclose(y[4:], h[4:] @ wa[1].T)


# ------------------------------------------------------------------ combine / whole layer
def _moe_per_token(inp, cfg, experts):
    """Full MoE output straight from the definition, one token at a time, with the
    same rounding points (h to BF16, each expert output row to BF16)."""
    ids, w = router.topk_route(inp["logits"], cfg.k)
    xf = bf16.bits_to_f64(inp["x"])
    w13f, w2f = bf16.bits_to_f64(inp["w13"]), bf16.bits_to_f64(inp["w2"])
    out = np.zeros((cfg.T, cfg.H))
    for t in range(cfg.T):
        for j in range(cfg.k):
            e = int(ids[t, j])
            if e not in experts:
                continue
            gu = w13f[e] @ xf[t]
            g, u = gu[:cfg.I], gu[cfg.I:]
            h = bf16.round_f64_to_bf16_value(g / (1 + np.exp(-g)) * u)
            y = bf16.round_f64_to_bf16_value(w2f[e] @ h)
            out[t] += w[t, j] * y
    return out


def test_layer_c1_equals_per_token_definition():
    cfg = W.CONFIGS["c1"]
    inp = W.gen_layer(cfg, 0)
    res = layer.rank_layer(inp, cfg.E, cfg.k, cfg.D, 0, 0.9, force=policy.BF16)
    want = _moe_per_token(inp, cfg, set(range(cfg.E)))
    assert np.allclose(res["out"], want, rtol=1e-9, atol=1e-12)
    assert res["expert_offsets"][-1] == res["rank_load"][0] == cfg.T * cfg.k


def test_rank_partial_outputs_sum_to_full_moe():
    cfg = W.scaled(W.CONFIGS["c1"], D=4, T=128)
    inp = W.gen_layer(cfg, 1)
    inp["w13"], inp["w2"] = W.gen_weights(cfg, 1, n_experts=cfg.E)
    total = np.zeros((cfg.T, cfg.H))
    nl = cfg.n_local
    for d in range(cfg.D):
        sub = dict(inp, w13=inp["w13"][d * nl:(d + 1) * nl], w2=inp["w2"][d * nl:(d + 1) * nl])
        res = layer.rank_layer(sub, cfg.E, cfg.k, cfg.D, d, 0.9, force=policy.BF16)
        total += res["out"]
        none_local = (res["assign_to_row"].reshape(cfg.T, cfg.k) < 0).all(axis=1)
        assert not res["out"][none_local].any()                    # exactly zero
    want = _moe_per_token(inp, cfg, set(range(cfg.E)))
    assert np.allclose(total, want, rtol=1e-9, atol=1e-12)


def test_layer_fp4_uses_dequantised_operands_and_is_close_to_bf16():
    cfg = W.CONFIGS["c1"]
    inp = W.gen_layer(cfg, 0)
    r4 = layer.rank_layer(inp, cfg.E, cfg.k, cfg.D, 0, 0.9, force=policy.FP4)
    r16 = layer.rank_layer(inp, cfg.E, cfg.k, cfg.D, 0, 0.9, force=policy.BF16)
    # activations are encoded after the gather: same codes as encoding x and gathering
    xq_tok, xs_tok = mxfp4.quantize(inp["x"])
    tok = r4["row_to_assign"].astype(np.int64) // cfg.k
    assert np.array_equal(r4["xq"], xq_tok[tok]) and np.array_equal(r4["xs"], xs_tok[tok])
    rel = np.linalg.norm(r4["out"] - r16["out"]) / np.linalg.norm(r16["out"])
    assert 0.05 < rel < 0.5                                         # FP4 noise is visible but bounded
