"""Pins for oracle.router and oracle.policy (CPU only): brute-force loops,
scipy's softmax, conservation invariants, closed forms of the AIMD recurrence,
the scenario of the paper's overview figure, and an exhaustive comparison with
the policy's literal ratio definitions evaluated in exact rationals."""
from fractions import Fraction
import itertools
import os

import numpy as np
import pytest
from scipy.special import softmax

import workloads as W
from oracle import router, policy


def _consts(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "policy_constants.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


# ------------------------------------------------------------------ router
def _topk_loops(logits, k):
    T, E = logits.shape
    ids = np.zeros((T, k), dtype=np.int32)
    for t in range(T):
        taken = set()
        for j in range(k):
            best = None
            for e in range(E):
                if e in taken:
                    continue
                if best is None or logits[t, e] > logits[t, best]:   # strict: lower index keeps ties
                    best = e
            taken.add(best)
            ids[t, j] = best
    return ids


def test_topk_ids_brute_force_with_ties():
    rng = np.random.default_rng(0)
    logits = rng.standard_normal((200, 16)).astype(np.float32)
    logits[:50] = np.round(logits[:50])            # many exact ties
    logits[50:60] = 0.0                            # all equal -> 0,1,2,...
    logits[60, 3] = -0.0
    ids, w = router.topk_route(logits, 4)
    assert np.array_equal(ids, _topk_loops(logits, 4))
    assert np.array_equal(ids[50], [0, 1, 2, 3])
    sel = np.take_along_axis(logits, ids.astype(np.int64), 1)
    assert (np.diff(sel, axis=1) <= 0).all()       # descending


def test_gate_weights_are_renormalised_softmax():
    rng = np.random.default_rng(1)
    logits = (rng.standard_normal((300, 64)) * 3).astype(np.float32)
    ids, w = router.topk_route(logits, 6)
    full = softmax(logits.astype(np.float64), axis=1)
    sel = np.take_along_axis(full, ids.astype(np.int64), 1)
    assert np.allclose(w, sel / sel.sum(1, keepdims=True), rtol=1e-12, atol=0)
    assert np.allclose(w.sum(1), 1.0, rtol=0, atol=1e-14)
    ids_all, w_all = router.topk_route(logits, 64)                 # k = E: plain softmax
    assert np.allclose(np.take_along_axis(full, ids_all.astype(np.int64), 1), w_all, rtol=1e-12)
    # extreme logits stay finite
    big = np.array([[1e4, -1e4, 0, 5e3]], dtype=np.float32)
    _, wb = router.topk_route(big, 2)
    assert np.array_equal(wb, [[1.0, 0.0]])


def test_counts_brute_force_and_conservation():
    cfg = W.CONFIGS["c1"]
    inp = W.gen_layer(cfg, 0)
    ids, _ = router.topk_route(inp["logits"], cfg.k)
    cnt, vis, load, rvis = router.route_counts(ids, inp["is_vision"], cfg.E, cfg.D)
    c2 = [0] * cfg.E
    v2 = [0] * cfg.E
    for t in range(cfg.T):
        for j in range(cfg.k):
            c2[ids[t, j]] += 1
            v2[ids[t, j]] += int(inp["is_vision"][t])
    assert list(cnt) == c2 and list(vis) == v2
    assert cnt.sum() == cfg.T * cfg.k == load.sum()
    assert vis.sum() == cfg.k * int(inp["is_vision"].sum())
    assert (vis <= cnt).all()
    # the +2.0 vision bias of this config makes experts 0-1 the hot, vision-heavy ones
    assert set(np.argsort(-cnt)[:2]) == {0, 1}


def test_counts_rank_grouping():
    rng = np.random.default_rng(2)
    ids = rng.integers(0, 12, (100, 3)).astype(np.int32)
    isv = rng.integers(0, 2, 100).astype(np.uint8)
    cnt, vis, load, rvis = router.route_counts(ids, isv, 12, 4)
    for d in range(4):
        m = (ids // 3) == d
        assert load[d] == m.sum()
        assert rvis[d] == (m & (isv[:, None] == 1)).sum()
    assert load.sum() == 300


# ------------------------------------------------------------------ policy
def test_policy_constants_match_paper(golden_dir):
    c = _consts(golden_dir)
    p = policy.PolicyConfig()
    assert (p.C, p.tau, p.Gamma, p.M_init, p.aimd_mul, p.aimd_add) == (
        c["C"], c["tau"], int(c["Gamma"]), c["M_init"], c["aimd_mul"], c["aimd_add"])
    assert policy.aimd_update(0.95, False, p) == c["M_cap"]


def test_aimd_closed_forms():
    p = policy.PolicyConfig()
    M = p.M_init
    for n in range(1, 30):                         # constant congestion: M_n = 0.9 * 2^-n, exactly
        M = policy.aimd_update(M, True, p)
        assert M == 0.9 * 2.0 ** (-n)
    M = 0.45
    seq = []
    for _ in range(8):
        M = policy.aimd_update(M, False, p)
        seq.append(M)
    assert np.allclose(seq, [0.55, 0.65, 0.75, 0.85, 0.95, 1.0, 1.0, 1.0], rtol=0, atol=1e-12)
    assert seq[-1] == 1.0
    # qualitative behaviour of the paper's AIMD appendix: fast fall, slow rise
    assert policy.aimd_update(0.9, True, p) < 0.9 - 3 * p.aimd_add


def test_overview_figure_scenario():
    """Two ranks overloaded, only one of them vision-dominant -> only that one goes FP4."""
    T, k, D = 8000, 1, 8
    ideal = T * k // D
    load = np.array([1.0, 1.6, 1.4, 0.7, 0.8, 0.9, 0.8, 0.8]) * ideal
    load = load.astype(np.int64)
    assert load.sum() == T * k
    rv = np.array([0.5, 0.95, 0.4, 0.5, 0.5, 0.5, 0.5, 0.5])
    vis = (rv * load).astype(np.int64)
    p = policy.PolicyConfig(aimd_enabled=False)                      # M stays 0.9
    prec, ib, M = policy.select_precision(load, vis, T, k, 0.9, p)
    assert list(prec) == [0, 1, 0, 0, 0, 0, 0, 0]
    assert ib == pytest.approx(1.6) and M == 0.9
    # with AIMD on, IB_global = 1.6 > tau halves M to 0.45 first; rank 2 (R_v 0.4) still BF16
    prec, ib, M = policy.select_precision(load, vis, T, k, 0.9, policy.PolicyConfig())
    assert list(prec) == [0, 1, 0, 0, 0, 0, 0, 0] and M == 0.45
    # decide-then-update: same decision here, same new M
    prec2, _, M2 = policy.select_precision(load, vis, T, k, 0.9, policy.PolicyConfig(update_first=False))
    assert list(prec2) == list(prec) and M2 == 0.45


def test_fixed_threshold_variants_and_gate_and_force():
    T, k, D = 4096, 2, 4
    load = np.array([4096, 2048, 1024, 1024])
    vis = np.array([1, 2048, 0, 1024])
    m1 = policy.PolicyConfig(aimd_enabled=False)
    prec, _, M = policy.select_precision(load, vis, T, k, 0.0, m1)   # M=0: every hotspot with a vision row
    assert list(prec) == [1, 0, 0, 0] and M == 0.0                   # rank 1: IB = 1.0, not > C
    load2 = np.array([3000, 3000, 1096, 1096]); vis2 = np.array([2200, 2000, 1096, 0])
    prec, _, _ = policy.select_precision(load2, vis2, T, k, 0.7, m1) # M=0.7: 0.733 yes, 0.667 no
    assert list(prec) == [1, 0, 0, 0]
    # LB gate: T <= Gamma -> all BF16, M untouched even under heavy imbalance
    prec, ib, M = policy.select_precision([4096, 0, 0, 0], [4096, 0, 0, 0], 2048, 2, 0.9, policy.PolicyConfig())
    assert list(prec) == [0, 0, 0, 0] and M == 0.9 and ib == 4.0
    prec, _, M = policy.select_precision([4098, 0, 0, 0], [4098, 0, 0, 0], 2049, 2, 0.9, policy.PolicyConfig())
    assert list(prec) == [1, 0, 0, 0] and M == 0.45
    # force overrides and leaves M alone
    for f in (policy.BF16, policy.FP4):
        prec, _, M = policy.select_precision(load, vis, T, k, 0.9, policy.PolicyConfig(), force=f)
        assert list(prec) == [f] * 4 and M == 0.9


def _literal_policy(load, vis, T, k, M, cfg):
    """The paper's definitions taken literally, in exact rationals: IB_d = Load_d /
    Ideal with Ideal the mean load, R_vd = N_vd / (N_vd + N_td), H = {IB_d > C},
    FP4 iff d in H and R_vd > M (M after the AIMD update)."""
    D = len(load)
    ideal = Fraction(sum(load), D)
    ib = [Fraction(l) / ideal for l in load]
    congested = max(ib) > Fraction(cfg.tau)
    Mn = Fraction(cfg.aimd_mul) * Fraction(M) if congested else min(Fraction(1), Fraction(M) + Fraction(cfg.aimd_add))
    out = []
    for d in range(D):
        if load[d] == 0:
            out.append(0)
            continue
        rv = Fraction(vis[d], load[d])
        out.append(1 if (ib[d] > Fraction(cfg.C) and rv > Mn) else 0)
    return out, float(max(ib)), congested


def test_policy_exhaustive_small_against_literal_ratios():
    cfg = policy.PolicyConfig(Gamma=0)
    n = 0
    for D in (2, 3):
        for total in range(1, 13):
            for load in itertools.product(range(total + 1), repeat=D):
                if sum(load) != total:
                    continue
                for vis in itertools.product(*[range(0, l + 1, max(1, l // 3)) for l in load]):
                    for M in (0.9, 0.45, 0.5, 0.0, 1.0):
                        prec, ib, Mn = policy.select_precision(load, vis, total, 1, M, cfg)
                        want, want_ib, congested = _literal_policy(load, vis, total, 1, M, cfg)
                        assert list(prec) == want, (load, vis, M)
                        assert ib == pytest.approx(want_ib, rel=1e-15)
                        assert Mn == (0.5 * M if congested else min(1.0, M + 0.1))
                        n += 1
    assert n > 5000


def test_policy_on_generated_configs_lands_in_paper_ranges():
    """The synthetic routing recipe gives the measured rank an imbalance and vision
    share inside the ranges the paper reports (device peak 2-3x+, hot rank > 90 % vision)."""
    cfg = W.scaled(W.CONFIGS["c2"], T=4096)
    x, isv = W.gen_tokens(W.scaled(cfg, H=32), 0)
    logits = W.gen_logits(cfg, 0, isv)
    ids, _ = router.topk_route(logits, cfg.k)
    _, _, load, rvis = router.route_counts(ids, isv, cfg.E, cfg.D)
    prec, ib, M = policy.select_precision(load, rvis, cfg.T, cfg.k, 0.9)
    assert np.argmax(load) == cfg.rank and 2.0 < ib < 4.5
    assert rvis[cfg.rank] / load[cfg.rank] > 0.88
    assert M == 0.45 and prec[cfg.rank] == policy.FP4
