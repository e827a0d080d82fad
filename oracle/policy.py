"""Modality-aware precision scheduling (paper Sec. "Real-time Modality-aware LB
Scheduling": runtime state IB_d, R_vd; hotspot set H; precision assignment;
AIMD update of M_d) and the LB gate (Sec. "Overhead-Aware Pipeline
Orchestration", paragraph "LB Gate").  Constants from Sec. "Setup":
C = 1, M_d initially 0.9, tau = 1.5, Gamma = 2048.

Readings taken where the paper is silent or ambiguous:
  * one scalar M serves all ranks (same initial value, same global update
    signal); there is no lower floor on M;
  * the gate compares the global batch's token count T (before top-k) with
    Gamma ("256 x 8 ranks" are per-rank token counts); "exceeds" is strict;
    when the gate is closed every rank runs BF16 and M is left untouched;
  * M is updated from this layer's IB_global first and the updated M decides
    this layer (update_first=True); update_first=False decides with the old M
    and updates afterwards;
  * `force` overrides the whole policy for benchmarking (FP4-All / Baseline
    variants of Sec. "Setup", Compared Methods) and leaves M untouched;
  * all compares are made without forming the ratios:
        IB_d > C         <=>  Load_d * D      > C   * (T*k)
        IB_global > tau  <=>  max Load_d * D  > tau * (T*k)
        R_vd > M         <=>  N_vd            > M   * Load_d
    each side evaluated in float64 (integers here are exact in float64).
"""
from dataclasses import dataclass
import numpy as np

BF16, FP4 = 0, 1
FORCE_NONE = -1


@dataclass
class PolicyConfig:
    C: float = 1.0
    tau: float = 1.5
    Gamma: int = 2048
    M_init: float = 0.9
    aimd_mul: float = 0.5
    aimd_add: float = 0.1
    aimd_enabled: bool = True      # False: fixed threshold (the ReaLB-m variants)
    update_first: bool = True


def aimd_update(M: float, congested: bool, cfg: PolicyConfig) -> float:
    """M <- 0.5*M under congestion, else min(1, M + 0.1)   (AIMD equation)."""
    if congested:
        return cfg.aimd_mul * M
    return min(1.0, M + cfg.aimd_add)


def select_precision(rank_load, rank_vis, T: int, k: int, M: float,
                     cfg: PolicyConfig = PolicyConfig(), force: int = FORCE_NONE):
    """Returns (prec[D] int32, IB_global float, M_after float)."""
    load = [int(v) for v in np.asarray(rank_load).reshape(-1)]
    vis = [int(v) for v in np.asarray(rank_vis).reshape(-1)]
    D = len(load)
    total = float(T * k)
    max_ld = float(max(load) * D) if D else 0.0
    ib_global = max_ld / total if total > 0 else 0.0
    if force != FORCE_NONE:
        return np.full(D, force, dtype=np.int32), ib_global, M
    if not (T > cfg.Gamma):                                   # LB gate closed
        return np.full(D, BF16, dtype=np.int32), ib_global, M
    congested = max_ld > cfg.tau * total
    M_new = aimd_update(M, congested, cfg) if cfg.aimd_enabled else M
    M_dec = M_new if cfg.update_first else M
    prec = np.zeros(D, dtype=np.int32)
    for d in range(D):
        hot = float(load[d] * D) > cfg.C * total              # d in H
        vision_heavy = float(vis[d]) > M_dec * float(load[d])  # R_vd > M
        prec[d] = FP4 if (hot and vision_heavy and load[d] > 0) else BF16
    return prec, ib_global, M_new
