"""Routing and profiling (paper Sec. "System Overview", stage 1; runtime state of
Sec. "Real-time Modality-aware LB Scheduling").

The paper only says that gating produces expert assignments and device-level
load statistics; top-k with gates renormalised over the selected experts is the
routing rule of both evaluated models and is what the workload description
fixes.  Readings taken where the paper is silent:
  * ties between equal logits go to the lower expert index; the k outputs are
    ordered by descending logit (ties ascending index);
  * logits are float32;
  * "token load on device d" counts routed (token, expert) assignments, i.e.
    the GEMM row count of that rank; experts map to ranks contiguously,
    rank(e) = e // n_local.
"""
import numpy as np


def topk_route(logits: np.ndarray, k: int):
    """ids[t, j] = index of the (j+1)-th largest logit of token t;
    w[t, j] = exp(l_j - l_max) / sum_{j' in top-k} exp(l_j' - l_max)  (float64),
    which equals a softmax over all experts renormalised over the top-k."""
    logits = np.asarray(logits, dtype=np.float32)
    T, E = logits.shape
    assert 1 <= k <= E
    assert np.isfinite(logits).all()
    order = np.argsort(-logits, axis=1, kind="stable")        # ties -> lower index first
    ids = order[:, :k].astype(np.int32)
    sel = np.take_along_axis(logits, ids.astype(np.int64), axis=1).astype(np.float64)
    ex = np.exp(sel - sel[:, :1])                              # column 0 is the row maximum
    w = ex / ex.sum(axis=1, keepdims=True)
    return ids, w


def route_counts(topk_ids: np.ndarray, is_vision: np.ndarray, E: int, D: int):
    """expert_cnt[e]  = #assignments routed to expert e,
    expert_vis[e]  = those whose token is a vision token,
    rank_load[d]   = Load_d  = sum of expert_cnt over the experts of rank d,
    rank_vis[d]    = N_vd    = sum of expert_vis over the experts of rank d
    (N_td = rank_load - rank_vis).  All int64."""
    ids = np.asarray(topk_ids, dtype=np.int64)
    T, k = ids.shape
    assert E % D == 0
    vis = np.repeat(np.asarray(is_vision).astype(bool), k)
    flat = ids.reshape(-1)
    expert_cnt = np.bincount(flat, minlength=E)
    expert_vis = np.bincount(flat[vis], minlength=E)
    n_local = E // D
    rank_load = expert_cnt.reshape(D, n_local).sum(axis=1)
    rank_vis = expert_vis.reshape(D, n_local).sum(axis=1)
    return expert_cnt, expert_vis, rank_load, rank_vis
