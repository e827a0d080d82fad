"""Seeded synthetic inputs for the ReaLB hot path (one EP rank's MoE layer).

This module only draws inputs: token activations, expert weights, router
logits and the vision/text flag per token, with the layer shapes of the two
models the paper evaluates (Sec. "Setup", Models: 64 and 128 routed experts)
and routing skew inside the ranges the paper reports for Kimi-VL on MMMU
(Sec. "High Dynamics of MMoE Routing": device peak 2-3x the mean, hottest
expert 2-12x the mean, hot-rank vision share above 90 %, others lower).
The paper's datasets, model weights and routing traces are not reproduced.

It holds none of the method's arithmetic (no top-k, no counts, no policy, no
FP4 encoding, no GEMM).  Both the CPU oracle's tests and the GPU tests / bench
feed the arrays produced here to their respective implementations.

BF16 tensors are carried as numpy uint16 bit patterns (numpy has no bfloat16).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

__all__ = [
    "LayerShape", "CONFIGS", "f32_to_bf16_bits", "gen_tokens", "gen_weights",
    "gen_logits", "gen_logits_c4", "gen_logits_trace", "gen_layer",
]


@dataclass(frozen=True)
class LayerShape:
    """One MoE layer + routing recipe.  n_local = E // D experts per rank."""
    name: str
    T: int            # tokens in the global batch (before top-k)
    E: int            # routed experts
    k: int            # experts per token
    D: int            # EP ranks
    H: int            # hidden size
    I: int            # SwiGLU intermediate size
    vision_frac: float
    logit_mode: str   # "c1" | "zipf"
    zipf_s: float = 0.0
    beta: float = 0.5
    rank: int = 0     # the measured rank

    @property
    def n_local(self) -> int:
        return self.E // self.D

    @property
    def A(self) -> int:
        return self.T * self.k


CONFIGS = {
    # tiny layer, one rank holds all experts; +2.0 logit bias on experts 0-1 for vision tokens
    "c1": LayerShape("c1", T=512, E=8, k=2, D=1, H=256, I=128, vision_frac=0.5, logit_mode="c1"),
    # Kimi-VL-A3B-shaped rank share (64 experts, top-6, 8 local)
    "c2": LayerShape("c2", T=16384, E=64, k=6, D=8, H=2048, I=1408, vision_frac=0.75,
                     logit_mode="zipf", zipf_s=1.1),
    # Qwen3-VL-30B-A3B-shaped rank share (128 experts, top-8, 16 local)
    "c3": LayerShape("c3", T=32768, E=128, k=8, D=8, H=2048, I=768, vision_frac=0.80,
                     logit_mode="zipf", zipf_s=1.2),
    # 8-rank imbalance simulation on the Kimi-shaped layer (logits from gen_logits_c4)
    "c4": LayerShape("c4", T=16384, E=64, k=6, D=8, H=2048, I=1408, vision_frac=0.70,
                     logit_mode="c4", zipf_s=1.1),
    # overlap stress on the Qwen-shaped rank
    "c5": LayerShape("c5", T=65536, E=128, k=8, D=8, H=2048, I=768, vision_frac=0.85,
                     logit_mode="zipf", zipf_s=1.2),
}


def scaled(cfg: LayerShape, **kw) -> LayerShape:
    """A copy of cfg with some fields replaced (used for reduced-size parity cases)."""
    return replace(cfg, **kw)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); return uint16 patterns.
    Storage-format conversion for the generated inputs only (finite values)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def _normal_bf16(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(-1)
    n = flat.size
    step = 1 << 24
    for s in range(0, n, step):
        m = min(step, n - s)
        v = rng.standard_normal(m, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        flat[s:s + m] = f32_to_bf16_bits(v)
    return out


def gen_tokens(cfg: LayerShape, seed: int):
    """x ~ N(0,1) as bf16 bits [T,H]; is_vision uint8 [T] with exactly
    round(vision_frac*T) ones at seeded random positions."""
    rng = np.random.default_rng([seed, 11])
    x = _normal_bf16(rng, (cfg.T, cfg.H), 1.0)
    nv = int(round(cfg.vision_frac * cfg.T))
    is_vision = np.zeros(cfg.T, dtype=np.uint8)
    is_vision[rng.permutation(cfg.T)[:nv]] = 1
    return x, is_vision


def gen_weights(cfg: LayerShape, seed: int, n_experts: int | None = None):
    """W13 bf16 bits [n, 2I, H] (gate rows first, then up rows) and W2 bf16 bits
    [n, H, I], both ~ N(0, 0.02)."""
    n = cfg.n_local if n_experts is None else n_experts
    rng = np.random.default_rng([seed, 23])
    w13 = _normal_bf16(rng, (n, 2 * cfg.I, cfg.H), 0.02)
    w2 = _normal_bf16(rng, (n, cfg.H, cfg.I), 0.02)
    return w13, w2


def _zipf_bias(E: int, s: float, beta: float, ranks: np.ndarray) -> np.ndarray:
    p = ranks.astype(np.float64) ** (-s)
    p /= p.sum()
    return (beta * np.log(E * p)).astype(np.float32)


def gen_logits(cfg: LayerShape, seed: int, is_vision: np.ndarray) -> np.ndarray:
    """Router logits f32 [T,E].

    "c1":   N(0,1), +2.0 on experts 0 and 1 for vision tokens.
    "zipf": N(0,1); vision tokens get += beta*ln(E*p_e), p_e ~ z_e^-s, where the
            measured rank's local experts hold Zipf ranks 1..n_local (seeded
            shuffle) and all other experts ranks n_local+1..E (seeded shuffle).
    """
    rng = np.random.default_rng([seed, 37])
    logits = rng.standard_normal((cfg.T, cfg.E), dtype=np.float32)
    vis = is_vision.astype(bool)
    if cfg.logit_mode == "c1":
        logits[np.ix_(vis, [0, 1])] += np.float32(2.0)
    elif cfg.logit_mode == "zipf":
        nl = cfg.n_local
        local = np.arange(cfg.rank * nl, (cfg.rank + 1) * nl)
        other = np.setdiff1d(np.arange(cfg.E), local)
        z = np.empty(cfg.E, dtype=np.int64)
        z[rng.permutation(local)] = np.arange(1, nl + 1)
        z[rng.permutation(other)] = np.arange(nl + 1, cfg.E + 1)
        logits[vis] += _zipf_bias(cfg.E, cfg.zipf_s, cfg.beta, z)[None, :]
    else:
        raise ValueError(f"gen_logits: mode {cfg.logit_mode!r}; use gen_logits_c4")
    return logits


def gen_logits_c4(cfg: LayerShape, iteration: int, is_vision: np.ndarray):
    """Per-iteration logits for the 8-rank imbalance simulation (seed 1000+it).
    With probability 1/2 "clustered": one uniformly drawn hot rank's experts take
    Zipf ranks 1..n_local, beta 0.5; else "scattered": Zipf ranks are a random
    permutation over all experts, beta 1.0.  Returns (logits, info dict)."""
    rng = np.random.default_rng([1000 + iteration, 41])
    logits = rng.standard_normal((cfg.T, cfg.E), dtype=np.float32)
    vis = is_vision.astype(bool)
    nl = cfg.n_local
    z = np.empty(cfg.E, dtype=np.int64)
    if rng.random() < 0.5:
        hot = int(rng.integers(cfg.D))
        local = np.arange(hot * nl, (hot + 1) * nl)
        other = np.setdiff1d(np.arange(cfg.E), local)
        z[rng.permutation(local)] = np.arange(1, nl + 1)
        z[rng.permutation(other)] = np.arange(nl + 1, cfg.E + 1)
        beta, kind = 0.5, "clustered"
    else:
        hot = -1
        z[rng.permutation(cfg.E)] = np.arange(1, cfg.E + 1)
        beta, kind = 1.0, "scattered"
    logits[vis] += _zipf_bias(cfg.E, cfg.zipf_s, beta, z)[None, :]
    return logits, {"kind": kind, "hot_rank": hot, "beta": beta}


def gen_logits_trace(cfg: LayerShape, iteration: int, is_vision: np.ndarray, block: int = 10):
    """Per-iteration logits of a longer trace whose imbalance comes and goes (seed 2000+it), for
    studying the threshold controller: blocks of `block` iterations cycle through "calm" (Zipf ranks
    scattered over all experts, beta 0.1: device peak close to the mean), "clustered" (one uniformly
    drawn hot rank, beta 0.5) and "scattered" (beta 1.0).  Returns (logits, info dict)."""
    rng = np.random.default_rng([2000 + iteration, 43])
    logits = rng.standard_normal((cfg.T, cfg.E), dtype=np.float32)
    vis = is_vision.astype(bool)
    nl = cfg.n_local
    z = np.empty(cfg.E, dtype=np.int64)
    regime = (iteration // block) % 3
    if regime == 1:
        hot = int(rng.integers(cfg.D))
        local = np.arange(hot * nl, (hot + 1) * nl)
        other = np.setdiff1d(np.arange(cfg.E), local)
        z[rng.permutation(local)] = np.arange(1, nl + 1)
        z[rng.permutation(other)] = np.arange(nl + 1, cfg.E + 1)
        beta, kind = 0.5, "clustered"
    else:
        hot = -1
        z[rng.permutation(cfg.E)] = np.arange(1, cfg.E + 1)
        beta, kind = (0.1, "calm") if regime == 0 else (1.0, "scattered")
    logits[vis] += _zipf_bias(cfg.E, cfg.zipf_s, beta, z)[None, :]
    return logits, {"kind": kind, "hot_rank": hot, "beta": beta}


def gen_layer(cfg: LayerShape, seed: int = 0, weight_seed: int | None = None):
    """All inputs of one layer call for cfg's measured rank, as a dict of numpy arrays."""
    x, is_vision = gen_tokens(cfg, seed)
    if cfg.logit_mode == "c4":
        logits, _ = gen_logits_c4(cfg, seed, is_vision)
    else:
        logits = gen_logits(cfg, seed, is_vision)
    w13, w2 = gen_weights(cfg, seed if weight_seed is None else weight_seed)
    return {"x": x, "is_vision": is_vision, "logits": logits, "w13": w13, "w2": w2}
