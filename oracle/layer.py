"""One EP rank's MoE layer, the oracle's steps chained in the order of the
paper's pipeline (Sec. "System Overview", stages 1-4): route and profile ->
precision plan -> (FP4 only) encode the rank's expert weights and routed
activations -> group rows by expert -> expert FFN -> weighted combine.
"""
import numpy as np
from . import router, policy, mxfp4, permute, ffn


def rank_layer(inp: dict, E: int, k: int, D: int, rank: int, M: float,
               cfg: policy.PolicyConfig = policy.PolicyConfig(), force: int = policy.FORCE_NONE):
    """inp: dict with x (bf16 bits [T,H]), is_vision, logits, w13, w2 (the rank's
    local experts).  Returns a dict of every intermediate the parity tests compare."""
    T = inp["x"].shape[0]
    n_local = E // D
    ids, w = router.topk_route(inp["logits"], k)
    cnt, vis, load, rvis = router.route_counts(ids, inp["is_vision"], E, D)
    prec, ib, M_after = policy.select_precision(load, rvis, T, k, M, cfg, force)
    off, r2a, a2r = permute.permute_indices(ids, rank, n_local)
    xperm = permute.gather_rows(inp["x"], r2a, k)
    out = {"topk_ids": ids, "topk_w": w, "expert_cnt": cnt, "expert_vis": vis,
           "rank_load": load, "rank_vis": rvis, "prec": prec, "ib_global": ib, "M_after": M_after,
           "expert_offsets": off, "row_to_assign": r2a, "assign_to_row": a2r, "xperm": xperm}
    if int(prec[rank]) == policy.FP4:
        w13q, w13s = mxfp4.quantize(inp["w13"])
        w2q, w2s = mxfp4.quantize(inp["w2"])
        xq, xs = mxfp4.quantize(xperm)
        hq, hs, y = ffn.ffn_fp4(xq, xs, w13q, w13s, w2q, w2s, off)
        out.update(w13q=w13q, w13s=w13s, w2q=w2q, w2s=w2s, xq=xq, xs=xs, hq=hq, hs=hs)
    else:
        h_bits, y = ffn.ffn_bf16(xperm, inp["w13"], inp["w2"], off)
        out.update(h_bits=h_bits)
    y_bits = ffn.to_bf16_bits(y)
    o = ffn.combine(y_bits, a2r, w, T, k)
    out.update(y=y, y_bits=y_bits, out=o, out_bits=ffn.to_bf16_bits(o))
    return out
