"""GPU parity for the two multi-call workloads, through the calls bench.py times for them.

Config 4 (8 simulated EP ranks run one after the other, realb_rank_forward): the partial outputs of the
eight ranks, summed in FP32, must equal the oracle's full MoE layer (all 64 experts on one rank) -- the
sum-over-ranks invariant of the result combination -- and the policy's plan for the iteration must be the
oracle's; the hot rank is then run in FP4 through the same call and compared row by row.

Config 5 (48 layers of distinct weights on a Qwen3-VL-shaped rank, 65536 tokens): three weight sets of
the seeded sequence (layers 0, 23, 47) go through realb_layer_forward with the encoder on the side
stream; indices, weight codes and scales are compared in full and bit-exactly, the GEMM outputs on a
seeded 4096-row sample; the call with pre-encoded weights (overlap = 2), which the bench uses as the
"nothing exposed" baseline, must reproduce the same rows bit for bit."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import bf16 as obf, ffn as offn, layer as olayer, mxfp4 as omx, permute as operm, policy as opol, router as orouter
from gpu_helpers import BF16_TOL, ROW_TOL, FP4_E2E_TOL, FP4_TOL, GATE_W_RTOL, rel_fro, row_report, same, say

pytestmark = pytest.mark.gpu


def _say(msg):
    say("gpu-c4c5", msg)


def test_config4_sum_over_ranks_is_the_full_layer():
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config
    cfg = W.CONFIGS["c4"]
    it = 0
    _say(f"c4: inputs T={cfg.T} E={cfg.E} D={cfg.D}, iteration {it}")
    xb, isv_np = W.gen_tokens(cfg, 0)
    logits, info = W.gen_logits_c4(cfg, it, isv_np)
    wsets = [W.gen_weights(cfg, 100 + d) for d in range(cfg.D)]
    rcfg = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
    ctx = R.Context(rcfg)
    buf = R.LayerBuffers(rcfg, cfg.T)
    x = R.bf16_from_bits(xb)
    lg = torch.from_numpy(logits).cuda()
    isv = torch.from_numpy(isv_np).cuda()

    # routing statistics and the plan of this iteration
    ctx.route_stats(lg, isv, buf)
    ctx.M = rcfg.M_init
    prec, ib, M = ctx.select_precision(buf, cfg.T)
    ids, w = orouter.topk_route(logits, cfg.k)
    cnt, vis, load, rvis = orouter.route_counts(ids, isv_np, cfg.E, cfg.D)
    want = opol.select_precision(load, rvis, cfg.T, cfg.k, rcfg.M_init)
    assert same(buf.topk_ids.cpu().numpy(), ids)
    assert np.allclose(buf.topk_w.cpu().numpy().astype(np.float64), w, rtol=GATE_W_RTOL, atol=1e-9)
    assert same(buf.rank_load.cpu().numpy(), load) and same(buf.rank_vis.cpu().numpy(), rvis)
    assert list(prec) == list(want[0]) and ib == want[1] and M == want[2]
    _say(f"c4: {info['kind']} skew, IB_global {ib:.2f}, plan {list(prec)}, M {M}")

    # every rank in BF16 through realb_rank_forward; FP32 sum of the partial outputs
    total = torch.zeros((cfg.T, cfg.H), dtype=torch.float32, device="cuda")
    rows_seen = 0
    for d in range(cfg.D):
        w13, w2 = (R.bf16_from_bits(a) for a in wsets[d])
        io = ctx.make_io(lg, isv, x, w13, w2, buf, d, overlap=True)
        buf.out.fill_(float("nan"))
        ctx.rank_forward(io, R.BF16)
        torch.cuda.synchronize()
        off, r2a, a2r = operm.permute_indices(ids, d, cfg.n_local)
        assert same(buf.expert_offsets.cpu().numpy(), off) and same(buf.assign_to_row.cpu().numpy(), a2r)
        assert int(off[-1]) == int(load[d])
        rows_seen += int(off[-1])
        total += buf.out.float()
        _say(f"c4: rank {d} BF16 done, {int(off[-1])} rows")
    assert rows_seen == cfg.T * cfg.k
    _say("c4: oracle full layer (64 experts on one rank, BF16)")
    inp_all = {"x": xb, "is_vision": isv_np, "logits": logits,
               "w13": np.concatenate([ws[0] for ws in wsets]), "w2": np.concatenate([ws[1] for ws in wsets])}
    o = olayer.rank_layer(inp_all, cfg.E, cfg.k, 1, 0, rcfg.M_init, force=opol.BF16)
    got = total.double().cpu().numpy()
    fro = rel_fro(got, o["out"])
    per_tok = np.linalg.norm(got - o["out"], axis=1) / np.linalg.norm(o["out"], axis=1)
    _say(f"c4: sum over the 8 ranks vs the full layer: rel fro {fro:.3e}, worst token {per_tok.max():.3e}")
    assert fro <= BF16_TOL and per_tok.max() <= BF16_TOL

    # the hottest rank in FP4 through the same call
    hot = int(np.argmax(load))
    w13b, w2b = wsets[hot]
    w13, w2 = R.bf16_from_bits(w13b), R.bf16_from_bits(w2b)
    io = ctx.make_io(lg, isv, x, w13, w2, buf, hot, overlap=True)
    buf.y_rows.fill_(float("nan"))
    ctx.rank_forward(io, R.FP4)
    torch.cuda.synchronize()
    _say(f"c4: rank {hot} FP4 done; oracle for that rank")
    of = olayer.rank_layer({"x": xb, "is_vision": isv_np, "logits": logits, "w13": w13b, "w2": w2b}, cfg.E, cfg.k, cfg.D, hot,
                           rcfg.M_init, force=opol.FP4)
    Rr = int(of["expert_offsets"][-1])
    assert same(buf.expert_offsets.cpu().numpy(), of["expert_offsets"]) and same(buf.row_to_assign.cpu().numpy()[:Rr], of["row_to_assign"])
    assert same(buf.w13_q.cpu().numpy(), omx.pack(of["w13q"])) and same(buf.w2_q.cpu().numpy(), omx.pack(of["w2q"]))
    hq = omx.unpack(buf.h_mid.view(torch.uint8).reshape(-1)[: buf.max_rows * (cfg.I // 2)].reshape(buf.max_rows, cfg.I // 2)[:Rr].cpu().numpy())
    hs = R.scales_to_canonical(buf.h_s, Rr, cfg.I)
    y = obf.bits_to_f64(R.bits_from_bf16(buf.y_rows[:Rr]))
    y_st = offn.down_fp4(hq, hs, of["w2q"], of["w2s"], of["expert_offsets"])
    staged, e2e = rel_fro(y, y_st), rel_fro(y, of["y"])
    wr, nb, ex = row_report(y, y_st)
    _say(f"c4: rank {hot} FP4, all {Rr} rows: staged rel fro {staged:.3e}, end to end {e2e:.3e}, worst row {wr:.3e}, outside the bound {nb}")
    assert staged <= FP4_TOL and e2e <= FP4_E2E_TOL and wr <= ROW_TOL and nb == 0
    assert torch.isnan(buf.y_rows[Rr:Rr + 4096].float()).all()
    out = obf.bits_to_f64(R.bits_from_bf16(buf.out))
    assert rel_fro(out, of["out"]) <= FP4_E2E_TOL
    ctx.close()


def test_config5_three_weight_sets_and_pre_encoded_call():
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config
    cfg = W.CONFIGS["c5"]
    _say(f"c5: inputs T={cfg.T} E={cfg.E} n_local={cfg.n_local}")
    xb, isv_np = W.gen_tokens(cfg, 0)
    logits = W.gen_logits(cfg, 0, isv_np)
    rcfg = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
    ctx = R.Context(rcfg)
    buf = R.LayerBuffers(rcfg, cfg.T)
    x = R.bf16_from_bits(xb)
    lg = torch.from_numpy(logits).cuda()
    isv = torch.from_numpy(isv_np).cuda()
    ids, w = orouter.topk_route(logits, cfg.k)
    cnt, vis, load, rvis = orouter.route_counts(ids, isv_np, cfg.E, cfg.D)
    off, r2a, a2r = operm.permute_indices(ids, cfg.rank, cfg.n_local)
    Rr = int(off[-1])
    tok = r2a.astype(np.int64) // cfg.k
    _say(f"c5: {Rr} rows on the rank; oracle encodes the tokens")
    xq_tok, xs_tok = omx.quantize_packed(xb)
    rng = np.random.default_rng(505)
    # 4096 sampled rows: the first and last row of every expert segment plus seeded random rows
    edge = [int(v) for e in range(cfg.n_local) if off[e + 1] > off[e] for v in (off[e], off[e + 1] - 1)]
    sample = np.unique(np.concatenate([np.array(edge, dtype=np.int64), rng.integers(0, Rr, 4096 - len(edge))]))
    seg_of = np.searchsorted(off, sample, side="right") - 1
    for layer in (0, 23, 47):
        _say(f"c5: layer {layer}: weights, layer_forward (encoder on the side stream)")
        w13b, w2b = W.gen_weights(cfg, layer)
        w13, w2 = R.bf16_from_bits(w13b), R.bf16_from_bits(w2b)
        buf.y_rows.fill_(float("nan"))
        io = ctx.make_io(lg, isv, x, w13, w2, buf, cfg.rank, force=R.FP4, overlap=1)
        assert ctx.layer_forward(io) == R.FP4
        torch.cuda.synchronize()
        assert same(buf.topk_ids.cpu().numpy(), ids)
        assert same(buf.expert_cnt.cpu().numpy(), cnt) and same(buf.rank_load.cpu().numpy(), load) and same(buf.rank_vis.cpu().numpy(), rvis)
        assert same(buf.expert_offsets.cpu().numpy(), off)
        assert same(buf.row_to_assign.cpu().numpy()[:Rr], r2a) and same(buf.assign_to_row.cpu().numpy(), a2r)
        _say(f"c5: layer {layer}: oracle encodes the weights")
        w13q, w13s = omx.quantize(w13b)
        w2q, w2s = omx.quantize(w2b)
        assert same(buf.w13_q.cpu().numpy(), omx.pack(w13q))
        assert same(R.scales_to_canonical(buf.w13_s, cfg.n_local * 2 * cfg.I, cfg.H).reshape(w13s.shape), w13s)
        assert same(buf.w2_q.cpu().numpy(), omx.pack(w2q))
        assert same(R.scales_to_canonical(buf.w2_s, cfg.n_local * cfg.H, cfg.I).reshape(w2s.shape), w2s)
        has_local = (a2r.reshape(cfg.T, cfg.k) >= 0).any(axis=1)
        assert same(buf.x_q.cpu().numpy()[:cfg.T][has_local], xq_tok[has_local])
        sel = torch.from_numpy(sample).cuda()
        hq_all = buf.h_mid.view(torch.uint8).reshape(-1)[: buf.max_rows * (cfg.I // 2)].reshape(buf.max_rows, cfg.I // 2)
        hq_g = omx.unpack(hq_all[sel].cpu().numpy())
        hs_g = R.scales_to_canonical(buf.h_s, Rr, cfg.I)[sample]
        yg = obf.bits_to_f64(R.bits_from_bf16(buf.y_rows[sel]))
        y_st = np.zeros_like(yg); y_e2e = np.zeros_like(yg)
        flips = 0
        for e in np.unique(seg_of):
            m = seg_of == e
            seg = [0, int(m.sum())]
            t = tok[sample[m]]
            hq, hs, y = offn.ffn_fp4(omx.unpack(xq_tok[t]), xs_tok[t], w13q[e:e + 1], w13s[e:e + 1], w2q[e:e + 1], w2s[e:e + 1], seg)
            flips += int((hq_g[m] != hq).sum())
            y_e2e[m] = y
            y_st[m] = offn.down_fp4(hq_g[m], hs_g[m], w2q[e:e + 1], w2s[e:e + 1], seg)
        staged, e2e = rel_fro(yg, y_st), rel_fro(yg, y_e2e)
        wr, nb, ex = row_report(yg, y_st)
        _say(f"c5: layer {layer}: {sample.size} sampled rows: staged rel fro {staged:.3e}, end to end {e2e:.3e}, worst row {wr:.3e}, "
             f"outside the bound {nb}, h code flips {flips / hq_g.size:.2e}")
        assert np.isfinite(yg).all()
        assert staged <= FP4_TOL and e2e <= FP4_E2E_TOL and wr <= ROW_TOL and nb == 0 and flips / hq_g.size <= 1e-3
        assert torch.isnan(buf.y_rows[Rr:Rr + 4096].float()).all()
    # weights encoded beforehand (overlap = 2): same rows and outputs, bit for bit, and the codes are only read
    ref_y = buf.y_rows[:Rr].clone(); ref_out = buf.out.clone(); ref_wq = buf.w13_q.clone()
    buf.y_rows.fill_(float("nan")); buf.out.fill_(float("nan"))
    io = ctx.make_io(lg, isv, x, w13, w2, buf, cfg.rank, force=R.FP4, overlap=2)
    assert ctx.layer_forward(io) == R.FP4
    torch.cuda.synchronize()
    assert torch.equal(buf.y_rows[:Rr].view(torch.int16), ref_y.view(torch.int16))
    assert torch.equal(buf.out.view(torch.int16), ref_out.view(torch.int16))
    assert torch.equal(buf.w13_q, ref_wq)
    _say("c5: pre-encoded call reproduces the rows bit for bit")
    ctx.close()


def test_policy_variants_choose_the_oracles_fp4_sets():
    """The four policy variants of the threshold study (AIMD with either update order, the fixed thresholds M = 0 and
    M = 0.7) on two seeded iterations of the simulated trace -- a clustered and a scattered one -- with the routing
    statistics taken from the GPU and the state carried from the first iteration to the second: the FP4 sets, IB_global
    and M must be the oracle's, through the context call and through the host function."""
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config, select_precision_host
    cfg = W.CONFIGS["c4"]
    _, isv_np = W.gen_tokens(cfg, 0)
    isv = torch.from_numpy(isv_np).cuda()
    variants = {"aimd_update_first": dict(aimd_enabled=1, M_init=0.9, update_first=1),
                "aimd_decide_first": dict(aimd_enabled=1, M_init=0.9, update_first=0),
                "fixed_m1": dict(aimd_enabled=0, M_init=0.0, update_first=1),
                "fixed_m2": dict(aimd_enabled=0, M_init=0.7, update_first=1)}
    iterations = (10, 20)                                    # clustered block, scattered block of the trace generator
    stats = []
    rcfg0 = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
    ctx0 = R.Context(rcfg0)
    buf = R.LayerBuffers(rcfg0, cfg.T)
    for it in iterations:
        logits, info = W.gen_logits_trace(cfg, it, isv_np)
        ctx0.route_stats(torch.from_numpy(logits).cuda(), isv, buf)
        torch.cuda.synchronize()
        ids, _ = orouter.topk_route(logits, cfg.k)
        _, _, load, rvis = orouter.route_counts(ids, isv_np, cfg.E, cfg.D)
        assert same(buf.rank_load.cpu().numpy(), load) and same(buf.rank_vis.cpu().numpy(), rvis)
        stats.append((buf.rank_load.clone(), buf.rank_vis.clone(), load, rvis, info["kind"]))
    ctx0.close()
    assert {s[4] for s in stats} == {"clustered", "scattered"}
    fired = 0
    for name, kw in variants.items():
        rcfg = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
        rcfg.aimd_enabled, rcfg.M_init, rcfg.update_first = kw["aimd_enabled"], kw["M_init"], kw["update_first"]
        ctx = R.Context(rcfg)
        pc = opol.PolicyConfig(aimd_enabled=bool(kw["aimd_enabled"]), M_init=kw["M_init"], update_first=bool(kw["update_first"]))
        M_or = M_host = kw["M_init"]
        for load_d, vis_d, load, rvis, kind in stats:
            buf.rank_load.copy_(load_d); buf.rank_vis.copy_(vis_d)
            prec, ib, M_ctx = ctx.select_precision(buf, cfg.T)
            want = opol.select_precision(load, rvis, cfg.T, cfg.k, M_or, pc)
            M_or = want[2]
            ph, ibh, M_host = select_precision_host(rcfg, load, rvis, cfg.T, M_host)
            _say(f"policy {name} on a {kind} iteration: FP4 ranks {list(np.nonzero(prec)[0])}, IB_global {ib:.3f}, M {M_ctx}")
            assert list(prec) == list(want[0]) == list(ph)
            assert ib == want[1] == ibh and M_ctx == want[2] == M_host == ctx.M
            fired += int(np.sum(prec))
        ctx.close()
    assert fired > 0                                         # the cases are not vacuous: some variant converts some rank
