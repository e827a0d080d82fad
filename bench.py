#!/usr/bin/env python3
"""Benchmark of the ReaLB rank-layer hot path on one MI355X.

A step is one pass of the whole path -- route_stats, select_precision,
quantize_experts_fp4, permute, grouped_moe_ffn, combine --
over one synthetic batch that is already resident in HBM.

Default workload: the Kimi-VL-A3B-shaped rank share (64 experts, top-6, 8 local,
H 2048, I 1408, 16384 prefill tokens, 75 % vision, Zipf(1.1) skew towards this
rank's experts), forced to the FP4 path.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c1]
                  [--no-cpu-baseline] [--detail PATH]

Further reports (each prints its own JSON line; weights are drawn on the device,
N(0, 0.02), because only timing is taken):
  --workload c4   8 simulated EP ranks run one after the other on the one GPU, 20 seeded
                  iterations with the vision skew redrawn, AIMD state carried: max-over-ranks
                  layer time, all-BF16 versus the policy's mixed-precision plan.
  --workload c5   48 layers with distinct BF16 weight sets on a Qwen3-VL-shaped rank, 65536
                  tokens: per-layer time with the weight encoding on the side stream, on the
                  main stream, and skipped (weights encoded beforehand) -> exposed encoding time.
  --workload gate-sweep [--shape c2|c3]
                  the measured rank's layer time with FP4 forced (weight encoding included) and with BF16
                  forced, for batch sizes T = 64 .. 65536 (prefixes of one seeded batch): the smallest T from
                  which FP4 stays faster is this machine's value of the LB gate Gamma.
  --workload format-gap
                  quantization error (relative Frobenius, on the tensors and on a product X W^T) of MXFP4, the
                  format the GEMMs run on, against the paper's NVFP4 (groups of 16, E4M3 scale, global scale),
                  both encoded by this library's kernels, on synthetic weights, activations and a heavy-tailed
                  tensor; and the two encoders' throughput.
  --workload policy-ablation [--iterations N]
                  the 8-rank simulation over a longer trace; every rank is timed in both precisions each
                  iteration, and the policy variants (AIMD, fixed thresholds M = 0 and M = 0.7, decide-then-update,
                  FP4 everywhere) are evaluated on the same measurements: max-rank layer ms and the share of
                  rank-layers run in FP4.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"fp4": 10100.0, "bf16": 2500.0}     # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0
PREROLL_MS = 150.0                                  # untimed steps before the timed region, beyond --warmup
ENCODE_MODES = ("prefetch", "speculative", "side", "main")
MODE_ID = {"speculative": 3, "side": 1, "main": 0}


class LayerRun:
    """One workload's inputs, context and buffers on the device, and its step functions."""

    def __init__(self, workload, args, torch, W, R, default_config):
        self.torch, self.R, self.args = torch, R, args
        cfg = self.cfg = W.CONFIGS[workload]
        self.inp = W.gen_layer(cfg, 0)
        self.rcfg = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
        self.ctx = R.Context(self.rcfg)
        self.buf = R.LayerBuffers(self.rcfg, cfg.T)
        self.lg = torch.from_numpy(self.inp["logits"]).cuda()
        self.isv = torch.from_numpy(self.inp["is_vision"]).cuda()
        self.x, self.w13, self.w2 = (R.bf16_from_bits(self.inp[n]) for n in ("x", "w13", "w2"))
        self.reserve = args.reserve_cus
        self._pair = None

    def close(self):
        self.ctx.prefetch_join()
        self.torch.cuda.synchronize()
        self.ctx.close()

    def stepper(self, fp4: bool, mode: str):
        """A function that runs one whole rank-layer step.  mode "prefetch": the steady state of a layer pipeline --
        two layers with distinct weights alternate, each call consumes the FP4 weights the previous call encoded beside
        its GEMMs and encodes the other layer's weights beside its own (every step still encodes one full weight set)."""
        R, ctx = self.R, self.ctx
        force = R.FP4 if fp4 else R.BF16
        if not (fp4 and mode == "prefetch"):
            io = ctx.make_io(self.lg, self.isv, self.x, self.w13, self.w2, self.buf, self.cfg.rank, force=force, overlap=MODE_ID[mode])
            return lambda: ctx.layer_forward(io)
        if self._pair is None:
            import workloads as W
            wB = tuple(R.bf16_from_bits(a) for a in W.gen_weights(self.cfg, 1))
            self._pair = ([(self.w13, self.w2), wB], [R.WeightBuffers(self.rcfg), R.WeightBuffers(self.rcfg)])
        ws, wbufs = self._pair
        ios = []
        for i in (0, 1):
            io = ctx.make_io(self.lg, self.isv, self.x, ws[i][0], ws[i][1], self.buf, self.cfg.rank, force=force, overlap=4)
            ctx.use_weight_buffers(io, wbufs[i])
            ctx.set_prefetch(io, ws[1 - i][0], ws[1 - i][1], wbufs[1 - i], self.reserve)
            ios.append(io)
        ctx.quantize_experts_fp4(ws[0][0], ws[0][1], wbufs[0])           # the first layer has nobody to prefetch for it
        state = {"i": 0}

        def step():
            ctx.layer_forward(ios[state["i"]])
            state["i"] ^= 1
        return step

    def stage_pass(self, step, steps):
        """Mean GPU ms per stage of the layer call over `steps` steps (library-recorded events)."""
        ctx = self.ctx
        ctx.stage_timing(True)
        acc = {}
        for _ in range(steps):
            step()
            for n, v in ctx.stage_ms().items():
                acc[n] = acc.get(n, 0.0) + v
        ctx.stage_timing(False)
        return {n: v / steps for n, v in acc.items()}

    def brief(self, fp4: bool, mode: str, warm: int = 30, steps: int = 30):
        """A short timing of the layer in one precision: ms per step, FFN rate, GEMM stage times."""
        torch = self.torch
        step = self.stepper(fp4, mode)
        for _ in range(warm):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        st = self.stage_pass(step, 10)
        self.ctx.prefetch_join()
        rows = int(self.buf.expert_offsets[-1].item())
        flops = 6.0 * rows * self.cfg.H * self.cfg.I
        peak = PEAK_TFLOPS["fp4" if fp4 else "bf16"]
        gemm = flops / ((st["gate_up"] + st["down"]) * 1e-3) / 1e12
        return {"layer_ms": ms, "rows_on_rank": rows, "step_tflops": flops / (ms * 1e-3) / 1e12, "encode_mode": mode if fp4 else None,
                "gate_up_ms": st["gate_up"], "down_ms": st["down"], "grouped_gemm_tflops": gemm, "grouped_gemm_frac_of_peak": gemm / peak,
                "gate_up_frac_of_peak": 4.0 * rows * self.cfg.H * self.cfg.I / (st["gate_up"] * 1e-3) / 1e12 / peak}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20, help="untimed steps first (a fixed 150 ms pre-roll follows in any case: the clocks need about 100 ms of load to settle)")
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "gate-sweep", "policy-ablation", "format-gap"],
                    help="c2 (default) is the headline line; c4 = 8-rank imbalance simulation, c5 = 48-layer overlap stress, "
                         "gate-sweep = FP4 vs BF16 layer time over the batch size (locates the LB gate), "
                         "policy-ablation = AIMD / fixed-threshold variants on a longer simulated trace, "
                         "format-gap = quantization error of the MXFP4 mapping against the paper's NVFP4")
    ap.add_argument("--shape", default="c2", choices=["c2", "c3"], help="layer shape of the gate sweep")
    ap.add_argument("--iterations", type=int, default=100, help="trace length of the policy ablation")
    ap.add_argument("--precision", default="fp4", choices=["fp4", "bf16"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--encode-mode", default="speculative", choices=list(ENCODE_MODES),
                    help="where the FP4 weight encoding runs: speculative (default) = side stream ahead of the decision, beside the routing and "
                         "index kernels; prefetch = layer pipeline, each step encodes the next layer's weights on the side stream beside "
                         "its own GEMMs; main = caller's "
                         "stream after the decision; side = side stream after the decision (under the permutation).  The step is timed "
                         "in all of them, in rotated order, and reported under extra")
    ap.add_argument("--reserve-cus", type=int, default=0, help="compute units the GEMMs leave to the encoder in prefetch mode")
    ap.add_argument("--only-headline", action="store_true",
                    help="time the headline placement only (profiling runs: every launch of a kernel then belongs to the same placement)")
    ap.add_argument("--no-compare", action="store_true", help="skip the brief BF16 pass and the c3 pair folded into the default line")
    ap.add_argument("--gemm-tile", type=int, default=0, choices=[0, 2, 8, 16], help="grouped-GEMM block tile selector (0 = automatic)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 512 MiB device copy (untimed) so that a counter run can scale FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--detail", default=None, help="write the per-kernel breakdown (JSON) to this path")
    return ap.parse_args()


def event_ms(fn, steps, torch):
    """Average duration of fn() on the current stream, HIP events around each call."""
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return sum(ts) / len(ts), ts[len(ts) // 2]


def cpu_baseline(cfg, inp, prec_fp4: bool, budget_s: float = 12.0):
    """The oracle, untuned, on a bounded sample of the same workload: routing of the
    whole batch, then -- one local expert after the other until `budget_s` seconds
    are spent or the rank's experts are exhausted -- weight encoding, permutation,
    FFN and combine of that expert's rows."""
    import numpy as np
    from oracle import router, permute, mxfp4, ffn
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    t0 = time.perf_counter()
    ids, w = router.topk_route(inp["logits"], cfg.k)
    router.route_counts(ids, inp["is_vision"], cfg.E, cfg.D)
    nl = cfg.n_local
    rows, done = 0, 0
    for e in range(nl):
        off, r2a, a2r = permute.permute_indices(ids, cfg.rank * nl + e, 1)
        xperm = permute.gather_rows(inp["x"], r2a, cfg.k)
        w13, w2 = inp["w13"][e:e + 1], inp["w2"][e:e + 1]
        if prec_fp4:
            w13q, w13s = mxfp4.quantize(w13)
            w2q, w2s = mxfp4.quantize(w2)
            xq, xs = mxfp4.quantize(xperm)
            _, _, y = ffn.ffn_fp4(xq, xs, w13q, w13s, w2q, w2s, off)
        else:
            _, y = ffn.ffn_bf16(xperm, w13, w2, off)
        out = ffn.combine(ffn.to_bf16_bits(y), a2r, w, cfg.T, cfg.k)
        ffn.to_bf16_bits(out)
        rows += int(off[-1])
        done += 1
        if time.perf_counter() - t0 >= budget_s:
            break
    dt = time.perf_counter() - t0
    flops = 6.0 * rows * cfg.H * cfg.I
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"routing of all {cfg.T} tokens, then weight encoding, permutation, FP64 FFN and combine for "
                      f"{done} of the rank's {nl} experts ({rows} rows), {dt:.1f} s", "seconds": dt, "rows": rows}


def _device_weights(torch, n, H, I, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    w13 = (torch.randn((n, 2 * I, H), generator=g, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
    w2 = (torch.randn((n, H, I), generator=g, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
    return w13, w2


def run_c4(args):
    """Simulated 8-rank EP imbalance (latency objective T_MoE = max_i T_i of the paper's
    problem formulation): every rank's share runs serially on the one GPU."""
    import numpy as np
    import torch
    import workloads as W
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config
    cfg = W.CONFIGS["c4"]
    iters = 20
    rcfg = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
    ctx = R.Context(rcfg)
    buf = R.LayerBuffers(rcfg, cfg.T)
    xb, isv_np = W.gen_tokens(cfg, 0)
    x = R.bf16_from_bits(xb)
    isv = torch.from_numpy(isv_np).cuda()
    weights = [_device_weights(torch, cfg.n_local, cfg.H, cfg.I, 100 + d) for d in range(cfg.D)]
    reps = max(1, min(args.steps, 5))
    per_iter = []
    ctx.M = rcfg.M_init
    for it in range(iters):
        logits_np, info = W.gen_logits_c4(cfg, it, isv_np)
        lg = torch.from_numpy(logits_np).cuda()
        ctx.route_stats(lg, isv, buf)
        prec, ib, M = ctx.select_precision(buf, cfg.T)
        load = buf.rank_load.cpu().numpy()
        vis = buf.rank_vis.cpu().numpy()
        t_bf16, t_plan = [], []
        for d in range(cfg.D):
            w13, w2 = weights[d]
            io = ctx.make_io(lg, isv, x, w13, w2, buf, d, overlap=True)
            for which, p in (("bf16", R.BF16), ("plan", int(prec[d]))):
                if which == "plan" and p == R.BF16:
                    t_plan.append(t_bf16[-1])
                    continue
                ctx.rank_forward(io, p)                      # warm-up
                avg, _ = event_ms(lambda: ctx.rank_forward(io, p), reps, torch)
                (t_bf16 if which == "bf16" else t_plan).append(avg)
        per_iter.append({"iteration": it, "kind": info["kind"], "hot_rank": info["hot_rank"], "ib_global": round(ib, 3),
                         "M": M, "fp4_ranks": [int(d) for d in np.nonzero(prec)[0]],
                         "rank_vision_share": [round(float(v) / max(int(l), 1), 3) for v, l in zip(vis, load)],
                         "rank_ms_bf16": [round(t, 4) for t in t_bf16], "rank_ms_plan": [round(t, 4) for t in t_plan],
                         "max_ms_bf16": max(t_bf16), "max_ms_plan": max(t_plan),
                         "straggler_bf16": int(np.argmax(t_bf16)), "straggler_plan": int(np.argmax(t_plan))})
    mb = float(np.mean([p["max_ms_bf16"] for p in per_iter]))
    mp = float(np.mean([p["max_ms_plan"] for p in per_iter]))
    best = max(p["max_ms_bf16"] / p["max_ms_plan"] for p in per_iter)
    result = {"metric": "max-rank MoE layer ms (mean over 20 iterations of max over 8 simulated ranks), mixed-precision plan",
              "value": mp, "unit": "ms", "n_gpus": 1, "steps": iters, "warmup": 1, "ms_per_step": mp,
              "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16 / fp4 per rank (policy)",
              "data": "synthetic",
              "config": {"workload": "c4: Kimi-VL-shaped layer, 64 experts top-6, 8 ranks x 8 experts run serially, T=16384, "
                                     "70% vision, skew redrawn per iteration, AIMD carried"},
              "extra": {"max_rank_ms_all_bf16": mb, "max_rank_ms_plan": mp, "mean_speedup": mb / mp, "best_iteration_speedup": best,
                        "iterations_with_fp4": sum(1 for p in per_iter if p["fp4_ranks"]),
                        "paper_context": "paper: average MoE layer latency 1.51 -> 1.36 ms, rank-level up to 1.29x (8x RTX 5090)"}}
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump({"result": result, "iterations": per_iter}, f, indent=1)
    ctx.close()
    print(json.dumps(result))


def run_c5(args):
    """Overlap stress: how much of the on-the-fly weight transformation stays exposed when it
    runs on the side stream under the permutation (the paper hides it under dispatch)."""
    import numpy as np
    import torch
    import workloads as W
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config
    cfg = W.CONFIGS["c5"]
    layers = 48
    rcfg = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
    ctx = R.Context(rcfg)
    buf = R.LayerBuffers(rcfg, cfg.T)
    xb, isv_np = W.gen_tokens(cfg, 0)
    x = R.bf16_from_bits(xb)
    isv = torch.from_numpy(isv_np).cuda()
    lg = torch.from_numpy(W.gen_logits(cfg, 0, isv_np)).cuda()
    weights = [_device_weights(torch, cfg.n_local, cfg.H, cfg.I, 200 + l) for l in range(layers)]
    ios = {mode: [ctx.make_io(lg, isv, x, w13, w2, buf, cfg.rank, force=R.FP4, overlap=mode) for (w13, w2) in weights]
           for mode in (0, 1, 3)}

    def sweep(mode):
        for l in range(layers):
            ctx.layer_forward(ios[mode][l])

    def timed(mode):
        sweep(mode)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(max(1, min(args.steps, 5))):
            sweep(mode)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / (layers * max(1, min(args.steps, 5)))

    # cross-layer prefetch: layer l consumes what layer l-1's call encoded beside its GEMMs and encodes layer l+1's
    # weights beside its own; the GEMMs' persistent grids leave `reserve` compute units to the encoder
    pair = [R.WeightBuffers(rcfg), R.WeightBuffers(rcfg)]
    ms_prefetch = {}
    for reserve in ((args.reserve_cus,) if args.steps < 3 else (0, 8, 16, 24, 32, 48)):
        pios = []
        for l in range(layers):
            io = ctx.make_io(lg, isv, x, weights[l][0], weights[l][1], buf, cfg.rank, force=R.FP4, overlap=4)
            ctx.use_weight_buffers(io, pair[l & 1])
            nw = weights[(l + 1) % layers]
            ctx.set_prefetch(io, nw[0], nw[1], pair[(l + 1) & 1], reserve)
            pios.append(io)
        ios[("prefetch", reserve)] = pios
        ctx.quantize_experts_fp4(weights[0][0], weights[0][1], pair[0])
        ms_prefetch[reserve] = timed(("prefetch", reserve))
        ctx.prefetch_join()
        torch.cuda.synchronize()
    best_reserve = min(ms_prefetch, key=ms_prefetch.get)
    ms_overlap = timed(1)
    ms_seq = timed(0)
    ms_spec = timed(3)
    # weights encoded beforehand: one layer's buffers reused (the GEMMs read the same bytes each time)
    io2 = ctx.make_io(lg, isv, x, weights[0][0], weights[0][1], buf, cfg.rank, force=R.FP4, overlap=0)
    ctx.layer_forward(io2)
    io2.overlap = 2
    torch.cuda.synchronize()
    reps = layers * max(1, min(args.steps, 5))
    ctx.layer_forward(io2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        ctx.layer_forward(io2)
    torch.cuda.synchronize()
    ms_noquant = (time.perf_counter() - t0) * 1e3 / reps
    qms, _ = event_ms(lambda: ctx.quantize_experts_fp4(weights[1][0], weights[1][1], buf), 20, torch)
    n_w = cfg.n_local * 3 * cfg.H * cfg.I
    rows = int(buf.expert_offsets[-1].item())
    ms_pf = ms_prefetch[best_reserve]
    result = {"metric": "per-layer ms over 48 layers of distinct weights, FP4 path, each layer's weights encoded beside the previous layer's GEMMs",
              "value": ms_pf, "unit": "ms", "n_gpus": 1, "steps": layers, "warmup": layers, "ms_per_step": ms_pf,
              "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
              "dtype": "fp4 (MXFP4 E2M1 + E8M0/32, fp32 accumulate)", "data": "synthetic",
              "config": {"workload": "c5: Qwen3-VL-shaped rank, 128 experts top-8, 16 local, H=2048 I=768, T=65536 tokens, "
                                     "85% vision, 48 distinct BF16 weight sets"},
              "extra": {"rows_on_rank": rows, "layer_ms_prefetch_by_reserved_cus": {str(k_): round(v, 5) for k_, v in ms_prefetch.items()},
                        "reserved_cus": best_reserve, "exposed_encoding_ms_prefetch": ms_pf - ms_noquant,
                        "layer_ms_overlap": ms_overlap, "layer_ms_sequential": ms_seq,
                        "layer_ms_weights_pre_encoded": ms_noquant, "exposed_encoding_ms_overlap": ms_overlap - ms_noquant,
                        "exposed_encoding_ms_sequential": ms_seq - ms_noquant, "layer_ms_speculative": ms_spec,
                        "exposed_encoding_ms_speculative": ms_spec - ms_noquant, "encoder_alone_ms": qms,
                        "encoder_alone_gbs": n_w * 2.53125 / (qms * 1e-3) / 1e9,
                        "paper_context": "paper: hiding the transformation is worth 3% end to end (ReaLB vs ReaLB-seq)"}}
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump({"result": result}, f, indent=1)
    ctx.close()
    print(json.dumps(result))


def run_gate_sweep(args):
    """Batch-threshold study (the paper's LB gate, Sec. "LB Gate"): below some batch size the GEMMs no
    longer dominate and switching to FP4, which costs the weight transformation, does not pay."""
    import numpy as np
    import torch
    import workloads as W
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config
    base = W.CONFIGS[args.shape]
    T_max = 65536
    cfg = W.scaled(base, T=T_max)
    rcfg = default_config(T_max, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
    ctx = R.Context(rcfg)
    buf = R.LayerBuffers(rcfg, T_max)
    xb, isv_np = W.gen_tokens(cfg, 0)
    logits_np = W.gen_logits(cfg, 0, isv_np)
    x_all = R.bf16_from_bits(xb)
    isv_all = torch.from_numpy(isv_np).cuda()
    lg_all = torch.from_numpy(logits_np).cuda()
    w13, w2 = _device_weights(torch, cfg.n_local, cfg.H, cfg.I, 300)
    steps = max(5, min(args.steps, 30))
    rows_out, gamma = [], None
    for T in (64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384, 32768, 65536):
        x, isv, lg = x_all[:T], isv_all[:T], lg_all[:T]
        ms = {}
        for name, force, mode in (("bf16", R.BF16, 3), ("fp4", R.FP4, 3), ("fp4_side", R.FP4, 1)):
            io = ctx.make_io(lg, isv, x, w13, w2, buf, cfg.rank, force=force, overlap=mode)
            io.T = T
            for _ in range(3):
                ctx.layer_forward(io)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                ctx.layer_forward(io)
            torch.cuda.synchronize()
            ms[name] = (time.perf_counter() - t0) * 1e3 / steps
        rows = int(buf.expert_offsets[-1].item())
        rows_out.append({"T": T, "rows_on_rank": rows, "ms_bf16": round(ms["bf16"], 5), "ms_fp4": round(ms["fp4"], 5),
                         "ms_fp4_encode_after_decision": round(ms["fp4_side"], 5),
                         "fp4_speedup": round(ms["bf16"] / ms["fp4"], 3),
                         "fp4_speedup_encode_after_decision": round(ms["bf16"] / ms["fp4_side"], 3)})
    gamma_side = None
    for r in reversed(rows_out):                      # smallest T from which FP4 stays faster
        if r["fp4_speedup"] > 1.0:
            gamma = r["T"]
        else:
            break
    for r in reversed(rows_out):
        if r["fp4_speedup_encode_after_decision"] > 1.0:
            gamma_side = r["T"]
        else:
            break
    result = {"metric": "LB gate on MI355X: smallest batch size T from which the FP4 layer (weight encoding included) stays faster than BF16",
              "value": gamma, "unit": "tokens", "n_gpus": 1, "steps": steps, "warmup": 3, "ms_per_step": None,
              "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16 vs fp4", "data": "synthetic",
              "config": {"workload": f"gate-sweep on the {args.shape} layer shape ({cfg.E} experts top-{cfg.k}, {cfg.n_local} local, "
                                     f"H={cfg.H} I={cfg.I}), hot rank, prefixes of one seeded 65536-token batch"},
              "extra": {"gate_with_encoding_after_the_decision": gamma_side, "sweep": rows_out, "paper_context": "paper: Gamma = 2048 tokens (256 per rank x 8 ranks) on RTX 5090"}}
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump({"result": result}, f, indent=1)
    ctx.close()
    print(json.dumps(result))


def run_policy_ablation(args):
    """AIMD against the fixed-threshold variants (the paper's ReaLB-m1 / -m2) and the other update
    order, on one longer simulated trace: every rank is timed in both precisions, so that all variants
    are evaluated on identical measurements."""
    import numpy as np
    import torch
    import workloads as W
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config, select_precision_host
    cfg = W.CONFIGS["c4"]
    iters = args.iterations
    rcfg = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
    ctx = R.Context(rcfg)
    buf = R.LayerBuffers(rcfg, cfg.T)
    xb, isv_np = W.gen_tokens(cfg, 0)
    x = R.bf16_from_bits(xb)
    isv = torch.from_numpy(isv_np).cuda()
    weights = [_device_weights(torch, cfg.n_local, cfg.H, cfg.I, 100 + d) for d in range(cfg.D)]
    reps = 3
    t_b = np.zeros((iters, cfg.D)); t_f = np.zeros((iters, cfg.D))
    loads = np.zeros((iters, cfg.D), dtype=np.int64); viss = np.zeros((iters, cfg.D), dtype=np.int64)
    kinds = []
    for it in range(iters):
        logits_np, info = W.gen_logits_trace(cfg, it, isv_np)
        kinds.append(info["kind"])
        lg = torch.from_numpy(logits_np).cuda()
        ctx.route_stats(lg, isv, buf)
        torch.cuda.synchronize()
        loads[it] = buf.rank_load.cpu().numpy(); viss[it] = buf.rank_vis.cpu().numpy()
        for d in range(cfg.D):
            w13, w2 = weights[d]
            io = ctx.make_io(lg, isv, x, w13, w2, buf, d, overlap=True)
            for p, arr in ((R.BF16, t_b), (R.FP4, t_f)):
                ctx.rank_forward(io, p)
                arr[it, d], _ = event_ms(lambda: ctx.rank_forward(io, p), reps, torch)

    def variant(name, aimd, M0, update_first, force=R.FORCE_NONE):
        c = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
        c.aimd_enabled, c.M_init, c.update_first = aimd, M0, update_first
        M, tmax, traj = M0, [], []
        nf4 = {"calm": 0, "clustered": 0, "scattered": 0}
        for it in range(iters):
            prec, ib, M = select_precision_host(c, loads[it], viss[it], cfg.T, M, force)
            t = np.where(np.asarray(prec) == R.FP4, t_f[it], t_b[it])
            tmax.append(float(t.max())); nf4[kinds[it]] += int(np.sum(np.asarray(prec) == R.FP4)); traj.append(round(M, 3))
        per_kind = {k: round(nf4[k] / max(1, kinds.count(k) * cfg.D), 4) for k in nf4}
        ms_kind = {k: round(float(np.mean([tmax[i] for i in range(iters) if kinds[i] == k] or [0.0])), 5) for k in nf4}
        return {"variant": name, "max_rank_ms": float(np.mean(tmax)), "max_rank_ms_by_regime": ms_kind,
                "fp4_share_of_rank_layers": sum(nf4.values()) / (iters * cfg.D), "fp4_share_by_regime": per_kind,
                "M_trajectory_first_40": traj[:40]}

    base = float(np.mean(t_b.max(axis=1)))
    variants = [variant("ReaLB (AIMD, update then decide)", 1, 0.9, 1),
                variant("AIMD, decide then update", 1, 0.9, 0),
                variant("fixed M = 0 (ReaLB-m1)", 0, 0.0, 1),
                variant("fixed M = 0.7 (ReaLB-m2)", 0, 0.7, 1),
                variant("fixed M = 0.9", 0, 0.9, 1),
                variant("FP4 on every rank", 0, 0.9, 1, force=R.FP4)]
    for v in variants:
        v["speedup_vs_all_bf16"] = base / v["max_rank_ms"]
    best = float(np.mean(np.minimum(t_b, t_f).max(axis=1)))
    result = {"metric": "max-rank MoE layer ms over a simulated trace, AIMD policy",
              "value": variants[0]["max_rank_ms"], "unit": "ms", "n_gpus": 1, "steps": iters, "warmup": 1,
              "ms_per_step": variants[0]["max_rank_ms"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
              "dtype": "bf16 / fp4 per rank (policy)", "data": "synthetic",
              "config": {"workload": f"policy-ablation: c4's 8-rank layer over a {iters}-iteration trace whose imbalance comes and goes "
                                     "(blocks of 10 iterations: calm / clustered / scattered), every rank timed in both precisions"},
              "extra": {"max_rank_ms_all_bf16": base, "max_rank_ms_per_rank_minimum": best,
                        "max_rank_ms_all_bf16_by_regime": {k: round(float(np.mean([t_b[i].max() for i in range(iters) if kinds[i] == k] or [0.0])), 5)
                                                           for k in ("calm", "clustered", "scattered")},
                        "ib_global_by_regime": {k: round(float(np.mean([loads[i].max() * cfg.D / (cfg.T * cfg.k) for i in range(iters) if kinds[i] == k] or [0.0])), 3)
                                                for k in ("calm", "clustered", "scattered")},
                        "variants": variants,
                        "ib_global_mean": float(np.mean(loads.max(axis=1) * cfg.D / (cfg.T * cfg.k))),
                        "paper_context": "paper: ReaLB 1.32x / m1 1.33x / m2 1.22x end to end on Kimi-VL MMMU; accuracy drops more with m1"}}
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump({"result": result}, f, indent=1)
    ctx.close()
    print(json.dumps(result))


def run_format_gap(args):
    """What the mapping of the paper's NVFP4 onto MXFP4 costs in accuracy, on synthetic tensors.  Both
    encodings come from the library's kernels; decoding and the reference products are analysis code
    (torch, FP32/FP64), not part of the product path."""
    import numpy as np
    import torch
    import workloads as W
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import scales_to_canonical
    cfg = W.CONFIGS["c2"]
    e2m1 = torch.tensor([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0, -0.0, -0.5, -1.0, -1.5, -2.0, -3.0, -4.0, -6.0],
                        dtype=torch.float64, device="cuda")

    def codes_to_values(q):
        lo, hi = (q & 0xF).long(), (q >> 4).long()
        return torch.stack([e2m1[lo], e2m1[hi]], dim=-1).reshape(q.shape[0], -1)

    def dec_mx(q, s, rows, K):
        sc = torch.from_numpy(scales_to_canonical(s, rows, K).astype(np.int64)).cuda()
        return (codes_to_values(q).reshape(rows, K // 32, 32) * torch.ldexp(torch.ones((), dtype=torch.float64, device="cuda"), sc - 127)[..., None]).reshape(rows, K)

    def dec_nv(q, s, g, rows, K):
        b = s.long()
        e, m = b >> 3, b & 7
        val = torch.where(e == 0, m.double() * 2.0 ** -9, (1 + m.double() / 8) * torch.ldexp(torch.ones((), dtype=torch.float64, device="cuda"), e - 7))
        s_eff = (val.float() * np.float32(g)).double()
        return (codes_to_values(q).reshape(rows, K // 16, 16) * s_eff[..., None]).reshape(rows, K)

    rng = np.random.default_rng(77)
    w = R.bf16_from_bits(W.gen_weights(cfg, 0, n_experts=1)[0][0])                        # [2I, H] ~ N(0, 0.02)
    xa = R.bf16_from_bits(W.gen_tokens(W.scaled(cfg, T=4096), 0)[0])                       # [4096, H] ~ N(0, 1)
    ht = rng.standard_normal((4096, cfg.H)).astype(np.float32)
    ht[rng.integers(4096, size=400), rng.integers(cfg.H, size=400)] *= 30.0                # heavy tail: 0.005 % outliers x30
    ht = R.bf16_from_bits(W.f32_to_bf16_bits(ht))
    report = {}
    dec = {}
    for name, t in (("weights N(0,0.02)", w), ("activations N(0,1)", xa), ("activations with x30 outliers", ht)):
        rows, K = t.shape
        ref = t.double()
        q, s = R.quantize_rows_fp4(t)
        mx = dec_mx(q, s, rows, K)
        g = float(np.float32(np.float32(float(R.amax_bf16(t).cpu()[0])) / np.float32(6.0 * 448.0)))
        qn, sn = R.quantize_rows_nvfp4(t, g)
        nv = dec_nv(qn, sn, g, rows, K)
        dec[name] = (ref, mx, nv)
        fro = lambda a: float(torch.linalg.norm(a - ref) / torch.linalg.norm(ref))
        t_mx, _ = event_ms(lambda: R.quantize_rows_fp4(t), 20, torch)
        t_nv, _ = event_ms(lambda: R.quantize_rows_nvfp4(t, g), 20, torch)
        report[name] = {"shape": [rows, K], "rel_fro_error_mxfp4": fro(mx), "rel_fro_error_nvfp4": fro(nv),
                        "bytes_per_element_mxfp4": 0.5 + 1 / 32, "bytes_per_element_nvfp4": 0.5 + 1 / 16,
                        "encoder_gbs_mxfp4": rows * K * (2 + 0.5 + 1 / 32) / (t_mx * 1e-3) / 1e9,
                        "encoder_gbs_nvfp4": rows * K * (2 + 0.5 + 1 / 16) / (t_nv * 1e-3) / 1e9}
    prod = {}
    for xname in ("activations N(0,1)", "activations with x30 outliers"):
        xr, xm, xn = dec[xname]
        wr, wm, wn = dec["weights N(0,0.02)"]
        exact = xr @ wr.T
        fro = lambda a: float(torch.linalg.norm(a - exact) / torch.linalg.norm(exact))
        prod[xname + " x weights^T"] = {"rel_fro_error_mxfp4": fro(xm @ wm.T), "rel_fro_error_nvfp4": fro(xn @ wn.T)}
    worst = max(v["rel_fro_error_mxfp4"] / v["rel_fro_error_nvfp4"] for v in prod.values())
    result = {"metric": "W4A4 product error of MXFP4 relative to NVFP4 (ratio of relative Frobenius errors, worst case)",
              "value": worst, "unit": "x", "n_gpus": 1, "steps": 20, "warmup": 1, "ms_per_step": None, "higher_is_better": False,
              "scaling": "weak", "vs_baseline": None, "dtype": "fp4 encodings of bf16 tensors", "data": "synthetic",
              "config": {"workload": "format-gap: Kimi-shaped expert weights [2816,2048], 4096 activation rows, and the same with outliers"},
              "extra": {"tensors": report, "products": prod}}
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump({"result": result}, f, indent=1)
    print(json.dumps(result))


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (one EP rank's share per GPU); --gpus {args.gpus} is not supported",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import workloads as W
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.gemm_tile:
        from paper_2604_19503_amd.binding import set_gemm_tile
        set_gemm_tile(args.gemm_tile)
    if args.workload == "c4":
        return run_c4(args)
    if args.workload == "c5":
        return run_c5(args)
    if args.workload == "gate-sweep":
        return run_gate_sweep(args)
    if args.workload == "policy-ablation":
        return run_policy_ablation(args)
    if args.workload == "format-gap":
        return run_format_gap(args)
    cfg = W.CONFIGS[args.workload]
    fp4 = args.precision == "fp4"
    lr = LayerRun(args.workload, args, torch, W, R, default_config)
    mode = args.encode_mode if fp4 else "main"

    # ---- warm-up: the driver's W steps, then a fixed, declared pre-roll (the clocks need about 100 ms of load to settle)
    step = lr.stepper(fp4, mode)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    preroll_steps = 0
    while (time.perf_counter() - t0) * 1e3 < PREROLL_MS:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
        preroll_steps += 20
    preroll_ms = (time.perf_counter() - t0) * 1e3

    # ---- timed region: exactly K steps of the headline placement.  The other placements of the weight encoding are
    #      timed beside it in rotated order (K steps each as well, in `rounds` chunks), so that no placement always
    #      runs first or last.
    modes = [mode] + [m for m in ENCODE_MODES if m != mode] if (fp4 and not args.only_headline) else [mode]
    steppers = {m: (step if m == mode else lr.stepper(fp4, m)) for m in modes}
    rounds = max(1, min(4, args.steps // 10))             # chunks of at least 10 steps: a chunk's first step starts on an idle GPU
    chunk = [args.steps // rounds + (1 if r < args.steps % rounds else 0) for r in range(rounds)]
    total = {m: 0.0 for m in modes}
    for r in range(rounds):
        order = modes[r % len(modes):] + modes[:r % len(modes)]
        for m in order:
            f = steppers[m]
            if m != mode or r > 0:
                f(); f()                                  # (switching placements: two untimed steps)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(chunk[r]):
                f()
            torch.cuda.synchronize()
            total[m] += time.perf_counter() - t1
    lr.ctx.prefetch_join()
    by_mode = {m: total[m] * 1e3 / args.steps for m in modes}
    ms_step = by_mode[mode]
    rows = int(lr.buf.expert_offsets[-1].item())
    H, I, T, k = cfg.H, cfg.I, cfg.T, cfg.k
    ffn_flops = 6.0 * rows * H * I

    # ---- the stages of the very call the step makes, timed by events the library records at its stage boundaries
    #      (a separate pass of K steps: the events cost a few microseconds per call)
    layer_stages = lr.stage_pass(step, args.steps)

    # ---- the entry points one by one on the same stream (separate pass)
    n_w = cfg.n_local * 3 * H * I
    ctx, buf, x, w13, w2, lg, isv = lr.ctx, lr.buf, lr.x, lr.w13, lr.w2, lr.lg, lr.isv
    force = R.FP4 if fp4 else R.BF16
    tok_local = int((buf.assign_to_row.view(T, k) >= 0).any(dim=1).sum().item())
    stages = {}

    def add(name, fn, work, unit_kind):
        avg, med = event_ms(fn, args.steps, torch)
        stages[name] = {"ms": avg, "ms_median": med, "work": work, "kind": unit_kind}

    add("route_stats", lambda: ctx.route_stats(lg, isv, buf), T * (4 * cfg.E + 1 + 8 * k), "bytes")
    add("quantize_experts_fp4", lambda: ctx.quantize_experts_fp4(w13, w2, buf), n_w * 2.53125, "bytes")
    row_out = (H // 2 + H // 32 + 4) if fp4 else (2 * H + 4)
    add("permute", lambda: ctx.permute(x, buf, cfg.rank, force), tok_local * 2 * H + 4 * T * k + rows * row_out, "bytes")
    add("ffn_gate_up", lambda: ctx.grouped_moe_ffn_gate_up(force, w13, buf), 4.0 * rows * H * I, "flops")
    add("ffn_down", lambda: ctx.grouped_moe_ffn_down(force, w2, buf), 2.0 * rows * H * I, "flops")
    add("combine", lambda: ctx.combine(buf), rows * 2 * H + T * 8 * k + T * 2 * H, "bytes")
    for st in stages.values():
        st["rate"] = st["work"] / (st["ms"] * 1e-3) / (1e12 if st["kind"] == "flops" else 1e9)
        st["unit"] = "TFLOP/s" if st["kind"] == "flops" else "GB/s"

    # ---- roofline of the dominant kernel of the step: the gate/up GEMM as the layer call launches it (rows fetched
    #      through row_to_assign), from the stage pass above
    peak = PEAK_TFLOPS[args.precision]
    gu_ms, dn_ms = layer_stages["gate_up"], layer_stages["down"]
    gu_rate = 4.0 * rows * H * I / (gu_ms * 1e-3) / 1e12
    dn_rate = 2.0 * rows * H * I / (dn_ms * 1e-3) / 1e12
    kernel = f"ffn_gemm256_kernel<{str(fp4).lower()}, true, true>"
    roofline = {"kernel": kernel, "what": "gate/up grouped GEMM + SwiGLU as launched by realb_layer_forward (activation rows fetched through row_to_assign)",
                "bound": "mfma", "achieved": gu_rate, "peak": peak, "unit": "TFLOP/s", "frac": gu_rate / peak, "traffic": None, "ms": gu_ms}
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")      # HBM bytes per launch from the committed counter runs, keyed by kernel
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            roofline["traffic"] = json.load(f).get(f"{args.workload}_{args.precision}:{kernel}")
    if args.calibrate_copy:
        src = torch.ones(128 << 20, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)                      # 512 MiB read + 512 MiB written per launch
        torch.cuda.synchronize()
        del src, dst

    ffn_ms = gu_ms + dn_ms
    extra = {
        "rows_on_rank": rows,
        "preroll_ms": round(preroll_ms, 1), "preroll_steps": preroll_steps,
        "grouped_gemm_tflops": ffn_flops / (ffn_ms * 1e-3) / 1e12,
        "grouped_gemm_frac_of_peak": ffn_flops / (ffn_ms * 1e-3) / 1e12 / peak,
        "gate_up_frac_of_peak": gu_rate / peak, "down_tflops": dn_rate, "down_frac_of_peak": dn_rate / peak,
        "down_frac_of_hbm": (rows * (2 * H + (I * 17 / 32 if fp4 else 2 * I)) / (dn_ms * 1e-3) / 1e9) / PEAK_HBM_GBS,
        "quantizer_gbs": stages["quantize_experts_fp4"]["rate"],
        "quantizer_frac_of_hbm": stages["quantize_experts_fp4"]["rate"] / PEAK_HBM_GBS,
        "layer_ms": ms_step,
        "layer_ms_by_encode_mode": {k_: round(v, 5) for k_, v in by_mode.items()},
        "layer_stages_ms": {n: round(v, 5) for n, v in layer_stages.items()},
        "entry_point_ms": {n: round(st["ms"], 5) for n, st in stages.items()},
    }
    if fp4 and mode == "prefetch":
        extra["reserve_cus"] = lr.reserve
    # ---- the other half of the metric ("BF16 vs FP4") and the Qwen-shaped layer, briefly, in the same run
    if not args.no_compare and args.workload == "c2":
        other = lr.brief(not fp4, "main" if fp4 else args.encode_mode)
        extra["same_layer_" + ("bf16" if fp4 else "fp4")] = other
        extra["fp4_speedup_over_bf16"] = (other["layer_ms"] / ms_step) if fp4 else (ms_step / other["layer_ms"])
        lr3 = LayerRun("c3", args, torch, W, R, default_config)
        extra["c3"] = {"fp4": lr3.brief(True, args.encode_mode), "bf16": lr3.brief(False, "main")}
        extra["c3"]["fp4_speedup_over_bf16"] = extra["c3"]["bf16"]["layer_ms"] / extra["c3"]["fp4"]["layer_ms"]
        lr3.close()
    result = {
        "metric": "grouped-GEMM TFLOP/s of the rank's SwiGLU FFN (6*R*H*I flop) over the whole rank-layer step",
        "value": ffn_flops / (ms_step * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4 (MXFP4 E2M1 + E8M0/32, fp32 accumulate)" if fp4 else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {cfg.E} experts top-{cfg.k}, {cfg.n_local} local, H={H} I={I}, "
                               f"T={T} tokens, {int(cfg.vision_frac * 100)}% vision, precision {args.precision} forced, "
                               f"weight encoding mode {mode}"},
        "roofline": roofline,
        "extra": extra,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, lr.inp, fp4)
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump({"result": result, "stages": stages}, f, indent=1)
    lr.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
