#!/usr/bin/env python3
"""Benchmark of the ReaLB rank-layer hot path on one MI355X.

A step is one pass of the whole path -- route_stats, select_precision,
quantize_experts_fp4 (side stream, overlapped with) permute, grouped_moe_ffn,
combine -- over one synthetic batch that is already resident in HBM.

Default workload: the Kimi-VL-A3B-shaped rank share (64 experts, top-6, 8 local,
H 2048, I 1408, 16384 prefill tokens, 75 % vision, Zipf(1.1) skew towards this
rank's experts), forced to the FP4 path.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c1]
                  [--no-cpu-baseline] [--detail PATH]
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3"])
    ap.add_argument("--precision", default="fp4", choices=["fp4", "bf16"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true")
    ap.add_argument("--gemm-tile", type=int, default=0, choices=[0, 2, 8], help="grouped-GEMM block tile selector (0 = automatic)")
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
    cfg = W.CONFIGS[args.workload]
    fp4 = args.precision == "fp4"
    force = R.FP4 if fp4 else R.BF16
    inp = W.gen_layer(cfg, 0)
    rcfg = default_config(cfg.T, cfg.E, cfg.k, cfg.D, cfg.H, cfg.I)
    ctx = R.Context(rcfg)
    buf = R.LayerBuffers(rcfg, cfg.T)
    lg = torch.from_numpy(inp["logits"]).cuda()
    isv = torch.from_numpy(inp["is_vision"]).cuda()
    x, w13, w2 = (R.bf16_from_bits(inp[n]) for n in ("x", "w13", "w2"))
    io = ctx.make_io(lg, isv, x, w13, w2, buf, cfg.rank, force=force, overlap=not args.no_overlap)

    def step():
        ctx.layer_forward(io)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps
    rows = int(buf.expert_offsets[-1].item())
    H, I, T, k = cfg.H, cfg.I, cfg.T, cfg.k
    ffn_flops = 6.0 * rows * H * I

    # ---- per-kernel breakdown on the same stream (separate pass, not part of the timed steps)
    n_w = cfg.n_local * 3 * H * I
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
    on_path = [n for n in stages if fp4 or n != "quantize_experts_fp4"]
    dom = max(on_path, key=lambda n: stages[n]["ms"])
    d = stages[dom]
    if d["kind"] == "flops":
        peak = PEAK_TFLOPS[args.precision]
        roofline = {"kernel": dom, "bound": "mfma", "achieved": d["rate"], "peak": peak, "unit": "TFLOP/s",
                    "frac": d["rate"] / peak, "traffic": None, "ms": d["ms"]}
    else:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": d["rate"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": d["rate"] / PEAK_HBM_GBS, "traffic": None, "ms": d["ms"]}

    # measured HBM traffic of the dominant kernel, if a counter summary for this workload is committed
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            roofline["traffic"] = json.load(f).get(f"{args.workload}_{args.precision}_{dom}")
    if args.calibrate_copy:
        src = torch.ones(128 << 20, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)                      # 512 MiB read + 512 MiB written per launch
        torch.cuda.synchronize()
        del src, dst

    ffn_ms = stages["ffn_gate_up"]["ms"] + stages["ffn_down"]["ms"]
    extra = {
        "rows_on_rank": rows,
        "grouped_gemm_tflops": ffn_flops / (ffn_ms * 1e-3) / 1e12,
        "grouped_gemm_frac_of_peak": ffn_flops / (ffn_ms * 1e-3) / 1e12 / PEAK_TFLOPS[args.precision],
        "quantizer_gbs": stages["quantize_experts_fp4"]["rate"],
        "quantizer_frac_of_hbm": stages["quantize_experts_fp4"]["rate"] / PEAK_HBM_GBS,
        "layer_ms": ms_step,
        "stages_ms": {n: round(s["ms"], 5) for n, s in stages.items()},
    }
    result = {
        "metric": "grouped-GEMM TFLOP/s of the rank's SwiGLU FFN (6*R*H*I flop) over the whole rank-layer step",
        "value": ffn_flops / (ms_step * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4 (MXFP4 E2M1 + E8M0/32, fp32 accumulate)" if fp4 else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {cfg.E} experts top-{cfg.k}, {cfg.n_local} local, H={H} I={I}, "
                               f"T={T} tokens, {int(cfg.vision_frac * 100)}% vision, precision {args.precision} forced, "
                               f"overlap {'off' if args.no_overlap else 'on'}"},
        "roofline": roofline,
        "extra": extra,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, inp, fp4)
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump({"result": result, "stages": stages}, f, indent=1)
    ctx.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
