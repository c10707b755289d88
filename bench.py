#!/usr/bin/env python3
"""Benchmark of the convolution hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config {1..5}] [--no-cpu-baseline]

A step is one pass of the whole hot path over one batch of synthetic input: for
every layer of the workload, input transform -> Winograd-domain GEMM -> output
transform (or the 1x1 GEMM / direct kernel), with the scheme chosen by the
pre-inference planner.  Inputs, weights and prepared weights are resident in HBM
before the timed region.  One JSON line is printed.
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

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
STAGE_NAMES = ["filter_transform", "input_transform", "gemm", "output_transform"]


def stage_work(layer, scheme, info, mnn):
    """Algorithmic work per launch of each per-inference stage: (flops, bytes)."""
    N, C, K = layer.n, layer.c_in, layer.c_out
    Ho, Wo = layer.h_out, layer.w_out
    out = {}
    if scheme.kind == mnn.SCHEME_WINOGRAD:
        a, n, P = info["alpha"], info["tile_n"], info["p"]
        a2 = a * a
        out["input_transform"] = (4.0 * a ** 3 * C * P, 4.0 * (N * C * layer.h * layer.w + a2 * C * P))
        out["gemm"] = (2.0 * a2 * K * C * P, 4.0 * a2 * (K * C + C * P + K * P))
        out["output_transform"] = (2.0 * (n * a2 + n * n * a) * K * P, 4.0 * (a2 * K * P + N * K * Ho * Wo))
    elif scheme.kind == mnn.SCHEME_GEMM1X1:
        HW = layer.h * layer.w
        out["gemm"] = (2.0 * N * K * C * HW, 4.0 * (N * C * HW + N * K * HW + K * C))
    else:
        out["gemm"] = (float(layer.direct_flops),
                       4.0 * (N * C * layer.h * layer.w + N * K * Ho * Wo + K * C * layer.kh * layer.kw))
    return out


def cpu_baseline(layers):
    """The float64 oracle, as it stands, timed on the host cores over the same workload."""
    import oracle
    from conv_workloads import draw
    flops, secs = 0.0, 0.0
    names = []
    budget_s = 40.0
    for layer in layers:
        sample = layer
        # bound the sample: keep whole images, drop images until the estimate fits the budget
        est = layer.direct_flops / 5e9
        if est > budget_s / len(layers):
            keep = max(1, int(layer.n * (budget_s / len(layers)) / est))
            sample = layer.with_batch(keep)
        x, w, b = draw(sample)
        t0 = time.perf_counter()
        oracle.conv2d(x, w, b, stride=sample.stride, pad=sample.pad, dil=sample.dil)
        secs += time.perf_counter() - t0
        flops += sample.direct_flops
        names.append(f"{sample.name}[N={sample.n}]")
    return {"value": flops / secs / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "one float64 direct-convolution pass over " + ", ".join(names), "seconds": round(secs, 3)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--force", type=str, default="", help="force a scheme: direct | gemm | F<n>  (default: planner)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); it has no multi-GPU path", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2002_12418_amd as mnn
    from conv_workloads import CONFIG_TITLES, config_layers, draw

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    layers = config_layers(args.config)
    opt = None
    if args.force:
        f = args.force.lower()
        if f == "direct":
            opt = mnn.Options(force_kind=mnn.SCHEME_DIRECT)
        elif f == "gemm":
            opt = mnn.Options(force_kind=mnn.SCHEME_GEMM1X1)
        elif f.startswith("f"):
            opt = mnn.Options(force_kind=mnn.SCHEME_WINOGRAD, force_tile_n=int(f[1:]))
        else:
            raise SystemExit(f"unknown --force {args.force}")

    stream = torch.cuda.current_stream()
    work = []
    for layer in layers:
        x, w, b = draw(layer)
        xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
        layer_opt = opt
        if opt is not None and layer.stride != 1 and opt.force_kind == mnn.SCHEME_WINOGRAD:
            layer_opt = mnn.Options(force_kind=mnn.SCHEME_DIRECT)
        plan = mnn.ConvPlan.for_layer(layer, options=layer_opt, stream=stream)
        y = torch.empty(plan.out_shape, dtype=torch.float32, device="cuda")
        plan.run(xd, wd, bd, y, stream=stream)      # prepares the weights (filter transform) once
        work.append((layer, plan, xd, wd, bd, y))
    torch.cuda.synchronize()

    def step():
        for layer, plan, xd, wd, bd, y in work:
            plan.run(xd, wd, bd, y, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    total_flops = float(sum(l.direct_flops for l in layers))
    ms_per_step = elapsed / args.steps * 1e3
    value = total_flops * args.steps / elapsed / 1e9

    # ---- per-kernel durations from HIP events on the launch stream (instrumented pass, same work)
    iters = max(5, min(args.steps, 50))
    per_layer = []
    stage_tot = {s: {"ms": 0.0, "flops": 0.0, "bytes": 0.0, "launches": 0} for s in STAGE_NAMES}
    for layer, plan, xd, wd, bd, y in work:
        ms = plan.run_timed(xd, wd, bd, y, iters=iters, stream=stream)
        sch = plan.scheme
        sw = stage_work(layer, sch, plan.info, mnn)
        entry = {"layer": layer.name, "scheme": sch.label(layer.kh),
                 "planner_ms": {c.label(layer.kh): round(c.est_ms, 4) for c in plan.candidates if c.est_ms >= 0},
                 "stage_ms": {STAGE_NAMES[i]: round(ms[i], 5) for i in range(1, 4) if ms[i] > 0},
                 "filter_ms_one_off": round(ms[0], 5)}
        lay_ms = sum(ms[1:4])
        entry["ms"] = round(lay_ms, 5)
        entry["gflops_direct_count"] = round(layer.direct_flops / (lay_ms * 1e-3) / 1e9, 1) if lay_ms > 0 else None
        for name, (fl, by) in sw.items():
            i = STAGE_NAMES.index(name)
            st = stage_tot[name]
            st["ms"] += ms[i]; st["flops"] += fl; st["bytes"] += by; st["launches"] += 1
            entry.setdefault("stage_rate", {})[name] = {
                "TFLOP/s": round(fl / (ms[i] * 1e-3) / 1e12, 2) if ms[i] > 0 else None,
                "GB/s": round(by / (ms[i] * 1e-3) / 1e9, 1) if ms[i] > 0 else None}
        per_layer.append(entry)

    dominant = max(STAGE_NAMES[1:], key=lambda s: stage_tot[s]["ms"])
    st = stage_tot[dominant]
    gemm_like = dominant == "gemm"
    if gemm_like:
        ach = st["flops"] / (st["ms"] * 1e-3) / 1e12
        roofline = {"kernel": "gemm_f32_kernel (Winograd-domain / 1x1 / direct)", "bound": "mfma", "achieved": round(ach, 2),
                    "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_FP32_MFMA_TFLOPS, 4),
                    "traffic": None}
    else:
        ach = st["bytes"] / (st["ms"] * 1e-3) / 1e9
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None}
    roofline["avg_launch_ms"] = round(st["ms"] / max(1, st["launches"]), 5)
    roofline["stages"] = {
        s: {"ms_per_step": round(v["ms"], 5),
            "TFLOP/s": round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) if v["ms"] > 0 else None,
            "GB/s": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] > 0 else None,
            "frac_mfma": round(v["flops"] / (v["ms"] * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4) if v["ms"] > 0 else None,
            "frac_hbm": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4) if v["ms"] > 0 else None}
        for s, v in stage_tot.items() if v["launches"]}

    out = {
        "metric": "conv GFLOP/s (direct-FLOP count)", "value": round(value, 1), "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": CONFIG_TITLES[args.config], "layers": [l.name for l in layers],
                   "batch": layers[0].n, "scheme": args.force or "planner"},
        "ms_per_layer": {e["layer"]: e["ms"] for e in per_layer},
        "roofline": roofline,
        "layers": per_layer,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layers)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
