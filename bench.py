#!/usr/bin/env python3
"""Benchmark of the fused-block hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of the workload:
every fusion block of the network executed once by `xl_run(fused=1)`, inputs
already resident in HBM.  The same step with `fused=0` (one kernel per layer,
intermediates through HBM) is timed beside it for the speedup.  Prints ONE JSON
line.  Inputs are seeded synthetic tensors (xl_workloads.py).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3  # dense fp32 matrix cores
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix cores
CACHE_BYTES = 512 << 20        # rotate buffers over more than L2 + Infinity Cache (256 MB)
TUNE = True                    # xl_tune picks tiles by measurement once, outside the timed region


def time_steps(fn, steps, warmup, torch):
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(steps):
        fn(warmup + i)
    ev1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3
    return ev0.elapsed_time(ev1) / steps, wall / steps


def bench_workload(cfg, steps, warmup, torch, np, W, Session, cold=True, precision=0):
    wl = cfg if isinstance(cfg, W.Workload) else W.config(cfg)
    x, params = W.make_tensors(wl)
    s = Session(wl, x, params, tune=TUNE, precision=precision)
    in_bytes = x.nbytes
    out_bytes = int(np.prod(wl.shapes[wl.output_id])) * 4
    sets = 1
    if cold:
        sets = max(1, min(64, -(-CACHE_BYTES // (in_bytes + out_bytes))))
    xs = [s.x] + [s.x.clone() for _ in range(sets - 1)]
    ys = [s.y] + [torch.empty_like(s.y) for _ in range(sets - 1)]

    def fused(i):
        s.run(True, xs[i % sets], ys[i % sets])

    def unfused(i):
        s.run(False, xs[i % sets], ys[i % sets])

    ms_f, wall_f = time_steps(fused, steps, warmup, torch)
    ms_u, _ = time_steps(unfused, steps, warmup, torch)
    groups = [s.plan.query(g) for g in range(s.plan.num_groups)]
    bytes_f = sum(g["bytes_fused"] for g in groups)
    bytes_u = sum(g["bytes_unfused"] for g in groups)
    flops = sum(g["flops"] for g in groups)
    res = {
        "workload": wl.name, "batch": wl.batch,
        "ms_fused": ms_f, "ms_unfused": ms_u, "wall_ms_fused": wall_f,
        "images_per_s": wl.batch / ms_f * 1e3,
        "speedup_vs_unfused": ms_u / ms_f,
        "launches_fused": s.plan.num_launches(True), "launches_unfused": s.plan.num_launches(False),
        "alg_bytes_fused": bytes_f, "alg_bytes_unfused": bytes_u, "flops": flops,
        "hbm_gbs_alg": bytes_f / ms_f / 1e6,
        "hbm_frac": bytes_f / ms_f / 1e6 / HBM_PEAK_GBS,
        "tflops": flops / ms_f / 1e9,
        "mfma_frac": flops / ms_f / 1e9 / MFMA_FP32_PEAK_TFLOPS,
        "buffer_sets": sets,
    }
    if precision:
        res["split_bf16_blocks"] = sum(1 for g in groups if g["precision"] == 1)
        res["blocks_total"] = len(groups)
    return res, s, wl, x, params


def cpu_baseline(cfg, W, np, budget_s=15.0):
    """The oracle as it stands, on a bounded sample of the same workload."""
    from oracle import xlo
    wl_full = W.config(cfg)
    n = wl_full.batch
    sample_n = max(1, min(n, 8))
    wl = W.config(cfg, n=sample_n)
    x, params = W.make_tensors(wl)
    xlo.forward(wl, x, params)        # warm-up pass (also builds the C library if needed)
    reps, t_total = 0, 0.0
    while t_total < budget_s and reps < 50:
        t0 = time.perf_counter()
        xlo.forward(wl, x, params)
        t_total += time.perf_counter() - t0
        reps += 1
    return {"value": sample_n * reps / t_total, "unit": "images/s", "cores": xlo.num_threads(), "kind": "oracle",
            "sample": f"{reps} passes of {wl.name} at batch {sample_n} (full batch {n}), {t_total:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=5, help="benchmark config number 1..5 timed as the headline")
    ap.add_argument("--headline-only", action="store_true", help="skip the per-config table reported under 'blocks'")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: one 256 MiB copy (calibration), then 3 fused and 3 unfused steps")
    ap.add_argument("--warm", action="store_true", help="reuse one buffer set (cache-resident) instead of rotating")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-tune", action="store_true", help="use the planner's cost-model choice without xl_tune")
    ap.add_argument("--precision", choices=["fp32", "bf16x3"], default="fp32",
                    help="arithmetic of the headline run; bf16x3 times the split-bf16 mode alone (for profiles)")
    ap.add_argument("--no-bf16x3", action="store_true",
                    help="skip the separate report of the split-bf16 precision mode (three bf16 matrix operations per product)")
    args = ap.parse_args()
    global TUNE
    TUNE = not args.no_tune
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (images are independent; batch sharding needs no "
              "collective); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import xl_workloads as W
    from paper_2007_06000_amd.session import Session

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libxl has no CPU path", file=sys.stderr)
        sys.exit(2)

    if args.traffic_probe:
        traffic_probe(args.workload, torch, np, W, Session)
        return

    prec = 1 if args.precision == "bf16x3" else 0
    if prec:
        args.no_bf16x3 = True
    res, s, wl, x, params = bench_workload(args.workload, args.steps, args.warmup, torch, np, W, Session,
                                           cold=not args.warm, precision=prec)

    # roofline of the dominant kernel of the headline workload
    roof = dominant_kernel_roofline(args.workload, res, args, torch, np, W, Session, precision=prec)

    out = {
        "metric": "images/sec per fused block + HBM GB/s vs roofline; speedup over unfused",
        "value": res["images_per_s"], "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_fused"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 hi+lo operands (3 products), f32 accumulate" if prec else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "launches_per_step": res["launches_fused"],
                   "buffers": "rotating (cold)" if not args.warm else "single set (warm)",
                   "tiles": "xl_tune (measured)" if TUNE else "cost model"},
        "speedup_vs_unfused": res["speedup_vs_unfused"],
        "ms_per_step_unfused": res["ms_unfused"],
        "hbm_gbs_algorithmic": res["hbm_gbs_alg"],
        "fp32_tflops": res["tflops"], "fp32_mfma_frac": res["mfma_frac"],
        "paper_context": {"fused_structures_speedup": 2.02, "squeezenet_speedup": 1.57,
                          "hardware": "TITAN Xp / Tesla P4, vs cuDNN v7"},
        "roofline": roof,
    }
    if not args.headline_only:
        blocks = []
        for c in (1, 2, 3, 4, 5):
            if c == args.workload:
                blocks.append({k: res[k] for k in res})
                continue
            r, *_ = bench_workload(c, args.steps, args.warmup, torch, np, W, Session, cold=not args.warm, precision=prec)
            blocks.append(r)
        # the paper's four fused structures (its Table 1; b.1 is the family of config 3), at batch 32
        table1 = {"table1_a1": W.straight_generic(32, 192, 28, 28, 16, 1, 0, 1, 32, 5, 2, 1),
                  "table1_a2": W.depthwise_pointwise(32, 16, 80, 80, 16),
                  "table1_c1": W.merge_two_producers(32)}
        for tag, wl in table1.items():
            try:
                r, *_ = bench_workload(wl, args.steps, args.warmup, torch, np, W, Session, cold=not args.warm, precision=prec)
                r["workload"] = tag + ":" + r["workload"]
            except Exception as e:      # an extra row must not take the headline down
                r = {"workload": tag, "error": repr(e)}
            blocks.append(r)
        out["blocks"] = blocks
    if not args.no_bf16x3:
        try:
            # reduced-precision operand mode, reported apart from the fp32 headline: same workloads, same
            # tolerance against the oracle, other arithmetic and other roofline denominator
            rb, *_ = bench_workload(args.workload, args.steps, args.warmup, torch, np, W, Session, cold=not args.warm,
                                    precision=1)
            b3 = {"arithmetic": "operands split into hi + lo bf16, 3 bf16 matrix operations per product, fp32 accumulate",
                  "workload": rb["workload"], "value": rb["images_per_s"], "unit": "images/s",
                  "ms_per_step": rb["ms_fused"], "ms_per_step_unfused": rb["ms_unfused"],
                  "speedup_vs_unfused": rb["speedup_vs_unfused"], "speedup_vs_fp32": res["ms_fused"] / rb["ms_fused"],
                  "split_bf16_blocks": rb["split_bf16_blocks"], "blocks_total": rb["blocks_total"],
                  "roofline": dominant_kernel_roofline(args.workload, rb, args, torch, np, W, Session, precision=1)}
            if not args.headline_only:
                b3["blocks"] = []
                for c in (2, 3, 4):
                    r, *_ = bench_workload(c, args.steps, args.warmup, torch, np, W, Session, cold=not args.warm, precision=1)
                    b3["blocks"].append({k: r[k] for k in ("workload", "batch", "ms_fused", "ms_unfused", "images_per_s",
                                                           "speedup_vs_unfused", "tflops", "split_bf16_blocks")})
            out["bf16x3"] = b3
        except Exception as e:      # the headline stands on its own
            out["bf16x3"] = {"error": repr(e)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, W, np)
    print(json.dumps(out))


def traffic_probe(cfg, torch, np, W, Session):
    """Work for the two counter passes (FETCH_SIZE, WRITE_SIZE): a copy of known size to scale the
    counters by, then the fused and the unfused path on cold buffers."""
    n = 64 << 20
    a = torch.ones(n, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    wl = W.config(cfg)
    x, params = W.make_tensors(wl)
    s = Session(wl, x, params, tune=TUNE)
    torch.empty(12345, dtype=torch.float32, device="cuda").fill_(1.0)     # marker: measured passes start here
    for fused in (True, False):
        for _ in range(3):
            xs, ys = s.x.clone(), torch.empty_like(s.y)
            torch.cuda.synchronize()
            s.run(fused, xs, ys)
            torch.cuda.synchronize()
    groups = [s.plan.query(g) for g in range(s.plan.num_groups)]
    print(json.dumps({"probe": wl.name, "copy_bytes_read": n * 4, "copy_bytes_written": n * 4,
                      "launches_fused": s.plan.num_launches(True), "launches_unfused": s.plan.num_launches(False),
                      "alg_bytes_fused": sum(g["bytes_fused"] for g in groups),
                      "alg_bytes_unfused": sum(g["bytes_unfused"] for g in groups)}))


def measured_traffic(kernel_name):
    """HBM bytes per launch of the dominant kernel from the committed counter summary, or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for ln in open(path):
        f = ln.split()
        if len(f) >= 3 and f[0] == kernel_name and not ln.startswith("#"):
            return float(f[1]) + float(f[2])
    return None


def dominant_kernel_roofline(cfg, res, args, torch, np, W, Session, precision=0):
    """Time the block that dominates the headline workload on its own (one
    kernel launch per step) and price it against the roofline that bounds it.
    precision = 1: the split-bf16 kernels, priced against the dense bf16 matrix
    peak divided by the three operations a product costs."""
    mfma_peak = MFMA_BF16_PEAK_TFLOPS / 3.0 if precision else MFMA_FP32_PEAK_TFLOPS
    wl_full = W.config(cfg)
    x, params = W.make_tensors(wl_full)
    s = Session(wl_full, x, params, tune=False, precision=precision)
    groups = [s.plan.query(g) for g in range(s.plan.num_groups)]
    if len(groups) == 1:
        g = groups[0]
        ms = res["ms_fused"]
        name = wl_full.name
    else:
        # the block with the largest roofline time, rebuilt as a workload of its own
        def t_roof(g):
            return max(g["flops"] / (mfma_peak * 1e12), g["bytes_fused"] / (HBM_PEAK_GBS * 1e9))
        gi = max(range(len(groups)), key=lambda i: t_roof(groups[i]))
        g = groups[gi]
        sub = W.subgraph(wl_full, gi)
        xs, ps = W.make_tensors(sub)
        ss = Session(sub, xs, ps, tune=TUNE, precision=precision)
        in_b, out_b = xs.nbytes, int(np.prod(sub.shapes[sub.output_id])) * 4
        sets = max(1, min(64, -(-CACHE_BYTES // (in_b + out_b)))) if not args.warm else 1
        bx = [ss.x] + [ss.x.clone() for _ in range(sets - 1)]
        by = [ss.y] + [torch.empty_like(ss.y) for _ in range(sets - 1)]
        ms, _ = time_steps(lambda i: ss.run(True, bx[i % sets], by[i % sets]), args.steps, args.warmup, torch)
        g = ss.plan.query(0)
        name = sub.name
    t_m = g["flops"] / (mfma_peak * 1e12)
    t_h = g["bytes_fused"] / (HBM_PEAK_GBS * 1e9)
    if t_m >= t_h:
        ach = g["flops"] / ms / 1e9
        r = {"bound": "mfma", "achieved": ach, "peak": mfma_peak, "unit": "TFLOP/s",
             "frac": ach / mfma_peak, "traffic": None if precision else measured_traffic(name), "kernel": name,
             "kernel_ms": ms, "flops_per_launch": g["flops"], "bytes_per_launch": g["bytes_fused"]}
        if precision:
            r["peak_note"] = "bf16 dense matrix peak 2500 TFLOP/s / 3 operations per product; flops = 2*MAC of the layer"
        return r
    ach = g["bytes_fused"] / ms / 1e6
    return {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
            "traffic": measured_traffic(name), "kernel": name, "kernel_ms": ms,
            "flops_per_launch": g["flops"], "bytes_per_launch": g["bytes_fused"]}


if __name__ == "__main__":
    main()
