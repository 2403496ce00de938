#!/usr/bin/env python3
"""Benchmark of the fused-block hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of the workload:
every fusion block of the network executed once by `xl_run(fused=1)`, inputs
already resident in HBM.  The same step with `fused=0` (one kernel per layer,
intermediates through HBM) is timed beside it for the speedup.  Prints ONE JSON
line.  Inputs are seeded synthetic tensors (xl_workloads.py).

What the line holds besides the contract fields:
  per_launch   one row per kernel launch of the fused step of the headline workload, in launch order:
               layers, adopted launch configuration (kernel variant, tile, workgroup size, split),
               average duration from events around that launch (xl_profile), FLOPs, algorithmic bytes,
               binding roofline and fraction, and the time of the same layers run one kernel each
  roofline     the launch with the largest share of the step, priced against the roofline that bounds it,
               plus the fraction of the whole step ("step_frac": all launches' roofline time / ms_per_step)
  peaks        published peaks and what this machine sustains on a copy kernel and on register-only loops
  blocks       the five benchmark configs, scaled-batch variants of configs 1-2 (marked: not the config)
               and the paper's Table 1 structures at batch 32 and batch 1, each with bound / frac / median / min
  bf16x3       the split-bf16 operand mode, reported apart
  cpu_baseline the oracle on the host cores (all cores and one thread)
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
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
    """EXACTLY `steps` timed steps between two synchronisations; also the duration of every single step
    from events recorded between them (no synchronisation inside the timed region)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    for e in ev:            # an event gets its device resources at its first record: not inside the timed region
        e.record()
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    # rehearsal: the timed loop once, untimed and complete with its events, so that whatever the runtime sizes by the
    # number of launches in flight (the host runs many steps ahead of the device) has its size before the clock starts
    for i in range(steps):
        fn(warmup + i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        fn(warmup + i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3
    each = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    return {"mean": ev[0].elapsed_time(ev[steps]) / steps, "median": statistics.median(each), "min": min(each),
            "max": max(each), "slowest_step": each.index(max(each)), "wall": wall / steps,
            "slowest5": sorted(((round(t, 3), i) for i, t in enumerate(each)), reverse=True)[:5]}


def bound_of(flops, nbytes, mfma_peak):
    """Which roofline binds a block and its roofline time in ms."""
    t_m = flops / (mfma_peak * 1e12) * 1e3
    t_h = nbytes / (HBM_PEAK_GBS * 1e9) * 1e3
    return ("mfma", t_m) if t_m >= t_h else ("hbm", t_h)


def group_layers(plan, wl, g):
    """Layer indices of block g of the plan (blocks are in graph order; layers outside every declared block are
    blocks of their own)."""
    q = plan.query(g)
    for grp in wl.groups:
        if grp.layers[0] == q["first_layer"]:
            return list(grp.layers)
    return list(range(q["first_layer"], q["first_layer"] + q["nlayers"]))


def switched_blocks(plan, wl):
    return [g for g in range(plan.num_groups) if len(group_layers(plan, wl, g)) > 1 and not plan.block_is_fused(g)]


def launch_rows(s, mfma_peak, reps):
    """Per-block table of the fused step: xl_profile durations joined with the plan's facts.  A block that
    xl_tune switched to layer-by-layer execution is several launches; its row sums them."""
    plan, wl = s.plan, s.workload
    us_f = plan.profile(s.tensor_ptrs, s.workspace.data_ptr(), s.stream, True, reps)
    us_u = plan.profile(s.tensor_ptrs, s.workspace.data_ptr(), s.stream, False, reps)
    layer_us = {}
    for l, t in enumerate(us_u):
        layer_us[plan.candidate_info(False, l)["first_layer"]] = t
    rows, by_group = [], {}
    for l, t in enumerate(us_f):
        info = plan.candidate_info(True, l)
        g = info["group"]
        if g in by_group:           # a further layer of a block run layer by layer
            r = by_group[g]
            r["us"] += t
            r["launches"] += 1
            r["variant"].append(info["variant"])
            continue
        q = plan.query(g)
        layers = group_layers(plan, wl, g)
        fused = plan.block_is_fused(g) or len(layers) == 1
        bound, t_roof = bound_of(q["flops"], q["bytes_fused"], mfma_peak)
        r = {
            "launch": l, "launches": 1,
            "layers": f"{wl.layers[layers[0]].name}..{wl.layers[layers[-1]].name}" if len(layers) > 1 else wl.layers[layers[0]].name,
            "mode": ["single", "straight", "split", "merge"][q["mode"]], "runs_fused": fused,
            "us": t, "us_unfused_layers": sum(layer_us.get(i, 0.0) for i in layers),
            "flops": q["flops"], "alg_bytes": q["bytes_fused"], "alg_bytes_unfused": q["bytes_unfused"],
            "bound": bound, "roofline_us": t_roof * 1e3,
            "variant": [info["variant"]], "candidate": info["candidate"], "tile": [info["tile_h"], info["tile_w"]],
            "threads": info["threads"], "cout_split": info["cout_split"], "lds_bytes": info["lds_bytes"],
            "redundancy": q["redundancy"] if fused else 1.0,
        }
        by_group[g] = r
        rows.append(r)
    for r in rows:
        t = r["us"]
        r["frac"] = r["roofline_us"] / t if t > 0 else None
        r["mfma_frac"] = r["flops"] / (t * 1e-6) / (mfma_peak * 1e12) if t > 0 else None
        r["hbm_frac"] = r["alg_bytes"] / (t * 1e-6) / (HBM_PEAK_GBS * 1e9) if t > 0 else None
        if len(r["variant"]) == 1:
            r["variant"] = r["variant"][0]
    return rows, us_u


def apply_candidates(plan, saved):
    """Adopt a saved launch configuration: first which blocks run layer by layer (that fixes the launch list of
    the fused path), then the candidate of every launch."""
    for g in range(plan.num_groups):
        plan.set_block_fused(g, g not in saved["layer_by_layer_blocks"])
    for fused, launch, cand in saved["candidates"]:
        plan.select_candidate(bool(fused), launch, cand)


def bench_workload(cfg, steps, warmup, torch, np, W, Session, cold=True, precision=0, candidates=None, fused_only=False,
                   per_launch=False):
    wl = cfg if isinstance(cfg, W.Workload) else W.config(cfg)
    x, params = W.make_tensors(wl)
    s = Session(wl, x, params, tune=TUNE and candidates is None, precision=precision)
    if candidates is not None:
        apply_candidates(s.plan, candidates)
    mfma_peak = MFMA_BF16_PEAK_TFLOPS / 3.0 if precision else MFMA_FP32_PEAK_TFLOPS
    in_bytes = x.nbytes
    out_bytes = int(np.prod(wl.shapes[wl.output_id])) * 4
    ws_bytes = s.plan.workspace_bytes()
    sets = 1
    if cold:
        # inputs, outputs AND workspaces (intermediates between kernels, filters) rotate over more than the caches hold
        sets = max(1, min(64, -(-CACHE_BYTES // (in_bytes + out_bytes + ws_bytes))))
        if sets == 1 and ws_bytes > (64 << 20):
            sets = 2
    xs = [s.x] + [s.x.clone() for _ in range(sets - 1)]
    ys = [s.y] + [torch.empty_like(s.y) for _ in range(sets - 1)]
    wss = [0] + [s.add_workspace() for _ in range(sets - 1)]

    def fused(i):
        s.run(True, xs[i % sets], ys[i % sets], wss[i % sets])

    def unfused(i):
        s.run(False, xs[i % sets], ys[i % sets], wss[i % sets])

    tf = time_steps(fused, steps, warmup, torch)
    tu = tf if fused_only else time_steps(unfused, steps, warmup, torch)
    ms_f, ms_u = tf["mean"], tu["mean"]
    groups = [s.plan.query(g) for g in range(s.plan.num_groups)]
    bytes_f = sum(g["bytes_fused"] for g in groups)
    bytes_u = sum(g["bytes_unfused"] for g in groups)
    flops = sum(g["flops"] for g in groups)
    # the roofline time of the step is the sum over its launches (they run one after the other)
    t_roof = sum(bound_of(g["flops"], g["bytes_fused"], mfma_peak)[1] for g in groups if g["bytes_fused"] > 0)
    bound = bound_of(flops, bytes_f, mfma_peak)[0] if len(groups) == 1 else "per launch"
    res = {
        "workload": wl.name, "batch": wl.batch,
        "ms_fused": ms_f, "ms_fused_median": tf["median"], "ms_fused_min": tf["min"], "ms_fused_max": tf["max"],
        "slowest_step": tf["slowest_step"], "slowest5": tf["slowest5"],
        "ms_unfused": ms_u, "ms_unfused_median": tu["median"], "ms_unfused_min": tu["min"], "wall_ms_fused": tf["wall"],
        "images_per_s": wl.batch / ms_f * 1e3,
        "speedup_vs_unfused": ms_u / ms_f,
        "launches_fused": s.plan.num_launches(True), "launches_unfused": s.plan.num_launches(False),
        "alg_bytes_fused": bytes_f, "alg_bytes_unfused": bytes_u, "flops": flops,
        "hbm_gbs_alg": bytes_f / ms_f / 1e6,
        "hbm_frac": bytes_f / ms_f / 1e6 / HBM_PEAK_GBS,
        "tflops": flops / ms_f / 1e9,
        "mfma_frac": flops / ms_f / 1e9 / mfma_peak,
        "bound": bound, "roofline_ms": t_roof, "frac": t_roof / ms_f,
        "buffer_sets": sets,
        "blocks_run_layer_by_layer": [wl.layers[group_layers(s.plan, wl, g)[0]].name for g in switched_blocks(s.plan, wl)],
        "adopted": [{k: s.plan.candidate_info(True, l)[k] for k in ("variant", "candidate", "tile_h", "tile_w", "threads",
                                                                      "cout_split", "lds_bytes")}
                    for l in range(s.plan.num_launches(True))],
    }
    if precision:
        res["split_bf16_blocks"] = sum(1 for g in groups if g["precision"] == 1)
        res["blocks_total"] = len(groups)
    if per_launch:
        res["per_launch"], _ = launch_rows(s, mfma_peak, max(5, steps))
    return res, s, wl, x, params


def cpu_baseline(cfg, W, np, budget_s=12.0):
    """The oracle as it stands, on a bounded sample of the same workload: all host cores, then one thread."""
    from oracle import xlo
    wl_full = W.config(cfg)
    n = wl_full.batch
    sample_n = max(1, min(n, 8))
    wl = W.config(cfg, n=sample_n)
    x, params = W.make_tensors(wl)
    xlo.forward(wl, x, params)        # warm-up pass (also builds the C library if needed)
    cores = xlo.num_threads()
    reps, t_total = 0, 0.0
    while t_total < budget_s and reps < 50:
        t0 = time.perf_counter()
        xlo.forward(wl, x, params)
        t_total += time.perf_counter() - t0
        reps += 1
    out = {"value": sample_n * reps / t_total, "unit": "images/s", "cores": cores, "kind": "oracle",
           "sample": f"{reps} passes of {wl.name} at batch {sample_n} (full batch {n}), {t_total:.1f} s"}
    # one thread: one image is enough (seconds per pass)
    wl1 = W.config(cfg, n=1)
    x1, p1 = W.make_tensors(wl1)
    xlo.set_num_threads(1)
    try:
        reps1, t1 = 0, 0.0
        while t1 < budget_s / 2 and reps1 < 10:
            t0 = time.perf_counter()
            xlo.forward(wl1, x1, p1)
            t1 += time.perf_counter() - t0
            reps1 += 1
        out["value_1_thread"] = reps1 / t1
        out["sample_1_thread"] = f"{reps1} passes at batch 1, {t1:.1f} s"
    finally:
        xlo.set_num_threads(cores)
    return out


def measured_peaks(torch):
    from paper_2007_06000_amd import binding
    n = 512 << 20
    a = torch.ones(n // 4, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    m = binding.xl_measure_peaks(b.data_ptr(), a.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
    del a, b
    return {"published": {"hbm_gbs": HBM_PEAK_GBS, "mfma_f32_tflops": MFMA_FP32_PEAK_TFLOPS, "mfma_bf16_tflops": MFMA_BF16_PEAK_TFLOPS,
                          "valu_f32_tflops_not_packed": 78.6},
            "measured": m, "how": "xl_measure_peaks: 512 MiB copy kernel (read + written bytes); register-only loops of "
                                  "independent operations on every compute unit; fastest of 5 launches"}


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
    ap.add_argument("--save-candidates", metavar="FILE",
                    help="after tuning, write the adopted candidate of every launch of the headline workload to FILE")
    ap.add_argument("--load-candidates", metavar="FILE",
                    help="adopt the candidates listed in FILE instead of tuning (for profiler runs: no candidate launches)")
    ap.add_argument("--fused-only", action="store_true", help="time the fused step only (for profiler runs)")
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

    candidates = None
    if args.load_candidates:
        candidates = json.load(open(args.load_candidates))

    if args.traffic_probe:
        traffic_probe(args.workload, torch, np, W, Session, candidates)
        return

    prec = 1 if args.precision == "bf16x3" else 0
    if prec:
        args.no_bf16x3 = True
    profiler_run = args.fused_only
    res, s, wl, x, params = bench_workload(args.workload, args.steps, args.warmup, torch, np, W, Session,
                                           cold=not args.warm, precision=prec, candidates=candidates,
                                           fused_only=args.fused_only, per_launch=not profiler_run)
    if args.save_candidates:
        cands = []
        for fused in (1, 0):
            for l in range(s.plan.num_launches(bool(fused))):
                cands.append([fused, l, s.plan.candidate_info(bool(fused), l)["candidate"]])
        json.dump({"workload": wl.name, "batch": wl.batch, "precision": args.precision,
                   "layer_by_layer_blocks": switched_blocks(s.plan, wl),
                   "candidates": cands}, open(args.save_candidates, "w"))
    if profiler_run:
        print(json.dumps({"profiler_run": wl.name, "ms_per_step": res["ms_fused"], "steps": args.steps, "adopted": res["adopted"]}))
        return

    mfma_peak = MFMA_BF16_PEAK_TFLOPS / 3.0 if prec else MFMA_FP32_PEAK_TFLOPS
    rows = res.pop("per_launch")
    roof = dominant_launch_roofline(rows, res, mfma_peak, prec)

    out = {
        "metric": "images/sec per fused block + HBM GB/s vs roofline; speedup over unfused",
        "value": res["images_per_s"], "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_fused"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 hi+lo operands (3 products), f32 accumulate" if prec else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "launches_per_step": res["launches_fused"],
                   "blocks_run_layer_by_layer": res["blocks_run_layer_by_layer"],
                   "buffers": "inputs, outputs and workspaces rotate over > 512 MB (cold)" if not args.warm else "single set (warm)",
                   "tiles": ("xl_tune (measured, median of 5)" if TUNE else "cost model") if candidates is None else "from file"},
        "ms_per_step_median": res["ms_fused_median"], "ms_per_step_min": res["ms_fused_min"],
        "speedup_vs_unfused": res["speedup_vs_unfused"],
        "ms_per_step_unfused": res["ms_unfused"],
        "hbm_gbs_algorithmic": res["hbm_gbs_alg"],
        "fp32_tflops": res["tflops"], "fp32_mfma_frac": res["mfma_frac"],
        "paper_context": {"fused_structures_speedup": 2.02, "squeezenet_speedup": 1.57,
                          "hardware": "TITAN Xp / Tesla P4, vs cuDNN v7"},
        "roofline": roof,
        "per_launch": rows,
        "per_launch_note": "us: average over xl_profile's runs, events around each launch on the launch stream, same buffers "
                           "every run; frac = roofline_us / us against the published peaks; us_unfused_layers: the block's "
                           "layers one kernel each",
        "target_60pct": {"met_by": [r["layers"] for r in rows if r["frac"] and r["frac"] >= 0.6],
                         "missed_by": [r["layers"] for r in rows if r["frac"] and r["frac"] < 0.6]},
        "peaks": measured_peaks(torch),
    }
    m = out["peaks"]["measured"]
    if not prec and m["mfma_f32_tflops"] > 0:
        out["roofline"]["frac_vs_measured_peak"] = (roof["achieved"] / m["mfma_f32_tflops"] if roof["bound"] == "mfma"
                                                    else roof["achieved"] / m["copy_gbs"])
        out["fp32_mfma_frac_vs_measured_peak"] = res["tflops"] / m["mfma_f32_tflops"]
    if not args.headline_only:
        blocks = []
        for c in (1, 2, 3, 4, 5):
            if c == args.workload:
                blocks.append({k: res[k] for k in res})
                continue
            r, *_ = bench_workload(c, args.steps, args.warmup, torch, np, W, Session, cold=not args.warm, precision=prec)
            blocks.append(r)
        # configs 1 and 2 are launch-latency sized: the same per-image shapes at a batch that runs for >= 100 us, so
        # that a roofline fraction means something -- NOT the benchmark configs
        extra = {"cfg1_scaled_batch": W.config(1, n=8192), "cfg2_scaled_batch": W.config(2, n=512),
                 # the paper's four fused structures (its Table 1; b.1 is the family of config 3), at batch 32 and at the
                 # paper's own batch 1
                 "table1_a1": W.straight_generic(32, 192, 28, 28, 16, 1, 0, 1, 32, 5, 2, 1),
                 "table1_a2": W.depthwise_pointwise(32, 16, 80, 80, 16),
                 "table1_c1": W.merge_two_producers(32),
                 "table1_a1_batch1": W.straight_generic(1, 192, 28, 28, 16, 1, 0, 1, 32, 5, 2, 1),
                 "table1_a2_batch1": W.depthwise_pointwise(1, 16, 80, 80, 16),
                 "table1_b1_batch1": W.config(3, n=1),
                 "table1_c1_batch1": W.merge_two_producers(1),
                 "cfg4_batch1": W.config(4, n=1)}
        for tag, w2 in extra.items():
            try:
                r, *_ = bench_workload(w2, args.steps, args.warmup, torch, np, W, Session, cold=not args.warm, precision=prec)
                r["workload"] = tag + ":" + r["workload"]
                if "scaled_batch" in tag:
                    r["not_the_config"] = True
            except Exception as e:      # an extra row must not take the headline down
                r = {"workload": tag, "error": repr(e)}
            blocks.append(r)
        out["blocks"] = blocks
    if not args.no_bf16x3:
        try:
            # reduced-precision operand mode, reported apart from the fp32 headline: same workloads, same
            # tolerance against the oracle, other arithmetic and other roofline denominator
            rb, *_ = bench_workload(args.workload, args.steps, args.warmup, torch, np, W, Session, cold=not args.warm,
                                    precision=1, per_launch=True)
            rows_b = rb.pop("per_launch")
            b3 = {"arithmetic": "operands split into hi + lo bf16, 3 bf16 matrix operations per product, fp32 accumulate",
                  "workload": rb["workload"], "value": rb["images_per_s"], "unit": "images/s",
                  "ms_per_step": rb["ms_fused"], "ms_per_step_unfused": rb["ms_unfused"],
                  "speedup_vs_unfused": rb["speedup_vs_unfused"], "speedup_vs_fp32": res["ms_fused"] / rb["ms_fused"],
                  "split_bf16_blocks": rb["split_bf16_blocks"], "blocks_total": rb["blocks_total"],
                  "roofline": dominant_launch_roofline(rows_b, rb, MFMA_BF16_PEAK_TFLOPS / 3.0, 1),
                  "per_launch": rows_b}
            if not args.headline_only:
                b3["blocks"] = []
                for c in (2, 3, 4):
                    r, *_ = bench_workload(c, args.steps, args.warmup, torch, np, W, Session, cold=not args.warm, precision=1)
                    b3["blocks"].append({k: r[k] for k in ("workload", "batch", "ms_fused", "ms_unfused", "images_per_s",
                                                           "speedup_vs_unfused", "tflops", "bound", "frac", "split_bf16_blocks")})
            out["bf16x3"] = b3
        except Exception as e:      # the headline stands on its own
            out["bf16x3"] = {"error": repr(e)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, W, np)
    print(json.dumps(out))


def traffic_probe(cfg, torch, np, W, Session, candidates):
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
    s = Session(wl, x, params, tune=TUNE and candidates is None)
    if candidates is not None:
        apply_candidates(s.plan, candidates)
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


def measured_traffic(layers):
    """HBM bytes per launch of the dominant launch from the committed counter summary (profiles/hbm_traffic.txt:
    lines `<first layer>..<last layer> <fetch bytes> <write bytes>`), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for ln in open(path):
        f = ln.split()
        if len(f) >= 3 and f[0] == layers and not ln.startswith("#"):
            return float(f[1]) + float(f[2])
    return None


def dominant_launch_roofline(rows, res, mfma_peak, precision):
    """The launch with the largest share of the step, priced against the roofline that bounds it.  Duration: the
    launch's average from events around it (xl_profile), measured in this process right after the timed steps."""
    r = max(rows, key=lambda q: q["us"])
    share = r["us"] / sum(q["us"] for q in rows)
    if r["bound"] == "mfma":
        ach, peak, unit = r["flops"] / (r["us"] * 1e-6) / 1e12, mfma_peak, "TFLOP/s"
    else:
        ach, peak, unit = r["alg_bytes"] / (r["us"] * 1e-6) / 1e9, HBM_PEAK_GBS, "GB/s"
    out = {"bound": r["bound"], "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
           "traffic": None if precision else measured_traffic(r["layers"]),
           "kernel": r["layers"], "launch": r["launch"], "kernel_us": r["us"], "share_of_step": share,
           "flops_per_launch": r["flops"], "bytes_per_launch": r["alg_bytes"],
           "step_frac": res["frac"], "step_roofline_ms": res["roofline_ms"],
           "sum_of_launches_ms": sum(q["us"] for q in rows) / 1e3}
    if precision:
        out["peak_note"] = "bf16 dense matrix peak 2500 TFLOP/s / 3 operations per product; flops = 2*MAC of the layer"
    return out


if __name__ == "__main__":
    main()
