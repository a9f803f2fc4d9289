#!/usr/bin/env python3
"""Throughput of the fused pipelines on one MI355X.

A step is one pass of the whole hot path: the five synthetic pipelines, each
executed as its fused clusters (fc_run_fused), inputs resident in HBM.  The
reported value is the fused-traffic lower bound of a step (every external input
byte once + every output byte once) divided by the time of a step.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--configs 1,2,3,4,5]

One JSON line goes to stdout; a table per pipeline goes to stderr.
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

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published peak
ROTATE_BYTES = 1 << 30       # cycle through input sets until at least this much is touched between
#                              two uses of the same set (the 256 MiB memory-side cache must not serve a pipeline)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def source_hash() -> str:
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2407_13585_amd", "csrc", "*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def measured_traffic(workload: str):
    """HBM bytes per launch from the committed counter summary, or None when the kernel
    sources have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
    if not os.path.exists(path):
        return None
    table, sha = {}, None
    for line in open(path):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "source_sha256":
            sha = t[1]
        else:
            table[t[0]] = int(t[2]) + int(t[4])
    if sha != source_hash():
        return None
    return table.get(workload)


def gather_ceiling(fc, DeviceProgram, np, torch):
    """Rate of bare random 4-byte gathers (index stream + gather + fold, no arithmetic) for three
    table sizes: the ceiling the memory system puts on the gather pipelines."""
    from workloads import Graph
    out = {}
    for logn in (20, 22, 24):
        n = 1 << logn
        rng = np.random.default_rng(logn)
        g = Graph()
        g.add("idx", "input", "i32", (n,))
        g.add("xs", "input", "f32", (n,))
        g.add("zs", "gather", "f32", (n,), args=("idx", "xs"))
        g.add("r", "fold", "f32", (1,), fn="add", args=("zs",), output=True)
        part = fc.fc_plan(g, "bytes")
        sets = max(2, (1 << 30) // (8 * n))
        progs = [DeviceProgram(g, {"idx": rng.permutation(n).astype(np.int32), "xs": np.ones(n, np.float32)}, part)
                 for _ in range(min(sets, 8))]
        for p in progs:
            p.run()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 16
        a.record()
        for r in range(reps):
            progs[r % len(progs)].run()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) / reps * 1e3
        out[f"table_2^{logn}_f32"] = {"us": round(us, 2), "Ggather/s": round(n / us / 1e3, 2), "kernel": progs[0].kernels()[0]}
        log(f"bare gather, table 2^{logn} floats: {us:8.1f} us  {n / us / 1e3:6.1f} G gathers/s")
    return out


def paper_examples(fc, DeviceProgram, np, torch):
    """The programs the paper times that can be rebuilt from its text (section 5, "Greedy
    counterexamples", and `singleLoop` of section 1): fused by fc_plan versus no fusion."""
    from workloads import paper_graphs as PG
    rng = np.random.default_rng(7)
    cases = {
        "greedyBottomUpBad(n=64, m=10^6)": (PG.greedy_bottom_up_bad(64, 1000000),
                                            {"xs": (1.0 + rng.uniform(-4, 4, 64) / 1e6).astype(np.float32)}),
        "greedyTopDownBad(n=2^24)": (PG.greedy_top_down_bad(1 << 24), {"as": rng.standard_normal(1 << 24).astype(np.float32)}),
        "singleLoop(n=2^24)": (PG.single_loop(1 << 24), {"as": rng.standard_normal(1 << 24).astype(np.float32)}),
    }
    out = {}
    for name, (g, ins) in cases.items():
        part = fc.fc_plan(g, "bytes")
        progs = {"fused": DeviceProgram(g, ins, part), "unfused": DeviceProgram(g, ins, None)}
        t = {}
        for tag, p in progs.items():
            p.run()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 10
            a.record()
            for _ in range(reps):
                p.run()
            b.record()
            torch.cuda.synchronize()
            t[tag] = a.elapsed_time(b) / reps * 1e3
        out[name] = {"fused_us": round(t["fused"], 1), "unfused_us": round(t["unfused"], 1),
                     "speedup": round(t["unfused"] / t["fused"], 2), "clusters": part.n_clusters,
                     "kernels": progs["fused"].kernels()}
        log(f"{name}: fused {t['fused']:9.1f} us ({part.n_clusters} kernels)  unfused {t['unfused']:9.1f} us  "
            f"speedup {t['unfused'] / t['fused']:6.2f}x")
        del progs
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--configs", default="1,2,3,4,5")
    ap.add_argument("--small", action="store_true", help="small sizes (debugging only; not a valid measurement)")
    ap.add_argument("--no-unfused", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--gather-ceiling", action="store_true",
                    help="also measure the rate of bare random gathers (no arithmetic) for three table sizes")
    ap.add_argument("--paper-examples", action="store_true",
                    help="also time the paper's small example programs, fused against unfused")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain copy kernel of known size (256 MiB in, 256 MiB out): the reference "
                         "that hardware counter readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: the library runs on one GPU; there is no multi-GPU path to measure (got --gpus %d)" % args.gpus)
        return 2

    import numpy as np
    import torch
    import paper_2407_13585_amd as fc
    from paper_2407_13585_amd.device import DeviceProgram, require_gpu
    from workloads import build

    dev = require_gpu()
    cfgs = [int(c) for c in args.configs.split(",")]

    # ---- build the workloads and the device programs --------------------------------------
    t0 = time.time()
    work, fused, unfused, kernels = {}, {}, {}, {}
    for c in cfgs:
        w = build(c, small=args.small)
        g, _ = fc.fc_duplicate(w.graph)
        part = fc.fc_plan(g, "bytes")
        footprint = sum(a.nbytes for a in w.inputs.values()) + 4 * sum(w.graph[o].size for o in w.graph.outputs())
        sets = max(2, min(8, -(-ROTATE_BYTES // max(footprint, 1))))
        fused[c] = [DeviceProgram(g, w.inputs, part) for _ in range(sets)]
        kernels[c] = fused[c][0].kernels()
        if not args.no_unfused:
            unfused[c] = DeviceProgram(w.graph, w.inputs, None)
        work[c] = w
        log(f"cfg{c}: {w.name} units={w.units} {w.unit_name}, LB={w.lb_bytes / 1e6:.1f} MB, "
            f"{part.n_clusters} fused cluster(s), {sets} rotating input sets: {kernels[c]}")
    log(f"setup {time.time() - t0:.1f}s")

    if args.calibrate:
        from workloads import Graph
        n = 1 << 26
        cg = Graph()
        cg.add("src", "input", "f32", (n,))
        cg.add("dst", "map", "f32", (n,), fn="ident", args=("src",), output=True)
        cal = DeviceProgram(cg, {"src": np.zeros(n, np.float32)}, fc.fc_plan(cg, "bytes"))
        for _ in range(3):
            cal.run()
        torch.cuda.synchronize()
        log(f"calibration copy: {cal.kernels()} moves {4 * n} B in and {4 * n} B out per launch")

    # pipeline 1 is 256 KiB and launch-latency bound; the same program at a bandwidth-sized n shows
    # what its kernel sustains (reported beside the step, not part of it)
    scaled = None
    if 1 in cfgs and not args.small:
        from workloads import configs as WC
        ws = WC.reverse_dot(n=1 << 26, seed=1)
        gs, _ = fc.fc_duplicate(ws.graph)
        ps = [DeviceProgram(gs, ws.inputs, fc.fc_plan(gs, "bytes")) for _ in range(3)]
        for p in ps:
            p.run()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for r in range(12):
            ps[r % 3].run()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) / 12 * 1e3
        gbs = ws.lb_bytes / us / 1e3
        scaled = {"n": 1 << 26, "kernel_us": round(us, 2), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
        log(f"cfg1 scaled to n=2^26: {us:9.1f} us  {gbs:8.1f} GB/s  {100 * gbs / HBM_PEAK_GBS:5.1f}% of HBM peak")
        del ps

    ceiling = gather_ceiling(fc, DeviceProgram, np, torch) if args.gather_ceiling else None
    examples = paper_examples(fc, DeviceProgram, np, torch) if args.paper_examples else None

    def one_step(s, events=None):
        for k, c in enumerate(cfgs):
            if events is not None:
                events[k].record()
            fused[c][s % len(fused[c])].run()
        if events is not None:
            events[len(cfgs)].record()

    # ---- timed region ----------------------------------------------------------------------
    for s in range(args.warmup):
        one_step(s)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(cfgs) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(args.warmup + s, ev[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    # per-pipeline kernel time from the HIP events on the launch stream
    kt = {c: [] for c in cfgs}
    for s in range(args.steps):
        for k, c in enumerate(cfgs):
            kt[c].append(ev[s][k].elapsed_time(ev[s][k + 1]))       # ms
    gpu_ms = {c: float(np.mean(kt[c])) for c in cfgs}
    gpu_med = {c: float(np.median(kt[c])) for c in cfgs}

    # ---- unfused arm: one kernel per combinator ---------------------------------------------
    unf_ms = {}
    if not args.no_unfused:
        for c in cfgs:
            p = unfused[c]
            reps = 3 if c == 5 else 5
            p.run()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                p.run()
            b.record()
            torch.cuda.synchronize()
            unf_ms[c] = a.elapsed_time(b) / reps

    # ---- CPU baseline: the oracle as it stands, one step on the host ------------------------
    cpu = None
    if not args.no_cpu:
        from oracle.interp import evaluate
        # whole steps, repeated until about ten seconds of host work have gone by (four at most)
        t0 = time.perf_counter()
        n_steps = 0
        while n_steps < 4 and (n_steps == 0 or time.perf_counter() - t0 < 10.0):
            for c in cfgs:
                evaluate(work[c].graph, work[c].inputs)
            n_steps += 1
        cpu_s = (time.perf_counter() - t0) / n_steps
        lb = sum(work[c].lb_bytes for c in cfgs)
        cpu = {"value": lb / cpu_s / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"{n_steps} whole steps (pipelines {args.configs} at the benchmarked sizes), {cpu_s:.2f} s each, "
                         f"numpy single thread, host has {os.cpu_count()} logical cores"}

    # ---- report ----------------------------------------------------------------------------
    lb_total = sum(work[c].lb_bytes for c in cfgs)
    per = {}
    for c in cfgs:
        w = work[c]
        gbs = w.lb_bytes / (gpu_ms[c] * 1e-3) / 1e9
        per[f"cfg{c}"] = {
            "kernel_ms": round(gpu_ms[c], 5), "kernel_ms_median": round(gpu_med[c], 5),
            "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
            f"{w.unit_name}/s": round(w.units / (gpu_ms[c] * 1e-3), 1), "lb_bytes": w.lb_bytes,
            "unfused_ms": round(unf_ms[c], 5) if c in unf_ms else None,
            "speedup_vs_unfused": round(unf_ms[c] / gpu_ms[c], 2) if c in unf_ms else None,
            "kernels": kernels[c], "traffic": measured_traffic(w.name),
        }
        log(f"cfg{c}: {gpu_ms[c] * 1e3:9.1f} us  {gbs:8.1f} GB/s  {100 * gbs / HBM_PEAK_GBS:5.1f}% of HBM peak  "
            + (f"unfused {unf_ms[c] * 1e3:10.1f} us  speedup {unf_ms[c] / gpu_ms[c]:6.2f}x" if c in unf_ms else ""))
    dom = max(cfgs, key=lambda c: gpu_ms[c])
    achieved = work[dom].lb_bytes / (gpu_ms[dom] * 1e-3) / 1e9
    out = {
        "metric": "fused pipeline GB/s (fused-traffic lower bound / time)",
        "value": round(lb_total / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": ("SMALL DEBUG SIZES " if args.small else "") +
                   "all five benchmark pipelines, fused: " + ", ".join(work[c].name for c in cfgs)},
        "gpu_sum_kernel_ms": round(sum(gpu_ms.values()), 5),
        "frac_hbm_peak": round(lb_total / (sum(gpu_ms.values()) * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "per_config": per,
        "roofline": {"bound": "hbm", "kernel": kernels[dom][0], "workload": work[dom].name,
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(work[dom].name),
                     "algorithmic_bytes": work[dom].lb_bytes},
        "cpu_baseline": cpu,
    }
    if scaled is not None:
        out["cfg1_scaled"] = scaled
    if ceiling is not None:
        out["gather_ceiling"] = ceiling
    if examples is not None:
        out["paper_examples"] = examples
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
