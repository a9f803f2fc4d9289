#!/usr/bin/env python3
"""Throughput of the fused pipelines on one MI355X.

A step is one pass of the whole hot path: the five synthetic pipelines, each
executed as its fused clusters (fc_run_fused), inputs resident in HBM.  The
reported value is the fused-traffic lower bound of a step (every external input
byte once + every output byte once) divided by the time of a step.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--configs 1,2,3,4,5]

One JSON line goes to stdout; a table per pipeline goes to stderr.  Beside the
step the run measures, each outside the timed region: the unfused arm (one kernel
per combinator), the single-pass kernels of the two gather pipelines (the
library's default for them visits the positions in another order), the
"materialise p" clustering of the stencil pipeline, a plain copy kernel (the
ceiling of the memory system), the oracle on the host (one core, then all
cores), and it compares the outputs of the timed programs with the oracle's.
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


# ---------------------------------------------------------------------------- host side (before the GPU is touched)
def oracle_outputs(work, cfgs):
    """One evaluation of every pipeline by the oracle; keeps the results the GPU run is checked against."""
    from oracle.interp import evaluate
    keep = {}
    for c in cfgs:
        env = evaluate(work[c].graph, work[c].inputs)
        keep[c] = {o: env[o] for o in work[c].graph.outputs()}
    return keep


def oracle_one_core(work, cfgs, budget_s=10.0, most=4):
    """Whole steps of the oracle, one numpy thread, until about budget_s have gone by."""
    from oracle.interp import evaluate
    t0 = time.perf_counter()
    n = 0
    while n < most and (n == 0 or time.perf_counter() - t0 < budget_s):
        for c in cfgs:
            evaluate(work[c].graph, work[c].inputs)
        n += 1
    return (time.perf_counter() - t0) / n, n


def oracle_all_cores(work, cfgs):
    """The oracle as it stands on every host core at once: P processes, each evaluates one
    whole step (the pipelines in a rotated order, so that their memory peaks do not coincide).
    The aggregate rate is P steps over the time until the last process is done.  Forked before
    anything touches the GPU; the children run numpy only."""
    import multiprocessing as mp
    from oracle.interp import evaluate
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    procs = max(1, min(cores, 16))
    ctx = mp.get_context("fork")
    start = ctx.Barrier(procs + 1)

    def worker(k):
        start.wait()
        order = cfgs[k % len(cfgs):] + cfgs[:k % len(cfgs)]
        for c in order:
            evaluate(work[c].graph, work[c].inputs)

    ps = [ctx.Process(target=worker, args=(k,)) for k in range(procs)]
    for p in ps:
        p.start()
    start.wait()
    t0 = time.perf_counter()
    for p in ps:
        p.join()
    wall = time.perf_counter() - t0
    if any(p.exitcode != 0 for p in ps):
        raise RuntimeError("a worker of the all-core oracle run failed: " + str([p.exitcode for p in ps]))
    return wall, procs


def verify(np, c, w, got, ref):
    """Outputs of the timed fused program of pipeline c against the oracle's, under the rules of the
    parity tests: integers exact, fp32 (+) folds 1e-5 relative, the segmented fold 1e-5 norm-wise,
    the stencil sum 1e-6 relative elementwise, max within 4 ulp."""
    F32 = np.float32
    if c in (1, 2):
        g, r = float(got["r"][0]), float(ref["r"][0])
        return abs(g - r) <= 1e-5 * abs(r), f"r gpu={g!r} oracle={r!r}"
    if c == 3:
        g, r = got["y"].astype(np.float64), ref["y"].astype(np.float64)
        e = float(np.linalg.norm(g - r)) / max(float(np.linalg.norm(r)), 1e-30)
        return e <= 1e-5, f"y relative 2-norm error {e:.2e}"
    if c == 4:
        count = int(ref["count"][0])
        ok = int(got["count"][0]) == count and np.array_equal(got["out"][:count], ref["out"][:count])
        return ok, f"count gpu={int(got['count'][0])} oracle={count}"
    g, r = got["out"].astype(np.float64), ref["out"].astype(np.float64)
    e = float(np.max(np.abs(g - r) / np.abs(r)))
    m_g, m_r = F32(got["m"][0]), F32(ref["m"][0])
    ok = e <= 1e-6 and abs(float(m_g) - float(m_r)) <= 4 * float(np.spacing(m_r))
    return ok, f"out max relative error {e:.2e}, m gpu={m_g!r} oracle={m_r!r}"


# ---------------------------------------------------------------------------- device side
def time_rotating(torch, progs, reps):
    """Mean time of a run in ms: every program warmed once, then `reps` runs that cycle through them."""
    for p in progs:
        p.run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for r in range(reps):
        progs[r % len(progs)].run()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def rotating_sets(nbytes, most=8):
    return max(2, min(most, -(-ROTATE_BYTES // max(int(nbytes), 1))))


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
        progs = [DeviceProgram(g, {"idx": rng.permutation(n).astype(np.int32), "xs": np.ones(n, np.float32)}, part)
                 for _ in range(rotating_sets(8 * n))]
        us = time_rotating(torch, progs, 16) * 1e3
        out[f"table_2^{logn}_f32"] = {"us": round(us, 2), "Ggather/s": round(n / us / 1e3, 2), "kernel": progs[0].kernels()[0]}
        log(f"bare gather, table 2^{logn} floats: {us:8.1f} us  {n / us / 1e3:6.1f} G gathers/s")
    return out


def paper_examples(fc, DeviceProgram, np, torch):
    """The programs the paper times that can be rebuilt from its text (section 5, "Greedy
    counterexamples", and `singleLoop` of section 1): fused by fc_plan versus no fusion.  The
    scalar that the paper's listings index out of an array (`zs!0`, `bs!0`) is a whole array
    added elementwise here (workloads/paper_graphs.py): the same clustering problem, not the
    same arithmetic, so the times are of that stand-in."""
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
        t = {tag: time_rotating(torch, [p], 10) * 1e3 for tag, p in progs.items()}
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
    ap.add_argument("--no-unfused", action="store_true", help="skip the comparison arms (unfused, single-pass, materialise p)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle on the host (and with it the check of the outputs)")
    ap.add_argument("--gather-ceiling", action="store_true",
                    help="also measure the rate of bare random gathers (no arithmetic) for three table sizes")
    ap.add_argument("--paper-examples", action="store_true",
                    help="also time the paper's small example programs, fused against unfused")
    ap.add_argument("--calibrate", action="store_true",
                    help="run the plain copy kernel a few more times under its own name: the reference that "
                         "hardware counter readings are scaled by (256 MiB in, 256 MiB out per launch)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: the library runs on one GPU; there is no multi-GPU path to measure (got --gpus %d)" % args.gpus)
        return 2

    import numpy as np
    from workloads import Graph, build, single_pass

    cfgs = [int(c) for c in args.configs.split(",")]
    t0 = time.time()
    work = {c: build(c, small=args.small) for c in cfgs}
    lb_total = sum(work[c].lb_bytes for c in cfgs)
    log(f"workloads built in {time.time() - t0:.1f}s")

    # ---- CPU baseline: the oracle as it stands, before anything touches the GPU ---------------
    cpu, expected = None, None
    if not args.no_cpu:
        t0 = time.perf_counter()
        expected = oracle_outputs(work, cfgs)
        first = time.perf_counter() - t0
        cpu_s, n_steps = oracle_one_core(work, cfgs, budget_s=max(0.0, 10.0 - first), most=3)
        all_s, procs = oracle_all_cores(work, cfgs)
        cpu = {"value": lb_total / cpu_s / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"{n_steps} whole steps (pipelines {args.configs} at the benchmarked sizes), {cpu_s:.2f} s each, "
                         f"numpy single thread, host has {os.cpu_count()} logical cores",
               "all_cores": {"value": procs * lb_total / all_s / 1e9, "unit": "GB/s", "cores": procs, "kind": "oracle",
                             "sample": f"{procs} processes at once, one whole step each (the same oracle, nothing shared "
                                       f"but the inputs), {all_s:.2f} s until the last is done; aggregate rate"}}
        log(f"oracle: one core {cpu_s:.2f} s per step ({cpu['value']:.2f} GB/s); {procs} processes {all_s:.2f} s "
            f"({cpu['all_cores']['value']:.2f} GB/s aggregate)")

    import torch
    import paper_2407_13585_amd as fc
    from paper_2407_13585_amd.device import DeviceProgram, require_gpu

    require_gpu()

    # ---- the device programs ------------------------------------------------------------------
    t0 = time.time()
    fused, kernels, arms = {}, {}, {c: {} for c in cfgs}
    for c in cfgs:
        w = work[c]
        g, _ = fc.fc_duplicate(w.graph)
        part = fc.fc_plan(g, "bytes")
        footprint = sum(a.nbytes for a in w.inputs.values()) + 4 * sum(w.graph[o].size for o in w.graph.outputs())
        fused[c] = [DeviceProgram(g, w.inputs, part) for _ in range(rotating_sets(footprint))]
        kernels[c] = fused[c][0].kernels()
        log(f"cfg{c}: {w.name} units={w.units} {w.unit_name}, LB={w.lb_bytes / 1e6:.1f} MB, "
            f"{part.n_clusters} fused cluster(s), {len(fused[c])} rotating input sets: {kernels[c]}")
        if args.no_unfused:
            continue
        # one kernel per combinator, every intermediate in memory; buffer sets rotate as for the fused arm
        arms[c]["unfused"] = [DeviceProgram(w.graph, w.inputs, None) for _ in range(rotating_sets(w.unfused_bytes, most=4))]
        if c in (2, 3):
            # the same cluster as one pass over its arrays, gathers issued in position order (FC_NODE_SINGLE_PASS)
            gs, _ = fc.fc_duplicate(single_pass(w.graph))
            ps = fc.fc_plan(gs, "bytes")
            arms[c]["single_pass"] = [DeviceProgram(gs, w.inputs, ps) for _ in range(len(fused[c]))]
        if c == 5:
            # the optimum of the paper's ILP proper (no work duplication): p stored by the cluster that folds it,
            # the stencil a second cluster that reads it back
            pm = fc.fc_plan(w.graph, "bytes")
            arms[c]["materialise_p"] = [DeviceProgram(w.graph, w.inputs, pm) for _ in range(2)]
    log(f"setup {time.time() - t0:.1f}s")

    # the ceiling of the memory system: a plain copy, 256 MiB in and 256 MiB out per launch
    n = 1 << (20 if args.small else 26)
    cg = Graph()
    cg.add("src", "input", "f32", (n,))
    cg.add("dst", "map", "f32", (n,), fn="ident", args=("src",), output=True)
    copy_part = fc.fc_plan(cg, "bytes")
    copies = [DeviceProgram(cg, {"src": np.zeros(n, np.float32)}, copy_part) for _ in range(3)]
    copy_ms = time_rotating(torch, copies, 12)
    copy_gbs = 8 * n / (copy_ms * 1e-3) / 1e9
    log(f"copy ceiling: {copies[0].kernels()} moves {4 * n} B in and {4 * n} B out in {copy_ms * 1e3:.1f} us: {copy_gbs:.0f} GB/s")
    if args.calibrate:
        for _ in range(3):
            copies[0].run()
        torch.cuda.synchronize()
    del copies

    # pipeline 1 is 256 KiB and launch-latency bound; the same program at a bandwidth-sized n shows
    # what its kernel sustains (reported beside the step, not part of it)
    scaled = None
    if 1 in cfgs and not args.small:
        from workloads import configs as WC
        ws = WC.reverse_dot(n=1 << 26, seed=1)
        gs, _ = fc.fc_duplicate(ws.graph)
        ps = [DeviceProgram(gs, ws.inputs, fc.fc_plan(gs, "bytes")) for _ in range(3)]
        us = time_rotating(torch, ps, 12) * 1e3
        gbs = ws.lb_bytes / us / 1e3
        scaled = {"n": 1 << 26, "kernel_us": round(us, 2), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                  "frac_copy_ceiling": round(gbs / copy_gbs, 4)}
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

    # ---- the outputs of the timed programs against the oracle --------------------------------
    verified = None
    if expected is not None:
        verified = True
        for c in cfgs:
            for k, prog in enumerate(fused[c]):
                prog.check()                                     # no bounded wait gave up
                got = {o: prog.fetch(o) for o in work[c].graph.outputs()}
                ok, what = verify(np, c, work[c], got, expected[c])
                if not ok:
                    verified = False
                    log(f"cfg{c}, input set {k}: the GPU result does not match the oracle: {what}")
        if not verified:
            log("bench.py: results do not match the oracle; no measurement is reported")
            return 1
        log("outputs of every timed program match the oracle")

    # ---- comparison arms, each timed on its own with rotating buffer sets ---------------------
    arm_ms = {c: {name: time_rotating(torch, progs, max(3, 12 // len(progs) * len(progs)) if c != 5 else 4)
                  for name, progs in arms[c].items()} for c in cfgs}
    arm_kernels = {c: {name: progs[0].kernels() for name, progs in arms[c].items() if name != "unfused"} for c in cfgs}

    # ---- report ----------------------------------------------------------------------------
    per = {}
    for c in cfgs:
        w = work[c]
        gbs = w.lb_bytes / (gpu_ms[c] * 1e-3) / 1e9
        unf = arm_ms[c].get("unfused")
        row = {
            "kernel_ms": round(gpu_ms[c], 5), "kernel_ms_median": round(gpu_med[c], 5),
            "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
            "frac_copy_ceiling": round(gbs / copy_gbs, 4),
            f"{w.unit_name}/s": round(w.units / (gpu_ms[c] * 1e-3), 1), "lb_bytes": w.lb_bytes,
            "unfused_ms": round(unf, 5) if unf else None,
            "speedup_vs_unfused": round(unf / gpu_ms[c], 2) if unf else None,
            "kernels": kernels[c], "traffic": measured_traffic(w.name),
        }
        if c == 1 and not args.small:
            row["note"] = "256 KiB: bound by the latency of a launch, not by bandwidth (see cfg1_scaled)"
        if "single_pass" in arm_ms[c]:
            sp = arm_ms[c]["single_pass"]
            row.update({"single_pass_ms": round(sp, 5), "single_pass_kernels": arm_kernels[c]["single_pass"],
                        "single_pass_GB/s": round(w.lb_bytes / (sp * 1e-3) / 1e9, 1),
                        "speedup_vs_unfused_single_pass": round(unf / sp, 2),
                        "note": "kernel_ms is the default kernel, which visits the gathered positions in another order than "
                                "the unfused arm does (so speedup_vs_unfused mixes fusion with locality); single_pass_ms is "
                                "the cluster as one pass with the gathers in position order, as in the unfused arm"})
        if "materialise_p" in arm_ms[c]:
            mp_ms = arm_ms[c]["materialise_p"]
            row.update({"materialise_p_ms": round(mp_ms, 5), "materialise_p_kernels": arm_kernels[c]["materialise_p"],
                        "speedup_vs_materialise_p": round(mp_ms / gpu_ms[c], 2),
                        "materialise_p_bytes": w.extra.get("materialise_p_bytes")})
        per[f"cfg{c}"] = row
        log(f"cfg{c}: {gpu_ms[c] * 1e3:9.1f} us  {gbs:8.1f} GB/s  {100 * gbs / HBM_PEAK_GBS:5.1f}% of HBM peak  "
            f"{100 * gbs / copy_gbs:5.1f}% of the copy ceiling  "
            + (f"unfused {unf * 1e3:10.1f} us  speedup {unf / gpu_ms[c]:6.2f}x" if unf else "")
            + (f"  single pass {arm_ms[c]['single_pass'] * 1e3:8.1f} us ({unf / arm_ms[c]['single_pass']:.2f}x)" if "single_pass" in arm_ms[c] else "")
            + (f"  materialise p {arm_ms[c]['materialise_p'] * 1e3:8.1f} us ({arm_ms[c]['materialise_p'] / gpu_ms[c]:.2f}x)" if "materialise_p" in arm_ms[c] else ""))
    dom = max(cfgs, key=lambda c: gpu_ms[c])
    achieved = work[dom].lb_bytes / (gpu_ms[dom] * 1e-3) / 1e9
    # the same sum with every cluster that has a single-pass form run in that form (gathers in position order, one
    # kernel, nothing sorted): what the step costs when each cluster is the one pass the paper describes
    sp_ms = {c: arm_ms[c].get("single_pass", gpu_ms[c]) for c in cfgs}
    single_pass_sum = sum(sp_ms.values()) if any("single_pass" in arm_ms[c] for c in cfgs) else None
    if single_pass_sum is not None:
        log(f"all pipelines: {sum(gpu_ms.values()) * 1e3:.1f} us with the default kernels ({lb_total / (sum(gpu_ms.values()) * 1e-3) / 1e9:.0f} GB/s), "
            f"{single_pass_sum * 1e3:.1f} us with the gather clusters as single passes ({lb_total / (single_pass_sum * 1e-3) / 1e9:.0f} GB/s)")
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
        "single_pass_clusters": None if single_pass_sum is None else {
            "gpu_sum_kernel_ms": round(single_pass_sum, 5), "GB/s": round(lb_total / (single_pass_sum * 1e-3) / 1e9, 1),
            "note": "the sum of the per-pipeline times with the gather pipelines' clusters run as single passes "
                    "(FC_NODE_SINGLE_PASS: one kernel, gathers in position order); `value` uses the default kernels, "
                    "which sort the gathered positions by table range first"},
        "copy_ceiling_GBs": round(copy_gbs, 1),
        "verified_against_oracle": verified,
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
