"""Coefficients of a linear cost function, fitted to measured run times.

Section 5.1 ("Runtime analysis") observes that none of the paper's cost functions models
run time well and proposes a linear combination of cost functions whose coefficients are
found by tuning.  This module does that for the machine it runs on: it executes several
legal clusterings of a set of programs, records the value of every cost function and the
time of each, fits non-negative coefficients (time ~ sum_k w_k * cost_k), and hands them
to fc_plan_weighted.  With the two columns used by default the coefficients have a plain
reading: `clusters` is the cost of one kernel launch, `bytes` the inverse of the bandwidth
the kernels sustain.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np

from . import binding as B


def candidate_partitions(graph) -> List[B.Partition]:
    """Clusterings worth timing: the optimum of every cost function, both greedy arms and no
    fusion, without repeats."""
    found, seen = [], set()

    def add(make):
        try:
            p = make()
        except B.FcError:
            return
        key = tuple(int(x) for x in p.pi)
        if key not in seen:
            seen.add(key)
            found.append(p)

    for cost in B.COST:
        add(lambda: B.fc_plan(graph, cost))
    for direction in ("top_down", "bottom_up"):
        add(lambda: B.fc_plan_greedy(graph, direction, "bytes"))
    add(lambda: B.fc_partition_trivial(graph))
    return found


def fit_weights(cost_vectors: np.ndarray, times: np.ndarray, columns: Sequence[str] = ("clusters", "bytes")) -> Dict[str, float]:
    """Non-negative least squares of times against the chosen cost columns."""
    from scipy.optimize import nnls
    cols = [B.COST[c] for c in columns]
    a = np.asarray(cost_vectors, dtype=np.float64)[:, cols]
    scale = np.maximum(a.max(axis=0), 1e-300)            # columns differ by many orders of magnitude
    w, _ = nnls(a / scale, np.asarray(times, dtype=np.float64))
    w = w / scale
    if not np.any(w > 0):
        raise ValueError("the samples do not determine any coefficient")
    return {c: float(x) for c, x in zip(columns, w)}


def time_partition(graph, inputs, partition, reps: int = 20) -> float:
    """Microseconds per run of the program under this clustering on the current GPU;
    raises FcError if a cluster has no kernel."""
    import torch
    from .device import DeviceProgram
    prog = DeviceProgram(graph, inputs, partition)
    for _ in range(3):
        prog.run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        prog.run()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps * 1e3


def tune(programs: Sequence[Tuple[object, dict]], columns: Sequence[str] = ("clusters", "bytes"), reps: int = 20):
    """programs: (graph, inputs) pairs.  Returns (weights, samples); samples lists, per timed
    clustering, the program index, its cluster numbers, its cost vector and its time in us."""
    samples = []
    for k, (graph, inputs) in enumerate(programs):
        for part in candidate_partitions(graph):
            try:
                us = time_partition(graph, inputs, part, reps)
            except B.FcError:
                continue                                   # legal, but some cluster has no kernel instance
            samples.append({"program": k, "pi": [int(x) for x in part.pi],
                            "costs": B.cost_vector(graph, part.pi), "us": us})
    if not samples:
        raise ValueError("no clustering of any program could be timed")
    weights = fit_weights(np.stack([s["costs"] for s in samples]), np.array([s["us"] for s in samples]), columns)
    return weights, samples
