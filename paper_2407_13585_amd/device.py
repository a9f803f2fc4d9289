"""Device-side plumbing for running a program: torch supplies memory and streams, nothing else.

`DeviceProgram` uploads the inputs of a workload, allocates the output (and, on
request, the intermediate) arrays and the scratch buffer, and calls
fc_run_fused / fc_run_unfused.  No combinator is evaluated here.
"""
from __future__ import annotations

from typing import Dict, Iterable, Optional

import numpy as np
import torch

from . import binding as B

_NP = {"f32": np.float32, "i32": np.int32}
_TORCH = {"f32": torch.float32, "i32": torch.int32}


def require_gpu() -> torch.device:
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: the HIP path has no CPU fallback")
    return torch.device("cuda:0")


class DeviceProgram:
    def __init__(self, graph, inputs: Dict[str, np.ndarray], partition: Optional[B.Partition] = None,
                 bind: Iterable[str] = (), device: Optional[torch.device] = None):
        """partition None = unfused execution.  `bind` names extra (intermediate) arrays
        to place in caller-visible tensors so they can be fetched."""
        self.device = device or require_gpu()
        self.graph = graph
        self.cg = B.CGraph(graph)
        self.partition = partition
        self.buffers: Dict[str, torch.Tensor] = {}
        by_name = {n.name: n for n in graph.nodes}
        for n in graph.nodes:
            if n.kind == "input":
                a = np.ascontiguousarray(inputs[n.name], dtype=_NP[n.dtype])
                if a.size != n.size:
                    raise ValueError(f"input {n.name}: expected {n.size} elements")
                # at least one element so that empty arrays still have a valid pointer
                t = torch.empty(max(a.size, 4), dtype=_TORCH[n.dtype], device=self.device)
                if a.size:
                    t[:a.size].copy_(torch.from_numpy(a.reshape(-1)))
                self.buffers[n.name] = t
        wanted = set(graph.outputs()) | set(bind)
        for n in reversed(graph.nodes):   # a fetched scatter needs its destination in a caller-visible tensor
            if n.kind == "scatter" and n.name in wanted:
                wanted.add(n.args[0])
        for n in graph.nodes:
            if n.name in wanted and n.kind not in ("input", "scatter"):
                self.buffers[n.name] = torch.zeros(max(n.size, 4), dtype=_TORCH[n.dtype], device=self.device)
        for n in graph.nodes:          # a scatter lives in the buffer of its destination (if the caller holds that one)
            if n.kind == "scatter" and by_name[n.args[0]].name in self.buffers:
                self.buffers[n.name] = self.buffers[by_name[n.args[0]].name]
        nbytes = B.fc_scratch_bytes(self.cg, partition)
        self.scratch = torch.zeros((nbytes + 3) // 4, dtype=torch.int32, device=self.device)
        self._bound = B.BoundRun(self.cg, partition, self.buffers, self.scratch)

    def run(self, stream: Optional[torch.cuda.Stream] = None) -> None:
        self._bound((stream or torch.cuda.current_stream(self.device)).cuda_stream)

    def fetch(self, name: str) -> np.ndarray:
        n = self.graph[name]
        torch.cuda.synchronize(self.device)
        t = self.buffers[name]
        return t[:n.size].cpu().numpy().reshape(n.shape).copy()

    def upload(self, name: str, a: np.ndarray) -> None:
        n = self.graph[name]
        a = np.ascontiguousarray(a, dtype=_NP[n.dtype]).reshape(-1)
        if a.size:
            self.buffers[name][:a.size].copy_(torch.from_numpy(a))

    def check(self, stream: Optional[torch.cuda.Stream] = None) -> None:
        """fc_check on this program's scratch buffer: synchronises the stream, raises FcError if a
        bounded wait gave up since the last check."""
        B.fc_check(self.scratch, (stream or torch.cuda.current_stream(self.device)).cuda_stream)

    def control_words(self) -> np.ndarray:
        """First words of the scratch control block: launch epoch, error flag."""
        torch.cuda.synchronize(self.device)
        return self.scratch[:4].cpu().numpy().copy()

    def kernels(self):
        k = self.partition.n_clusters if self.partition is not None else B.fc_partition_trivial(self.cg).n_clusters
        return [B.fc_cluster_kernel(self.cg, self.partition, i) for i in range(k)]
