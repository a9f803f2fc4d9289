"""ctypes binding of libfc.so: the calls of include/fc.h under the same names.

Argument marshalling only.  Every step of a program runs in the library's HIP
kernels; there is no Python or CPU fallback, and a missing library is an error.
Device memory and streams come from the caller (torch tensors or raw pointers).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from workloads.graph import Graph

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfc.so")

FC_MAX_ARGS = 6
FC_SCRATCH_CONTROL_BYTES = 1 << 23

KIND = {"input": 0, "map": 1, "generate": 2, "gather": 3, "fold": 4, "foldseg": 5,
        "scanl": 6, "scanr": 7, "scatter": 8, "force": 9}
DTYPE = {"f32": 0, "i32": 1}
FN = {"": 0, "ident": 1, "affine": 2, "sin_x_mul_x": 3, "sq_plus_one": 4, "mul2": 5, "add2": 6,
      "add3": 7, "add5": 8, "exp_neg": 9, "mod_eq": 10,
      "iota": 32, "iota_rev": 33, "clamp_shift_2d": 34, "row_of_2d": 35, "const_i32": 36}
OP = {"add": 64, "max": 65, "mul": 66, "overwrite": 67}
COST = {"clusters": 0, "fused_edges": 1, "arrays": 2, "reads": 3, "reads_writes": 4, "bytes": 5}
FC_PLAN_NO_SPLIT = 1
FC_PLAN_EXECUTABLE = 2
FC_PLAN_ANYTIME = 4
FC_NODE_OUTPUT = 1
FC_NODE_SINGLE_PASS = 2

ERRORS = {-1: "FC_E_BADGRAPH", -2: "FC_E_ILLEGAL_PARTITION", -3: "FC_E_UNSUPPORTED", -4: "FC_E_UNBOUND",
          -5: "FC_E_SCRATCH", -6: "FC_E_HIP", -7: "FC_E_ARG", -8: "FC_E_LIMIT", -9: "FC_E_DEVICE_WAIT"}


class FcError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"{ERRORS.get(code, code)}: {message}")
        self.code = code
        self.name = ERRORS.get(code, str(code))


class fc_node(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32), ("fn", C.c_int32),
                ("fparam", C.c_float * 2), ("iparam", C.c_int32 * 4),
                ("nargs", C.c_int32), ("arg", C.c_int32 * FC_MAX_ARGS),
                ("rank", C.c_int32), ("shape", C.c_int64 * 2), ("flags", C.c_uint32),
                ("infusible_args", C.c_uint32)]


class fc_graph(C.Structure):
    _fields_ = [("n", C.c_int32), ("nodes", C.POINTER(fc_node))]


class fc_partition(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("n_edges", C.c_int32),
                ("pi", C.POINTER(C.c_int32)), ("fused_away", C.POINTER(C.c_uint8)),
                ("order_out", C.POINTER(C.c_int32)), ("edge_unfused", C.POINTER(C.c_uint8)),
                ("n_clusters", C.c_int32), ("cost", C.c_double), ("proven", C.c_int32)]


class fc_buffer(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("bytes", C.c_int64)]


_lib = None


def _share_hip_runtime_with_torch() -> None:
    """Device pointers and streams come from the caller's torch, so the library must use
    the HIP runtime torch uses.  torch wheels ship their own libamdhip64.so; loading it
    first makes the dynamic loader resolve the library's libamdhip64.so.7 dependency to
    that same object (matched by SONAME) instead of a second runtime under /opt/rocm."""
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.submodule_search_locations:
        return
    path = os.path.join(list(spec.submodule_search_locations)[0], "lib", "libamdhip64.so")
    if os.path.exists(path):
        C.CDLL(path, mode=C.RTLD_GLOBAL)


def lib() -> C.CDLL:
    """Loads libfc.so; builds it first only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing and could not be built; there is no fallback path")
    _share_hip_runtime_with_torch()
    L = C.CDLL(_LIB_PATH)
    L.fc_last_error.restype = C.c_char_p
    PG, PP = C.POINTER(fc_graph), C.POINTER(fc_partition)
    L.fc_num_edges.argtypes = [PG, C.POINTER(C.c_int32)]
    L.fc_plan.argtypes = [PG, C.c_int, C.c_uint32, PP]
    L.fc_plan_weighted.argtypes = [PG, C.POINTER(C.c_double), C.c_uint32, PP]
    L.fc_plan_greedy.argtypes = [PG, C.c_int, C.c_int, C.c_uint32, PP]
    L.fc_partition_trivial.argtypes = [PG, PP]
    L.fc_partition_check.argtypes = [PG, PP, C.c_int, C.POINTER(C.c_double)]
    L.fc_duplicate.argtypes = [PG, C.POINTER(fc_node), C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.fc_scratch_bytes.argtypes = [PG, PP, C.POINTER(C.c_size_t)]
    L.fc_run_fused.argtypes = [PG, PP, C.POINTER(fc_buffer), C.c_void_p, C.c_size_t, C.c_void_p]
    L.fc_run_unfused.argtypes = [PG, C.POINTER(fc_buffer), C.c_void_p, C.c_size_t, C.c_void_p]
    L.fc_cluster_kernel.argtypes = [PG, PP, C.c_int32, C.c_char_p, C.c_size_t]
    L.fc_check.argtypes = [C.c_void_p, C.c_void_p]
    L.fc_run_fused_static.argtypes = [PG, PP, C.POINTER(fc_buffer), C.c_void_p]
    for f in ("fc_check", "fc_run_fused_static", "fc_num_edges", "fc_plan", "fc_plan_weighted", "fc_plan_greedy", "fc_partition_trivial", "fc_partition_check", "fc_duplicate",
              "fc_scratch_bytes", "fc_run_fused", "fc_run_unfused", "fc_cluster_kernel"):
        getattr(L, f).restype = C.c_int
    _lib = L
    return L


def _check(rc: int):
    if rc != 0:
        raise FcError(rc, lib().fc_last_error().decode())


# ------------------------------------------------------------------ graph marshalling
class CGraph:
    """fc_graph plus the storage it points to."""

    def __init__(self, graph: Graph):
        self.graph = graph
        self.names = [n.name for n in graph.nodes]
        ix = graph.index()
        self.nodes = (fc_node * max(len(graph.nodes), 1))()
        for i, n in enumerate(graph.nodes):
            c = self.nodes[i]
            c.kind, c.dtype = KIND[n.kind], DTYPE[n.dtype]
            if n.kind in ("fold", "foldseg", "scanl", "scanr", "scatter"):
                c.fn = OP[n.fn]
            else:
                c.fn = FN[n.fn]
            for k, v in enumerate(n.fparam[:2]):
                c.fparam[k] = float(v)
            for k, v in enumerate(n.iparam[:4]):
                c.iparam[k] = int(v)
            if len(n.args) > FC_MAX_ARGS:
                raise ValueError(f"{n.name}: too many arguments")
            c.nargs = len(n.args)
            for k, a in enumerate(n.args):
                c.arg[k] = ix[a]
            if len(n.shape) not in (1, 2):
                raise ValueError(f"{n.name}: rank must be 1 or 2")
            c.rank = len(n.shape)
            c.shape[0] = int(n.shape[0])
            c.shape[1] = int(n.shape[1]) if len(n.shape) == 2 else 1
            c.flags = (FC_NODE_OUTPUT if n.output else 0) | (FC_NODE_SINGLE_PASS if getattr(n, "single_pass", False) else 0)
            c.infusible_args = sum(1 << k for k in getattr(n, "infusible", ()))
        self.c = fc_graph(len(graph.nodes), self.nodes)
        self.n_edges = len(graph.edges())

    def ref(self):
        return C.byref(self.c)


def _cg(graph) -> CGraph:
    return graph if isinstance(graph, CGraph) else CGraph(graph)


@dataclass
class Partition:
    pi: np.ndarray
    fused_away: np.ndarray
    order_out: np.ndarray
    edge_unfused: np.ndarray
    n_clusters: int = 0
    cost: float = 0.0
    proven: bool = True          # False: the best clustering found when an anytime search ran out of budget

    def _c(self) -> fc_partition:
        self.pi = np.ascontiguousarray(self.pi, dtype=np.int32)
        self.fused_away = np.ascontiguousarray(self.fused_away, dtype=np.uint8)
        self.order_out = np.ascontiguousarray(self.order_out, dtype=np.int32)
        self.edge_unfused = np.ascontiguousarray(self.edge_unfused, dtype=np.uint8)
        p = fc_partition()
        p.n_nodes, p.n_edges = len(self.pi), len(self.edge_unfused)
        p.pi = self.pi.ctypes.data_as(C.POINTER(C.c_int32))
        p.fused_away = self.fused_away.ctypes.data_as(C.POINTER(C.c_uint8))
        p.order_out = self.order_out.ctypes.data_as(C.POINTER(C.c_int32))
        p.edge_unfused = self.edge_unfused.ctypes.data_as(C.POINTER(C.c_uint8))
        return p

    @staticmethod
    def empty(n_nodes: int, n_edges: int) -> "Partition":
        return Partition(np.zeros(n_nodes, np.int32), np.zeros(n_nodes, np.uint8),
                         np.zeros(n_nodes, np.int32), np.zeros(n_edges, np.uint8))


def _finish(part: Partition, cp: fc_partition) -> Partition:
    part.n_clusters, part.cost, part.proven = int(cp.n_clusters), float(cp.cost), bool(cp.proven)
    return part


# ------------------------------------------------------------------ the calls of fc.h
def fc_num_edges(graph) -> int:
    g = _cg(graph)
    n = C.c_int32()
    _check(lib().fc_num_edges(g.ref(), C.byref(n)))
    return n.value


def _plan_flags(no_split: bool, executable: bool, anytime: bool = False) -> int:
    return (FC_PLAN_NO_SPLIT if no_split else 0) | (FC_PLAN_EXECUTABLE if executable else 0) | (FC_PLAN_ANYTIME if anytime else 0)


def fc_plan(graph, cost: str = "bytes", no_split: bool = False, executable: bool = False, anytime: bool = False) -> Partition:
    """executable: choose among the clusterings the library has kernels for (FC_PLAN_EXECUTABLE).
    anytime: search for a few seconds at most and return the best clustering found (Partition.proven tells)."""
    g = _cg(graph)
    part = Partition.empty(len(g.names), g.n_edges)
    cp = part._c()
    _check(lib().fc_plan(g.ref(), COST[cost], _plan_flags(no_split, executable, anytime), C.byref(cp)))
    return _finish(part, cp)


def _weights(weights) -> "C.Array":
    """weights: {cost name: coefficient} or a sequence of len(COST) coefficients in fc_cost order."""
    if isinstance(weights, dict):
        unknown = set(weights) - set(COST)
        if unknown:
            raise ValueError(f"unknown cost functions {sorted(unknown)}")
        vec = [float(weights.get(k, 0.0)) for k in sorted(COST, key=COST.get)]
    else:
        vec = [float(x) for x in weights]
        if len(vec) != len(COST):
            raise ValueError(f"expected {len(COST)} weights")
    return (C.c_double * len(COST))(*vec)


def fc_plan_weighted(graph, weights, no_split: bool = False, executable: bool = False, anytime: bool = False) -> Partition:
    g = _cg(graph)
    part = Partition.empty(len(g.names), g.n_edges)
    cp = part._c()
    _check(lib().fc_plan_weighted(g.ref(), _weights(weights), _plan_flags(no_split, executable, anytime), C.byref(cp)))
    return _finish(part, cp)


def cost_vector(graph, pi: Sequence[int]) -> np.ndarray:
    """The values of all cost functions (fc_cost order) for the clustering with these cluster numbers."""
    g = _cg(graph)
    out = np.zeros(len(COST))
    for name, k in COST.items():
        part = Partition.empty(len(g.names), g.n_edges)
        part.pi[:] = np.asarray(pi, dtype=np.int32)
        cp = part._c()
        v = C.c_double()
        _check(lib().fc_partition_check(g.ref(), C.byref(cp), k, C.byref(v)))
        out[k] = v.value
    return out


def fc_plan_greedy(graph, direction: str, cost: str = "bytes", no_split: bool = False, executable: bool = False) -> Partition:
    """direction: 'top_down' or 'bottom_up'."""
    g = _cg(graph)
    part = Partition.empty(len(g.names), g.n_edges)
    cp = part._c()
    d = {"top_down": 0, "bottom_up": 1}[direction]
    _check(lib().fc_plan_greedy(g.ref(), d, COST[cost], _plan_flags(no_split, executable), C.byref(cp)))
    return _finish(part, cp)


def fc_partition_trivial(graph) -> Partition:
    g = _cg(graph)
    part = Partition.empty(len(g.names), g.n_edges)
    cp = part._c()
    _check(lib().fc_partition_trivial(g.ref(), C.byref(cp)))
    return _finish(part, cp)


def fc_partition_check(graph, pi: Sequence[int], cost: str = "reads_writes") -> Partition:
    g = _cg(graph)
    part = Partition.empty(len(g.names), g.n_edges)
    part.pi[:] = np.asarray(pi, dtype=np.int32)
    cp = part._c()
    v = C.c_double()
    _check(lib().fc_partition_check(g.ref(), C.byref(cp), COST[cost], C.byref(v)))
    return _finish(part, cp)


def fc_duplicate(graph: Graph) -> Tuple[Graph, List[int]]:
    g = _cg(graph)
    cap = 8 * len(g.names) + 8
    out = (fc_node * cap)()
    origin = (C.c_int32 * cap)()
    n = C.c_int32()
    _check(lib().fc_duplicate(g.ref(), out, cap, C.byref(n), origin))
    src = g.graph
    new = Graph()
    seen: Dict[int, int] = {}
    new_names: List[str] = []
    for i in range(n.value):
        o = origin[i]
        k = seen.get(o, 0)
        seen[o] = k + 1
        base = src.nodes[o]
        name = base.name if k == 0 else f"{base.name}~{k}"
        new_names.append(name)
        new.add(name, base.kind, base.dtype, base.shape,
                fn=base.fn, fparam=base.fparam, iparam=base.iparam,
                args=tuple(new_names[out[i].arg[j]] for j in range(out[i].nargs)),
                output=bool(out[i].flags & FC_NODE_OUTPUT), infusible=base.infusible,
                single_pass=bool(out[i].flags & FC_NODE_SINGLE_PASS))
    return new, [origin[i] for i in range(n.value)]


def fc_scratch_bytes(graph, partition: Optional[Partition] = None) -> int:
    g = _cg(graph)
    b = C.c_size_t()
    cp = partition._c() if partition is not None else None
    _check(lib().fc_scratch_bytes(g.ref(), C.byref(cp) if cp is not None else None, C.byref(b)))
    return b.value


def _buffers(g: CGraph, buffers: Dict[str, object]):
    arr = (fc_buffer * max(len(g.names), 1))()
    for i, name in enumerate(g.names):
        b = buffers.get(name)
        if b is None:
            arr[i].ptr, arr[i].bytes = None, 0
        elif isinstance(b, tuple):
            arr[i].ptr, arr[i].bytes = int(b[0]) or None, int(b[1])
        else:                                   # a torch tensor (device memory owned by the caller)
            arr[i].ptr, arr[i].bytes = b.data_ptr() or None, b.numel() * b.element_size()
    return arr


def _scratch(scratch):
    if isinstance(scratch, tuple):
        return int(scratch[0]), int(scratch[1])
    return scratch.data_ptr(), scratch.numel() * scratch.element_size()


def fc_run_fused(graph, partition: Partition, buffers: Dict[str, object], scratch, stream: int = 0) -> None:
    """Enqueues the program on `stream` (a hipStream_t value); returns without synchronising."""
    g = _cg(graph)
    cp = partition._c()
    sp, sb = _scratch(scratch)
    _check(lib().fc_run_fused(g.ref(), C.byref(cp), _buffers(g, buffers), sp, sb, stream or None))


FC_STATIC_SCRATCH_BYTES = 32 << 20


def fc_run_fused_static(graph, partition: Partition, buffers: Dict[str, object], stream: int = 0) -> None:
    """fc_run_fused in the library's own static scratch buffer (no allocation anywhere)."""
    g = _cg(graph)
    cp = partition._c()
    _check(lib().fc_run_fused_static(g.ref(), C.byref(cp), _buffers(g, buffers), stream or None))


def fc_run_unfused(graph, buffers: Dict[str, object], scratch, stream: int = 0) -> None:
    g = _cg(graph)
    sp, sb = _scratch(scratch)
    _check(lib().fc_run_unfused(g.ref(), _buffers(g, buffers), sp, sb, stream or None))


class BoundRun:
    """fc_run_fused / fc_run_unfused with the arguments marshalled once: for callers that run
    one program on the same buffers many times.  partition None = fc_run_unfused."""

    def __init__(self, graph, partition: Optional[Partition], buffers: Dict[str, object], scratch):
        self._g = _cg(graph)
        self._part = partition
        self._cp = partition._c() if partition is not None else None
        self._bufs = _buffers(self._g, buffers)
        self._keep = (buffers, scratch)                 # the device memory must outlive the calls
        self._sp, self._sb = _scratch(scratch)
        self._lib = lib()

    def __call__(self, stream: int = 0) -> None:
        if self._cp is None:
            rc = self._lib.fc_run_unfused(self._g.ref(), self._bufs, self._sp, self._sb, stream or None)
        else:
            rc = self._lib.fc_run_fused(self._g.ref(), C.byref(self._cp), self._bufs, self._sp, self._sb,
                                        stream or None)
        if rc != 0:
            _check(rc)


def fc_check(scratch, stream: int = 0) -> None:
    """Synchronises `stream` and raises FcError (FC_E_DEVICE_WAIT) if a kernel that used `scratch`
    gave up a bounded wait since the last check."""
    sp = _scratch(scratch)[0] if scratch is not None else None
    _check(lib().fc_check(sp or None, stream or None))


def fc_cluster_kernel(graph, partition: Optional[Partition], cluster: int) -> str:
    g = _cg(graph)
    cp = partition._c() if partition is not None else None
    buf = C.create_string_buffer(4096)
    _check(lib().fc_cluster_kernel(g.ref(), C.byref(cp) if cp is not None else None, cluster, buf, 4096))
    return buf.value.decode()


def fc_last_error() -> str:
    return lib().fc_last_error().decode()
