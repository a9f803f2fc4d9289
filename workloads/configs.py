"""The five synthetic pipelines and their seeded inputs.

Each builder returns a `Workload`: the combinator program (a `Graph`), the host
input arrays, and the byte accounting used when throughput is reported.  The
programs take the patterns the paper discusses (map -> gather -> fold chains as
in `simple1` / `singleLoop`, "gather then fold back" as in its FlashAttention
remark, `filter` through scan + scatter, a producer shared by consumers that
read it in different orders); the paper's own benchmark programs are not
available, these stand in for them.

Nothing here evaluates a combinator: inputs are drawn from numpy's PCG64
(`default_rng(SEED0 + config)`), and only the *inputs* are produced.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, Optional

import numpy as np

from .graph import Graph

SEED0 = 20240713


@dataclass
class Workload:
    name: str
    graph: Graph
    inputs: Dict[str, np.ndarray]
    units: int                     # elements / nnz / grid points per pass
    unit_name: str
    lb_bytes: int                  # fused-traffic lower bound: every external input byte
    #                                once, every program output byte once
    unfused_bytes: int             # one kernel per combinator, every intermediate in HBM
    notes: str = ""
    extra: Dict[str, object] = field(default_factory=dict)


def _rng(cfg: int, seed: Optional[int]):
    return np.random.default_rng(SEED0 + cfg if seed is None else seed)


# --------------------------------------------------------------------------- cfg 1
def reverse_dot(n: int = 65536, seed: Optional[int] = None, xs: Optional[np.ndarray] = None) -> Workload:
    """ys = map(2x+1) xs; zs = gather(reverse index, ys); r = fold(+)(zipWith(*) ys zs)."""
    if xs is None:
        xs = _rng(1, seed).uniform(-1.0, 1.0, size=n).astype(np.float32)
    n = int(xs.shape[0])
    g = Graph()
    g.add("xs", "input", "f32", (n,))
    g.add("ys", "map", "f32", (n,), fn="affine", fparam=(2.0, 1.0), args=("xs",))
    g.add("idx", "generate", "i32", (n,), fn="iota_rev")
    g.add("zs", "gather", "f32", (n,), args=("idx", "ys"))
    g.add("ps", "map", "f32", (n,), fn="mul2", args=("ys", "zs"))
    g.add("r", "fold", "f32", (1,), fn="add", args=("ps",), output=True)
    return Workload("cfg1_reverse_dot", g, {"xs": xs}, n, "elements",
                    lb_bytes=4 * n + 4, unfused_bytes=40 * n + 4)


# --------------------------------------------------------------------------- cfg 2
def perm_gather_fold(n: int = 1 << 24, seed: Optional[int] = None,
                     xs: Optional[np.ndarray] = None, idx: Optional[np.ndarray] = None) -> Workload:
    """ys = map(sin x * x) xs; zs = gather(perm, ys); ws = map(z*z+1) zs; r = fold(+) ws."""
    rng = _rng(2, seed)
    if xs is None:
        xs = rng.standard_normal(size=n).astype(np.float32)
    n = int(xs.shape[0])
    if idx is None:
        idx = rng.permutation(n).astype(np.int32)
    m = int(idx.shape[0])
    g = Graph()
    g.add("xs", "input", "f32", (n,))
    g.add("idx", "input", "i32", (m,))
    g.add("ys", "map", "f32", (n,), fn="sin_x_mul_x", args=("xs",))
    g.add("zs", "gather", "f32", (m,), args=("idx", "ys"))
    g.add("ws", "map", "f32", (m,), fn="sq_plus_one", args=("zs",))
    g.add("r", "fold", "f32", (1,), fn="add", args=("ws",), output=True)
    return Workload("cfg2_perm_gather_fold", g, {"xs": xs, "idx": idx}, m, "elements",
                    lb_bytes=4 * n + 4 * m + 4, unfused_bytes=8 * n + 12 * m + 8 * m + 4 * m + 4)


# --------------------------------------------------------------------------- cfg 3
def spmv(rows: int = 1 << 22, mean_len: float = 16.0, seed: Optional[int] = None,
         lengths: Optional[np.ndarray] = None, ncols: Optional[int] = None) -> Workload:
    """y = foldSeg(+)(zipWith(*) vals (gather(col, x)), off): CSR sparse matrix-vector product."""
    rng = _rng(3, seed)
    if lengths is None:
        lengths = rng.poisson(mean_len, size=rows)
    lengths = np.asarray(lengths, dtype=np.int64)
    rows = int(lengths.shape[0])
    ncols = rows if ncols is None else int(ncols)
    off = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(lengths, out=off[1:])          # input preparation: the row descriptor
    nnz = int(off[-1])
    if nnz >= 2 ** 31:
        raise ValueError("nnz does not fit int32 offsets")
    col = rng.integers(0, max(ncols, 1), size=nnz, dtype=np.int32)
    vals = rng.uniform(-1.0, 1.0, size=nnz).astype(np.float32)
    x = rng.uniform(-1.0, 1.0, size=ncols).astype(np.float32)
    g = Graph()
    g.add("x", "input", "f32", (ncols,))
    g.add("col", "input", "i32", (nnz,))
    g.add("vals", "input", "f32", (nnz,))
    g.add("off", "input", "i32", (rows + 1,))
    g.add("g", "gather", "f32", (nnz,), args=("col", "x"))
    g.add("p", "map", "f32", (nnz,), fn="mul2", args=("vals", "g"))
    g.add("y", "foldseg", "f32", (rows,), fn="add", args=("p", "off"), output=True)
    return Workload("cfg3_spmv", g,
                    {"x": x, "col": col, "vals": vals, "off": off.astype(np.int32)},
                    nnz, "nnz",
                    lb_bytes=8 * nnz + 4 * (rows + 1) + 4 * ncols + 4 * rows,
                    unfused_bytes=28 * nnz + 8 * rows + 4,
                    extra={"rows": rows, "nnz": nnz})


# --------------------------------------------------------------------------- cfg 4
def compaction(n: int = 1 << 26, seed: Optional[int] = None, v: Optional[np.ndarray] = None,
               modulus: int = 3, residue: int = 0, fill: int = -1) -> Workload:
    """flags = map(v mod 3 == 0) v; offs = scanl(+) flags; out = scatter v to offs where flag."""
    if v is None:
        v = _rng(4, seed).integers(0, 2 ** 31, size=n, dtype=np.int32)
    v = np.asarray(v, dtype=np.int32)
    n = int(v.shape[0])
    dest = np.full(n, fill, dtype=np.int32)
    g = Graph()
    g.add("v", "input", "i32", (n,))
    g.add("dest", "input", "i32", (n,))
    g.add("flags", "map", "i32", (n,), fn="mod_eq", iparam=(modulus, residue), args=("v",))
    g.add("offs", "scanl", "i32", (n,), fn="add", args=("flags",))
    g.add("count", "fold", "i32", (1,), fn="add", args=("flags",), output=True)
    g.add("out", "scatter", "i32", (n,), fn="overwrite",
          args=("dest", "offs", "v", "flags"), output=True)
    # the number of kept elements is a property of the input, needed for the byte count
    kept = int(np.count_nonzero((v.astype(np.int64) % modulus) == residue))
    return Workload("cfg4_compaction", g, {"v": v, "dest": dest}, n, "elements",
                    lb_bytes=4 * n + 4 * kept + 4,
                    unfused_bytes=28 * n + 4 * kept + 4 * n + 4,
                    extra={"kept": kept})


# --------------------------------------------------------------------------- cfg 5
def stencil_max(h: int = 8192, w: int = 8192, seed: Optional[int] = None,
                grid: Optional[np.ndarray] = None) -> Workload:
    """p = map(exp(-x)) grid; out = p + pN + pS + pW + pE (clamped); m = fold(max) p."""
    if grid is None:
        grid = _rng(5, seed).uniform(0.0, 1.0, size=(h, w)).astype(np.float32)
    h, w = int(grid.shape[0]), int(grid.shape[1])
    g = Graph()
    g.add("grid", "input", "f32", (h, w))
    g.add("p", "map", "f32", (h, w), fn="exp_neg", args=("grid",))
    for nm, (di, dj) in (("N", (-1, 0)), ("S", (1, 0)), ("W", (0, -1)), ("E", (0, 1))):
        g.add("i" + nm, "generate", "i32", (h, w), fn="clamp_shift_2d", iparam=(di, dj))
        g.add("p" + nm, "gather", "f32", (h, w), args=("i" + nm, "p"))
    g.add("out", "map", "f32", (h, w), fn="add5", args=("p", "pN", "pS", "pW", "pE"), output=True)
    g.add("m", "fold", "f32", (1,), fn="max", args=("p",), output=True)
    pts = h * w
    return Workload("cfg5_stencil_max", g, {"grid": grid}, pts, "points",
                    lb_bytes=8 * pts + 4, unfused_bytes=100 * pts + 4,
                    extra={"materialise_p_bytes": 16 * pts + 4})


BUILDERS: Dict[int, Callable[..., Workload]] = {
    1: reverse_dot, 2: perm_gather_fold, 3: spmv, 4: compaction, 5: stencil_max,
}

# sizes at which the CPU oracle finishes in well under a second; ragged on purpose
SMALL = {
    1: dict(n=65536),
    2: dict(n=100003),
    3: dict(rows=20011),
    4: dict(n=300007),
    5: dict(h=197, w=331),
}


def build(cfg: int, small: bool = False, **kw) -> Workload:
    args = dict(SMALL[cfg]) if small else {}
    args.update(kw)
    return BUILDERS[cfg](**args)
