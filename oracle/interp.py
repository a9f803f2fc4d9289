"""CPU oracle: a plain, unfused interpreter of the combinator language.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module;
only the tests, the smoke check and the CPU-baseline leg of the bench do.  It
shares no code with the HIP library and never calls it.

Fusion is semantics preserving (paper section 3: a cluster is just several
combinators executed in one loop), so what a fused program must compute is by
definition what the unfused program computes.  The oracle is therefore the plain
definition: every node of the program, in program order, is evaluated into a
fully materialised host array by one simple whole-array step per combinator
(paper section 2, "Language").  There is no blocking, fusion or reordering.

Precision rules
  * fp32 element functions built from + - * and compares are evaluated in fp32,
    every operation rounded on its own (numpy never contracts a*b+c).
  * sin and exp are evaluated in fp64 and rounded once to fp32.
  * a fold / segmented fold with (+) over fp32 accumulates in fp64 and returns the
    fp64 value (the reference the 1e-5 bound is measured against); so does a
    scatter that combines fp32 values with (+); max and all integer work are exact.

Readings taken where the paper leaves a choice
  * scanl is exclusive and identity seeded (element i combines the elements
    before it, not itself); scanr is its mirror image; a two-dimensional array
    is scanned row by row.
  * fold takes the identity of its operator as initial value, so an empty fold
    (and an empty segment of foldSeg) yields that identity.
  * a fold whose result has shape (1,) reduces the flattened input; otherwise it
    reduces the innermost dimension.
  * foldSeg (only named in the paper) folds the flat value array over the
    segments [off[r], off[r+1]).
  * values that are not finite (the paper says nothing about them): every element
    function and (+) follow IEEE-754 operation by operation, so a NaN, or infinities
    of both signs, among the summands of a fold / segmented fold / scan prefix give
    NaN and infinities of one sign give that infinity; max is IEEE-754 maxNum, which
    treats a NaN operand as missing (the maximum of the other values; the identity
    -inf when there are none).  Either rule gives one result whatever the order of
    evaluation, which a parallel fold needs.  Partial sums that overflow fp32 although
    the exact sum is finite are outside the comparison (the reference sums in fp64).
  * scatter(f, dest, src): src is the SoA tuple (index, value[, flag]); for every
    element in source order with a non-zero flag, dest[index] becomes
    f(dest[index], value); f = overwrite means "the new value wins" and then the
    indices of the kept elements must be distinct; an index out of range is an
    error here (undefined in the paper).

Parity pins live in tests/test_oracle_pins.py; "parity unpinned": the exact fp32
value of sin / exp based maps (only a tolerance is fixed).
"""
from __future__ import annotations

from typing import Dict

import numpy as np

F32 = np.float32


# --------------------------------------------------------------------- element functions
def _map(fn, fparam, iparam, args):
    if fn == "ident":
        return args[0].copy()
    if fn == "affine":                      # a*x + b, two roundings
        a, b = F32(fparam[0]), F32(fparam[1])
        return (a * args[0]) + b
    if fn == "sin_x_mul_x":                 # fl32(sin(x)) * x
        x = args[0]
        s = np.sin(x.astype(np.float64)).astype(F32)
        return s * x
    if fn == "sq_plus_one":                 # z*z + 1
        z = args[0]
        return (z * z) + F32(1.0)
    if fn == "mul2":
        return args[0] * args[1]
    if fn == "add2":
        return args[0] + args[1]
    if fn == "add3":
        return (args[0] + args[1]) + args[2]
    if fn == "add5":                        # fixed left-to-right order
        return (((args[0] + args[1]) + args[2]) + args[3]) + args[4]
    if fn == "exp_neg":                     # fl32(exp(-x))
        return np.exp(-args[0].astype(np.float64)).astype(F32)
    if fn == "mod_eq":                      # 1 where v mod k == r (v >= 0)
        k, r = int(iparam[0]), int(iparam[1])
        v = args[0]
        if v.size and int(v.min()) < 0:
            raise ValueError("mod_eq is defined on non-negative integers only")
        return ((v.astype(np.int64) % k) == r).astype(np.int32)
    raise ValueError(f"unknown map function {fn}")


def _generate(fn, shape, iparam):
    n = int(np.prod(shape)) if len(shape) else 1
    if fn == "iota":
        return np.arange(n, dtype=np.int64).astype(np.int32).reshape(shape)
    if fn == "iota_rev":
        return (n - 1 - np.arange(n, dtype=np.int64)).astype(np.int32).reshape(shape)
    if fn == "clamp_shift_2d":              # (i, j) -> clamp(i+di) * W + clamp(j+dj)
        h, w = shape
        di, dj = int(iparam[0]), int(iparam[1])
        i = np.clip(np.arange(h, dtype=np.int64) + di, 0, h - 1)
        j = np.clip(np.arange(w, dtype=np.int64) + dj, 0, w - 1)
        return (i[:, None] * w + j[None, :]).astype(np.int32)
    if fn == "row_of_2d":                   # (i, j) -> i
        h, w = shape
        return np.repeat(np.arange(h, dtype=np.int64), w).astype(np.int32).reshape(shape)
    if fn == "const_i32":
        return np.full(shape, int(iparam[0]), dtype=np.int32)
    raise ValueError(f"unknown generate function {fn}")


# --------------------------------------------------------------------- reductions
def _acc(a, dtype):
    """Accumulation type: fp64 for fp32 data, int64 for int32 data."""
    return a.astype(np.float64) if dtype == "f32" else a.astype(np.int64)


def _identity(op, dtype):
    if op == "add":
        return 0.0 if dtype == "f32" else 0
    if op == "mul":
        return 1.0 if dtype == "f32" else 1
    if op == "max":
        return -np.inf if dtype == "f32" else np.iinfo(np.int32).min
    raise ValueError(f"unknown reducer {op}")


def _reduce(op, a, dtype, axis=None):
    z = _identity(op, dtype)
    a = _acc(a, dtype)
    if op == "add":
        return np.add.reduce(a, axis=axis, initial=z)
    if op == "mul":
        return np.multiply.reduce(a, axis=axis, initial=z)
    # max over fp32 is IEEE-754 maxNum: a NaN operand counts as missing, the other operand is
    # the result (np.fmax); with integers fmax is the plain maximum
    return np.fmax.reduce(a, axis=axis, initial=z)


def _finish(r, dtype):
    r = np.atleast_1d(np.asarray(r))
    if dtype == "i32":
        if r.size and (r.max() > np.iinfo(np.int32).max or r.min() < np.iinfo(np.int32).min):
            raise OverflowError("int32 reduction overflowed")
        return r.astype(np.int32)
    return r.astype(np.float64)


def _fold(op, a, dtype, out_shape):
    if tuple(out_shape) == (1,):
        return _finish(_reduce(op, a.reshape(-1), dtype), dtype)
    if tuple(out_shape) != tuple(a.shape[:-1]):
        raise ValueError("fold reduces the innermost dimension")
    return _finish(_reduce(op, a, dtype, axis=-1), dtype).reshape(out_shape)


def _foldseg(op, vals, off, dtype):
    off = off.astype(np.int64)
    rows = off.shape[0] - 1
    if rows < 0:
        raise ValueError("the offsets array needs at least one entry")
    if np.any(np.diff(off) < 0) or off[0] < 0 or off[-1] > vals.size:
        raise ValueError("segment offsets must be non-decreasing and inside the value array")
    a = _acc(vals.reshape(-1), dtype)
    out = np.full(rows, _identity(op, dtype), dtype=a.dtype)
    # one reduction per non-empty segment [off[r], off[r+1]); an empty segment keeps
    # the identity.  Empty segments lie between two non-empty ones without taking an
    # element, so consecutive non-empty starts delimit exactly the non-empty segments.
    nonempty = np.nonzero(off[1:] > off[:-1])[0]
    if nonempty.size:
        ufunc = {"add": np.add, "mul": np.multiply, "max": np.fmax}[op]
        out[nonempty] = ufunc.reduceat(a[:int(off[-1])], off[:-1][nonempty])
    return _finish(out, dtype)


def _scan(op, a, dtype, reverse):
    """Exclusive (+) scan; a multidimensional array is scanned row by row, i.e. along its
    innermost dimension (section 2, scanl / scanr)."""
    if op != "add":
        raise ValueError("scan supports (+) only")
    rows = _acc(a.reshape(-1, a.shape[-1]) if a.ndim > 1 else a.reshape(1, -1), dtype)
    if reverse:
        rows = rows[:, ::-1]
    out = np.zeros_like(rows)
    if rows.shape[1]:
        np.cumsum(rows[:, :-1], axis=1, out=out[:, 1:])   # exclusive: element i combines the elements before it
    if reverse:
        out = out[:, ::-1]
    if dtype == "i32":
        if out.size and out.max() > np.iinfo(np.int32).max:
            raise OverflowError("int32 scan overflowed")
        return out.astype(np.int32).reshape(a.shape)
    return out.astype(F32).reshape(a.shape)


def _scatter(fn, dest, idx, val, flag):
    out = dest.copy().reshape(-1)
    idx = idx.reshape(-1).astype(np.int64)
    val = val.reshape(-1)
    keep = np.ones(idx.shape[0], dtype=bool) if flag is None else (flag.reshape(-1) != 0)
    ki, kv = idx[keep], val[keep]
    if ki.size and (ki.min() < 0 or ki.max() >= out.shape[0]):
        raise IndexError("scatter index out of range")
    if fn == "overwrite":
        if np.unique(ki).size != ki.size:
            raise ValueError("overwrite scatter needs distinct destination indices")
        out[ki] = kv
    elif fn == "add":
        if out.dtype == F32:
            # fp32 sums depend on the order of the updates, which the paper leaves open
            # (section 2, scatter); the reference is the sum accumulated in fp64, as for folds
            out = out.astype(np.float64)
            np.add.at(out, ki, kv.astype(np.float64))
        else:
            np.add.at(out, ki, kv)           # sequential in source order; exact
    else:
        raise ValueError(f"unknown scatter function {fn}")
    return out.reshape(dest.shape)


# --------------------------------------------------------------------- interpreter
def _as_elem(a, dtype):
    """Value of an array when an element function or a gather reads it."""
    if dtype == "f32" and a.dtype != F32:
        return a.astype(F32)
    return a


def evaluate(graph, inputs: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    """Evaluate every node of `graph`; returns {node name: array}."""
    env: Dict[str, np.ndarray] = {}
    by_name = {n.name: n for n in graph.nodes}
    for n in graph.nodes:
        args = [env[a] for a in n.args]
        adt = [by_name[a].dtype for a in n.args]
        if n.kind == "input":
            a = np.asarray(inputs[n.name])
            want = F32 if n.dtype == "f32" else np.int32
            if a.dtype != want or tuple(a.shape) != tuple(n.shape):
                raise ValueError(f"input {n.name}: expected {want} {n.shape}, got {a.dtype} {a.shape}")
            v = a
        elif n.kind == "map":
            ea = [_as_elem(a, d) for a, d in zip(args, adt)]
            if any(tuple(a.shape) != tuple(n.shape) for a in ea):
                raise ValueError(f"{n.name}: map arguments must have the shape of the result")
            v = _map(n.fn, n.fparam, n.iparam, ea)
        elif n.kind == "generate":
            v = _generate(n.fn, tuple(n.shape), n.iparam)
        elif n.kind == "gather":
            idx, src = args[0].reshape(-1).astype(np.int64), _as_elem(args[1], adt[1]).reshape(-1)
            if idx.size and (idx.min() < 0 or idx.max() >= src.shape[0]):
                raise IndexError(f"{n.name}: gather index out of range")
            v = src[idx].reshape(n.shape)
        elif n.kind == "fold":
            v = _fold(n.fn, _as_elem(args[0], adt[0]), n.dtype, n.shape)
        elif n.kind == "foldseg":
            v = _foldseg(n.fn, _as_elem(args[0], adt[0]), args[1], n.dtype)
        elif n.kind in ("scanl", "scanr"):
            v = _scan(n.fn, _as_elem(args[0], adt[0]), n.dtype, reverse=(n.kind == "scanr"))
        elif n.kind == "scatter":
            flag = args[3] if len(args) > 3 else None
            v = _scatter(n.fn, args[0], args[1], _as_elem(args[2], adt[2]), flag)
        elif n.kind == "force":
            v = args[0].copy()
        else:
            raise ValueError(n.kind)
        env[n.name] = v
    return env
