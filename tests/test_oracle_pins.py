"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these re-types the oracle's own formulas on the same path: each is a
closed form, a law of the combinators (paper section 2), a special case that
collapses to another routine, or a pure-Python brute force on tiny inputs.
A planted mistake in the oracle (dropped term, wrong index or sign, swapped
gather operands, inclusive instead of exclusive scan, unclamped border) makes at
least one of them fail.
"""
import math

import numpy as np
import pytest

from oracle.interp import evaluate
from workloads import Graph, build
from workloads import configs as C

F32 = np.float32


def run(g, inputs):
    return evaluate(g, inputs)


# ---------------------------------------------------------------- map / generate / gather laws
def test_identity_gather_is_noop():
    rng = np.random.default_rng(1)
    a = rng.standard_normal(1000).astype(F32)
    g = Graph()
    g.add("a", "input", "f32", (1000,))
    g.add("i", "generate", "i32", (1000,), fn="iota")
    g.add("b", "gather", "f32", (1000,), args=("i", "a"))
    assert np.array_equal(run(g, {"a": a})["b"], a)


def test_reverse_twice_is_identity_and_reverse_matches_slice():
    # reverse = gather over generate(n-1-i)  (section 2, `reverse`)
    a = np.arange(17, dtype=np.int32) * 3 + 1
    g = Graph()
    g.add("a", "input", "i32", (17,))
    g.add("i", "generate", "i32", (17,), fn="iota_rev")
    g.add("b", "gather", "i32", (17,), args=("i", "a"))
    g.add("c", "gather", "i32", (17,), args=("i", "b"))
    env = run(g, {"a": a})
    assert np.array_equal(env["b"], a[::-1])
    assert np.array_equal(env["c"], a)
    assert env["i"][0] == 16 and env["i"][16] == 0


def test_gather_argument_roles():
    # gather(is, as)[j] = as[is[j]]: the first argument indexes, the second is read
    src = np.array([10, 20, 30, 40], dtype=np.int32)
    idx = np.array([3, 3, 0], dtype=np.int32)
    g = Graph()
    g.add("src", "input", "i32", (4,))
    g.add("idx", "input", "i32", (3,))
    g.add("b", "gather", "i32", (3,), args=("idx", "src"))
    assert run(g, {"src": src, "idx": idx})["b"].tolist() == [40, 40, 10]


def test_gather_out_of_range_is_an_error():
    g = Graph()
    g.add("src", "input", "i32", (4,))
    g.add("idx", "input", "i32", (1,))
    g.add("b", "gather", "i32", (1,), args=("idx", "src"))
    with pytest.raises(IndexError):
        run(g, {"src": np.zeros(4, np.int32), "idx": np.array([4], np.int32)})


def test_permutation_gather_preserves_multiset_and_commutes_with_map():
    # `simple1`: gather(is, map f xs) == map f (gather(is, xs)), bit for bit
    rng = np.random.default_rng(2)
    n = 4099
    xs = rng.standard_normal(n).astype(F32)
    idx = rng.permutation(n).astype(np.int32)
    g = Graph()
    g.add("xs", "input", "f32", (n,))
    g.add("idx", "input", "i32", (n,))
    g.add("a", "map", "f32", (n,), fn="affine", fparam=(2.0, 1.0), args=("xs",))
    g.add("b", "gather", "f32", (n,), args=("idx", "a"))
    g.add("gx", "gather", "f32", (n,), args=("idx", "xs"))
    g.add("b2", "map", "f32", (n,), fn="affine", fparam=(2.0, 1.0), args=("gx",))
    env = run(g, {"xs": xs, "idx": idx})
    assert np.array_equal(env["b"], env["b2"])
    assert np.array_equal(np.sort(env["gx"]), np.sort(xs))


def test_gather_of_gather_composes():
    # `simple2`: gather(is2, gather(is1, xs)) == gather(gather(is2, is1), xs)
    rng = np.random.default_rng(3)
    xs = rng.integers(0, 1000, 50, dtype=np.int32)
    is1 = rng.integers(0, 50, 70, dtype=np.int32)
    is2 = rng.integers(0, 70, 31, dtype=np.int32)
    g = Graph()
    g.add("xs", "input", "i32", (50,))
    g.add("is1", "input", "i32", (70,))
    g.add("is2", "input", "i32", (31,))
    g.add("a", "gather", "i32", (70,), args=("is1", "xs"))
    g.add("b", "gather", "i32", (31,), args=("is2", "a"))
    g.add("ii", "gather", "i32", (31,), args=("is2", "is1"))
    g.add("b2", "gather", "i32", (31,), args=("ii", "xs"))
    env = run(g, {"xs": xs, "is1": is1, "is2": is2})
    assert np.array_equal(env["b"], env["b2"])


def test_affine_rounds_twice_not_fused():
    # 2x+1 with separate roundings differs from the single rounding of a fused
    # multiply-add for some x; pick one by search and pin the two-rounding value
    a, b = F32(1.0000001), F32(1.0)
    found = None
    for k in range(1, 4000):
        x = F32(1.0) + F32(k) * F32(2.0 ** -23)
        two = F32(F32(a * x) + b)
        one = F32(np.float64(a) * np.float64(x) + np.float64(b))
        if two != one:
            found = (x, two)
            break
    assert found is not None
    x, two = found
    g = Graph()
    g.add("x", "input", "f32", (1,))
    g.add("y", "map", "f32", (1,), fn="affine", fparam=(float(a), float(b)), args=("x",))
    assert run(g, {"x": np.array([x], F32)})["y"][0] == two


def test_transcendental_maps_against_math_module():
    xs = np.array([0.0, 0.5, -1.25, 3.0, 1e-3], dtype=F32)
    g = Graph()
    g.add("x", "input", "f32", (5,))
    g.add("s", "map", "f32", (5,), fn="sin_x_mul_x", args=("x",))
    g.add("e", "map", "f32", (5,), fn="exp_neg", args=("x",))
    g.add("q", "map", "f32", (5,), fn="sq_plus_one", args=("x",))
    env = run(g, {"x": xs})
    for i, x in enumerate(xs.tolist()):
        assert env["s"][i] == F32(F32(math.sin(x)) * F32(x))
        assert env["e"][i] == F32(math.exp(-x))
        assert env["q"][i] == F32(F32(F32(x) * F32(x)) + F32(1))
    assert env["s"][0] == 0 and env["e"][0] == 1 and env["q"][0] == 1


# ---------------------------------------------------------------- fold
def _fold_graph(n, fn="add", dtype="f32"):
    g = Graph()
    g.add("a", "input", dtype, (n,))
    g.add("r", "fold", dtype, (1,), fn=fn, args=("a",))
    return g


def test_fold_closed_forms():
    n = 100000
    c = F32(0.1)
    env = run(_fold_graph(n), {"a": np.full(n, c, F32)})
    assert env["r"][0] == pytest.approx(n * float(c), rel=1e-13)
    env = run(_fold_graph(n, dtype="i32"), {"a": np.arange(n, dtype=np.int32) % 7})
    assert int(env["r"][0]) == (n // 7) * 21 + sum(range(n % 7))
    with pytest.raises(OverflowError):                        # int32 results are checked, not wrapped
        run(_fold_graph(3, dtype="i32"), {"a": np.full(3, 2 ** 30, np.int32)})
    env = run(_fold_graph(1000, dtype="i32"), {"a": np.arange(1000, dtype=np.int32)})
    assert int(env["r"][0]) == 1000 * 999 // 2
    # empty fold = identity of the operator
    assert run(_fold_graph(0), {"a": np.zeros(0, F32)})["r"][0] == 0.0
    assert run(_fold_graph(0, "max"), {"a": np.zeros(0, F32)})["r"][0] == -np.inf


def test_fold_accumulates_in_fp64_not_fp32():
    # 2^24 + 1 + 1 ... in fp32 would stall at 2^24
    a = np.ones(5, F32)
    a[0] = F32(2.0 ** 24)
    assert run(_fold_graph(5), {"a": a})["r"][0] == 2.0 ** 24 + 4


def test_fold_of_affine_map_is_linear():
    # fold(+)(map(2x+1) xs) = 2*sum(xs) + n up to the fp32 rounding of each element
    rng = np.random.default_rng(4)
    n = 5000
    xs = (rng.integers(-512, 512, n) / 1024.0).astype(F32)   # 2x+1 exact in fp32
    g = Graph()
    g.add("xs", "input", "f32", (n,))
    g.add("ys", "map", "f32", (n,), fn="affine", fparam=(2.0, 1.0), args=("xs",))
    g.add("r", "fold", "f32", (1,), fn="add", args=("ys",))
    assert run(g, {"xs": xs})["r"][0] == 2.0 * float(np.sum(xs.astype(np.float64))) + n


def test_fold_brute_force_tiny():
    rng = np.random.default_rng(5)
    for n in range(1, 9):
        a = rng.standard_normal(n).astype(F32)
        acc = 0.0
        mx = -math.inf
        for v in a.tolist():
            acc += v
            mx = max(mx, v)
        assert run(_fold_graph(n), {"a": a})["r"][0] == pytest.approx(acc, rel=1e-15, abs=1e-15)
        assert run(_fold_graph(n, "max"), {"a": a})["r"][0] == mx


def test_row_fold_reduces_innermost_dimension():
    a = np.arange(12, dtype=np.int32).reshape(3, 4)
    g = Graph()
    g.add("a", "input", "i32", (3, 4))
    g.add("r", "fold", "i32", (3,), fn="add", args=("a",))
    assert run(g, {"a": a})["r"].tolist() == [6, 22, 38]


def test_cfg1_closed_form_and_reversal_invariance():
    n = 4096
    c = F32(0.375)
    w = C.reverse_dot(xs=np.full(n, c, F32))
    assert evaluate(w.graph, w.inputs)["r"][0] == n * (2 * 0.375 + 1) ** 2
    rng = np.random.default_rng(6)
    xs = rng.uniform(-1, 1, n).astype(F32)
    r1 = evaluate(C.reverse_dot(xs=xs).graph, {"xs": xs})["r"][0]
    r2 = evaluate(C.reverse_dot(xs=xs[::-1].copy()).graph, {"xs": xs[::-1].copy()})["r"][0]
    assert r1 == pytest.approx(r2, rel=1e-13)
    # brute force
    ys = [float(F32(F32(2) * x + F32(1))) for x in xs]
    acc = 0.0
    for i in range(n):
        acc += float(F32(F32(ys[i]) * F32(ys[n - 1 - i])))
    assert r1 == pytest.approx(acc, rel=1e-13)


def test_cfg2_identity_vs_random_permutation():
    rng = np.random.default_rng(7)
    n = 20000
    xs = rng.standard_normal(n).astype(F32)
    ident = np.arange(n, dtype=np.int32)
    perm = rng.permutation(n).astype(np.int32)
    r_id = evaluate(C.perm_gather_fold(xs=xs, idx=ident).graph, {"xs": xs, "idx": ident})["r"][0]
    r_pm = evaluate(C.perm_gather_fold(xs=xs, idx=perm).graph, {"xs": xs, "idx": perm})["r"][0]
    assert r_id == pytest.approx(r_pm, rel=1e-12)
    # direct evaluation without any gather
    z = (np.sin(xs.astype(np.float64)).astype(F32) * xs)
    wz = (z * z + F32(1)).astype(np.float64)
    assert r_id == pytest.approx(math.fsum(wz.tolist()), rel=1e-13)


# ---------------------------------------------------------------- foldSeg / SpMV
def test_spmv_unit_values_give_row_lengths():
    w = C.spmv(rows=3000, seed=11)
    ins = dict(w.inputs)
    ins["vals"] = np.ones_like(ins["vals"])
    ins["x"] = np.ones_like(ins["x"])
    y = evaluate(w.graph, ins)["y"]
    assert np.array_equal(y, np.diff(ins["off"]).astype(np.float64))


def test_spmv_diagonal_is_elementwise_product():
    n = 1000
    rng = np.random.default_rng(12)
    w = C.spmv(lengths=np.ones(n, np.int64), seed=12)
    ins = dict(w.inputs)
    ins["col"] = np.arange(n, dtype=np.int32)
    y = evaluate(w.graph, ins)["y"]
    assert np.array_equal(y.astype(F32), ins["vals"] * ins["x"])


def test_spmv_vs_dense_and_empty_rows():
    lengths = np.array([0, 3, 0, 0, 5, 1, 0, 40, 2, 0], dtype=np.int64)
    w = C.spmv(lengths=lengths, seed=13, ncols=10)
    ins = w.inputs
    rows = len(lengths)
    dense = np.zeros((rows, 10), dtype=np.float64)
    for r in range(rows):
        for k in range(ins["off"][r], ins["off"][r + 1]):
            dense[r, ins["col"][k]] += float(F32(ins["vals"][k] * ins["x"][ins["col"][k]]))
    y = evaluate(w.graph, ins)["y"]
    assert y.shape == (rows,)
    assert np.allclose(y, dense.sum(axis=1), rtol=1e-14, atol=1e-15)
    assert all(y[r] == 0.0 for r in range(rows) if lengths[r] == 0)


def test_spmv_row_sums_total_and_single_row():
    w = C.spmv(rows=2000, seed=14)
    env = evaluate(w.graph, w.inputs)
    assert math.fsum(env["y"].tolist()) == pytest.approx(
        math.fsum(env["p"].astype(np.float64).tolist()), rel=1e-12)
    # all elements in one row = a plain fold
    nnz = int(w.inputs["off"][-1])
    w1 = C.spmv(lengths=np.array([nnz], np.int64), seed=14, ncols=2000)
    y1 = evaluate(w1.graph, w1.inputs)
    assert y1["y"][0] == pytest.approx(math.fsum(y1["p"].astype(np.float64).tolist()), rel=1e-13)


def test_foldseg_max_and_leading_trailing_empty():
    vals = np.array([1, 5, 2, 9, 4], dtype=np.int32)
    off = np.array([0, 0, 2, 2, 5, 5], dtype=np.int32)
    g = Graph()
    g.add("v", "input", "i32", (5,))
    g.add("off", "input", "i32", (6,))
    g.add("y", "foldseg", "i32", (5,), fn="max", args=("v", "off"))
    y = run(g, {"v": vals, "off": off})["y"]
    lo = np.iinfo(np.int32).min
    assert y.tolist() == [lo, 5, lo, 9, lo]
    g2 = Graph()
    g2.add("v", "input", "i32", (5,))
    g2.add("off", "input", "i32", (6,))
    g2.add("y", "foldseg", "i32", (5,), fn="add", args=("v", "off"))
    assert run(g2, {"v": vals, "off": off})["y"].tolist() == [0, 6, 0, 15, 0]


# ---------------------------------------------------------------- scan / scatter / compaction
def test_scan_is_exclusive():
    a = np.array([3, 1, 4, 1, 5, 9, 2, 6], dtype=np.int32)
    g = Graph()
    g.add("a", "input", "i32", (8,))
    g.add("l", "scanl", "i32", (8,), fn="add", args=("a",))
    g.add("r", "scanr", "i32", (8,), fn="add", args=("a",))
    env = run(g, {"a": a})
    run_sum, expect = 0, []
    for v in a.tolist():
        expect.append(run_sum)
        run_sum += v
    assert env["l"].tolist() == expect
    # scanr: everything later
    assert env["r"].tolist() == [sum(a.tolist()[i + 1:]) for i in range(8)]
    ones = np.ones(1000, np.int32)
    g1 = Graph()
    g1.add("a", "input", "i32", (1000,))
    g1.add("l", "scanl", "i32", (1000,), fn="add", args=("a",))
    assert np.array_equal(run(g1, {"a": ones})["l"], np.arange(1000, dtype=np.int32))


def test_scan_of_a_two_dimensional_array_scans_every_row():
    # section 2 (scanl / scanr): in a multidimensional array the scan is performed over each row
    rng = np.random.default_rng(31)
    a = rng.integers(0, 100, size=(5, 7), dtype=np.int32)
    g = Graph()
    g.add("a", "input", "i32", (5, 7))
    g.add("l", "scanl", "i32", (5, 7), fn="add", args=("a",))
    g.add("r", "scanr", "i32", (5, 7), fn="add", args=("a",))
    env = run(g, {"a": a})
    for i in range(5):
        row = a[i].tolist()
        assert env["l"][i].tolist() == [sum(row[:j]) for j in range(7)]
        assert env["r"][i].tolist() == [sum(row[j + 1:]) for j in range(7)]
    # rows do not leak into each other: the first column of scanl and the last of scanr are zero
    assert not env["l"][:, 0].any() and not env["r"][:, -1].any()
    # a single row is the one-dimensional scan
    g1 = Graph()
    g1.add("a", "input", "i32", (1, 7))
    g1.add("l", "scanl", "i32", (1, 7), fn="add", args=("a",))
    assert run(g1, {"a": a[:1]})["l"][0].tolist() == [sum(a[0].tolist()[:j]) for j in range(7)]


def test_scan_of_fp32_is_the_exactly_summed_prefix_rounded_once():
    # the reference of an fp32 (+) scan: every prefix summed without rounding error, then rounded
    # to fp32 once.  Pinned by exact rational arithmetic on a short array, by inputs whose
    # prefixes are representable (powers of two, ones), and by scanr = scanl of the mirror image.
    from fractions import Fraction
    rng = np.random.default_rng(33)
    a = (rng.standard_normal(40) * 10.0 ** rng.integers(-6, 6, size=40)).astype(np.float32)
    g = Graph()
    g.add("a", "input", "f32", (40,))
    g.add("l", "scanl", "f32", (40,), fn="add", args=("a",))
    g.add("r", "scanr", "f32", (40,), fn="add", args=("a",))
    env = run(g, {"a": a})
    exact = [Fraction(float(v)) for v in a]
    for i in range(40):
        before, after = sum(exact[:i], Fraction(0)), sum(exact[i + 1:], Fraction(0))
        # the double nearest to the rational sum, then the float nearest to that double: with 40
        # terms of at most 24 bits the double is exact or one rounding away, which the fp32
        # rounding absorbs except on a tie; allow the neighbouring float
        for got, want in ((env["l"][i], before), (env["r"][i], after)):
            assert abs(Fraction(float(got)) - want) <= Fraction(float(np.spacing(np.float32(abs(float(want)))))) / 2 + Fraction(1, 10 ** 40)
    assert env["l"].dtype == np.float32 and env["l"][0] == 0.0 and env["r"][-1] == 0.0
    halves = np.array([2.0 ** -k for k in range(24)], dtype=np.float32)
    g2 = Graph()
    g2.add("a", "input", "f32", (24,))
    g2.add("l", "scanl", "f32", (24,), fn="add", args=("a",))
    assert run(g2, {"a": halves})["l"].tolist() == [0.0] + [2.0 - 2.0 ** -(k - 1) for k in range(1, 24)]
    ones = np.ones(5000, np.float32)
    g3 = Graph()
    g3.add("a", "input", "f32", (5000,))
    g3.add("l", "scanl", "f32", (5000,), fn="add", args=("a",))
    g3.add("r", "scanr", "f32", (5000,), fn="add", args=("a",))
    env3 = run(g3, {"a": ones})
    assert np.array_equal(env3["l"], np.arange(5000, dtype=np.float32))
    assert np.array_equal(env3["r"], np.arange(5000, dtype=np.float32)[::-1])
    # two dimensions: every row on its own
    b = rng.standard_normal((3, 9)).astype(np.float32)
    g4 = Graph()
    g4.add("a", "input", "f32", (3, 9))
    g4.add("l", "scanl", "f32", (3, 9), fn="add", args=("a",))
    l4 = run(g4, {"a": b})["l"]
    for i in range(3):
        g5 = Graph()
        g5.add("a", "input", "f32", (9,))
        g5.add("l", "scanl", "f32", (9,), fn="add", args=("a",))
        assert np.array_equal(l4[i], run(g5, {"a": b[i]})["l"])


def test_compaction_invariants():
    w = C.compaction(n=50021, seed=21)
    env = evaluate(w.graph, w.inputs)
    v, flags, offs, out = w.inputs["v"], env["flags"], env["offs"], env["out"]
    count = int(env["count"][0])
    assert offs[0] == 0
    assert np.array_equal(np.diff(offs), flags[:-1])
    assert count == int(offs[-1] + flags[-1])                             # count = scan total
    keep = [int(x) for x in v.tolist() if x % 3 == 0]                    # stable filtered subsequence
    assert count == len(keep)
    assert out[:count].tolist() == keep
    assert np.all(out[count:] == -1)                                      # untouched part of dest
    # statistical pin on the generator + predicate: p = 715827883 / 2^31
    p = 715827883 / 2 ** 31
    assert abs(count - 50021 * p) < 4 * math.sqrt(50021 * p * (1 - p))


def test_compaction_closed_form_iota():
    n = 1000
    w = C.compaction(v=np.arange(n, dtype=np.int32))
    env = evaluate(w.graph, w.inputs)
    count = int(env["count"][0])
    assert count == (n + 2) // 3
    assert env["out"][:count].tolist() == [3 * k for k in range(count)]


def test_scatter_semantics():
    g = Graph()
    g.add("dest", "input", "i32", (6,))
    g.add("i", "input", "i32", (4,))
    g.add("x", "input", "i32", (4,))
    g.add("f", "input", "i32", (4,))
    g.add("o", "scatter", "i32", (6,), fn="overwrite", args=("dest", "i", "x", "f"))
    g.add("a", "scatter", "i32", (6,), fn="add", args=("dest", "i", "x"))
    ins = {"dest": np.arange(6, dtype=np.int32) * 100,
           "i": np.array([5, 0, 5, 2], np.int32), "x": np.array([1, 2, 3, 4], np.int32),
           "f": np.array([1, 1, 0, 1], np.int32)}
    env = run(g, ins)
    assert env["o"].tolist() == [2, 100, 4, 300, 400, 1]
    assert env["a"].tolist() == [2, 100, 204, 300, 400, 504]       # colliding (+) combines
    assert ins["dest"].tolist() == [0, 100, 200, 300, 400, 500]    # the oracle works on a copy
    ins2 = dict(ins, f=np.ones(4, np.int32))
    with pytest.raises(ValueError):
        run(g, ins2)                                                # colliding overwrite is rejected
    with pytest.raises(IndexError):
        run(g, dict(ins, i=np.array([6, 0, 5, 2], np.int32)))


def test_scatter_add_fp32_reference_is_the_exact_sum():
    # fp32 (+) with colliding indices: the update order is not fixed (section 2, scatter), so the
    # reference is the sum in fp64.  A histogram of ones has a closed form; a large start value
    # followed by many small ones shows that nothing is rounded away on the way.
    n, k = 100000, 7
    g = Graph()
    g.add("dest", "input", "f32", (k,))
    g.add("i", "input", "i32", (n,))
    g.add("x", "input", "f32", (n,))
    g.add("h", "scatter", "f32", (k,), fn="add", args=("dest", "i", "x"))
    idx = (np.arange(n) % k).astype(np.int32)
    env = run(g, {"dest": np.zeros(k, F32), "i": idx, "x": np.ones(n, F32)})
    assert env["h"].dtype == np.float64
    assert env["h"].tolist() == [float(len(range(j, n, k))) for j in range(k)]
    dest = np.zeros(k, F32)
    dest[3] = F32(2.0 ** 26)                       # one more is below half an ulp of this in fp32
    env = run(g, {"dest": dest, "i": np.full(n, 3, np.int32), "x": np.ones(n, F32)})
    assert env["h"][3] == 2.0 ** 26 + n and not env["h"][[0, 1, 2, 4, 5, 6]].any()
    # brute force, with a flag
    rng = np.random.default_rng(5)
    g2 = Graph()
    g2.add("dest", "input", "f32", (5,))
    g2.add("i", "input", "i32", (40,))
    g2.add("x", "input", "f32", (40,))
    g2.add("f", "input", "i32", (40,))
    g2.add("h", "scatter", "f32", (5,), fn="add", args=("dest", "i", "x", "f"))
    ins = {"dest": rng.standard_normal(5).astype(F32), "i": rng.integers(0, 5, 40, dtype=np.int32),
           "x": rng.standard_normal(40).astype(F32), "f": rng.integers(0, 2, 40, dtype=np.int32)}
    want = [float(d) for d in ins["dest"]]
    for j, x, f in zip(ins["i"].tolist(), ins["x"].tolist(), ins["f"].tolist()):
        if f:
            want[j] += x
    assert np.allclose(run(g2, ins)["h"], want, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- stencil + max
def test_stencil_constant_grid_pins_clamping():
    c = F32(0.3)
    w = C.stencil_max(grid=np.full((7, 9), c, F32))
    env = evaluate(w.graph, w.inputs)
    e = F32(math.exp(-float(c)))
    assert np.all(env["out"] == F32(F32(F32(F32(e + e) + e) + e) + e))   # borders included
    assert env["m"][0] == float(e)


def test_stencil_brute_force_and_max_monotone():
    rng = np.random.default_rng(31)
    for (h, w_) in ((3, 3), (1, 8), (5, 1), (4, 6)):
        grid = rng.uniform(0, 1, (h, w_)).astype(F32)
        wk = C.stencil_max(grid=grid)
        env = evaluate(wk.graph, wk.inputs)
        p = [[F32(math.exp(-float(grid[i, j]))) for j in range(w_)] for i in range(h)]
        for i in range(h):
            for j in range(w_):
                n_, s_ = p[max(i - 1, 0)][j], p[min(i + 1, h - 1)][j]
                w__, e_ = p[i][max(j - 1, 0)], p[i][min(j + 1, w_ - 1)]
                want = F32(F32(F32(F32(p[i][j] + n_) + s_) + w__) + e_)
                assert env["out"][i, j] == want, (h, w_, i, j)
        assert env["m"][0] == float(F32(math.exp(-float(grid.min()))))


def test_stencil_row_only_grid():
    # a grid that depends on the row only: west and east terms equal the centre
    h, w_ = 6, 5
    grid = np.repeat(np.linspace(0, 1, h, dtype=F32)[:, None], w_, axis=1)
    wk = C.stencil_max(grid=grid)
    env = evaluate(wk.graph, wk.inputs)
    assert np.array_equal(env["pW"], env["p"]) and np.array_equal(env["pE"], env["p"])
    assert np.array_equal(env["pN"][1:], env["p"][:-1]) and np.array_equal(env["pN"][0], env["p"][0])
    assert np.array_equal(env["pS"][:-1], env["p"][1:]) and np.array_equal(env["pS"][-1], env["p"][-1])


def test_all_small_configs_evaluate():
    for c in (1, 2, 3, 4, 5):
        w = build(c, small=True)
        env = evaluate(w.graph, w.inputs)
        for o in w.graph.outputs():
            assert env[o].shape == tuple(w.graph[o].shape)


# ---------------------------------------------------------------- the remaining vocabulary, one pin each
def test_mul_reducer_against_python_products():
    # fold / row fold / foldSeg with (*): exact rational products of short arrays (every value is
    # a small integer or a power of two, so the fp64 product is the exact one), and the identity 1
    from fractions import Fraction
    rng = np.random.default_rng(41)
    for n in range(0, 9):
        a = rng.integers(-3, 4, n).astype(F32)
        a[a == 0] = F32(2.0)
        want = Fraction(1)
        for v in a.tolist():
            want *= Fraction(v)
        assert Fraction(float(run(_fold_graph(n, "mul"), {"a": a})["r"][0])) == want
    pw = np.array([2.0 ** k for k in (3, -5, 7, -2, 0, 1)], dtype=F32)
    assert run(_fold_graph(6, "mul"), {"a": pw})["r"][0] == 2.0 ** 4
    # a sign and a zero: the product is not a sum in disguise
    assert run(_fold_graph(3, "mul"), {"a": np.array([-1.5, 2.0, 4.0], F32)})["r"][0] == -12.0
    assert run(_fold_graph(3, "mul"), {"a": np.array([5.0, 0.0, 7.0], F32)})["r"][0] == 0.0
    # rows of a two-dimensional array, each on its own
    a2 = np.array([[1, 2, 3, 4], [2, 2, 2, 2], [-1, 1, -1, 5]], dtype=F32)
    g = Graph()
    g.add("a", "input", "f32", (3, 4))
    g.add("r", "fold", "f32", (3,), fn="mul", args=("a",))
    assert run(g, {"a": a2})["r"].tolist() == [24.0, 16.0, 5.0]
    # int32 products
    gi = Graph()
    gi.add("a", "input", "i32", (2, 3))
    gi.add("r", "fold", "i32", (2,), fn="mul", args=("a",))
    assert run(gi, {"a": np.array([[2, 3, 5], [-7, 1, 11]], np.int32)})["r"].tolist() == [30, -77]
    # segments, the empty ones yielding the identity of (*)
    gs = Graph()
    gs.add("v", "input", "f32", (5,))
    gs.add("off", "input", "i32", (5,))
    gs.add("y", "foldseg", "f32", (4,), fn="mul", args=("v", "off"))
    y = run(gs, {"v": np.array([2, 3, 5, 7, 11], F32), "off": np.array([0, 2, 2, 5, 5], np.int32)})["y"]
    assert y.tolist() == [6.0, 1.0, 385.0, 1.0]


def test_add2_add3_round_after_every_addition_in_argument_order():
    # element by element against F32(F32(a + b) + c); the triples are picked so that the other
    # association, and a single rounding at the end, give another value
    a = np.array([1e8, 1.0, 0.1, 16777216.0, -3.5], dtype=F32)
    b = np.array([-1e8, 2.0 ** -24, 0.2, 1.0, 3.5], dtype=F32)
    c = np.array([1.0, 2.0 ** -24, 0.3, 1.0, 2.0 ** -30], dtype=F32)
    g = Graph()
    for nm in "abc":
        g.add(nm, "input", "f32", (5,))
    g.add("s2", "map", "f32", (5,), fn="add2", args=("a", "b"))
    g.add("s3", "map", "f32", (5,), fn="add3", args=("a", "b", "c"))
    g.add("d2", "map", "f32", (5,), fn="add2", args=("b", "c"))          # arguments are not swapped or reused
    env = run(g, {"a": a, "b": b, "c": c})
    differs = 0
    for i in range(5):
        x, y, z = float(a[i]), float(b[i]), float(c[i])
        assert env["s2"][i] == F32(x + y)                                 # the sum of two floats in fp64 rounds once: exact
        assert env["s3"][i] == F32(float(F32(x + y)) + z)
        assert env["d2"][i] == F32(y + z)
        differs += env["s3"][i] != F32(x + float(F32(y + z)))
    assert differs >= 2                                                   # the pin can tell (a+b)+c from a+(b+c)
    assert env["s3"][0] == 1.0 and env["s3"][3] == 16777216.0


def test_row_of_2d_and_const_i32_against_nested_loops():
    h, w = 3, 5
    g = Graph()
    g.add("r", "generate", "i32", (h, w), fn="row_of_2d")
    g.add("k", "generate", "i32", (h, w), fn="const_i32", iparam=(-7,))
    g.add("k1", "generate", "i32", (4,), fn="const_i32", iparam=(2147483647,))
    env = run(g, {})
    for i in range(h):
        for j in range(w):
            assert env["r"][i, j] == i and env["k"][i, j] == -7
    assert env["r"].dtype == np.int32 and env["k"].dtype == np.int32 and env["r"].shape == (h, w)
    assert env["k1"].tolist() == [2147483647] * 4
    # the row index picks rows: gathering a column vector by it repeats every entry along its row
    g2 = Graph()
    g2.add("xs", "input", "f32", (h,))
    g2.add("r", "generate", "i32", (h, w), fn="row_of_2d")
    g2.add("big", "gather", "f32", (h, w), args=("r", "xs"))
    xs = np.array([1.5, -2.0, 4.0], F32)
    assert run(g2, {"xs": xs})["big"].tolist() == [[v] * w for v in xs.tolist()]


def test_force_and_ident_are_bit_identical_copies():
    # bit patterns survive (a negative zero, a NaN with a payload, a denormal), for both types,
    # and the result is a new array: later writes to one side do not show in the other
    bits = np.array([0x80000000, 0x7fc12345, 0x00000001, 0x3f800000, 0xff800000], dtype=np.uint32)
    xf = bits.view(F32)
    xi = np.array([-2 ** 31, -1, 0, 7, 2 ** 31 - 1], dtype=np.int32)
    g = Graph()
    g.add("xf", "input", "f32", (5,))
    g.add("xi", "input", "i32", (5,))
    g.add("ff", "force", "f32", (5,), args=("xf",))
    g.add("fi", "force", "i32", (5,), args=("xi",))
    g.add("mf", "map", "f32", (5,), fn="ident", args=("xf",))
    g.add("mi", "map", "i32", (5,), fn="ident", args=("xi",))
    env = run(g, {"xf": xf, "xi": xi})
    for name in ("ff", "mf"):
        assert env[name].dtype == F32 and env[name].view(np.uint32).tolist() == bits.tolist()
        assert not np.shares_memory(env[name], xf)
    for name in ("fi", "mi"):
        assert env[name].dtype == np.int32 and env[name].tolist() == xi.tolist()
        assert not np.shares_memory(env[name], xi)


@pytest.mark.parametrize("k,r", [(2, 1), (3, 0), (4, 3), (7, 6), (5, 5), (5, 9), (1, 0), (1000003, 17)])
def test_mod_eq_against_python_remainders(k, r):
    rng = np.random.default_rng(k * 31 + r)
    v = np.concatenate([np.arange(0, 40), rng.integers(0, 2 ** 31, 200), [2 ** 31 - 1, 2 ** 31 - 2, k, k - 1 if k > 1 else 0, r]]).astype(np.int32)
    g = Graph()
    g.add("v", "input", "i32", (v.size,))
    g.add("f", "map", "i32", (v.size,), fn="mod_eq", iparam=(k, r), args=("v",))
    f = run(g, {"v": v})["f"]
    assert f.dtype == np.int32
    assert f.tolist() == [1 if int(x) % k == r else 0 for x in v.tolist()]
    if r >= k:
        assert not f.any()                                                # a residue outside [0, k) matches nothing


# ---------------------------------------------------------------- values that are not finite
def test_nonfinite_values_in_folds_scans_and_maps():
    # (+) follows IEEE-754: a NaN among the summands, or infinities of both signs, give NaN;
    # infinities of one sign give that infinity.  max is maxNum: a NaN counts as missing.
    # Each outcome is the same for every order of evaluation, which is checked on permutations.
    nan, inf = float("nan"), float("inf")
    rng = np.random.default_rng(43)
    base = rng.standard_normal(12).astype(F32)
    cases = {"nan": [3, nan], "pinf": [5, inf], "ninf": [7, -inf], "both": [2, inf, 9, -inf], "pinf_nan": [1, inf, 4, nan]}
    for name, spec in cases.items():
        a = base.copy()
        for pos, val in zip(spec[0::2], spec[1::2]):
            a[pos] = val
        for trial in range(4):
            b = a[rng.permutation(12)] if trial else a
            s = run(_fold_graph(12), {"a": b})["r"][0]
            m = run(_fold_graph(12, "max"), {"a": b})["r"][0]
            finite_max = max(v for v in b.tolist() if not math.isnan(v))
            assert m == finite_max, (name, trial)
            if name in ("nan", "both", "pinf_nan"):
                assert math.isnan(s), (name, trial)
            else:
                assert s == (inf if name == "pinf" else -inf), (name, trial)
    # nothing but NaN: the identity of max; a segment likewise, and one NaN does not leak into other segments
    assert run(_fold_graph(3, "max"), {"a": np.full(3, nan, F32)})["r"][0] == -inf
    gs = Graph()
    gs.add("v", "input", "f32", (6,))
    gs.add("off", "input", "i32", (4,))
    gs.add("s", "foldseg", "f32", (3,), fn="add", args=("v", "off"))
    gs.add("m", "foldseg", "f32", (3,), fn="max", args=("v", "off"))
    env = run(gs, {"v": np.array([1, nan, 2, 3, inf, 4], F32), "off": np.array([0, 2, 4, 6], np.int32)})
    assert math.isnan(env["s"][0]) and env["s"][1] == 5.0 and env["s"][2] == inf
    assert env["m"].tolist() == [1.0, 3.0, inf]
    # exclusive scan: a prefix is affected from the element after the special value on
    gl = Graph()
    gl.add("a", "input", "f32", (6,))
    gl.add("l", "scanl", "f32", (6,), fn="add", args=("a",))
    gl.add("r", "scanr", "f32", (6,), fn="add", args=("a",))
    env = run(gl, {"a": np.array([1, 2, inf, 4, nan, 8], F32)})
    assert env["l"][:3].tolist() == [0.0, 1.0, 3.0] and env["l"][3] == inf and env["l"][4] == inf and math.isnan(env["l"][5])
    assert math.isnan(env["r"][0]) and math.isnan(env["r"][3]) and env["r"][4] == 8.0 and env["r"][5] == 0.0
    # element functions: sin of an infinity is NaN, exp(-x) saturates to 0 and to +inf
    gm = Graph()
    gm.add("x", "input", "f32", (4,))
    gm.add("s", "map", "f32", (4,), fn="sin_x_mul_x", args=("x",))
    gm.add("e", "map", "f32", (4,), fn="exp_neg", args=("x",))
    with np.errstate(all="ignore"):
        env = run(gm, {"x": np.array([inf, -inf, nan, 1000.0], F32)})
    assert all(math.isnan(v) for v in env["s"][:3].tolist())
    assert env["e"][0] == 0.0 and env["e"][1] == inf and math.isnan(env["e"][2]) and env["e"][3] == 0.0
