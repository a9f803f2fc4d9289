"""The example programs of the paper (sections 1, 3.3, 3.4, 5), planned by fc_plan and executed
on the GPU, fused and unfused, against the CPU oracle."""
import numpy as np
import pytest

import parity as P
from oracle.interp import evaluate
from workloads import Graph
from workloads import paper_graphs as PG

pytestmark = pytest.mark.gpu
F32 = np.float32


def fc():
    import paper_2407_13585_amd as fc_
    return fc_


def device_program(*a, **kw):
    from paper_2407_13585_amd.device import DeviceProgram
    return DeviceProgram(*a, **kw)


def random_inputs(g, rng, index_ranges):
    ins = {}
    for n in g.nodes:
        if n.kind != "input":
            continue
        if n.dtype == "i32":
            hi = index_ranges.get(n.name, 1000)
            ins[n.name] = rng.integers(0, hi, size=n.shape, dtype=np.int32)
        else:
            ins[n.name] = rng.uniform(0.9, 1.1, size=n.shape).astype(F32)
    return ins


def check(g, ins, exact=(), folds=(), close=(), duplicate=False, expect_clusters=None):
    env = evaluate(g, ins)
    gp = g
    if duplicate:
        gp, _ = fc().fc_duplicate(g)
    part = fc().fc_plan(gp, "bytes")
    if expect_clusters is not None:
        assert part.n_clusters == expect_clusters
    runs = {"fused": device_program(gp, ins, part), "unfused": device_program(g, ins, None)}
    for tag, prog in runs.items():
        prog.run()
        for name in exact:
            P.assert_bit_exact(prog.fetch(name), env[name], f"{tag}/{name}")
        for name in folds:
            got, ref = prog.fetch(name).astype(np.float64), env[name].astype(np.float64)
            assert np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-30), f"{tag}/{name}"
        for name, rel in close:
            P.assert_close(prog.fetch(name), env[name], rel, f"{tag}/{name}")
        assert prog.control_words()[1] == 0
    return runs


def test_scatter_example_combining_scatter():
    rng = np.random.default_rng(1)
    g = PG.scatter_example()
    n = g["xs"].size
    ins = {"xs": rng.integers(0, n, size=n, dtype=np.int32)}       # colliding indices on purpose
    runs = check(g, ins, exact=("result",), expect_clusters=2)
    assert runs["fused"].kernels()[-1].startswith("scatter.add[")


def test_single_loop_is_one_kernel():
    rng = np.random.default_rng(2)
    g = PG.single_loop()
    runs = check(g, random_inputs(g, rng, {}), exact=("result",), expect_clusters=1)
    assert len(runs["fused"].kernels()) == 1


def test_single_loop_sizes():
    # the reversed read: whole tiles, a ragged tail, tile counts off the groups of the mirrored order
    rng = np.random.default_rng(12)
    for n in (1, 3, 4, 4096, 4100, 16 * 4096, 21 * 4096 + 4, 47 * 4096 + 1, 2070 * 4096 + 12):
        g = PG.single_loop(n)
        check(g, random_inputs(g, rng, {}), exact=("result",), expect_clusters=1)


def test_simple_programs():
    rng = np.random.default_rng(3)
    for make, ranges, out in ((PG.simple1, {"is": PG.N}, "bs"), (PG.simple2, {"is1": 2 * PG.N, "is2": PG.N}, "bs"),
                              (PG.simple3, {"is": PG.N}, "bs"), (PG.simple5, {"is": PG.N}, "cs")):
        g = make()
        check(g, random_inputs(g, rng, ranges), exact=(out,))
    g = PG.simple3()
    check(g, random_inputs(g, rng, {"is": PG.N}), exact=("as", "bs"), expect_clusters=2)


def test_simple4_gather_of_a_row_fold():
    rng = np.random.default_rng(4)
    for inner in (16, 5, 200, 4096):
        g = Graph()
        rows = 300
        g.add("is", "input", "i32", (rows // 2,))
        g.add("xs", "input", "f32", (rows, inner))
        g.add("as", "fold", "f32", (rows,), fn="add", args=("xs",))
        g.add("bs", "gather", "f32", (rows // 2,), args=("is", "as"), output=True)
        ins = random_inputs(g, rng, {"is": rows})
        runs = check(g, ins, folds=("bs",), expect_clusters=1)
        assert "@gather" in runs["fused"].kernels()[0]


def test_scan_then_gather_and_scanr():
    rng = np.random.default_rng(5)
    g = PG.scan_then_gather()
    check(g, random_inputs(g, rng, {"is": PG.N, "xs": 100}), exact=("bs",), expect_clusters=2)
    # scanr reads whole tiles in mirrored 128-bit groups when the length is a multiple of four
    for n in (1, 5, 4097, 100003, 100004, 3 * 12288, 12288 + 8):
        g = Graph()
        g.add("x", "input", "i32", (n,))
        g.add("z", "scanr", "i32", (n,), fn="add", args=("x",), output=True)
        g.add("y", "scanl", "i32", (n,), fn="add", args=("x",), output=True)
        ins = {"x": rng.integers(0, 50, size=n, dtype=np.int32)}
        env = evaluate(g, ins)
        part = fc().fc_partition_trivial(g)
        prog = device_program(g, ins, part)
        prog.run()
        P.assert_bit_exact(prog.fetch("z"), env["z"], f"scanr n={n}")
        P.assert_bit_exact(prog.fetch("y"), env["y"], f"scanl n={n}")


def test_scatter_add_fp32():
    # colliding fp32 sums: hardware atomics, update order not fixed; every destination within
    # 1e-5 of the sum of the magnitudes that went into it (the bound the row sums of SpMV use)
    rng = np.random.default_rng(10)
    for (n, k, flagged) in ((1, 1, False), (4099, 17, False), (1 << 20, 1000, True), (300001, 1 << 18, True)):
        g = Graph()
        g.add("dest", "input", "f32", (k,))
        g.add("i", "input", "i32", (n,))
        g.add("x", "input", "f32", (n,))
        args = ("dest", "i", "x")
        if flagged:
            g.add("f", "input", "i32", (n,))
            args += ("f",)
        g.add("h", "scatter", "f32", (k,), fn="add", args=args, output=True)
        ins = {"dest": rng.standard_normal(k).astype(F32), "i": rng.integers(0, k, n, dtype=np.int32),
               "x": rng.standard_normal(n).astype(F32)}
        if flagged:
            ins["f"] = rng.integers(0, 2, n, dtype=np.int32)
        env = evaluate(g, ins)
        keep = ins["f"] != 0 if flagged else np.ones(n, bool)
        scale = np.abs(ins["dest"]).astype(np.float64)
        np.add.at(scale, ins["i"][keep], np.abs(ins["x"][keep]).astype(np.float64))
        for part in (fc().fc_plan(g, "bytes"), None):
            prog = device_program(g, ins, part)
            prog.run()
            got = prog.fetch("h").astype(np.float64)
            assert np.all(np.abs(got - env["h"]) <= 1e-5 * scale + 1e-30), (n, k)
            assert prog.kernels()[-1].startswith("scatter.add[")


def prefix_scale(x, reverse):
    """Sum of the magnitudes that go into every exclusive prefix (suffix) of the rows of x."""
    a = np.abs(np.asarray(x, dtype=np.float64))
    a = a.reshape(-1, a.shape[-1]) if a.ndim > 1 else a.reshape(1, -1)
    if reverse:
        a = a[:, ::-1]
    sc = np.zeros_like(a)
    np.cumsum(a[:, :-1], axis=1, out=sc[:, 1:])
    return (sc[:, ::-1] if reverse else sc).reshape(np.asarray(x).shape)


def test_scans_of_fp32():
    # prefix sums of fp32 arrays: the same single pass with the aggregates travelling as bit
    # patterns.  The kernel adds in a fixed tree order, the reference sums exactly and rounds once:
    # every prefix within 1e-5 of the magnitudes summed (the bound of the folds).  Lengths around
    # the tile (8192), the 128-bit group and the group of 256 tiles; scanr with a length that is
    # and is not a multiple of four (mirrored 128-bit reads, or element by element).
    rng = np.random.default_rng(12)
    for n in (1, 3, 8191, 8192, 8193, 100003, 100004, (1 << 21) + 8192 * 3 + 5, 1 << 22):
        g = Graph()
        g.add("x", "input", "f32", (n,))
        g.add("l", "scanl", "f32", (n,), fn="add", args=("x",), output=True)
        g.add("r", "scanr", "f32", (n,), fn="add", args=("x",), output=True)
        ins = {"x": rng.standard_normal(n).astype(F32)}
        env = evaluate(g, ins)
        prog = device_program(g, ins, fc().fc_partition_trivial(g))
        for _ in range(2):                                       # the status words are reused
            prog.run()
            for name, rev in (("l", False), ("r", True)):
                got = prog.fetch(name).astype(np.float64)
                tol = 1e-5 * prefix_scale(ins["x"], rev) + 1e-30
                bad = np.flatnonzero(np.abs(got - env[name].astype(np.float64)) > tol)
                assert bad.size == 0, (n, name, bad[:5], got[bad[:5]], env[name][bad[:5]])
            assert prog.control_words()[1] == 0
        assert sorted(prog.kernels()) == ["scan[in0:f32]+offs", "scanr[in0:f32]+offs"]
    # positive terms of one size: the running sum grows to 2^22 times a term, the worst case for the
    # rounding of a sequential sum; the tree order stays far inside the bound
    n = 1 << 22
    g = Graph()
    g.add("x", "input", "f32", (n,))
    g.add("y", "map", "f32", (n,), fn="affine", fparam=(0.5, 0.25), args=("x",))
    g.add("l", "scanl", "f32", (n,), fn="add", args=("y",), output=True)
    ins = {"x": rng.uniform(0.0, 1.0, size=n).astype(F32)}
    env = evaluate(g, ins)
    for part in (fc().fc_plan(g, "bytes"), None):
        prog = device_program(g, ins, part)
        prog.run()
        got = prog.fetch("l").astype(np.float64)
        assert np.all(np.abs(got - env["l"].astype(np.float64)) <= 1e-5 * prefix_scale(env["y"], False) + 1e-30)
        if part is not None:
            assert prog.kernels() == ["scan[map2(in0:f32)]+offs"], prog.kernels()
    # two dimensions: row by row
    for (rows, w) in ((3, 1), (37, 16), (300, 17), (65, 65), (40, 1000), (7, 1025), (2, 70001)):
        g = Graph()
        g.add("x", "input", "f32", (rows, w))
        g.add("l", "scanl", "f32", (rows, w), fn="add", args=("x",), output=True)
        g.add("r", "scanr", "f32", (rows, w), fn="add", args=("x",), output=True)
        ins = {"x": rng.standard_normal((rows, w)).astype(F32)}
        env = evaluate(g, ins)
        prog = device_program(g, ins, fc().fc_partition_trivial(g))
        prog.run()
        for name, rev in (("l", False), ("r", True)):
            got = prog.fetch(name).astype(np.float64)
            assert np.all(np.abs(got - env[name].astype(np.float64)) <= 1e-5 * prefix_scale(ins["x"], rev) + 1e-30), (rows, w, name)
        assert all(k.startswith("rowscan") for k in prog.kernels())


def test_programs_whose_optimum_has_no_kernel_run_with_an_executable_plan():
    # the cheapest legal clustering of these programs contains a cluster the library has no
    # kernel for; planned with FC_PLAN_EXECUTABLE they run fused as far as the kernels go
    from test_chooser import unsupported_optimum_graphs
    rng = np.random.default_rng(14)
    for name, g in unsupported_optimum_graphs().items():
        ins = {n.name: (rng.integers(0, 2 ** 31, size=n.shape, dtype=np.int32) if n.dtype == "i32"
                        else rng.uniform(0.0, 1.0, size=n.shape).astype(F32)) for n in g.nodes if n.kind == "input"}
        env = evaluate(g, ins)
        with pytest.raises(fc().FcError):
            device_program(g, ins, fc().fc_plan(g, "bytes")).run()
        part = fc().fc_plan(g, "bytes", executable=True)
        prog = device_program(g, ins, part)
        prog.run()
        for out in g.outputs():
            got, ref = prog.fetch(out), env[out]
            node = g[out]
            if node.dtype == "i32":
                P.assert_bit_exact(got, ref, f"{name}/{out}")
            elif node.kind == "scanl":
                scale = prefix_scale(env[node.args[0]], False)
                assert np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= 1e-5 * scale + 1e-30), (name, out)
            elif node.kind == "fold" and node.fn == "add":
                scale = np.abs(env[node.args[0]].astype(np.float64)).sum()
                assert abs(float(got[0]) - float(ref[0])) <= 1e-5 * scale, (name, out)
            elif node.kind == "fold" and node.fn == "mul":
                assert abs(float(got[0]) - float(ref[0])) <= 1e-4 * abs(float(ref[0])), (name, out)
            elif node.kind == "fold":
                P.assert_bit_exact(got, ref, f"{name}/{out}")        # a maximum of exactly computed values
            else:
                P.assert_ulp(got, np.asarray(ref, dtype=np.float64).astype(F32), 4, f"{name}/{out}")
        assert prog.control_words()[1] == 0


class ProgramMaker:
    """Random element programs over a few inputs of one shape: every root a tree, so that the roots
    together with one consumer are one legal cluster."""

    def __init__(self, rng, shape):
        self.rng, self.shape = rng, tuple(shape)
        self.size = int(np.prod(shape))
        self.g, self.ins = Graph(), {}
        self.count = 0
        self.pool = {"f32": [], "i32": []}               # a handful of inputs, read from several places

    def fresh(self, prefix):
        self.count += 1
        return f"{prefix}{self.count}"

    def leaf_f32(self):
        rng, pool = self.rng, self.pool["f32"]
        if len(pool) == 3 or (pool and rng.integers(0, 2)):
            return pool[rng.integers(0, len(pool))]
        name = self.fresh("x")
        self.g.add(name, "input", "f32", self.shape)
        self.ins[name] = rng.uniform(0.0, 1.0, size=self.shape).astype(F32)
        pool.append(name)
        return name

    def leaf_i32(self):
        """Flat positions inside the arrays."""
        rng, pool = self.rng, self.pool["i32"]
        if len(pool) == 2:
            return pool[rng.integers(0, 2)]
        name = self.fresh("i")
        self.g.add(name, "input", "i32", self.shape)
        self.ins[name] = rng.integers(0, self.size, size=self.shape, dtype=np.int32)
        pool.append(name)
        return name

    def index(self, depth, root=False):
        rng = self.rng
        kind = rng.integers(1 if root else 0, 4 if depth > 0 else 3)
        if kind == 0:
            return self.leaf_i32()
        name = self.fresh("i")
        if kind == 1:
            self.g.add(name, "generate", "i32", self.shape, fn="iota_rev", output=root)
        elif kind == 2:
            self.g.add(name, "generate", "i32", self.shape, fn="iota", output=root)
        else:
            self.g.add(name, "gather", "i32", self.shape, args=(self.index(0), self.index(depth - 1)), output=root)
        return name

    def flags(self, depth):
        """Zeros and ones computed from positions."""
        name = self.fresh("f")
        k = int(self.rng.integers(2, 6))
        self.g.add(name, "map", "i32", self.shape, fn="mod_eq", iparam=(k, int(self.rng.integers(0, k))), args=(self.index(depth),))
        return name

    def value(self, depth, root=False):
        rng, g, shape = self.rng, self.g, self.shape
        kind = rng.integers(1 if root else 0, 8) if depth > 0 else 0
        if kind == 0:
            return self.leaf_f32()
        name = self.fresh("v")
        if kind in (1, 2):
            fn = ("affine", "sq_plus_one", "exp_neg", "sin_x_mul_x", "ident")[rng.integers(0, 5)]
            kw = {"fparam": (float(rng.uniform(0.5, 1.5)), float(rng.uniform(-0.5, 0.5)))} if fn == "affine" else {}
            g.add(name, "map", "f32", shape, fn=fn, args=(self.value(depth - 1),), output=root, **kw)
        elif kind in (3, 4):
            g.add(name, "map", "f32", shape, fn=("mul2", "add2")[rng.integers(0, 2)],
                  args=(self.value(depth - 1), self.value(depth - 1)), output=root)
        elif kind == 5:
            g.add(name, "map", "f32", shape, fn="add3", args=(self.value(depth - 1), self.value(0), self.value(depth - 1)),
                  output=root)
        else:
            g.add(name, "gather", "f32", shape, args=(self.index(1), self.value(depth - 1)), output=root)
        return name


def random_element_program(rng, n, n_stores, with_fold):
    """A cluster of maps, generates and gathers that ends in stored arrays and at most one fold."""
    pm = ProgramMaker(rng, (n,))
    for _ in range(n_stores):
        pm.value(3, root=True)                         # a stored array is computed by the cluster
    if with_fold:
        pm.g.add("total", "fold", "f32", (1,), fn=("add", "max")[rng.integers(0, 2)], args=(pm.value(3),), output=True)
    return pm.g, pm.ins


def test_interpreted_clusters_match_the_compiled_kernels():
    # random elementwise clusters run by the interpreting kernel as one cluster; the same
    # programs run one compiled kernel per combinator must give the same bits (the same device
    # functions in the same order); a fold within the bound of the folds
    rng = np.random.default_rng(2024)
    seen_interpreted = 0
    for trial in range(40):
        n = int(rng.choice([1, 255, 5000, 300001]))
        n_stores = int(rng.integers(0, 4))
        with_fold = bool(rng.integers(0, 2)) or n_stores == 0
        g, ins = random_element_program(rng, n, n_stores, with_fold)
        if sum(nd.kind != "input" for nd in g.nodes) > 20:
            continue
        pi = [0 if nd.kind == "input" else 1 for nd in g.nodes]
        try:
            part = fc().fc_partition_check(g, pi)
            name = fc().fc_cluster_kernel(g, part, 0)
        except fc().FcError:
            continue                                   # too large for one element program
        seen_interpreted += "interpreted" in name
        env = evaluate(g, ins)
        inter = [nd.name for nd in g.nodes if nd.kind != "input"]
        fused, unfused = device_program(g, ins, part), device_program(g, ins, None, bind=inter)
        fused.run()
        unfused.run()
        for out in g.outputs():
            got = fused.fetch(out)
            if g[out].kind == "fold":
                arg = env[g[out].args[0]].astype(np.float64)
                if g[out].fn == "add":
                    assert abs(float(got[0]) - float(env[out][0])) <= 1e-5 * np.abs(arg).sum() + 1e-30, (trial, name)
                else:
                    P.assert_bit_exact(got, unfused.fetch(out), f"{trial}/{out}")
            else:
                P.assert_bit_exact(got, unfused.fetch(out), f"trial {trial} {name} {out}")
                P.assert_close(got, env[out], 1e-4, f"{trial}/{out}", abs_=1e-5)
        assert fused.control_words()[1] == 0
    assert seen_interpreted >= 15
    # sum and maximum of one computed array, and of two different ones, in one pass
    for shared in (True, False):
        n = 70001
        g = Graph()
        g.add("x", "input", "f32", (n,))
        g.add("a", "map", "f32", (n,), fn="sin_x_mul_x", args=("x",), output=shared)
        g.add("b", "map", "f32", (n,), fn="exp_neg", args=("x",))
        g.add("s", "fold", "f32", (1,), fn="add", args=("a",), output=True)
        g.add("t", "fold", "f32", (1,), fn="max", args=("a" if shared else "b",), output=True)
        ins = {"x": rng.uniform(0, 1, n).astype(F32)}
        env = evaluate(g, ins)
        part = fc().fc_plan(g, "bytes")
        fused = device_program(g, ins, part)
        assert part.n_clusters == 1 and "interpreted" in fused.kernels()[0], fused.kernels()
        unfused = device_program(g, ins, None, bind=["a", "b"])
        for _ in range(2):                                   # two accumulators, one tag per launch
            fused.run()
            unfused.run()
            P.assert_fold(fused.fetch("s"), env["s"], "two folds: sum")
            P.assert_bit_exact(fused.fetch("t"), unfused.fetch("t"), "two folds: max")
            if shared:
                P.assert_bit_exact(fused.fetch("a"), unfused.fetch("a"), "two folds: stored array")
        assert fused.control_words()[1] == 0 and fused.control_words()[0] == 2
    # an array that is stored and folded is computed once (the store leaves the value for the fold)
    n = 100003
    g = Graph()
    for nm in "abc":
        g.add(nm, "input", "f32", (n,))
    g.add("i", "input", "i32", (n,))
    g.add("t", "map", "f32", (n,), fn="affine", fparam=(2.0, 1.0), args=("a",))
    g.add("u", "map", "f32", (n,), fn="mul2", args=("t", "b"))
    g.add("gc", "gather", "f32", (n,), args=("i", "c"))
    g.add("out", "map", "f32", (n,), fn="add2", args=("u", "gc"), output=True)
    g.add("tot", "fold", "f32", (1,), fn="add", args=("out",), output=True)
    ins = {k: rng.uniform(0, 1, n).astype(F32) for k in "abc"}
    ins["i"] = rng.integers(0, n, size=n, dtype=np.int32)
    env = evaluate(g, ins)
    part = fc().fc_plan(g, "bytes")
    fused = device_program(g, ins, part)
    assert part.n_clusters == 1 and "interpreted" in fused.kernels()[0]
    fused.run()
    P.assert_bit_exact(fused.fetch("out"), env["out"], "stored and folded: out")
    P.assert_fold(fused.fetch("tot"), env["tot"], "stored and folded: tot")
    assert fused.control_words()[1] == 0


def one_cluster(g):
    part = fc().fc_partition_check(g, [0 if nd.kind == "input" else 1 for nd in g.nodes])
    return part, fc().fc_cluster_kernel(g, part, 0)


class TooLarge(Exception):
    pass


def fused_and_unfused(g, ins):
    try:
        part, name = one_cluster(g)
    except fc().FcError as e:                            # deeper than the interpreter's stack, too many inputs
        assert e.name == "FC_E_UNSUPPORTED"
        raise TooLarge()
    inter = [nd.name for nd in g.nodes if nd.kind != "input"]
    fused, unfused = device_program(g, ins, part), device_program(g, ins, None, bind=inter)
    fused.run()
    unfused.run()
    assert fused.control_words()[1] == 0
    return fused, unfused, name


def test_every_consumer_takes_any_element_program():
    # segmented folds, scatters, scans (alone and as a compaction), row folds and row scans over
    # random element programs that no instance was compiled for: the instances over Interp<K, T> run
    # them.  Arrays that are stored, scanned or scattered agree bit for bit with the unfused arm (the
    # same device functions in the same order); sums within the bound of the folds.
    rng = np.random.default_rng(4242)
    names = []
    for trial in range(6):                                    # segmented fold of a computed array
        n = int(rng.choice([1000, 70001]))
        pm = ProgramMaker(rng, (n,))
        v = pm.value(3, root=False)
        if pm.g[v].kind == "input":
            continue
        rows = max(1, n // 9)
        cuts = np.sort(rng.integers(0, n + 1, size=rows - 1))
        off = np.concatenate([[0], cuts, [n]]).astype(np.int32)
        pm.g.add("off", "input", "i32", (rows + 1,))
        pm.ins["off"] = off
        pm.g.add("y", "foldseg", "f32", (rows,), fn=("add", "max")[trial % 2], args=(v, "off"), output=True)
        env = evaluate(pm.g, pm.ins)
        try:
            fused, unfused, name = fused_and_unfused(pm.g, pm.ins)
        except TooLarge:
            continue
        names.append(name)
        if trial % 2:
            P.assert_bit_exact(fused.fetch("y"), unfused.fetch("y"), name)
        else:
            P.assert_segmented(fused.fetch("y"), env["y"], env[v], off, name)
    for trial in range(8):                                    # scatter: computed index, value and flag
        n = int(rng.choice([999, 50003]))
        pm = ProgramMaker(rng, (n,))
        add, flagged, ints = bool(trial & 1), bool(trial & 2), bool(trial & 4)
        perm = rng.permutation(n).astype(np.int32)
        pm.g.add("perm", "input", "i32", (n,))
        pm.ins["perm"] = perm
        pm.g.add("where", "gather", "i32", (n,), args=(pm.index(1, root=False), "perm"))   # distinct only if the index is
        idx = "where" if add else None
        if not add:                                          # overwrite needs distinct indices: a permutation read backwards
            pm.g.add("back", "generate", "i32", (n,), fn="iota_rev")
            pm.g.add("where2", "gather", "i32", (n,), args=("back", "perm"))
            idx = "where2"
        val = pm.index(2, root=False) if ints else pm.value(2, root=False)
        if pm.g[val].kind == "input":
            continue
        dt = "i32" if ints else "f32"
        pm.g.add("dest", "input", dt, (n,))
        pm.ins["dest"] = (rng.integers(0, 100, size=n, dtype=np.int32) if ints else rng.uniform(0, 1, size=n).astype(F32))
        args = ("dest", idx, val) + ((pm.flags(1),) if flagged else ())
        pm.g.add("h", "scatter", dt, (n,), fn="add" if add else "overwrite", args=args, output=True)
        # nodes nothing reads would be clusters of their own
        g = prune(pm.g)
        ins = {k: v for k, v in pm.ins.items() if k in {nd.name for nd in g.nodes}}
        env = evaluate(g, ins)
        try:
            fused, unfused, name = fused_and_unfused(g, ins)
        except TooLarge:
            continue
        names.append(name)
        if add and not ints:
            keep = env[args[3]].reshape(-1) != 0 if flagged else np.ones(n, bool)
            scale = np.abs(ins["dest"]).astype(np.float64)
            np.add.at(scale, env[idx].reshape(-1)[keep], np.abs(env[val].reshape(-1)[keep]).astype(np.float64))
            assert np.all(np.abs(fused.fetch("h").astype(np.float64) - env["h"]) <= 1e-5 * scale + 1e-30), name
        else:
            P.assert_bit_exact(fused.fetch("h"), unfused.fetch("h"), name)
    for trial in range(6):                                    # scans of computed flags; compaction of computed values
        n = int(rng.choice([777, 12288 * 3 + 5, 200001]))
        pm = ProgramMaker(rng, (n,))
        flags = pm.flags(2)
        mode = trial % 3
        pm.g.add("offs", "scanl", "i32", (n,), fn="add", args=(flags,), output=(mode != 1))
        outs = ["offs"] if mode != 1 else []
        if mode >= 1:
            ints = bool(trial & 1)
            val = pm.index(2, root=False) if ints else pm.value(2, root=False)
            if pm.g[val].kind == "input":
                continue
            dt = "i32" if ints else "f32"
            pm.g.add("dest", "input", dt, (n,))
            pm.ins["dest"] = np.zeros(n, dtype=np.int32 if ints else F32)
            pm.g.add("out", "scatter", dt, (n,), fn="overwrite", args=("dest", "offs", val, flags), output=True)
            pm.g.add("count", "fold", "i32", (1,), fn="add", args=(flags,), output=True)
            outs += ["out", "count"]
        g = prune(pm.g)
        ins = {k: v for k, v in pm.ins.items() if k in {nd.name for nd in g.nodes}}
        try:
            fused, unfused, name = fused_and_unfused(g, ins)
        except TooLarge:
            continue
        names.append(name)
        for o in outs:
            P.assert_bit_exact(fused.fetch(o), unfused.fetch(o), f"{name}/{o}")
    for trial in range(4):                                    # prefix sums of a computed fp32 array
        n = int(rng.choice([5000, 8192 * 5 + 3]))
        pm = ProgramMaker(rng, (n,))
        v = pm.value(3, root=False)
        if pm.g[v].kind == "input":
            continue
        pm.g.add("l", "scanr" if trial & 1 else "scanl", "f32", (n,), fn="add", args=(v,), output=True)
        env = evaluate(pm.g, pm.ins)
        try:
            fused, unfused, name = fused_and_unfused(pm.g, pm.ins)
        except TooLarge:
            continue
        names.append(name)
        got = fused.fetch("l").astype(np.float64)
        assert np.all(np.abs(got - env["l"].astype(np.float64)) <= 1e-5 * prefix_scale(env[v], bool(trial & 1)) + 1e-30), name
    for trial in range(8):                                    # rows: folds and scans of computed 2-D arrays
        rows, w = [(37, 16), (5, 1000), (300, 17), (3, 5000)][trial % 4]
        pm = ProgramMaker(rng, (rows, w))
        if trial < 4:
            v = pm.value(3, root=False)
            if pm.g[v].kind == "input":
                continue
            fn = ("add", "max", "mul", "add")[trial]
            if fn == "mul":                                   # keep the product of a row in range
                pm.g.add("near1", "map", "f32", (rows, w), fn="affine", fparam=(1e-4, 1.0), args=(v,))
                v = "near1"
            pm.g.add("y", "fold", "f32", (rows,), fn=fn, args=(v,), output=True)
            env = evaluate(pm.g, pm.ins)
            try:
                fused, unfused, name = fused_and_unfused(pm.g, pm.ins)
            except TooLarge:
                continue
            got, ref = fused.fetch("y").astype(np.float64), env["y"].astype(np.float64)
            if fn == "max":
                P.assert_bit_exact(fused.fetch("y"), unfused.fetch("y"), name)
            elif fn == "add":
                assert np.all(np.abs(got - ref) <= 1e-5 * np.abs(env[v].astype(np.float64)).sum(axis=1) + 1e-30), name
            else:
                assert np.all(np.abs(got - ref) <= 1e-4 * np.abs(ref)), name
        else:
            flags = pm.flags(2)
            pm.g.add("l", "scanr" if trial & 1 else "scanl", "i32", (rows, w), fn="add", args=(flags,), output=True)
            try:
                fused, unfused, name = fused_and_unfused(pm.g, pm.ins)
            except TooLarge:
                continue
            P.assert_bit_exact(fused.fetch("l"), unfused.fetch("l"), name)
        names.append(name)
    generic = [k for k in names if "element programs interpreted" in k]
    assert len(generic) >= 20, names
    for shape in ("foldseg.", "scatter[", "scatter.add[", "scan[", "+scatter[", "+count", "scanr[", "rowfold.", "rowscan"):
        assert any(shape in k for k in generic), (shape, generic)


def prune(g):
    """The graph without the nodes no output depends on."""
    need, by_name = set(), {nd.name: nd for nd in g.nodes}
    stack = [nd.name for nd in g.nodes if nd.output]
    while stack:
        a = stack.pop()
        if a not in need:
            need.add(a)
            stack.extend(by_name[a].args)
    out = Graph()
    for nd in g.nodes:
        if nd.name in need:
            out.add(nd.name, nd.kind, nd.dtype, nd.shape, fn=nd.fn, fparam=nd.fparam, iparam=nd.iparam, args=nd.args, output=nd.output)
    return out


def random_program(rng, n, n_ops):
    """A random program over arrays of n elements that can be executed: arrays used as positions hold
    positions (inputs below n, iota, gathers of such), everything else is typed by what produced it."""
    g, ins = Graph(), {}
    pos, flags, ints, flts = [], [], [], []                  # positions, zeros and ones, any i32, f32
    for k in range(2):
        g.add(f"p{k}", "input", "i32", (n,))
        ins[f"p{k}"] = rng.integers(0, n, size=n, dtype=np.int32)
        pos.append(f"p{k}")
        g.add(f"x{k}", "input", "f32", (n,))
        ins[f"x{k}"] = rng.uniform(0.0, 1.0, size=n).astype(F32)
        flts.append(f"x{k}")
    g.add("perm", "input", "i32", (n,))
    ins["perm"] = rng.permutation(n).astype(np.int32)
    pick = lambda pool: str(pool[rng.integers(0, len(pool))])
    scattered = set()
    for k in range(n_ops):
        nm = f"t{k}"
        kind = str(rng.choice(["map1", "map1", "map2", "gen", "gatherp", "gatherf", "gatherf", "flags", "scani", "scanf",
                               "foldf", "foldi", "scatterf", "scatteri"]))
        if kind == "map1":
            fn = str(rng.choice(["affine", "sq_plus_one", "exp_neg", "sin_x_mul_x"]))
            kw = {"fparam": (float(rng.uniform(0.5, 1.0)), float(rng.uniform(0.0, 0.5)))} if fn == "affine" else {}
            g.add(nm, "map", "f32", (n,), fn=fn, args=(pick(flts),), **kw)
            flts.append(nm)
        elif kind == "map2":
            g.add(nm, "map", "f32", (n,), fn=str(rng.choice(["mul2", "add2"])), args=(pick(flts), pick(flts)))
            flts.append(nm)
        elif kind == "gen":
            g.add(nm, "generate", "i32", (n,), fn=str(rng.choice(["iota", "iota_rev"])))
            pos.append(nm)
        elif kind == "gatherp":
            g.add(nm, "gather", "i32", (n,), args=(pick(pos), pick(pos)))
            pos.append(nm)
        elif kind == "gatherf":
            g.add(nm, "gather", "f32", (n,), args=(pick(pos), pick(flts)))
            flts.append(nm)
        elif kind == "flags":
            m = int(rng.integers(2, 5))
            g.add(nm, "map", "i32", (n,), fn="mod_eq", iparam=(m, int(rng.integers(0, m))), args=(pick(pos + ints),))
            flags.append(nm)
        elif kind == "scani":
            g.add(nm, str(rng.choice(["scanl", "scanr"])), "i32", (n,), fn="add", args=(pick(flags or pos),))
            ints.append(nm)
        elif kind == "scanf":
            g.add(nm, str(rng.choice(["scanl", "scanr"])), "f32", (n,), fn="add", args=(pick(flts),))
            # prefix sums grow with n: bring them back to the size of the other values
            g.add(nm + "s", "map", "f32", (n,), fn="affine", fparam=(1.0 / n, 0.0), args=(nm,))
            flts.append(nm + "s")
        elif kind == "foldf":
            g.add(nm, "fold", "f32", (1,), fn=str(rng.choice(["add", "max"])), args=(pick(flts),), output=True)
        elif kind == "foldi":
            if flags and rng.integers(0, 2):
                g.add(nm, "fold", "i32", (1,), fn="add", args=(pick(flags),), output=True)      # a count
            else:
                g.add(nm, "fold", "i32", (1,), fn="max", args=(pick(flags + ints or pos),), output=True)
        else:
            f32 = kind == "scatterf"
            dests = [d for d in (flts if f32 else ints + flags) if d not in scattered and g[d].kind != "input"]
            if not dests:
                continue
            dest = pick(dests)
            scattered.add(dest)
            # overwrite at distinct positions (a permutation, or one read backwards); i32 may also combine anywhere
            if f32 or rng.integers(0, 2):
                g.add(nm + "b", "generate", "i32", (n,), fn="iota_rev")
                g.add(nm + "w", "gather", "i32", (n,), args=(nm + "b", "perm"))
                where, fn = nm + "w", "overwrite"
            else:
                where, fn = pick(pos), "add"
            # the destination is updated in place, so the scatter reads everything else from other arrays
            values = [v for v in (flts if f32 else flags + ints or pos) if v != dest] or pos
            if f32 and values is pos:
                continue
            others = [f for f in flags if f != dest]
            args = (dest, where, pick(values)) + ((pick(others),) if others and rng.integers(0, 2) else ())
            g.add(nm, "scatter", "f32" if f32 else "i32", (n,), fn=fn, args=args)
            # the scatter updates its destination in place: from here on the program names the result only
            for pool in (pos, flags, ints, flts):
                if dest in pool:
                    pool.remove(dest)
            (flts if f32 else ints).append(nm)
            scattered.add(nm)
        if sum(nd.kind != "input" for nd in g.nodes) >= 11:      # the chooser is exact: keep its search short
            break
    return g, ins


def with_outputs(g):
    """Every array nothing reads becomes a result (it is manifest anyway)."""
    read = {a for nd in g.nodes for a in nd.args}
    out = Graph()
    for nd in g.nodes:
        out.add(nd.name, nd.kind, nd.dtype, nd.shape, fn=nd.fn, fparam=nd.fparam, iparam=nd.iparam, args=nd.args,
                output=nd.output or (nd.kind != "input" and nd.name not in read))
    return out


@pytest.mark.parametrize("seed", range(24))
def test_random_programs_planned_and_run(seed):
    # whole programs: a random DAG over every combinator, planned by the ILP among the clusterings the
    # library runs, executed fused and unfused.  Integers agree exactly with the oracle; fp32 arrays agree
    # bit for bit between the two arms (same device functions in the same order) and closely with the
    # oracle; fp32 sums within the bound of the folds.
    rng = np.random.default_rng(7000 + seed)
    n = int(rng.choice([1000, 4097, 30001]))
    g, ins = random_program(rng, n, int(rng.integers(4, 11)))
    g = with_outputs(g)
    used = {a for nd in g.nodes for a in nd.args}
    ins = {k: v for k, v in ins.items()}
    env = evaluate(g, ins)
    part = fc().fc_plan(g, "bytes", executable=True)
    inter = [nd.name for nd in g.nodes if nd.kind != "input"]
    fused, unfused = device_program(g, ins, part), device_program(g, ins, None, bind=inter)
    fused.run()
    unfused.run()
    assert fused.control_words()[1] == 0 and unfused.control_words()[1] == 0
    for out in g.outputs():
        nd = g[out]
        got, ref = fused.fetch(out), env[out]
        what = f"seed {seed} {out} {fused.kernels()}"
        if nd.dtype == "i32":
            P.assert_bit_exact(got, ref, what)
        elif nd.kind == "fold" and nd.fn == "add":
            assert abs(float(got[0]) - float(ref[0])) <= 1e-5 * np.abs(env[nd.args[0]].astype(np.float64)).sum() + 1e-30, what
        else:
            P.assert_bit_exact(got, unfused.fetch(out), what)
            P.assert_close(got, ref, 2e-4, what, abs_=2e-5)


@pytest.mark.parametrize("n_ops", [30, 45, 70])
def test_large_programs_planned_anytime_and_run(n_ops):
    # programs of the size of the paper's benchmarks (section 5.2: 51 to 99 combinators): planned within
    # the time limit among the clusterings that run, executed fused (a dozen clusters, intermediates in
    # scratch) and one kernel per combinator; results as in test_random_programs_planned_and_run
    from test_chooser import pipeline_program
    n = 4096
    for seed in range(20):
        g = pipeline_program(np.random.default_rng(1000 * n_ops + seed), n_ops, n=n, tame=True)
        rng = np.random.default_rng(seed)
        ins = {nd.name: (rng.integers(0, n, size=n, dtype=np.int32) if nd.dtype == "i32" else rng.uniform(0.0, 1.0, size=n).astype(F32))
               for nd in g.nodes if nd.kind == "input"}
        g = with_outputs(g)
        with np.errstate(all="ignore"):
            env = evaluate(g, ins)
        if all(np.all(np.isfinite(v.astype(np.float64))) and np.all(np.abs(v.astype(np.float64)) < 1e4) for v in env.values()):
            break                                       # repeated squaring makes some programs overflow, or sin ill-conditioned
    else:
        pytest.skip("no program with finite results")
    part = fc().fc_plan(g, "bytes", executable=True, anytime=True)
    assert part.n_clusters <= (3 * n_ops) // 4
    inter = [nd.name for nd in g.nodes if nd.kind != "input"]
    fused, unfused = device_program(g, ins, part), device_program(g, ins, None, bind=inter)
    fused.run()
    unfused.run()
    assert fused.control_words()[1] == 0 and unfused.control_words()[1] == 0
    for out in g.outputs():
        nd = g[out]
        got, ref = fused.fetch(out), env[out]
        what = f"{n_ops} combinators, {out}"
        if nd.dtype == "i32":
            P.assert_bit_exact(got, ref, what)
        elif nd.kind == "fold":
            arg = env[nd.args[0]].astype(np.float64)
            assert abs(float(got[0]) - float(ref[0])) <= 1e-5 * np.abs(arg).sum() + 1e-30, what
        else:
            P.assert_bit_exact(got, unfused.fetch(out), what)
            P.assert_close(got, ref, 1e-3, what, abs_=1e-4)


def test_scan_clusters_that_also_store_what_they_scan():
    # diagonal fusion into a scan: the predicate is a result as well as scanned (and the compaction's
    # scatter and count may sit in the same cluster); stored straight from the registers it was loaded into
    rng = np.random.default_rng(21)
    for n in (5, 12288, 12288 * 2 + 8, 100003):
        for shape in ("offsets", "compaction", "computed", "right"):
            g = Graph()
            g.add("v", "input", "i32", (n,))
            if shape == "computed":                          # no compiled instance: the element programs are interpreted
                g.add("back", "generate", "i32", (n,), fn="iota_rev")
                g.add("vv", "gather", "i32", (n,), args=("back", "v"))
                g.add("flags", "map", "i32", (n,), fn="mod_eq", iparam=(4, 1), args=("vv",), output=True)
            else:
                g.add("flags", "map", "i32", (n,), fn="mod_eq", iparam=(3, 0), args=("v",), output=True)
            g.add("offs", "scanr" if shape == "right" else "scanl", "i32", (n,), fn="add", args=("flags",),
                  output=shape != "compaction")
            outs = ["flags"] + (["offs"] if shape != "compaction" else [])
            if shape in ("compaction", "computed"):
                g.add("dest", "input", "i32", (n,))
                g.add("out", "scatter", "i32", (n,), fn="overwrite", args=("dest", "offs", "v", "flags"), output=True)
                g.add("count", "fold", "i32", (1,), fn="add", args=("flags",), output=True)
                outs += ["out", "count"]
            ins = {"v": rng.integers(0, 2 ** 31, size=n, dtype=np.int32), "dest": np.zeros(n, np.int32)}
            ins = {k: v for k, v in ins.items() if k in {nd.name for nd in g.nodes}}
            env = evaluate(g, ins)
            part = fc().fc_plan(g, "bytes")
            prog = device_program(g, ins, part)
            assert part.n_clusters == 1 and "+input" in prog.kernels()[0], prog.kernels()
            assert ("interpreted" in prog.kernels()[0]) == (shape in ("computed", "right"))
            prog.run()
            for o in outs:
                P.assert_bit_exact(prog.fetch(o), env[o], f"{shape} n={n} {o}")
            assert prog.control_words()[1] == 0


def test_fp32_scans_that_also_store_what_they_scan():
    # the same for fp32: `affine` under scanl has a compiled instance, the others run with the element
    # program interpreted; both arrays agree bit for bit with the unfused arm (same additions in the same
    # tree), the stored array with the oracle as its map allows, the prefixes within the bound of the folds
    rng = np.random.default_rng(22)
    for n in (7, 8192, 8192 * 3 + 4, 50001):
        for fn, right in (("affine", False), ("affine", True), ("exp_neg", False), ("sq_plus_one", True)):
            g = Graph()
            g.add("v", "input", "f32", (n,))
            kw = {"fparam": (0.5, 0.25)} if fn == "affine" else {}
            g.add("w", "map", "f32", (n,), fn=fn, args=("v",), output=True, **kw)
            g.add("sums", "scanr" if right else "scanl", "f32", (n,), fn="add", args=("w",), output=True)
            ins = {"v": rng.uniform(-1.0, 1.0, size=n).astype(F32)}
            env = evaluate(g, ins)
            part = fc().fc_plan(g, "bytes")
            fused, unfused = device_program(g, ins, part), device_program(g, ins, None)
            assert part.n_clusters == 1 and "+input" in fused.kernels()[0], fused.kernels()
            assert ("interpreted" in fused.kernels()[0]) == (fn != "affine" or right)
            fused.run()
            unfused.run()
            what = f"{fn} right={right} n={n}"
            for o in ("w", "sums"):
                P.assert_bit_exact(fused.fetch(o), unfused.fetch(o), what + " " + o)
            if fn == "exp_neg":
                P.assert_ulp(fused.fetch("w"), np.asarray(env["w"], dtype=np.float64).astype(F32), 4, what)
            else:
                P.assert_bit_exact(fused.fetch("w"), env["w"], what)
            scale = prefix_scale(env["w"], right)
            err = np.abs(fused.fetch("sums").astype(np.float64) - env["sums"].astype(np.float64))
            assert np.all(err <= 1e-5 * scale + 1e-30), what
            assert fused.control_words()[1] == 0


def test_row_scans_that_also_store_what_they_scan():
    # two-dimensional arrays: every row scanned on its own, the scanned array a result as well
    rng = np.random.default_rng(23)
    for shape in ((1, 300), (200, 777), (3000, 17), (5, 5000)):
        for dtype, fn, right in (("i32", "mod_eq", False), ("i32", "mod_eq", True), ("f32", "sq_plus_one", False), ("f32", "affine", True)):
            g = Graph()
            g.add("v", "input", dtype, shape)
            kw = {"iparam": (3, 0)} if fn == "mod_eq" else {"fparam": (0.5, 0.25)} if fn == "affine" else {}
            g.add("w", "map", dtype, shape, fn=fn, args=("v",), output=True, **kw)
            g.add("sums", "scanr" if right else "scanl", dtype, shape, fn="add", args=("w",), output=True)
            ins = {"v": rng.integers(0, 2 ** 31, size=shape, dtype=np.int32) if dtype == "i32"
                   else rng.uniform(-1.0, 1.0, size=shape).astype(F32)}
            env = evaluate(g, ins)
            part = fc().fc_plan(g, "bytes")
            fused, unfused = device_program(g, ins, part), device_program(g, ins, None)
            assert part.n_clusters == 1 and "+input" in fused.kernels()[0], fused.kernels()
            fused.run()
            unfused.run()
            what = f"{shape} {dtype} right={right}"
            for o in ("w", "sums"):
                P.assert_bit_exact(fused.fetch(o), unfused.fetch(o), what + " " + o)
            P.assert_bit_exact(fused.fetch("w"), env["w"], what)
            if dtype == "i32":
                P.assert_bit_exact(fused.fetch("sums"), env["sums"], what)
            else:
                err = np.abs(fused.fetch("sums").astype(np.float64) - env["sums"].astype(np.float64))
                assert np.all(err <= 1e-5 * prefix_scale(env["w"], right) + 1e-30), what


def test_row_scans():
    # scans of two-dimensional arrays run row by row; row lengths on both sides of the
    # 16-lane / wave / workgroup variants, ragged against their step, with and without a fused producer
    rng = np.random.default_rng(9)
    for (rows, w) in ((1, 5), (3, 1), (37, 16), (300, 17), (129, 64), (65, 65), (40, 1000), (9, 1024), (7, 1025),
                      (5, 5000), (2, 70001), (2051, 33)):
        g = Graph()
        g.add("x", "input", "i32", (rows, w))
        g.add("l", "scanl", "i32", (rows, w), fn="add", args=("x",), output=True)
        g.add("r", "scanr", "i32", (rows, w), fn="add", args=("x",), output=True)
        ins = {"x": rng.integers(0, 1000, size=(rows, w), dtype=np.int32)}
        env = evaluate(g, ins)
        prog = device_program(g, ins, fc().fc_partition_trivial(g))
        prog.run()
        P.assert_bit_exact(prog.fetch("l"), env["l"], f"scanl {rows}x{w}")
        P.assert_bit_exact(prog.fetch("r"), env["r"], f"scanr {rows}x{w}")
        if rows > 1:
            assert all(k.startswith("rowscan") for k in prog.kernels())
    # producer fused into the row scan: offsets of the kept elements inside every row
    g = Graph()
    g.add("v", "input", "i32", (200, 777))
    g.add("flags", "map", "i32", (200, 777), fn="mod_eq", iparam=(3, 0), args=("v",))
    g.add("offs", "scanl", "i32", (200, 777), fn="add", args=("flags",), output=True)
    ins = {"v": rng.integers(0, 2 ** 31, size=(200, 777), dtype=np.int32)}
    runs = check(g, ins, exact=("offs",), expect_clusters=1)
    assert runs["fused"].kernels() == ["rowscan[map10(in0:i32)]+offs"]


def test_greedy_bottom_up_bad_contracts_the_large_array():
    rng = np.random.default_rng(6)
    for (n, m) in ((64, 4096), (7, 130), (1000, 16), (3, 10000), (64, 65536), (5, 1000003), (2, 1 << 20)):
        g = PG.greedy_bottom_up_bad(n, m)
        # values so close to 1 that the product over a row of any length stays in range
        ins = {"xs": (1.0 + rng.uniform(-4.0, 4.0, size=n) / m).astype(F32)}
        runs = check(g, ins, folds=("result",), expect_clusters=2)
        assert runs["fused"].kernels()[0].startswith("rowfold.add.f32+mul.f32[")
        # the large array never reaches memory in the fused plan
        gi = g.index()
        part = fc().fc_plan(g, "bytes")
        assert part.fused_away[gi["large"]] == 1 and part.fused_away[gi["is"]] == 1


def test_greedy_top_down_bad():
    rng = np.random.default_rng(7)
    g = PG.greedy_top_down_bad()
    check(g, random_inputs(g, rng, {}), folds=("result",), expect_clusters=2)


def test_diagonal_cluster_two_stores():
    rng = np.random.default_rng(8)
    n = 10007
    g = Graph()
    g.add("as", "input", "f32", (n,))
    g.add("bs", "map", "f32", (n,), fn="affine", fparam=(2.0, 0.5), args=("as",), output=True)
    g.add("cs", "map", "f32", (n,), fn="affine", fparam=(-1.5, 1.0), args=("bs",), output=True)
    ins = {"as": rng.standard_normal(n).astype(F32)}
    runs = check(g, ins, exact=("bs", "cs"), expect_clusters=1)
    assert runs["fused"].kernels()[0].count("store[") == 2


def test_tuned_cost_weights():
    # section 5.1: a linear combination of cost functions with coefficients found by tuning.
    # Clusterings of three programs are timed, launch cost and inverse bandwidth fitted, and the
    # plans of the fitted cost function must run correctly and be about as fast as the best
    # clustering that was timed.
    from paper_2407_13585_amd import tune
    rng = np.random.default_rng(11)
    programs = []
    for g in (PG.single_loop(1 << 22), PG.greedy_top_down_bad(1 << 22), PG.greedy_bottom_up_bad(64, 1 << 16)):
        ins = random_inputs(g, rng, {})
        if "xs" in ins and g["xs"].shape == (64,):
            ins["xs"] = (1.0 + rng.uniform(-4.0, 4.0, size=64) / (1 << 16)).astype(F32)
        programs.append((g, ins))
    weights, samples = tune.tune(programs, reps=10)
    assert set(weights) == {"clusters", "bytes"} and all(w >= 0 for w in weights.values()) and weights["bytes"] > 0
    # between 1 and 20 TB/s, and a launch costs less than 50 us: the coefficients have their physical meaning
    assert 1e12 < 1e6 / weights["bytes"] < 2e13 and weights["clusters"] < 50.0
    for k, (g, ins) in enumerate(programs):
        part = fc().fc_plan_weighted(g, weights)
        env = evaluate(g, ins)
        prog = device_program(g, ins, part)
        prog.run()
        for name in g.outputs():
            got, ref = prog.fetch(name).astype(np.float64), np.asarray(env[name], dtype=np.float64)
            assert np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-30), name
        best = min(s["us"] for s in samples if s["program"] == k)
        assert tune.time_partition(g, ins, part, reps=10) <= 1.3 * best + 5.0
