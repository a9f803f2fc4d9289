"""Parity of the HIP path (through the C ABI) with the CPU oracle, on the GPU.

Every case runs the same seeded inputs through oracle.interp.evaluate and through
fc_run_fused / fc_run_unfused and compares element by element under the rules of
tests/parity.py.
"""
import numpy as np
import pytest

import parity as P
from oracle.interp import evaluate
from workloads import Graph, build
from workloads import configs as C

pytestmark = pytest.mark.gpu

F32 = np.float32

# comparison rule per node of the five pipelines
RULES = {
    1: {"ys": "exact", "idx": "exact", "zs": "exact", "ps": "exact", "r": "fold"},
    2: {"ys": ("ulp", 4), "zs": ("ulp", 4), "ws": ("rel", 2e-6), "r": "fold"},
    3: {"g": "exact", "p": "exact", "y": "segmented"},
    4: {"flags": "exact", "offs": "exact", "count": "exact", "out": "exact"},
    5: {"p": ("ulp", 4), "iN": "exact", "iS": "exact", "iW": "exact", "iE": "exact",
        "pN": ("ulp", 4), "pS": ("ulp", 4), "pW": ("ulp", 4), "pE": ("ulp", 4),
        "out": ("rel", 1e-6), "m": ("ulp", 4)},
}


def fc():
    import paper_2407_13585_amd as fc_
    return fc_


def device_program(*a, **kw):
    from paper_2407_13585_amd.device import DeviceProgram
    return DeviceProgram(*a, **kw)


def compare(cfg, w, env, prog, names, tag):
    for name in names:
        rule = RULES[cfg][name]
        got, ref = prog.fetch(name), env[name]
        what = f"{w.name}/{tag}/{name}"
        if rule == "exact":
            P.assert_bit_exact(got, ref, what)
        elif rule == "fold":
            P.assert_fold(got, ref, what)
        elif rule == "segmented":
            P.assert_segmented(got, ref, env["p"], w.inputs["off"], what)
        elif rule[0] == "ulp":
            P.assert_ulp(got, np.asarray(ref, dtype=np.float64).astype(F32), rule[1], what)
        elif rule[0] == "rel":
            P.assert_close(got, ref, rule[1], what)


def plan(graph, duplicate):
    if duplicate:
        graph, _ = fc().fc_duplicate(graph)
    return graph, fc().fc_plan(graph, "bytes")


def run_all_modes(cfg, w, env=None):
    env = env or evaluate(w.graph, w.inputs)
    outs = w.graph.outputs()
    results = {}
    for dup in (True, False):
        g, part = plan(w.graph, dup)
        prog = device_program(g, w.inputs, part)
        prog.run()
        compare(cfg, w, env, prog, outs, "fused-dup" if dup else "fused-strict")
        results["dup" if dup else "strict"] = {o: prog.fetch(o) for o in outs}
        assert prog.control_words()[1] == 0          # no bounded wait gave up
    inter = [n.name for n in w.graph.nodes if n.kind != "input"]
    prog = device_program(w.graph, w.inputs, None, bind=inter)
    prog.run()
    compare(cfg, w, env, prog, inter, "unfused")
    results["unfused"] = {o: prog.fetch(o) for o in outs}
    return results


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_small_configs_match_oracle(cfg):
    w = build(cfg, small=True)
    res = run_all_modes(cfg, w)
    # fusion never changes element values: stored arrays agree bit for bit across arms
    for o in w.graph.outputs():
        if RULES[cfg][o] in ("exact",) or o == "out":
            P.assert_bit_exact(res["dup"][o], res["unfused"][o], f"{w.name}: fused vs unfused {o}")
            P.assert_bit_exact(res["strict"][o], res["unfused"][o], f"{w.name}: strict vs unfused {o}")


def test_plans_have_the_expected_shape():
    k = {}
    for cfg in (1, 2, 3, 4, 5):
        w = build(cfg, small=True)
        _, strict = plan(w.graph, False)
        _, dup = plan(w.graph, True)
        k[cfg] = (strict.n_clusters, dup.n_clusters)
    # without duplication a producer read in two orders stays manifest (cfg 1, cfg 5)
    assert k == {1: (2, 1), 2: (1, 1), 3: (1, 1), 4: (1, 1), 5: (2, 1)}


# ------------------------------------------------------------------ values that are not finite
@pytest.mark.parametrize("n", [37, 70001])
def test_nonfinite_values_are_compared_by_class(n):
    # an infinity and a NaN among the inputs of fold(+), fold(max), the fp32 scans and a segmented
    # fold (+ and max), fused and one kernel per combinator.  (+) is IEEE addition, max is maxNum
    # (a NaN counts as missing): both give one result whatever the order of evaluation.
    rng = np.random.default_rng(n)
    for special in ((np.inf, np.nan), (np.inf, -np.inf), (-np.inf, None), (np.nan, None)):
        x = rng.uniform(-1.0, 1.0, n).astype(F32)
        x[n // 3] = special[0]
        if special[1] is not None:
            x[(2 * n) // 3] = special[1]
        rows = max(1, n // 9)
        cuts = np.sort(rng.integers(0, n + 1, rows - 1))
        off = np.concatenate([[0], cuts, [n]]).astype(np.int32)
        g = Graph()
        g.add("x", "input", "f32", (n,))
        g.add("off", "input", "i32", (rows + 1,))
        g.add("s", "fold", "f32", (1,), fn="add", args=("x",), output=True)
        g.add("m", "fold", "f32", (1,), fn="max", args=("x",), output=True)
        g.add("l", "scanl", "f32", (n,), fn="add", args=("x",), output=True)
        g.add("r", "scanr", "f32", (n,), fn="add", args=("x",), output=True)
        g.add("ys", "foldseg", "f32", (rows,), fn="add", args=("x", "off"), output=True)
        g.add("ym", "foldseg", "f32", (rows,), fn="max", args=("x", "off"), output=True)
        ins = {"x": x, "off": off}
        with np.errstate(all="ignore"):
            env = evaluate(g, ins)
        assert not np.all(np.isfinite(env["l"])) and not np.isfinite(env["s"][0])      # the case is not vacuous
        finite_abs = np.where(np.isfinite(x), np.abs(x), F32(0)).astype(np.float64)
        for tag, part in (("fused", fc().fc_plan(g, "bytes", executable=True)), ("unfused", None)):
            prog = device_program(g, ins, part)
            prog.run()
            what = f"n={n} special={special} {tag}"
            P.assert_fold(prog.fetch("s"), env["s"], what + " fold(+)")
            P.assert_bit_exact(prog.fetch("m"), env["m"].astype(F32), what + " fold(max)")
            P.assert_bit_exact(prog.fetch("ym"), env["ym"].astype(F32), what + " foldSeg(max)")
            P.assert_segmented(prog.fetch("ys"), env["ys"], x, off, what + " foldSeg(+)")
            for name, scale in (("l", np.concatenate([[0.0], np.cumsum(finite_abs)[:-1]])),
                                ("r", np.concatenate([np.cumsum(finite_abs[::-1])[::-1][1:], [0.0]]))):
                got, ref = prog.fetch(name), env[name]
                finite = P.same_class(got, ref, what + " scan " + name)
                err = np.abs(np.where(finite, got, 0).astype(np.float64) - np.where(finite, ref, 0).astype(np.float64))
                assert np.all(err <= 1e-5 * scale + 1e-30), what + " scan " + name
            assert prog.control_words()[1] == 0


# ------------------------------------------------------------------ ragged sizes, tiles, edges
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 255, 4095, 4096, 4097, 8191, 12289, 1 << 20,
                               # tile counts around the groups of 16 the mirrored tile order forms
                               16 * 4096, 17 * 4096 + 4, 33 * 4096 + 3, 38 * 4096 + 2052, 2100 * 4096 + 8])
def test_fold_sizes(n):
    w = C.reverse_dot(n=n, seed=100 + n)
    run_all_modes(1, w)
    w = C.perm_gather_fold(n=n, seed=200 + n)
    run_all_modes(2, w)


@pytest.mark.parametrize("n", [1, 3, 4, 4095, 4096, 4097, 65536 + 17, 3 * 4096, (1 << 20) + 5])
def test_compaction_sizes(n):
    run_all_modes(4, C.compaction(n=n, seed=300 + n))


def test_compaction_degenerate_flags():
    n = 50000
    for v in (np.zeros(n, np.int32) + 3, np.zeros(n, np.int32) + 1, np.arange(n, dtype=np.int32)):
        run_all_modes(4, C.compaction(v=v))


@pytest.mark.parametrize("modulus,residue", [(1, 0), (2, 0), (2, 1), (3, 2), (4, 3), (6, 0), (6, 4), (7, 6), (12, 8),
                                             (1000, 999), (65536, 123), (3 << 20, 5), (2 ** 31 - 1, 17), (5, 5), (5, 9)])
def test_compaction_moduli(modulus, residue):
    # the predicate is evaluated without a division (even and odd moduli, powers of two, a
    # residue outside [0, modulus) that matches nothing); kept fractions from all to none
    # cross the size of the buffer that holds a tile's kept elements
    rng = np.random.default_rng(400 + modulus % 1000 + residue)
    n = 70001
    v = rng.integers(0, 2 ** 31, size=n, dtype=np.int32)
    v[: n // 3] = (v[: n // 3] // modulus) * modulus + residue if residue < modulus else v[: n // 3]
    v = np.abs(v.astype(np.int64)) % (2 ** 31)
    v[:8] = [0, 1, 2, 2 ** 31 - 1, 2 ** 31 - 2, modulus % 2 ** 31, max(residue, 0) % 2 ** 31, 3]
    run_all_modes(4, C.compaction(v=v.astype(np.int32), modulus=modulus, residue=residue))


def test_empty_inputs():
    w = C.reverse_dot(xs=np.zeros(0, F32))
    env = evaluate(w.graph, w.inputs)
    for part in (plan(w.graph, True), (w.graph, None)):
        prog = device_program(part[0], w.inputs, part[1])
        prog.run()
        assert prog.fetch("r")[0] == 0.0 == env["r"][0]
    w = C.compaction(v=np.zeros(0, np.int32))
    g, part = plan(w.graph, True)
    prog = device_program(g, w.inputs, part)
    prog.run()
    assert prog.fetch("count")[0] == 0
    w = C.spmv(lengths=np.zeros(0, np.int64), ncols=4, seed=1)
    g, part = plan(w.graph, True)
    prog = device_program(g, w.inputs, part)
    prog.run()
    assert prog.fetch("y").shape == (0,)


@pytest.mark.parametrize("lengths", [
    [0, 0, 0], [1], [5000], [0, 17, 0, 16, 15, 33, 1, 0], [16] * 1000, [0] * 100 + [3] + [0] * 100,
    list(range(0, 70)), [100000, 0, 1, 0, 100000],
])
def test_spmv_row_shapes(lengths):
    lengths = np.asarray(lengths, dtype=np.int64)
    w = C.spmv(lengths=lengths, seed=int(lengths.sum()) % 1000 + 400, ncols=max(int(lengths.max()), 8))
    run_all_modes(3, w)


def test_spmv_skewed_rows():
    rng = np.random.default_rng(77)
    lengths = np.minimum(rng.zipf(1.5, size=5000), 20000).astype(np.int64)
    run_all_modes(3, C.spmv(lengths=lengths, seed=78, ncols=5000))


@pytest.mark.parametrize("rows,ncols,mean_len", [(20000, 1200000, 8.0), (16384 + 77, (1 << 22) - 5, 5.0),
                                                  (70001, 3000001, 3.0)])
def test_spmv_column_blocked(rows, ncols, mean_len):
    # a gathered table of more than one and at most four L2s takes the column-blocked kernel:
    # four workgroups per unit of 256 rows, partial row sums handed over through memory.
    # Row counts off the unit size, empty rows, a table that is not a multiple of the range.
    rng = np.random.default_rng(rows)
    lengths = rng.poisson(mean_len, size=rows)
    lengths[rng.integers(0, rows, size=rows // 50)] = 0
    lengths[rng.integers(0, rows, size=20)] = 3000            # a few long rows
    w = C.spmv(lengths=lengths, seed=rows + 1, ncols=ncols)
    env = evaluate(w.graph, w.inputs)
    g, part = plan(w.graph, False)
    prog = device_program(g, w.inputs, part)
    assert "column-blocked" in prog.kernels()[0], prog.kernels()
    for k in range(3):                                        # flags and workspace are reused launch after launch
        if k:
            # other values every time: a partial row sum left over from the launch before
            # would now be a wrong one
            w.inputs["vals"] = rng.uniform(-1.0, 1.0, size=w.inputs["vals"].shape).astype(F32)
            w.inputs["x"] = rng.uniform(-1.0, 1.0, size=w.inputs["x"].shape).astype(F32)
            prog.upload("vals", w.inputs["vals"])
            prog.upload("x", w.inputs["x"])
            env = evaluate(w.graph, w.inputs)
        prog.run()
        compare(3, w, env, prog, w.graph.outputs(), "column-blocked")
        assert prog.control_words()[1] == 0
    run_all_modes(3, w, env)


@pytest.mark.parametrize("shape", ["uniform", "crowded", "long rows", "empty ends", "one column", "many ranges"])
def test_spmv_sorted_through_lds(shape):
    # from four million elements on, over a table that no L2 holds, the segmented fold sorts its elements by
    # table range, gathers from LDS and puts the values back in place (four kernels, everything between
    # them in scratch).  Columns spread evenly, columns that crowd into few ranges or one (slots overflow:
    # those elements go through the tiles' lists), rows longer than several tiles, rows that end exactly
    # on a tile boundary, runs of empty rows at both ends and around tile boundaries, a table that is cut
    # into many short ranges, element counts off the tile and off the 128-bit group.
    rng = np.random.default_rng(len(shape) * 1000 + 7)
    rows, ncols = 300001, 1500007
    lengths = rng.poisson(16.0, size=rows).astype(np.int64)
    if shape == "long rows":
        lengths[rng.integers(0, rows, size=6)] = 40000
        lengths[:1024] = 16                                   # row 1024 starts on a tile boundary ...
        lengths[1024] = 16384 * 3
        lengths[1025:1035] = 0                                # ... ends on one, and empty rows follow
    elif shape == "empty ends":
        lengths[:5000] = 0
        lengths[-7000:] = 0
        lengths[60000:90000] = 0
        lengths[30000:30100] = 2000
    elif shape == "many ranges":
        ncols = (1 << 24) - 3
    w = C.spmv(lengths=lengths, seed=11, ncols=ncols)
    nnz = w.inputs["col"].shape[0]
    assert nnz >= 1 << 22
    if shape == "crowded":
        w.inputs["col"] = np.where(rng.random(nnz) < 0.9, rng.integers(0, 3000, size=nnz), rng.integers(0, ncols, size=nnz)).astype(np.int32)
    elif shape == "one column":
        w.inputs["col"] = np.full(nnz, ncols - 1, dtype=np.int32)
    env = evaluate(w.graph, w.inputs)
    g, part = plan(w.graph, False)
    prog = device_program(g, w.inputs, part)
    assert "sorted through LDS" in prog.kernels()[0], prog.kernels()
    for k in range(2):                                        # the scratch arrays are rewritten launch after launch
        if k:
            w.inputs["vals"] = rng.uniform(-1.0, 1.0, size=nnz).astype(F32)
            w.inputs["x"] = rng.uniform(-1.0, 1.0, size=ncols).astype(F32)
            w.inputs["col"] = np.ascontiguousarray(w.inputs["col"][::-1])
            for name in ("vals", "x", "col"):
                prog.upload(name, w.inputs[name])
            env = evaluate(w.graph, w.inputs)
        prog.run()
        compare(3, w, env, prog, w.graph.outputs(), "sorted")
        assert prog.control_words()[1] == 0
        first = prog.fetch("y").copy()
        prog.run()                                            # every sum has a fixed order: the same bits again
        P.assert_bit_exact(prog.fetch("y"), first, "sorted: second launch")
    run_all_modes(3, w, env)


@pytest.mark.parametrize("table,m,spread", [(2200003, 2200003, "permutation"), (3000000, (1 << 21) + 4099, "uniform"),
                                            (2000001, (1 << 21) + 8197, "skewed"), (1 << 22, (1 << 21) + 2, "one"),
                                            (3000017, (1 << 21) + 77, "middle")])
def test_perm_gather_binned(table, m, spread):
    # a fold over a gather from a table of more than one L2 sorts the indices by table range
    # first (two kernels, the entries in scratch).  A permutation, repeated indices, indices
    # that crowd into one range or one position (more than a slot takes: the remainder is
    # evaluated on the spot), lengths off the tile and off the 128-bit group.
    rng = np.random.default_rng(table + m)
    xs = rng.standard_normal(size=table).astype(F32)
    if spread == "permutation":
        idx = rng.permutation(table).astype(np.int32)
    elif spread == "uniform":
        idx = rng.integers(0, table, size=m, dtype=np.int32)
    elif spread == "skewed":
        idx = np.where(rng.random(m) < 0.9, rng.integers(0, 5000, size=m), rng.integers(0, table, size=m)).astype(np.int32)
    elif spread == "middle":
        idx = np.where(rng.random(m) < 0.7, rng.integers(table // 2, table // 2 + 70000, size=m),
                       rng.integers(0, table, size=m)).astype(np.int32)
    else:
        idx = np.full(m, table - 1, dtype=np.int32)
    w = C.perm_gather_fold(xs=xs, idx=idx)
    env = evaluate(w.graph, w.inputs)
    g, part = plan(w.graph, False)
    prog = device_program(g, w.inputs, part)
    assert "binned" in prog.kernels()[0], prog.kernels()
    for k in range(3):                                        # counts and entries are rewritten launch after launch
        if k:
            w.inputs["xs"] = rng.standard_normal(size=table).astype(F32)
            w.inputs["idx"] = np.ascontiguousarray(w.inputs["idx"][::-1])
            prog.upload("xs", w.inputs["xs"])
            prog.upload("idx", w.inputs["idx"])
            env = evaluate(w.graph, w.inputs)
        prog.run()
        compare(2, w, env, prog, w.graph.outputs(), "binned")
        assert prog.control_words()[1] == 0
        first = prog.fetch("r").copy()
        prog.run()                                            # every sum has a fixed order: the same bits again
        P.assert_bit_exact(prog.fetch("r"), first, "binned: second launch")
    run_all_modes(2, w, env)


def test_single_pass_flag_keeps_the_gathers_in_position_order():
    # FC_NODE_SINGLE_PASS on the fold: the cluster runs as one pass with every gather issued at the
    # position that asks for it, also where the library would by default sort the indices by table
    # range (fold) or read the streams once per column range (segmented fold).  Same oracle, same bounds.
    from workloads import single_pass
    rng = np.random.default_rng(91)
    table, m = 3000017, (1 << 21) + 77
    w = C.perm_gather_fold(xs=rng.standard_normal(size=table).astype(F32), idx=rng.integers(0, table, size=m, dtype=np.int32))
    env = evaluate(w.graph, w.inputs)
    for marked, variant in ((False, "binned"), (True, None)):
        g = single_pass(w.graph) if marked else w.graph
        g, part = plan(g, False)
        prog = device_program(g, w.inputs, part)
        assert (variant in prog.kernels()[0]) if variant else ("{" not in prog.kernels()[0]), prog.kernels()
        prog.run()
        compare(2, w, env, prog, w.graph.outputs(), "single-pass" if marked else "default")
    lengths = rng.poisson(6.0, size=40000)
    w = C.spmv(lengths=lengths, seed=92, ncols=2500000)
    env = evaluate(w.graph, w.inputs)
    for marked, variant in ((False, "column-blocked"), (True, None)):
        g = single_pass(w.graph) if marked else w.graph
        g, part = plan(g, True)                               # the flag survives the duplication rewrite
        prog = device_program(g, w.inputs, part)
        assert (variant in prog.kernels()[0]) if variant else ("{" not in prog.kernels()[0]), prog.kernels()
        prog.run()
        compare(3, w, env, prog, w.graph.outputs(), "single-pass" if marked else "default")


@pytest.mark.parametrize("table,m", [(1048600, 1 << 21), ((1 << 24), (1 << 21) + 8192), (5000000, (1 << 21) + 4096),
                                     (1234567, (1 << 21) + 4100), ((1 << 25) + 5, (1 << 21) + 1),
                                     ((1 << 24) - 12345, (1 << 23) + 4100), ((1 << 24), (1 << 23) + 32768 + 3),
                                     (9000001, 4500001)])
def test_perm_gather_binned_sizes(table, m):
    # table sizes just above one L2, at 64 MiB and beyond (ranges larger than half an L2); position counts that
    # are whole tiles, whole passes, and a pass with four elements in it.  Tables of up to 2^24 elements with
    # at least half as many positions take the kernels that keep a table range in LDS (ranges of a power of
    # two and of any other length, a last range that is shorter, a last tile that is all but empty).
    rng = np.random.default_rng(table ^ m)
    w = C.perm_gather_fold(xs=rng.standard_normal(size=table).astype(F32), idx=rng.integers(0, table, size=m, dtype=np.int32))
    env = evaluate(w.graph, w.inputs)
    g, part = plan(w.graph, False)
    prog = device_program(g, w.inputs, part)
    assert "binned" in prog.kernels()[0], prog.kernels()
    assert ("LDS" in prog.kernels()[0]) == (table <= 1 << 24 and 2 * m >= table), prog.kernels()
    prog.run()
    compare(2, w, env, prog, w.graph.outputs(), "binned")
    assert prog.control_words()[1] == 0


@pytest.mark.parametrize("hw", [(1, 4), (1, 8), (2, 4), (3, 3), (1, 1), (5, 7), (33, 248), (34, 252), (64, 256),
                                (65, 1000), (7, 1004), (100, 2048), (31, 996)])
def test_stencil_shapes(hw):
    run_all_modes(5, C.stencil_max(h=hw[0], w=hw[1], seed=500 + hw[0] * 7 + hw[1]))


def test_stencil_constant_grid_borders():
    w = C.stencil_max(grid=np.full((40, 500), F32(0.25)))
    res = run_all_modes(5, w)
    assert np.all(res["dup"]["out"] == res["dup"]["out"][0, 0])


# ------------------------------------------------------------------ scratch reuse
def test_repeated_runs_share_scratch():
    for cfg in (2, 4, 5):
        w = build(cfg, small=True)
        env = evaluate(w.graph, w.inputs)
        g, part = plan(w.graph, True)
        prog = device_program(g, w.inputs, part)
        for rep in range(4):
            if cfg == 4:
                prog.upload("dest", w.inputs["dest"])
            prog.run()
            compare(cfg, w, env, prog, w.graph.outputs(), f"rep{rep}")
        words = prog.control_words()
        assert words[1] == 0
        assert words[0] == 4            # one tagged launch per run


def test_two_streams_each_with_its_own_scratch():
    # launches that overlap in time must not share a scratch buffer; with one each they may: two streams
    # (default priority) with two and three programs, whose kernels wait for other workgroups
    import torch
    rng = np.random.default_rng(79)
    big = 2200003
    items = [(4, C.compaction(n=3000001, seed=9)),
             (3, C.spmv(lengths=rng.poisson(8.0, size=20000), seed=6, ncols=1200000)),
             (2, C.perm_gather_fold(xs=rng.standard_normal(size=big).astype(F32), idx=rng.permutation(big).astype(np.int32))),
             (5, build(5, small=True)),
             # a second column-blocked fold, on the other stream than the first: two launches whose workgroups wait for partners
             (3, C.spmv(lengths=rng.poisson(12.0, size=60000), seed=7, ncols=1500000))]
    progs = []
    for cfg, w in items:
        g, part = plan(w.graph, True)
        progs.append(device_program(g, w.inputs, part))
    assert "column-blocked" in progs[1].kernels()[0] and "column-blocked" in progs[4].kernels()[0]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(6):
        for k, p in enumerate(progs):
            p.run(streams[k % 2])                 # a program (and its scratch buffer) stays on one stream
    torch.cuda.synchronize()
    for (cfg, w), p in zip(items, progs):
        compare(cfg, w, evaluate(w.graph, w.inputs), p, w.graph.outputs(), "two streams")
        words = p.control_words()
        assert words[1] == 0 and words[0] >= 6


def test_step_replays_from_a_hip_graph():
    # fc_run_fused only enqueues kernels (no allocation, no host synchronisation, no memset), so a
    # caller can capture a step into a HIP graph.  Captured here: the five pipelines at small sizes
    # plus the two kernels that hand data over through scratch (column-blocked SpMV, fold over sorted
    # gather indices).  Every replay runs on other input values, with eager copies and
    # synchronisations in between, and is checked against the oracle.
    import torch
    rng = np.random.default_rng(77)
    items = []
    for cfg in (1, 2, 3, 4, 5):
        items.append((cfg, build(cfg, small=True), True))
    lengths = rng.poisson(8.0, size=20000)
    items.append((3, C.spmv(lengths=lengths, seed=5, ncols=1200000), False))
    big = 2200003
    items.append((2, C.perm_gather_fold(xs=rng.standard_normal(size=big).astype(F32), idx=rng.permutation(big).astype(np.int32)), False))
    progs = []
    for cfg, w, dup in items:
        g, part = plan(w.graph, dup)
        progs.append(device_program(g, w.inputs, part))
    assert "column-blocked" in progs[5].kernels()[0] and "binned" in progs[6].kernels()[0]
    for p in progs:                                           # first launches outside the capture
        p.run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        for p in progs:
            p.run()
    for rep in range(3):
        for (cfg, w, dup), p in zip(items, progs):
            for name, a in list(w.inputs.items()):
                if a.dtype == F32:                            # other values every time
                    w.inputs[name] = (a * F32(0.5) + rng.uniform(-0.1, 0.1, size=a.shape).astype(F32)).astype(F32)
                p.upload(name, w.inputs[name])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (cfg, w, dup), p in zip(items, progs):
            env = evaluate(w.graph, w.inputs)
            compare(cfg, w, env, p, w.graph.outputs(), f"replay{rep}")
            assert p.control_words()[1] == 0


def test_fusion_rule_clusters_execute():
    """`simple1`, `simple2`, reverse and a diagonal cluster, each as one kernel."""
    rng = np.random.default_rng(9)
    n, m = 5003, 3001
    xs = rng.standard_normal(n).astype(F32)
    is1 = rng.integers(0, n, m, dtype=np.int32)
    is2 = rng.integers(0, m, 777, dtype=np.int32)
    g = Graph()
    g.add("xs", "input", "f32", (n,))
    g.add("is", "input", "i32", (m,))
    g.add("as", "map", "f32", (n,), fn="affine", fparam=(3.0, -0.5), args=("xs",))
    g.add("bs", "gather", "f32", (m,), args=("is", "as"), output=True)
    part = fc().fc_plan(g, "bytes")
    assert part.n_clusters == 1 and part.fused_away[2] == 1
    prog = device_program(g, {"xs": xs, "is": is1}, part)
    prog.run()
    P.assert_bit_exact(prog.fetch("bs"), evaluate(g, {"xs": xs, "is": is1})["bs"], "simple1")

    g = Graph()
    g.add("is1", "input", "i32", (m,))
    g.add("is2", "input", "i32", (777,))
    g.add("xs", "input", "f32", (n,))
    g.add("as", "gather", "f32", (m,), args=("is1", "xs"))
    g.add("bs", "gather", "f32", (777,), args=("is2", "as"), output=True)
    part = fc().fc_plan(g, "bytes")
    assert part.n_clusters == 1
    ins = {"xs": xs, "is1": is1, "is2": is2}
    prog = device_program(g, ins, part)
    prog.run()
    P.assert_bit_exact(prog.fetch("bs"), evaluate(g, ins)["bs"], "simple2")


# ------------------------------------------------------------------ the largest arrays the library takes
@pytest.mark.timeout(900)
def test_arrays_of_two_to_the_31_minus_one_elements():
    # The inputs repeat a seeded block, less the very last element (a ragged tail of three): what the oracle
    # computes on one block then fixes every output of the whole array -- the kept elements repeat, the
    # offsets of repetition k are the block's plus k times its count, a sum is the block's times the repetitions.
    B, reps = 1 << 24, 128
    n = B * reps - 1
    rng = np.random.default_rng(77)

    block = rng.integers(0, 2 ** 31, size=B, dtype=np.int32)
    wb = C.compaction(v=block)
    eb = evaluate(wb.graph, wb.inputs)
    count_b = int(eb["count"][0])
    kept_b = eb["out"][:count_b]
    count = reps * count_b - int(eb["flags"][B - 1])
    g = Graph()
    g.add("v", "input", "i32", (n,))
    g.add("dest", "input", "i32", (n,))
    g.add("flags", "map", "i32", (n,), fn="mod_eq", iparam=(3, 0), args=("v",))
    g.add("offs", "scanl", "i32", (n,), fn="add", args=("flags",))
    g.add("count", "fold", "i32", (1,), fn="add", args=("flags",), output=True)
    g.add("out", "scatter", "i32", (n,), fn="overwrite", args=("dest", "offs", "v", "flags"), output=True)
    ins = {"v": np.tile(block, reps)[:n], "dest": np.full(n, -1, np.int32)}
    want_out = np.full(n, -1, np.int32)
    want_out[:count] = np.tile(kept_b, reps)[:count]
    want_offs = (eb["offs"][None, :] + (np.arange(reps, dtype=np.int32) * np.int32(count_b))[:, None]).reshape(-1)[:n]
    for fused in (True, False):
        part = fc().fc_plan(g, "bytes") if fused else None
        prog = device_program(g, ins, part, bind=() if fused else ["flags", "offs"])
        prog.run()
        what = "fused" if fused else "unfused"
        assert int(prog.fetch("count")[0]) == count, what
        P.assert_bit_exact(prog.fetch("out"), want_out, what + " out")
        if not fused:
            P.assert_bit_exact(prog.fetch("offs"), want_offs, "offs")
        assert prog.control_words()[1] == 0
        del prog
    del ins, want_out, want_offs

    # reversed dot product: position i meets position n-1-i, which lies B-2-i (mod B) into the block
    xb = rng.uniform(-1.0, 1.0, size=B).astype(F32)
    gb = Graph()
    gb.add("xs", "input", "f32", (B,))
    gb.add("idx", "input", "i32", (B,))
    gb.add("ys", "map", "f32", (B,), fn="affine", fparam=(2.0, 1.0), args=("xs",))
    gb.add("zs", "gather", "f32", (B,), args=("idx", "ys"))
    gb.add("ps", "map", "f32", (B,), fn="mul2", args=("ys", "zs"))
    gb.add("r", "fold", "f32", (1,), fn="add", args=("ps",), output=True)
    eb = evaluate(gb, {"xs": xb, "idx": ((B - 2 - np.arange(B)) % B).astype(np.int32)})
    last = float(eb["ys"][B - 1])
    want = reps * float(eb["r"][0]) - last * last        # the missing position would have met itself
    w = C.reverse_dot(xs=np.tile(xb, reps)[:n])
    for dup in (True, False):
        gg, part = plan(w.graph, dup)
        prog = device_program(gg, w.inputs, part)
        prog.run()
        P.assert_fold(prog.fetch("r"), np.array([want]), "reversed dot product at 2^31-1")
        assert prog.control_words()[1] == 0
        del prog


@pytest.mark.timeout(900)
def test_segments_that_end_at_two_to_the_31_minus_one():
    # 2^27 rows over 2^31 - 1 elements: a block of 2^20 rows with exactly 2^24 elements, repeated; the last
    # row is one element short.  A row's sum takes its terms in an order that depends on the row alone, so
    # every repetition must give the bits of the first, and the first is compared with the oracle.
    Rb, reps, ncols = 1 << 20, 128, 1 << 20
    rng = np.random.default_rng(78)
    lengths = rng.poisson(16.0, size=Rb).astype(np.int64)
    diff = (1 << 24) - int(lengths.sum())
    rows_to_change = np.flatnonzero(lengths > 1)[:abs(diff)]
    lengths[rows_to_change] += 1 if diff > 0 else -1
    lengths[-1] = max(lengths[-1], 2); lengths[0] += (1 << 24) - int(lengths.sum())
    assert lengths.sum() == 1 << 24 and lengths.min() >= 0
    def graph_of(nnz, rows):
        g = Graph()
        g.add("x", "input", "f32", (ncols,))
        g.add("col", "input", "i32", (nnz,))
        g.add("vals", "input", "f32", (nnz,))
        g.add("off", "input", "i32", (rows + 1,))
        g.add("g", "gather", "f32", (nnz,), args=("col", "x"))
        g.add("p", "map", "f32", (nnz,), fn="mul2", args=("vals", "g"))
        g.add("y", "foldseg", "f32", (rows,), fn="add", args=("p", "off"), output=True)
        return g

    wb = C.spmv(lengths=lengths, ncols=ncols, seed=78)
    eb = evaluate(wb.graph, wb.inputs)
    # the block with its last row one element short
    off_s = wb.inputs["off"].copy(); off_s[-1] -= 1
    es = evaluate(graph_of((1 << 24) - 1, Rb), {"x": wb.inputs["x"], "col": wb.inputs["col"][:-1],
                                               "vals": wb.inputs["vals"][:-1], "off": off_s})

    nnz, rows = (1 << 31) - 1, Rb * reps
    off = (wb.inputs["off"][None, :-1].astype(np.int64) + (np.arange(reps, dtype=np.int64) << 24)[:, None]).reshape(-1)
    off = np.append(off, nnz).astype(np.int32)
    ins = {"x": wb.inputs["x"], "col": np.tile(wb.inputs["col"], reps)[:nnz], "vals": np.tile(wb.inputs["vals"], reps)[:nnz],
           "off": off}
    g = graph_of(nnz, rows)
    for fused in (True, False):
        prog = device_program(g, ins, fc().fc_plan(g, "bytes") if fused else None)
        prog.run()
        y = prog.fetch("y").reshape(reps, Rb)
        what = "fused" if fused else "unfused"
        P.assert_segmented(y[0], eb["y"], eb["p"], wb.inputs["off"], what + " first repetition")
        assert np.array_equal(y[1:-1].view(np.int32), np.broadcast_to(y[0].view(np.int32), (reps - 2, Rb))), what
        assert np.array_equal(y[-1, :-1].view(np.int32), y[0, :-1].view(np.int32)), what
        P.assert_segmented(y[-1, -1:], es["y"][-1:], es["p"][off_s[-2]:], np.array([0, off_s[-1] - off_s[-2]]), what + " last row")
        del prog


# ------------------------------------------------------------------ full sizes (the launch shapes the bench times)
@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_configs_match_oracle(cfg):
    w = build(cfg)
    env = evaluate(w.graph, w.inputs)
    g, part = plan(w.graph, True)
    prog = device_program(g, w.inputs, part)
    prog.run()
    compare(cfg, w, env, prog, w.graph.outputs(), "full-fused")
    del prog
    prog = device_program(w.graph, w.inputs, None)
    prog.run()
    compare(cfg, w, env, prog, w.graph.outputs(), "full-unfused")
