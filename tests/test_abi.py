"""The C ABI: every function include/fc.h declares is exported, and the host-side checks
reject bad input with the documented error codes before any device work is enqueued."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

import paper_2407_13585_amd as fc
from paper_2407_13585_amd import binding as B
from workloads import Graph, build
from workloads import paper_graphs as PG

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"fc_plan", "fc_run_fused", "fc_run_unfused", "fc_last_error"} <= set(names)
    lib = B.lib()
    for name in names:
        assert hasattr(lib, name), name


def test_header_is_plain_c_and_struct_layout_matches_the_binding(tmp_path):
    # fc.h must compile as C; the sizes and a few offsets gcc gives its PODs must equal ctypes' layout
    src = tmp_path / "layout.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "fc.h"\n'
        'int main(void){printf("%zu %zu %zu %zu %zu %zu %zu\\n", sizeof(fc_node), sizeof(fc_buffer), sizeof(fc_graph),'
        ' sizeof(fc_partition), offsetof(fc_node, shape), offsetof(fc_node, infusible_args),'
        ' offsetof(fc_partition, cost)); return 0;}\n')
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = [int(x) for x in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    assert got == [ctypes.sizeof(B.fc_node), ctypes.sizeof(B.fc_buffer), ctypes.sizeof(B.fc_graph),
                   ctypes.sizeof(B.fc_partition), B.fc_node.shape.offset, B.fc_node.infusible_args.offset,
                   B.fc_partition.cost.offset]


def expect(code, fn, *a, **kw):
    with pytest.raises(fc.FcError) as e:
        fn(*a, **kw)
    assert e.value.name == code, str(e.value)
    return str(e.value)


def test_bad_graphs_are_rejected():
    g = Graph()
    g.add("a", "input", "f32", (8,))
    g.add("b", "input", "f32", (9,))
    g.add("c", "map", "f32", (8,), fn="add2", args=("a", "b"))        # zipWith of unequal sizes
    expect("FC_E_BADGRAPH", fc.fc_plan, g)
    g = Graph()
    g.add("a", "input", "f32", (8,))
    g.add("i", "input", "f32", (8,))
    g.add("c", "gather", "f32", (8,), args=("i", "a"))                # float indices
    expect("FC_E_BADGRAPH", fc.fc_plan, g)
    g = Graph()
    g.add("a", "input", "f32", (8,))
    g.add("c", "map", "f32", (8,), fn="mul2", args=("a",))            # arity
    expect("FC_E_BADGRAPH", fc.fc_plan, g)
    g = Graph()
    g.add("a", "input", "i32", (8,))
    g.add("o", "input", "i32", (3,))
    g.add("y", "foldseg", "i32", (3,), fn="add", args=("a", "o"))     # offsets need rows + 1 entries
    expect("FC_E_BADGRAPH", fc.fc_plan, g)


def test_run_checks_come_before_any_launch():
    w = build(2, small=True)
    g = w.graph
    part = fc.fc_plan(g, "bytes")
    fake = (0x10000000, 1 << 30)          # never dereferenced: every call below fails validation first
    bufs = {n.name: fake for n in g.nodes if n.kind == "input" or n.output}
    expect("FC_E_SCRATCH", fc.fc_run_fused, g, part, bufs, (0, 0))
    expect("FC_E_SCRATCH", fc.fc_run_fused, g, part, bufs, (0x10000001, 1 << 30))
    expect("FC_E_SCRATCH", fc.fc_run_fused, g, part, bufs, (0x10000000, 1024))
    missing = dict(bufs)
    del missing["idx"]
    expect("FC_E_UNBOUND", fc.fc_run_fused, g, part, missing, fake)
    small = dict(bufs, xs=(0x10000000, 16))
    expect("FC_E_UNBOUND", fc.fc_run_fused, g, part, small, fake)
    odd = dict(bufs, xs=(0x10000004, 1 << 30))
    expect("FC_E_UNBOUND", fc.fc_run_fused, g, part, odd, fake)
    bad = fc.Partition(part.pi.copy(), part.fused_away, part.order_out, part.edge_unfused)
    bad.pi[2] = 5                          # ys after its consumer
    expect("FC_E_ILLEGAL_PARTITION", fc.fc_run_fused, g, bad, bufs, fake)
    # unfused needs room for every intermediate
    expect("FC_E_SCRATCH", fc.fc_run_unfused, g, bufs, (0x10000000, B.FC_SCRATCH_CONTROL_BYTES))


def test_scatter_that_reads_its_destination_is_refused():
    # the destination is updated in place; a scatter that took its values (or indices, or flags)
    # from the same array would read what it is overwriting
    g = Graph()
    g.add("d", "input", "i32", (16,))
    g.add("i", "input", "i32", (16,))
    g.add("h", "scatter", "i32", (16,), fn="add", args=("d", "i", "d"), output=True)
    expect("FC_E_BADGRAPH", fc.fc_plan, g, "bytes")
    g = Graph()
    g.add("d", "input", "i32", (16,))
    g.add("v", "input", "i32", (16,))
    g.add("h", "scatter", "i32", (16,), fn="overwrite", args=("d", "d", "v"), output=True)
    expect("FC_E_BADGRAPH", fc.fc_plan, g, "bytes")


def test_unsupported_cluster_is_reported_not_executed():
    # a legal clustering with a cluster no kernel is built for: prefix sums and the total of a computed fp32 array
    g = Graph()
    g.add("x", "input", "f32", (64,))
    g.add("y", "map", "f32", (64,), fn="affine", fparam=(2.0, 1.0), args=("x",))
    g.add("l", "scanl", "f32", (64,), fn="add", args=("y",), output=True)
    g.add("t", "fold", "f32", (1,), fn="add", args=("y",), output=True)
    part = fc.fc_plan(g, "bytes")
    assert part.n_clusters == 1
    msg = expect("FC_E_UNSUPPORTED", fc.fc_cluster_kernel, g, part, 0)
    assert "scan of f32" in msg
    fake = (0x10000000, 1 << 30)
    bufs = {n.name: fake for n in g.nodes}
    expect("FC_E_UNSUPPORTED", fc.fc_run_fused, g, part, bufs, fake)


def test_elementwise_cluster_without_a_compiled_kernel_is_interpreted():
    # maps, generates and gathers ending in stored arrays and at most one fold always run: the
    # element programs travel as code when no compiled instance has their shape
    g = Graph()
    g.add("a", "input", "f32", (64,))
    g.add("b", "input", "f32", (64,))
    g.add("ea", "map", "f32", (64,), fn="exp_neg", args=("a",))
    g.add("sb", "map", "f32", (64,), fn="sin_x_mul_x", args=("b",))
    g.add("out", "map", "f32", (64,), fn="mul2", args=("ea", "sb"), output=True)
    part = fc.fc_plan(g, "bytes")
    assert part.n_clusters == 1
    assert fc.fc_cluster_kernel(g, part, 0) == "store[map5(map9(in0:f32),map3(in1:f32))] {interpreted}"
    # a program of the benchmark keeps its compiled kernel
    w = build(2, small=True)
    assert "interpreted" not in fc.fc_cluster_kernel(w.graph, fc.fc_plan(w.graph, "bytes"), 0)
    # too deep for the interpreter's stack of gathers: four gathers inside one another
    g = Graph()
    g.add("x", "input", "f32", (64,))
    prev = "x"
    for k in range(4):
        g.add(f"i{k}", "input", "i32", (64,))
        g.add(f"g{k}", "gather", "f32", (64,), args=(f"i{k}", prev), output=(k == 3))
        prev = f"g{k}"
    pi = [0, 0, 1, 0, 1, 0, 1, 0, 1]
    part = fc.fc_partition_check(g, pi)
    expect("FC_E_UNSUPPORTED", fc.fc_cluster_kernel, g, part, 0)


def test_scratch_bytes_and_kernel_names():
    w = build(5, small=True)
    g2, _ = fc.fc_duplicate(w.graph)
    part = fc.fc_plan(g2, "bytes")
    fused = fc.fc_scratch_bytes(g2, part)
    unfused = fc.fc_scratch_bytes(w.graph, None)
    pts = w.units
    assert fused >= B.FC_SCRATCH_CONTROL_BYTES and unfused >= B.FC_SCRATCH_CONTROL_BYTES + 10 * 4 * pts
    name = fc.fc_cluster_kernel(g2, part, 0)
    assert name.startswith("store[") and "fold.max.f32" in name
    assert fc.fc_num_edges(w.graph) == len(w.graph.edges())
    trivial = fc.fc_partition_trivial(w.graph)
    assert trivial.n_clusters == len([n for n in w.graph.nodes if n.kind != "input"])
    assert not trivial.fused_away.any()


def test_workspace_of_the_column_blocked_segmented_fold_is_part_of_scratch():
    # graph only, no data: an SpMV-shaped cluster over a 6 MiB table takes the column-blocked
    # kernel, which hands partial row sums over through 32 bytes of scratch per row
    rows, ncols, nnz = 100000, 1500000, 800000
    g = Graph()
    g.add("x", "input", "f32", (ncols,))
    g.add("col", "input", "i32", (nnz,))
    g.add("vals", "input", "f32", (nnz,))
    g.add("off", "input", "i32", (rows + 1,))
    g.add("g", "gather", "f32", (nnz,), args=("col", "x"))
    g.add("p", "map", "f32", (nnz,), fn="mul2", args=("vals", "g"))
    g.add("y", "foldseg", "f32", (rows,), fn="add", args=("p", "off"), output=True)
    part = fc.fc_plan(g, "bytes")
    assert part.n_clusters == 1 and "column-blocked" in fc.fc_cluster_kernel(g, part, 0)
    need = fc.fc_scratch_bytes(g, part)
    assert need >= B.FC_SCRATCH_CONTROL_BYTES + 32 * rows
    fake = (0x10000000, 1 << 30)
    bufs = {n.name: fake for n in g.nodes if n.kind == "input" or n.output}
    expect("FC_E_SCRATCH", fc.fc_run_fused, g, part, bufs, (0x10000000, B.FC_SCRATCH_CONTROL_BYTES + 32 * rows - 256))
    # a table that fits one L2 keeps the plain kernel and needs no workspace
    g2 = Graph()
    g2.add("x", "input", "f32", (1000,))
    g2.add("col", "input", "i32", (nnz,))
    g2.add("vals", "input", "f32", (nnz,))
    g2.add("off", "input", "i32", (rows + 1,))
    g2.add("g", "gather", "f32", (nnz,), args=("col", "x"))
    g2.add("p", "map", "f32", (nnz,), fn="mul2", args=("vals", "g"))
    g2.add("y", "foldseg", "f32", (rows,), fn="add", args=("p", "off"), output=True)
    part2 = fc.fc_plan(g2, "bytes")
    assert "column-blocked" not in fc.fc_cluster_kernel(g2, part2, 0)
    # (the figure allows for an output the caller leaves unbound, nothing more)
    assert fc.fc_scratch_bytes(g2, part2) == need - 32 * rows


def test_workspace_of_the_sorted_segmented_fold_is_part_of_scratch():
    # graph only, no data: from four million elements on, over a table that no L2 holds (up to 2^24 elements),
    # an SpMV-shaped cluster sorts its elements through LDS; the sorted offsets and positions (2 + 2 bytes), the
    # gathered values (4 bytes), all with the slots' slack, and room for every element on its tile's overflow
    # list (6 bytes) live in scratch.  The static scratch buffer is too small for it and says so.
    def program(rows, ncols, nnz):
        g = Graph()
        g.add("x", "input", "f32", (ncols,))
        g.add("col", "input", "i32", (nnz,))
        g.add("vals", "input", "f32", (nnz,))
        g.add("off", "input", "i32", (rows + 1,))
        g.add("g", "gather", "f32", (nnz,), args=("col", "x"))
        g.add("p", "map", "f32", (nnz,), fn="mul2", args=("vals", "g"))
        g.add("y", "foldseg", "f32", (rows,), fn="add", args=("p", "off"), output=True)
        return g
    nnz = (1 << 22) + 5
    fake = (0x10000000, 1 << 30)
    for ncols in (1 << 22, 1500007, (1 << 24) - 3):
        g = program(300000, ncols, nnz)
        part = fc.fc_plan(g, "bytes")
        assert part.n_clusters == 1 and "sorted through LDS" in fc.fc_cluster_kernel(g, part, 0)
        need = fc.fc_scratch_bytes(g, part) - B.FC_SCRATCH_CONTROL_BYTES
        assert 14 * nnz <= need <= 19 * nnz, (ncols, need / nnz)
        bufs = {n.name: fake for n in g.nodes if n.kind == "input" or n.output}
        expect("FC_E_SCRATCH", fc.fc_run_fused, g, part, bufs, (0x10000000, B.FC_SCRATCH_CONTROL_BYTES + 13 * nnz))
        expect("FC_E_LIMIT", fc.fc_run_fused_static, g, part, bufs)
    # fewer elements, a table beyond 2^24 elements, or the single-pass flag: other kernels
    from workloads import single_pass
    for g in (program(100000, 1 << 22, (1 << 22) - 1), program(300000, (1 << 24) + 1, nnz), single_pass(program(300000, 1 << 22, nnz))):
        part = fc.fc_plan(g, "bytes")
        assert "sorted through LDS" not in fc.fc_cluster_kernel(g, part, 0)


def test_workspace_of_the_fold_over_sorted_gather_indices_is_part_of_scratch():
    # graph only, no data: a fold over a gather from a 16 MiB table takes the kernel pair that sorts
    # the indices by table range first; the sorted indices live in scratch
    def program(table, m):
        g = Graph()
        g.add("xs", "input", "f32", (table,))
        g.add("idx", "input", "i32", (m,))
        g.add("ys", "map", "f32", (table,), fn="sin_x_mul_x", args=("xs",))
        g.add("zs", "gather", "f32", (m,), args=("idx", "ys"))
        g.add("ws", "map", "f32", (m,), fn="sq_plus_one", args=("zs",))
        g.add("r", "fold", "f32", (1,), fn="add", args=("ws",), output=True)
        return g
    m = 1 << 22
    fake = (0x10000000, 1 << 30)
    # up to 2^24 table elements the entries are 16-bit offsets into a table range (96 per 64 positions: 3 bytes
    # a position), beyond that whole indices (320 words per 256: 5 bytes a position)
    for table, variant, per_position in ((1 << 22, "LDS", 3), (1 << 25, "binned", 5)):
        g = program(table, m)
        part = fc.fc_plan(g, "bytes")
        assert part.n_clusters == 1 and variant in fc.fc_cluster_kernel(g, part, 0), fc.fc_cluster_kernel(g, part, 0)
        assert ("LDS" in fc.fc_cluster_kernel(g, part, 0)) == (variant == "LDS")
        need = fc.fc_scratch_bytes(g, part)
        assert B.FC_SCRATCH_CONTROL_BYTES + per_position * m <= need < B.FC_SCRATCH_CONTROL_BYTES + (per_position + 1) * m
        bufs = {n.name: fake for n in g.nodes if n.kind == "input" or n.output}
        expect("FC_E_SCRATCH", fc.fc_run_fused, g, part, bufs, (0x10000000, B.FC_SCRATCH_CONTROL_BYTES + (per_position - 1) * m))
    # a table that fits one L2, or few positions: gathered directly, no workspace
    for table, count in ((1 << 20, m), (1 << 22, 1 << 20)):
        small = program(table, count)
        part = fc.fc_plan(small, "bytes")
        assert "binned" not in fc.fc_cluster_kernel(small, part, 0)
        assert fc.fc_scratch_bytes(small, part) < B.FC_SCRATCH_CONTROL_BYTES + 4096


def test_duplicate_keeps_program_meaning():
    from oracle.interp import evaluate
    for cfg in (1, 5):
        w = build(cfg, small=True)
        g2, origin = fc.fc_duplicate(w.graph)
        assert len(g2.nodes) > len(w.graph.nodes)
        a, b = evaluate(w.graph, w.inputs), evaluate(g2, w.inputs)
        for o in w.graph.outputs():
            assert np.array_equal(a[o], b[o])
        for i, n in enumerate(g2.nodes):
            assert n.kind == w.graph.nodes[origin[i]].kind


def test_bench_refuses_more_than_one_gpu():
    # one GPU is all the library uses: asked for more, the benchmark says so and measures nothing
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "one GPU" in p.stderr and p.stdout.strip() == ""


def test_the_unfused_clustering_exists_wherever_a_clustering_does():
    # a reader of a scatter's destination that comes after the scatter in program order: the
    # clusters are numbered so that it still runs before the scatter (section 4.1: every other
    # use of the destination sits in an earlier cluster)
    n = 64
    g = Graph()
    g.add("dest", "input", "i32", (n,))
    g.add("idx", "input", "i32", (n,))
    g.add("val", "input", "i32", (n,))
    g.add("s", "scatter", "i32", (n,), fn="add", args=("dest", "idx", "val"), output=True)
    g.add("m", "map", "i32", (n,), fn="ident", args=("dest",), output=True)
    assert fc.fc_plan(g, "bytes").n_clusters == 2
    t = fc.fc_partition_trivial(g)
    ix = g.index()
    assert t.n_clusters == 2 and t.pi[ix["m"]] < t.pi[ix["s"]]
    assert fc.fc_scratch_bytes(g, None) >= B.FC_SCRATCH_CONTROL_BYTES
    # random programs with scatters: whenever fc_plan finds a clustering, the unfused one exists too,
    # is legal, and keeps program order where no scatter forces otherwise
    from test_chooser import random_graph
    seen = 0
    for seed in range(120):
        rng = np.random.default_rng(5000 + seed)
        g = random_graph(rng, int(rng.integers(3, 9)))
        try:
            fc.fc_plan(g, "reads_writes", no_split=True)
        except fc.FcError:
            with pytest.raises(fc.FcError):
                fc.fc_partition_trivial(g)
            continue
        t = fc.fc_partition_trivial(g)
        ops = [k for k, nd in enumerate(g.nodes) if nd.kind != "input"]
        assert t.n_clusters == len(ops) and len({int(t.pi[k]) for k in ops}) == len(ops)
        assert fc.fc_partition_check(g, [int(v) for v in t.pi]).n_clusters == len(ops)
        if not any(nd.kind == "scatter" for nd in g.nodes):
            assert [int(t.pi[k]) for k in ops] == sorted(int(t.pi[k]) for k in ops)
        seen += any(nd.kind == "scatter" for nd in g.nodes)
    assert seen >= 20


def test_check_rejects_a_scratch_buffer_that_cannot_be_one():
    # host-side argument checks only: nothing is enqueued
    expect("FC_E_SCRATCH", fc.fc_check, (0x10000010, B.FC_SCRATCH_CONTROL_BYTES))   # not 256-byte aligned


@pytest.mark.gpu
def test_check_reports_and_clears_a_wait_that_gave_up():
    # The error word is planted from the host (no kernel is made to give up a wait): fc_check
    # must turn it into FC_E_DEVICE_WAIT once, clear it, and leave the launch counter alone,
    # so that the scratch buffer keeps working.
    import torch
    from oracle.interp import evaluate
    from paper_2407_13585_amd.device import DeviceProgram
    w = build(4, small=True)
    prog = DeviceProgram(w.graph, w.inputs, fc.fc_plan(w.graph, "bytes"))
    prog.run()
    prog.check()                                                       # a clean run: FC_OK
    epoch = int(prog.control_words()[0])
    assert epoch >= 1 and prog.control_words()[1] == 0
    prog.scratch[1] = 1
    torch.cuda.synchronize()
    msg = expect("FC_E_DEVICE_WAIT", prog.check)
    assert "invalid" in msg
    assert prog.control_words().tolist()[:2] == [epoch, 0]
    prog.check()                                                       # cleared: the next check is clean
    prog.run()
    prog.check()
    env = evaluate(w.graph, w.inputs)
    assert np.array_equal(prog.fetch("out"), env["out"]) and int(prog.fetch("count")[0]) == int(env["count"][0])


def test_single_pass_flag_selects_the_kernel_that_keeps_position_order():
    # host only: the matcher's choice for the two gather pipelines at their benchmark sizes
    from workloads import single_pass
    for cfg, variant in ((2, "binned"), (3, "sorted through LDS")):
        w = build(cfg)
        default = fc.fc_plan(w.graph, "bytes")
        assert variant in fc.fc_cluster_kernel(w.graph, default, 0)
        g = single_pass(w.graph)
        marked = fc.fc_plan(g, "bytes")
        assert marked.n_clusters == 1 and "{" not in fc.fc_cluster_kernel(g, marked, 0)
        # the single pass needs no workspace beyond the control block
        assert fc.fc_scratch_bytes(g, marked) < fc.fc_scratch_bytes(w.graph, default)
