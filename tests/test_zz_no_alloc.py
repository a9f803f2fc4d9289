"""fc_run_fused_static: fc_run_fused for callers that cannot allocate (its scratch is a static
array inside the library).  Checked through the C ABI against fc_run_fused on the same inputs,
two calls in a row, the second with a smaller input, so that what the first call left in the
shared buffer is there when the second runs."""
import numpy as np
import pytest

import parity as P
from workloads import Graph
from workloads import configs as C

pytestmark = pytest.mark.gpu

F32 = np.float32


def programs(scale):
    """(name, graph, inputs, duplicate producers?) of the cluster shapes that use scratch: a fold's
    partials, a scan's tile words with the compaction's scatter, a manifest intermediate placed in
    scratch (the strict plan of the reversed dot product keeps `ys`), a segmented fold."""
    n = 300007 if scale else 70001
    yield "reverse-dot", C.reverse_dot(n=n, seed=7 + scale), True
    yield "reverse-dot-strict", C.reverse_dot(n=n + 13, seed=8 + scale), False
    yield "perm-gather-fold", C.perm_gather_fold(n=n, seed=9 + scale), True
    yield "compaction", C.compaction(n=3 * n + 5, seed=10 + scale), True
    yield "spmv", C.spmv(rows=n // 10, seed=11 + scale), True
    yield "stencil-max", C.stencil_max(h=197 if scale else 61, w=331 if scale else 77, seed=12 + scale), True


def test_static_scratch_gives_the_results_of_a_caller_buffer():
    import torch
    import paper_2407_13585_amd as fc
    from paper_2407_13585_amd import binding as B
    from paper_2407_13585_amd.device import DeviceProgram
    stream = torch.cuda.current_stream().cuda_stream
    for scale in (1, 0):                                   # the second round is the smaller one
        for name, w, dup in programs(scale):
            g = fc.fc_duplicate(w.graph)[0] if dup else w.graph
            part = fc.fc_plan(g, "bytes")
            assert fc.fc_scratch_bytes(g, part) <= B.FC_STATIC_SCRATCH_BYTES
            ref = DeviceProgram(g, w.inputs, part)         # its own scratch buffer, fc_run_fused
            ref.run()
            got = DeviceProgram(g, w.inputs, part)         # used for its input and output tensors only
            for rep in range(2):
                for o in g.outputs():
                    if g[o].kind != "scatter":
                        got.buffers[o].fill_(0)
                fc.fc_run_fused_static(g, part, got.buffers, stream)
                fc.fc_check(None, stream)                  # synchronises; no bounded wait gave up
                for o in g.outputs():
                    P.assert_bit_exact(got.fetch(o), ref.fetch(o), f"{name} scale={scale} rep={rep} {o}")


def test_static_scratch_refuses_programs_that_need_more():
    # nothing is enqueued: the pointers are never used
    import paper_2407_13585_amd as fc
    from paper_2407_13585_amd import binding as B
    n = 1 << 24                                            # the unbound intermediate alone takes 64 MiB
    g = Graph()
    g.add("x", "input", "f32", (n,))
    g.add("y", "map", "f32", (n,), fn="sq_plus_one", args=("x",))
    g.add("z", "scanl", "f32", (n,), fn="add", args=("y",), output=True)
    g.add("r", "fold", "f32", (1,), fn="add", args=("y",), output=True)
    part = fc.fc_partition_trivial(g)
    assert fc.fc_scratch_bytes(g, part) > B.FC_STATIC_SCRATCH_BYTES
    fake = (0x10000000, 1 << 30)
    with pytest.raises(fc.FcError) as e:
        fc.fc_run_fused_static(g, part, {"x": fake, "z": fake, "r": fake})
    assert e.value.name == "FC_E_LIMIT" and "static" in str(e.value)


def test_static_scratch_runs_replay_from_a_hip_graph():
    # what the entry point is for: a step captured into a HIP graph (no allocation may happen under
    # capture).  The first calls are made outside the capture (the buffer's address is looked up
    # then); every replay runs on other input values and is checked against the oracle.
    import torch
    import paper_2407_13585_amd as fc
    from oracle.interp import evaluate
    from paper_2407_13585_amd.device import DeviceProgram
    from workloads import build
    rng = np.random.default_rng(5)
    items = []
    for cfg in (1, 2, 3, 4, 5):
        w = build(cfg, small=True)
        g, _ = fc.fc_duplicate(w.graph)
        part = fc.fc_plan(g, "bytes")
        items.append((cfg, w, g, part, DeviceProgram(g, w.inputs, part)))     # the tensors only
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for cfg, w, g, part, prog in items:
            fc.fc_run_fused_static(g, part, prog.buffers, side.cuda_stream)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for cfg, w, g, part, prog in items:
            fc.fc_run_fused_static(g, part, prog.buffers, torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        for cfg, w, g, part, prog in items:
            for name, a in list(w.inputs.items()):
                if a.dtype == F32:
                    w.inputs[name] = (a * F32(0.5) + rng.uniform(-0.1, 0.1, size=a.shape).astype(F32)).astype(F32)
                prog.upload(name, w.inputs[name])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        fc.fc_check(None, 0)
        for cfg, w, g, part, prog in items:
            env = evaluate(w.graph, w.inputs)
            for o in w.graph.outputs():
                got, ref = prog.fetch(o), env[o]
                what = f"{w.name} replay {rep} {o}"
                if g[o].dtype == "i32":
                    P.assert_bit_exact(got, ref, what)
                elif g[o].kind == "fold" and g[o].fn == "add":
                    P.assert_fold(got, ref, what)
                elif g[o].kind == "foldseg":
                    P.assert_segmented(got, ref, env["p"], w.inputs["off"], what)
                elif g[o].kind == "fold":                                  # max of exp(-x): within 4 ulp
                    P.assert_ulp(got, np.asarray(ref, dtype=np.float64).astype(F32), 4, what)
                else:
                    P.assert_close(got, ref, 1e-6, what)
