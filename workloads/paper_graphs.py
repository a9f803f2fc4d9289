"""Dependence graphs of the programs the paper uses as examples (sections 1, 3.3, 3.4 and 5).

Structure only: element functions are placeholders from the closed vocabulary,
chosen so that arities, shapes and dtypes are valid.  A use of an array through
indexing (`xs ! 0`) is an argument marked infusible, as in section 4.1.
"""
from __future__ import annotations

from .graph import Graph

N = 1024


def scatter_example() -> Graph:
    """section 3.4: as = map f xs; bs = map g xs; result = scatter(+, bs, as)."""
    g = Graph()
    g.add("xs", "input", "i32", (N,))
    g.add("as", "map", "i32", (N,), fn="ident", args=("xs",))
    g.add("bs", "map", "i32", (N,), fn="ident", args=("xs",))
    g.add("result", "scatter", "i32", (N,), fn="add", args=("bs", "as", "as"), output=True)
    return g


def single_loop(N: int = N) -> Graph:
    """section 1: bs = reverse as; cs = map f as; ds = map g cs; result = zipWith3 (+) bs cs ds."""
    g = Graph()
    g.add("as", "input", "f32", (N,))
    g.add("inds", "generate", "i32", (N,), fn="iota_rev")
    g.add("bs", "gather", "f32", (N,), args=("inds", "as"))
    g.add("cs", "map", "f32", (N,), fn="affine", fparam=(2.0, 0.0), args=("as",))
    g.add("ds", "map", "f32", (N,), fn="sq_plus_one", args=("cs",))
    g.add("result", "map", "f32", (N,), fn="add3", args=("bs", "cs", "ds"), output=True)
    return g


def simple1(output_as: bool = False) -> Graph:
    """section 3.3 simple1 (and simple3 when `as` is also a result)."""
    g = Graph()
    g.add("is", "input", "i32", (N // 2,))
    g.add("xs", "input", "f32", (N,))
    g.add("as", "map", "f32", (N,), fn="affine", fparam=(2.0, 1.0), args=("xs",), output=output_as)
    g.add("bs", "gather", "f32", (N // 2,), args=("is", "as"), output=True)
    return g


def simple3() -> Graph:
    return simple1(output_as=True)


def simple2() -> Graph:
    g = Graph()
    g.add("is1", "input", "i32", (N,))
    g.add("is2", "input", "i32", (N // 2,))
    g.add("xs", "input", "f32", (2 * N,))
    g.add("as", "gather", "f32", (N,), args=("is1", "xs"))
    g.add("bs", "gather", "f32", (N // 2,), args=("is2", "as"), output=True)
    return g


def simple4() -> Graph:
    """gather of a row-fold: the gather picks the row, the fold loops inside."""
    g = Graph()
    g.add("is", "input", "i32", (N // 2,))
    g.add("xs", "input", "f32", (N, 16))
    g.add("as", "fold", "f32", (N,), fn="add", args=("xs",))
    g.add("bs", "gather", "f32", (N // 2,), args=("is", "as"), output=True)
    return g


def simple5(produced_xs: bool = False) -> Graph:
    """one array read in order 0 and in a gather's order inside one loop."""
    g = Graph()
    g.add("is", "input", "i32", (N,))
    if produced_xs:
        g.add("src", "input", "f32", (N,))
        g.add("xs", "map", "f32", (N,), fn="exp_neg", args=("src",))
    else:
        g.add("xs", "input", "f32", (N,))
    g.add("as", "map", "f32", (N,), fn="sq_plus_one", args=("xs",))
    g.add("bs", "gather", "f32", (N,), args=("is", "xs"))
    g.add("cs", "map", "f32", (N,), fn="mul2", args=("as", "bs"), output=True)
    return g


def scan_then_gather() -> Graph:
    g = Graph()
    g.add("is", "input", "i32", (N,))
    g.add("xs", "input", "i32", (N,))
    g.add("as", "scanl", "i32", (N,), fn="add", args=("xs",))
    g.add("bs", "gather", "i32", (N,), args=("is", "as"), output=True)
    return g


def scanl_scanr(produced: bool = True) -> Graph:
    g = Graph()
    g.add("src", "input", "i32", (N,))
    x = "src"
    if produced:
        g.add("x", "map", "i32", (N,), fn="ident", args=("src",))
        x = "x"
    g.add("y", "scanl", "i32", (N,), fn="add", args=(x,), output=True)
    g.add("z", "scanr", "i32", (N,), fn="add", args=(x,), output=True)
    return g


def greedy_bottom_up_bad(n: int = 64, m: int = 4096) -> Graph:
    """section 5: a large gathered array that both folds can contract if they share a cluster."""
    g = Graph()
    g.add("xs", "input", "f32", (n,))
    g.add("is", "generate", "i32", (n, m), fn="row_of_2d")
    g.add("large", "gather", "f32", (n, m), args=("is", "xs"))
    g.add("ys", "fold", "f32", (n,), fn="add", args=("large",))
    g.add("zs", "fold", "f32", (n,), fn="mul", args=("large",))
    # result = map (\y -> y + zs!0) ys : zs is indexed, so that edge is infusible
    g.add("result", "map", "f32", (n,), fn="add2", args=("ys", "zs"), infusible=(1,), output=True)
    return g


def greedy_top_down_bad(N: int = N) -> Graph:
    """section 5: diagonal fusion of cs with bs versus vertical fusion of cs with es."""
    g = Graph()
    g.add("as", "input", "f32", (N,))
    g.add("bs", "map", "f32", (N,), fn="affine", fparam=(2.0, 0.0), args=("as",))
    g.add("cs", "map", "f32", (N,), fn="affine", fparam=(1.0, 1.0), args=("bs",))
    # ds = generate n (\i -> i + bs!0): bs is indexed, so the edge is infusible
    g.add("ds", "map", "f32", (N,), fn="ident", args=("bs",), infusible=(0,))
    g.add("es", "map", "f32", (N,), fn="add2", args=("cs", "ds"))
    g.add("result", "fold", "f32", (1,), fn="add", args=("es",), output=True)
    return g


ALL = {
    "scatter_example": scatter_example, "single_loop": single_loop, "simple1": simple1, "simple2": simple2,
    "simple3": simple3, "simple4": simple4, "simple5": simple5, "scan_then_gather": scan_then_gather,
    "scanl_scanr": scanl_scanr, "greedy_bottom_up_bad": greedy_bottom_up_bad,
    "greedy_top_down_bad": greedy_top_down_bad,
}
