"""Plain description of a combinator program: a topologically ordered list of nodes.

This module is data only.  It holds none of the arithmetic of the method: no
element function is evaluated here, no combinator is executed, no partition is
chosen.  Both the CPU oracle and the binding of the HIP library read these
descriptions; each turns the names below into its own representation.

Vocabulary (paper section 2, "Language", and Table 1):

kinds   input | map | generate | gather | fold | foldseg | scanl | scanr |
        scatter | force
        `map` is n-ary: after the array-of-structures to structure-of-arrays
        step a zipWith is a map over several equally sized arrays (section 2,
        last paragraph).
args    map:      the argument arrays, in the order the element function takes them
        gather:   (indices, source)          -- Table 1 row "gather"
        fold:     (values,)
        foldseg:  (values, offsets)          -- offsets has R+1 entries
        scanl/r:  (values,)
        scatter:  (dest, index, value[, flag])  -- src is the SoA tuple (index, value, flag)
        force:    (xs,)
fn      name of the element function, index function or reducer
dtype   'f32' | 'i32' element type of the array the node produces
shape   tuple of extents (row-major); a global fold produces shape (1,)
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

KINDS = ("input", "map", "generate", "gather", "fold", "foldseg",
         "scanl", "scanr", "scatter", "force")

# element functions of map nodes (arity in brackets)
MAP_FNS = ("ident", "affine", "sin_x_mul_x", "sq_plus_one", "mul2", "add2",
           "add3", "add5", "exp_neg", "mod_eq")
# index functions of generate nodes
GEN_FNS = ("iota", "iota_rev", "clamp_shift_2d", "row_of_2d", "const_i32")
# reducers of fold / foldseg / scan, combination functions of scatter
REDUCERS = ("add", "max", "mul")
SCATTER_FNS = ("overwrite", "add")


@dataclass(frozen=True)
class Node:
    name: str
    kind: str
    dtype: str
    shape: Tuple[int, ...]
    fn: str = ""
    fparam: Tuple[float, ...] = ()
    iparam: Tuple[int, ...] = ()
    args: Tuple[str, ...] = ()
    output: bool = False          # a result of the program: must be manifest
    infusible: Tuple[int, ...] = ()   # argument positions reached through `!`, force or foreign code
    single_pass: bool = False     # fold / foldseg: the cluster must be one pass over its arrays, gathers in position order

    def __post_init__(self):
        if self.kind not in KINDS:
            raise ValueError(f"unknown kind {self.kind!r}")
        if self.dtype not in ("f32", "i32"):
            raise ValueError(f"unknown dtype {self.dtype!r}")

    @property
    def size(self) -> int:
        n = 1
        for s in self.shape:
            n *= int(s)
        return n


@dataclass
class Graph:
    nodes: List[Node] = field(default_factory=list)

    def add(self, *a, **kw) -> str:
        node = Node(*a, **kw)
        if any(n.name == node.name for n in self.nodes):
            raise ValueError(f"duplicate node {node.name}")
        known = {n.name for n in self.nodes}
        for arg in node.args:
            if arg not in known:
                raise ValueError(f"{node.name}: argument {arg} not defined before use")
        self.nodes.append(node)
        return node.name

    def index(self) -> Dict[str, int]:
        return {n.name: i for i, n in enumerate(self.nodes)}

    def __getitem__(self, name: str) -> Node:
        for n in self.nodes:
            if n.name == name:
                return n
        raise KeyError(name)

    def edges(self) -> List[Tuple[int, int, int]]:
        """(producer index, consumer index, argument slot), consumers ascending,
        slots ascending: the edge numbering every partition array uses."""
        ix = self.index()
        out = []
        for b, n in enumerate(self.nodes):
            for k, a in enumerate(n.args):
                out.append((ix[a], b, k))
        return out

    def inputs(self) -> List[str]:
        return [n.name for n in self.nodes if n.kind == "input"]

    def outputs(self) -> List[str]:
        return [n.name for n in self.nodes if n.output]


def names(nodes: Sequence[Node]) -> List[str]:
    return [n.name for n in nodes]


def single_pass(graph: Graph) -> Graph:
    """The same program with every fold / foldseg marked `single_pass`."""
    from dataclasses import replace
    return Graph([replace(n, single_pass=True) if n.kind in ("fold", "foldseg") else n for n in graph.nodes])
