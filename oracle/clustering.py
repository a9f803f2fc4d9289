"""CPU oracle for the chooser: brute-force enumeration of all clusterings of a tiny program.

TEST INFRASTRUCTURE ONLY (see oracle/interp.py).  Shares no code with the HIP
library or its planner and never calls them.

A clustering is a set partition of the non-input combinators into clusters plus
an execution order of the clusters.  It is legal when it obeys the four rules of
section 3.4 ("Optimal Clustering") with the order annotations of Table 1 and of
section 4.2:

  1. every array that reaches memory (and the source tuple of a scatter) is
     produced in order 0 or 1 -- an array produced in the order of a gather must
     be fused away, i.e. every one of its consumers sits in its cluster;
  2. the relative order of producer and consumer is kept: the clusters can be
     sequenced so that every edge runs forwards (no cycle between clusters);
  3. an infusible edge (from a program input, out of force, into force, the
     destination of a scatter, out of a scatter, the offsets of foldSeg) never
     lies inside a cluster;
  4. temporal uniqueness of scatter: every other use of its destination sits in a
     strictly earlier cluster;
  and inside a cluster the orders agree over every fused edge: a consumer reads an
  argument in its own output order (map, fold, the index argument of a gather, the
  source tuple of a scatter, the values of foldSeg), in its own label (the source
  argument of a gather), or in order 0 / 1 (scanl / scanr).

The ILP of Fig. "Total ILP formulation" identifies a cluster with a value of pi, so
two unrelated groups of combinators may share a value; enumerating all set
partitions covers exactly those level sets.  Costs are evaluated on the partition
as section 4.1 ("Cost function") defines them:

  clusters      number of clusters (distinct values of pi over the combinators)
  fused_edges   number of fusible edges not fused over                    (sum of x)
  arrays        number of combinator results that reach memory            (sum of 1 - m)
  reads         for every array, the number of distinct (cluster, order) pairs
                that read it from memory (same cluster and same order share a load:
                horizontal fusion; different orders never share, `simple5`)
  reads_writes  reads + arrays
  bytes         reads_writes with every read and write weighted by the array's bytes
"""
from __future__ import annotations

from itertools import count
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

ORDERED_SAME = "same"      # read in the consumer's own output order
ORDERED_LABEL = "label"    # read in the order of the consuming gather
UNORDERED = "none"


def _edges(graph):
    ix = graph.index()
    out = []
    for b, n in enumerate(graph.nodes):
        for k, a in enumerate(n.args):
            out.append((ix[a], b, k))
    return out


def _fusible(graph, a, b, k) -> bool:
    na, nb = graph.nodes[a], graph.nodes[b]
    if k in nb.infusible:
        return False
    if na.kind in ("input", "force", "scatter"):
        return False
    if nb.kind == "force":
        return False
    if nb.kind == "scatter" and k == 0:
        return False
    if nb.kind == "foldseg" and k == 1:
        return False
    return True


def _read_order(graph, b, k):
    """How consumer b reads its k-th argument: ('same',), ('label', b), ('const', 0|1) or ('none',)."""
    kind = graph.nodes[b].kind
    if kind in ("map", "fold"):
        return ("same",)
    if kind == "gather":
        return ("same",) if k == 0 else ("label", b)
    if kind == "foldseg":
        return ("same",) if k == 0 else ("none",)
    if kind == "scanl":
        return ("const", 0)
    if kind == "scanr":
        return ("const", 1)
    if kind == "scatter":
        return ("none",) if k == 0 else ("same",)
    return ("none",)


def set_partitions(items: Sequence[int]) -> Iterable[List[List[int]]]:
    """All set partitions, by restricted growth."""
    items = list(items)
    if not items:
        yield []
        return

    def rec(i, blocks):
        if i == len(items):
            yield [list(b) for b in blocks]
            return
        for b in blocks:
            b.append(items[i])
            yield from rec(i + 1, blocks)
            b.pop()
        blocks.append([items[i]])
        yield from rec(i + 1, blocks)
        blocks.pop()

    yield from rec(0, [])


class Verdict:
    def __init__(self, legal: bool, why: str = "", orders: Optional[Dict[int, int]] = None,
                 fused_away: Optional[Dict[int, bool]] = None, sequence: Optional[List[int]] = None):
        self.legal, self.why, self.orders, self.fused_away, self.sequence = legal, why, orders, fused_away, sequence


def judge(graph, blocks: List[List[int]]) -> Verdict:
    """Is this set partition of the non-input nodes a legal clustering?"""
    n = len(graph.nodes)
    cluster = {}
    for c, blk in enumerate(blocks):
        for a in blk:
            cluster[a] = c
    for a in range(n):
        if graph.nodes[a].kind == "input":
            cluster[a] = -1 - a                        # every input in a "cluster" of its own, before everything
    edges = _edges(graph)
    # rule 3
    for (a, b, k) in edges:
        if cluster[a] == cluster[b] and not _fusible(graph, a, b, k):
            return Verdict(False, f"infusible edge {a}->{b} inside a cluster")
    # rules 2 and 4: the clusters must admit a sequence
    before = {c: set() for c in range(len(blocks))}    # before[c] = clusters that must precede c
    for (a, b, k) in edges:
        if cluster[a] >= 0 and cluster[a] != cluster[b]:
            before[cluster[b]].add(cluster[a])
    for j in range(n):
        if graph.nodes[j].kind != "scatter":
            continue
        d = graph.index()[graph.nodes[j].args[0]]
        for (a, b, k) in edges:
            if a == d and b != j:
                if cluster[b] == cluster[j]:
                    return Verdict(False, f"node {b} uses the destination of scatter {j} in the same cluster")
                before[cluster[j]].add(cluster[b])
    sequence, placed = [], set()
    while len(sequence) < len(blocks):
        ready = [c for c in range(len(blocks)) if c not in placed and before[c] <= placed]
        if not ready:
            return Verdict(False, "clusters cannot be sequenced")
        sequence.append(ready[0])
        placed.add(ready[0])
    # fused-away arrays: all consumers inside the cluster, not a program result
    fused_away = {}
    for a in range(n):
        cons = [(b, k) for (p, b, k) in edges if p == a]
        fused_away[a] = (graph.nodes[a].kind != "input" and not graph.nodes[a].output and len(cons) > 0
                         and all(cluster[b] == cluster[a] for b, _ in cons))
    # orders: propagate until nothing changes; None = still free
    order: Dict[int, Optional[int]] = {a: None for a in range(n)}
    labels = {}
    lab = count(2)
    for a in range(n):
        if graph.nodes[a].kind == "gather":
            labels[a] = next(lab)
    for a in range(n):
        if graph.nodes[a].kind == "scanl":
            order[a] = 0
        if graph.nodes[a].kind == "scanr":
            order[a] = 1
    fused = [(a, b, k) for (a, b, k) in edges if cluster[a] == cluster[b]]

    def assign(a, v):
        if order[a] is None:
            order[a] = v
            return True
        if order[a] != v:
            raise ValueError(a)
        return False

    try:
        changed = True
        while changed:
            changed = False
            for (a, b, k) in fused:
                ro = _read_order(graph, b, k)
                if ro[0] == "const":
                    changed |= assign(a, ro[1])
                elif ro[0] == "label":
                    changed |= assign(a, labels[b])
                elif ro[0] == "same":
                    if order[b] is not None:
                        changed |= assign(a, order[b])
                    elif order[a] is not None:
                        changed |= assign(b, order[a])
                else:
                    return Verdict(False, "fused over an unordered argument")
    except ValueError as e:
        return Verdict(False, f"orders conflict at node {e.args[0]}")
    # rule 1
    for a in range(n):
        needs01 = (not fused_away[a]) or graph.nodes[a].kind == "scatter"
        if needs01 and order[a] is not None and order[a] > 1:
            return Verdict(False, f"array {a} would be produced in a gathered order but reaches memory")
    final = {a: (0 if order[a] is None else order[a]) for a in range(n)}
    # free groups joined by "same" edges must end up equal: they do, all free ones become 0
    return Verdict(True, "", final, fused_away, sequence)


def cost(graph, blocks: List[List[int]], v: Verdict, kind: str) -> float:
    n = len(graph.nodes)
    cluster = {}
    for c, blk in enumerate(blocks):
        for a in blk:
            cluster[a] = c
    edges = _edges(graph)
    labels, lab = {}, count(2)
    for a in range(n):
        if graph.nodes[a].kind == "gather":
            labels[a] = next(lab)

    def nbytes(a):
        return 4 * graph.nodes[a].size

    def reads(weighted):
        total = 0.0
        for a in range(n):
            keys = set()
            for (p, b, k) in edges:
                if p != a or cluster.get(a, None) == cluster[b]:
                    continue
                ro = _read_order(graph, b, k)
                if ro[0] == "same":
                    o = v.orders[b]
                elif ro[0] == "label":
                    o = labels[b]
                elif ro[0] == "const":
                    o = ro[1]
                else:
                    o = ("unordered", b)
                keys.add((cluster[b], o))
            total += len(keys) * (nbytes(a) if weighted else 1)
        return total

    def writes(weighted):
        return float(sum((nbytes(a) if weighted else 1) for a in range(n)
                         if graph.nodes[a].kind != "input" and not v.fused_away[a]))

    if kind == "clusters":
        return float(len(blocks))
    if kind == "fused_edges":
        return float(sum(1 for (a, b, k) in edges if _fusible(graph, a, b, k) and cluster[a] != cluster[b]))
    if kind == "arrays":
        return writes(False)
    if kind == "reads":
        return reads(False)
    if kind == "reads_writes":
        return reads(False) + writes(False)
    if kind == "bytes":
        return reads(True) + writes(True)
    raise ValueError(kind)


def optimum(graph, kind: str) -> Tuple[float, List[List[List[int]]]]:
    """Minimum cost over all legal clusterings and every partition that attains it."""
    nodes = [i for i, nd in enumerate(graph.nodes) if nd.kind != "input"]
    best, arg = float("inf"), []
    for blocks in set_partitions(nodes):
        v = judge(graph, blocks)
        if not v.legal:
            continue
        c = cost(graph, blocks, v, kind)
        if c < best - 1e-9:
            best, arg = c, [blocks]
        elif abs(c - best) <= 1e-9:
            arg.append(blocks)
    return best, arg


def legal_partitions(graph) -> List[List[List[int]]]:
    nodes = [i for i, nd in enumerate(graph.nodes) if nd.kind != "input"]
    return [b for b in set_partitions(nodes) if judge(graph, b).legal]


def greedy(graph, direction: str, kind: str) -> Tuple[float, List[Tuple[int, int]]]:
    """The greedy comparison arms of section 5 ("Greedy"): walk the fusible edges from the top of
    the graph ('top_down': producers nearest the inputs first) or from the bottom ('bottom_up':
    consumers nearest the results first); fuse an edge if some legal clustering still fuses it
    together with all edges taken so far.  Returns the cost of the cheapest legal clustering that
    fuses the accepted edges, and those edges."""
    legal = legal_partitions(graph)

    def fuses(blocks, pairs):
        where = {a: c for c, blk in enumerate(blocks) for a in blk}
        return all(where[a] == where[b] for a, b in pairs)

    edges = [(a, b, k) for (a, b, k) in _edges(graph) if _fusible(graph, a, b, k)]
    if direction == "top_down":
        edges.sort(key=lambda e: (e[0], e[1]))
    elif direction == "bottom_up":
        edges.sort(key=lambda e: (-e[1], -e[0]))
    else:
        raise ValueError(direction)
    taken: List[Tuple[int, int]] = []
    for (a, b, k) in edges:
        trial = taken + [(a, b)]
        if any(fuses(p, trial) for p in legal):
            taken = trial
    best = min(cost(graph, p, judge(graph, p), kind) for p in legal if fuses(p, taken))
    return best, taken
