"""CPU oracle, part 1: the capacitated digraph and its brute-force invariants.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package;
it exists so the tests, the smoke check and the benchmark's CPU-baseline leg can
say what the right answer is.  It shares no code with the HIP library.

Model (paper section 3.1): every rank is a vertex, every link a directed arc
with a bandwidth-proportional capacity; a broadcast from root r is a set of
weighted spanning arborescences (directed spanning trees diverging from r) and
the best total weight equals the smallest capacity leaving any vertex set that
contains r (Edmonds; the paper cites it for the optimal rate).

Everything here is the plain definition written out (subset enumeration,
exhaustive parent assignment), usable only for small k.
"""
from __future__ import annotations

import itertools
from fractions import Fraction
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np


class Digraph:
    """k vertices, directed arcs with positive capacity; parallel arcs merged."""

    def __init__(self, k: int, arcs: Iterable[Tuple[int, int, float]]):
        if k < 1:
            raise ValueError("k must be positive")
        cap: Dict[Tuple[int, int], float] = {}
        for u, v, c in arcs:
            u, v, c = int(u), int(v), float(c)
            if not (0 <= u < k and 0 <= v < k) or u == v:
                raise ValueError(f"bad arc {u}->{v}")
            if not c > 0:
                raise ValueError(f"capacity of {u}->{v} must be positive")
            cap[(u, v)] = cap.get((u, v), 0.0) + c
        self.k = k
        self.cap = cap
        self.arcs: List[Tuple[int, int, float]] = [(u, v, cap[(u, v)]) for (u, v) in sorted(cap)]

    @classmethod
    def from_topology(cls, top) -> "Digraph":
        return cls(top.k, zip(top.src.tolist(), top.dst.tolist(), top.cap.tolist()))

    @property
    def m(self) -> int:
        return len(self.arcs)

    def in_neighbours(self, v: int) -> List[int]:
        return [u for (u, w, _) in self.arcs if w == v]

    def reachable_from(self, root: int) -> List[bool]:
        seen = [False] * self.k
        seen[root] = True
        stack = [root]
        while stack:
            u = stack.pop()
            for (a, b, _) in self.arcs:
                if a == u and not seen[b]:
                    seen[b] = True
                    stack.append(b)
        return seen


def min_root_cut(g: Digraph, root: int) -> float:
    """min over vertex sets S with root in S, S != V, of the capacity of arcs
    leaving S.  All 2^(k-1) sets are tried (vectorised over the sets)."""
    k = g.k
    if k == 1:
        return float("inf")
    masks = np.arange(1 << k, dtype=np.int64)
    ok = ((masks >> root) & 1 == 1) & (masks != (1 << k) - 1)
    masks = masks[ok]
    out = np.zeros(masks.shape[0], np.float64)
    for (u, v, c) in g.arcs:
        leaving = ((masks >> u) & 1 == 1) & ((masks >> v) & 1 == 0)
        out += np.where(leaving, c, 0.0)
    return float(out.min())


def is_spanning_arborescence(g: Digraph, root: int, parent: Sequence[int]) -> bool:
    """parent[v] is v's predecessor (parent[root] == -1).  True iff every
    non-root vertex has a parent joined to it by an arc of g and following
    parents from any vertex reaches the root (hence k-1 arcs, no cycle)."""
    k = g.k
    if len(parent) != k or parent[root] != -1:
        return False
    for v in range(k):
        if v == root:
            continue
        p = parent[v]
        if not (0 <= p < k) or (p, v) not in g.cap:
            return False
    for v in range(k):
        x, hops = v, 0
        while x != root:
            x = parent[x]
            hops += 1
            if hops > k:
                return False
    return True


def enumerate_arborescences(g: Digraph, root: int) -> List[Tuple[int, ...]]:
    """All spanning arborescences rooted at root, as parent tuples: every
    non-root vertex tries every in-neighbour; assignments with a cycle are
    dropped.  Exponential; small graphs only."""
    k = g.k
    others = [v for v in range(k) if v != root]
    choices = [g.in_neighbours(v) for v in others]
    if any(len(c) == 0 for c in choices):
        return []
    out = []
    parent = [-1] * k
    for combo in itertools.product(*choices):
        for v, p in zip(others, combo):
            parent[v] = p
        good = True
        for v in others:
            x, hops = v, 0
            while x != root:
                x = parent[x]
                hops += 1
                if hops > k:
                    good = False
                    break
            if not good:
                break
        if good:
            out.append(tuple(parent))
    return out


def count_arborescences_matrix_tree(g: Digraph, root: int) -> int:
    """Directed matrix-tree theorem: the number of spanning arborescences
    diverging from root is the determinant of (in-degree matrix - adjacency)
    with the root's row and column removed.  Exact rational elimination."""
    k = g.k
    L = [[Fraction(0)] * k for _ in range(k)]
    for (u, v, _) in g.arcs:
        L[v][v] += 1
        L[u][v] -= 1
    idx = [i for i in range(k) if i != root]
    M = [[L[i][j] for j in idx] for i in idx]
    n = len(M)
    det = Fraction(1)
    for c in range(n):
        piv = next((r for r in range(c, n) if M[r][c] != 0), None)
        if piv is None:
            return 0
        if piv != c:
            M[c], M[piv] = M[piv], M[c]
            det = -det
        det *= M[c][c]
        for r in range(c + 1, n):
            f = M[r][c] / M[c][c]
            if f != 0:
                for j in range(c, n):
                    M[r][j] -= f * M[c][j]
    assert det.denominator == 1
    return int(det)


def tree_arcs(root: int, parent: Sequence[int]) -> List[Tuple[int, int]]:
    """Arcs (parent -> child) of an arborescence."""
    return [(parent[v], v) for v in range(len(parent)) if v != root]


def children_of(parent: Sequence[int]) -> List[List[int]]:
    """Children lists in ascending vertex id (the fixed order in which a node
    folds its children's partial sums)."""
    k = len(parent)
    ch: List[List[int]] = [[] for _ in range(k)]
    for v in range(k):
        if parent[v] >= 0:
            ch[parent[v]].append(v)
    return ch


def max_integral_packing_exhaustive(g: Digraph, root: int,
                                    trees: Optional[List[Tuple[int, ...]]] = None) -> int:
    """Largest number of unit-weight arborescences (repeats allowed) that fit
    under the capacities, by exhaustive depth-first search over the full list
    of arborescences.  Tiny graphs only.  With integer capacities Edmonds'
    theorem says this equals min_root_cut."""
    if trees is None:
        trees = enumerate_arborescences(g, root)
    resid = dict(g.cap)
    best = 0

    def fits(t) -> bool:
        return all(resid[a] >= 1.0 - 1e-12 for a in tree_arcs(root, t))

    def rec(start: int, count: int) -> None:
        nonlocal best
        best = max(best, count)
        # no packing can exceed the residual capacity entering any vertex
        room = min(sum(c for (u, v), c in resid.items() if v == x)
                   for x in range(g.k) if x != root)
        if count + int(room + 1e-12) <= best:
            return
        for i in range(start, len(trees)):
            t = trees[i]
            if fits(t):
                for a in tree_arcs(root, t):
                    resid[a] -= 1.0
                rec(i, count + 1)
                for a in tree_arcs(root, t):
                    resid[a] += 1.0

    rec(0, 0)
    return best
