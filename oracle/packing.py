"""CPU oracle, part 2: packing spanning trees (paper sections 3.1, 3.2, 3.2.1, 3.5).

TEST INFRASTRUCTURE ONLY (see oracle/graph.py).  Shares no code with the HIP
library's packer; parity between the two is on invariants (feasibility, rate,
tree validity), never on which trees were chosen.

The paper describes the multiplicative-weight-update (MWU) packing in one
paragraph (section 3.2) and leaves its constants unstated.  Reading used here,
the Garg-Koenemann form of the fractional-packing family the paper cites:

  * every arc e carries a length l_e, initially delta / c_e;
  * repeat: find the minimum-length spanning arborescence T under l; add
    gamma = min_{e in T} c_e to T's weight; l_e <- l_e (1 + eps gamma / c_e)
    for e in T; stop once sum_e c_e l_e >= 1;
  * scale all weights down by the worst congestion max_e load_e / c_e, which
    makes the packing feasible (this is never weaker than the textbook scale
    factor log_{1+eps}((1+eps)/delta));
  * delta = (1+eps) ((1+eps) m)^(-1/eps).

Minimising the number of trees (section 3.2.1): weights restricted to a grid
g * {0,1,2,...} over MWU's candidate trees, maximise the total weight exactly
(depth-first branch and bound); start with g = 1 (the paper's 0/1 program;
multiplicity 2 of a tree stands for two identical unit trees) and relax by
halving g until the rate is within ``tol`` of MWU's rate.  The paper's
capacity constraint is printed with a strict '<'; it is read as '<=' because
the paper's own result (six unit trees on a graph whose root cut is six)
saturates the constraints.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

from .graph import Digraph, is_spanning_arborescence, tree_arcs

Tree = Tuple[int, ...]  # parent tuple, parent[root] == -1


# --------------------------------------------------------------------------
# minimum-length spanning arborescence (Chu-Liu / Edmonds), recursive form
# --------------------------------------------------------------------------
def min_arborescence(k: int, arcs: Sequence[Tuple[int, int, float]], root: int,
                     verts: Optional[Sequence[int]] = None) -> Optional[List[int]]:
    """Indices into ``arcs`` of a minimum-total-length spanning arborescence
    diverging from ``root`` over the vertices ``verts`` (default 0..k-1); None
    if some vertex cannot be reached.  Ties are broken towards the lowest arc
    index."""
    if verts is None:
        verts = list(range(k))
    # cheapest arc into every non-root vertex
    best: Dict[int, int] = {}
    for i, (u, v, w) in enumerate(arcs):
        if v == root or u == v:
            continue
        if v not in best or w < arcs[best[v]][2]:
            best[v] = i
    for v in verts:
        if v != root and v not in best:
            return None
    # look for a cycle among the chosen arcs
    cycle: Optional[List[int]] = None
    colour: Dict[int, int] = {}
    for s in verts:
        if s == root or s in colour:
            continue
        path = []
        x = s
        while x != root and x not in colour:
            colour[x] = s
            path.append(x)
            x = arcs[best[x]][0]
        if x != root and colour.get(x) == s:
            cycle = path[path.index(x):]
            break
    if cycle is None:
        return sorted(best.values())
    # contract the cycle into a fresh vertex and recurse
    in_cycle = set(cycle)
    c = max(verts) + 1
    new_arcs: List[Tuple[int, int, float]] = []
    origin: List[int] = []
    for i, (u, v, w) in enumerate(arcs):
        uu = c if u in in_cycle else u
        vv = c if v in in_cycle else v
        if uu == vv:
            continue
        if vv == c:
            w = w - arcs[best[v]][2]
        new_arcs.append((uu, vv, w))
        origin.append(i)
    sub = min_arborescence(k, new_arcs, root, [v for v in verts if v not in in_cycle] + [c])
    if sub is None:
        return None
    chosen = [origin[j] for j in sub]
    # the one chosen arc that enters the cycle displaces the cycle arc into the same vertex
    entered = next(arcs[i][1] for i in chosen if arcs[i][1] in in_cycle and arcs[i][0] not in in_cycle)
    chosen += [best[v] for v in cycle if v != entered]
    return sorted(chosen)


def _parents_from_arcs(k: int, arcs, idx: Sequence[int], root: int) -> Tree:
    parent = [-1] * k
    for i in idx:
        parent[arcs[i][1]] = arcs[i][0]
    return tuple(parent)


# --------------------------------------------------------------------------
# MWU fractional packing (section 3.2)
# --------------------------------------------------------------------------
def mwu_pack(g: Digraph, root: int, eps: float = 0.1) -> Tuple[List[Tree], List[float]]:
    """Approximate maximum fractional packing of arborescences rooted at root.
    Returns distinct trees and feasible weights; total weight >= (1-2 eps) of
    the optimum for small eps (checked against brute force in the tests)."""
    if not all(g.reachable_from(root)):
        raise ValueError("some vertex is unreachable from the root")
    m = g.m
    delta = (1.0 + eps) * ((1.0 + eps) * m) ** (-1.0 / eps)
    length = [delta / c for (_, _, c) in g.arcs]
    weight: Dict[Tree, float] = {}
    while sum(c * l for (_, _, c), l in zip(g.arcs, length)) < 1.0:
        arcs = [(u, v, length[i]) for i, (u, v, _) in enumerate(g.arcs)]
        idx = min_arborescence(g.k, arcs, root)
        gamma = min(g.arcs[i][2] for i in idx)
        t = _parents_from_arcs(g.k, g.arcs, idx, root)
        weight[t] = weight.get(t, 0.0) + gamma
        for i in idx:
            length[i] *= 1.0 + eps * gamma / g.arcs[i][2]
    trees = list(weight)
    w = [weight[t] for t in trees]
    load = arc_loads(g, trees, w, [root] * len(trees))
    congestion = max(load[a] / g.cap[a] for a in load)
    w = [x / congestion for x in w]
    return trees, w


# --------------------------------------------------------------------------
# fewer trees (section 3.2.1)
# --------------------------------------------------------------------------
def grid_max_packing(g: Digraph, root: int, cands: Sequence[Tree], unit: float,
                     node_budget: int = 200_000) -> Tuple[List[int], float]:
    """Maximise sum_i x_i * unit over integer x_i >= 0 subject to the arc
    capacities, by depth-first branch and bound over the candidate trees.
    Returns the multiplicities and the rate.  Exact unless the node budget runs
    out (then the best packing found so far)."""
    resid = dict(g.cap)
    arcs_of = [tree_arcs(root, t) for t in cands]
    n = len(cands)
    cur = [0] * n
    best_x = [0] * n
    best = 0
    nodes = 0
    non_root = [v for v in range(g.k) if v != root]

    def bound() -> int:
        room = min(sum(c for (u, v), c in resid.items() if v == x) for x in non_root)
        return int(math.floor(room / unit + 1e-9))

    cap_total = bound()  # no packing beats the smallest in-capacity

    def rec(i: int, count: int) -> bool:
        nonlocal best, best_x, nodes
        nodes += 1
        if count > best:
            best, best_x = count, cur.copy()
            if best >= cap_total:
                return True
        if i == n or nodes > node_budget or count + bound() <= best:
            return False
        most = int(math.floor(min(resid[a] for a in arcs_of[i]) / unit + 1e-9))
        for mult in range(most, -1, -1):
            for a in arcs_of[i]:
                resid[a] -= mult * unit
            cur[i] = mult
            done = rec(i + 1, count + mult)
            for a in arcs_of[i]:
                resid[a] += mult * unit
            cur[i] = 0
            if done:
                return True
        return False

    rec(0, 0)
    return best_x, best * unit


def prune(g: Digraph, root: int, trees: Sequence[Tree], weights: Sequence[float],
          tol: float = 0.05, min_unit: float = 1.0 / 64) -> Tuple[List[Tree], List[float]]:
    """Fewest-trees refinement of an MWU packing: grid program over its trees,
    unit 1, 1/2, 1/4, ... until the rate is within tol of MWU's rate."""
    target = (1.0 - tol) * sum(weights)
    order = sorted(range(len(trees)), key=lambda i: -weights[i])
    cands = [trees[i] for i in order]
    unit = 1.0
    best: Tuple[List[Tree], List[float]] = (list(trees), list(weights))
    while unit >= min_unit:
        x, rate = grid_max_packing(g, root, cands, unit)
        if rate >= target - 1e-9:
            keep = [(cands[i], x[i] * unit) for i in range(len(cands)) if x[i] > 0]
            best = ([t for t, _ in keep], [w for _, w in keep])
            break
        unit /= 2.0
    return best


def pack_trees(g: Digraph, root: int, eps: float = 0.1, tol: float = 0.05):
    """MWU then pruning.  Returns (roots, trees, weights)."""
    trees, w = mwu_pack(g, root, eps)
    trees, w = prune(g, root, trees, w, tol)
    return [root] * len(trees), trees, w


def one_hop_stars(g: Digraph):
    """Switch-like topologies (section 3.5): with m ranks, m one-hop trees, rank
    i the root of tree i, every other rank its direct child, each tree carrying
    1/m of the data.  Requires every arc i->j to exist."""
    k = g.k
    for i in range(k):
        for j in range(k):
            if i != j and (i, j) not in g.cap:
                raise ValueError("one-hop trees need a fully connected graph")
    roots = list(range(k))
    trees = [tuple(-1 if v == r else r for v in range(k)) for r in roots]
    return roots, trees, [1.0 / k] * k


# --------------------------------------------------------------------------
# validators for ANY packer's output
# --------------------------------------------------------------------------
def arc_loads(g: Digraph, trees: Sequence[Tree], weights: Sequence[float],
              roots: Sequence[int]) -> Dict[Tuple[int, int], float]:
    load = {a: 0.0 for a in g.cap}
    for t, w, r in zip(trees, weights, roots):
        for a in tree_arcs(r, t):
            load[a] += w
    return load


def check_packing(g: Digraph, roots: Sequence[int], trees: Sequence[Tree],
                  weights: Sequence[float], slack: float = 1e-9) -> float:
    """Raises AssertionError unless every tree is a spanning arborescence of g
    from its root, every weight is positive and no arc carries more than its
    capacity (packing LP of section 3.1).  Returns the rate sum(weights)."""
    assert len(roots) == len(trees) == len(weights) and len(trees) > 0
    for t, w, r in zip(trees, weights, roots):
        assert w > 0, "non-positive tree weight"
        assert is_spanning_arborescence(g, r, t), f"not a spanning arborescence: {t}"
    load = arc_loads(g, trees, weights, roots)
    for a, l in load.items():
        assert l <= g.cap[a] + slack, f"arc {a} overloaded: {l} > {g.cap[a]}"
    return float(sum(weights))
