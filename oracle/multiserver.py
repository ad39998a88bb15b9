"""CPU oracle, part 6: AllReduce across several servers (paper section 3.5, the
three-phase protocol) and the split between two classes of links (section 3.4).

TEST INFRASTRUCTURE ONLY (see oracle/graph.py).  Shares no code with the HIP
library.

What the paper fixes for n servers, each with its own packed local trees:
  1. the payload is partitioned by the local spanning trees; inside every
     server the root of a partition's tree reduces the partition over that tree;
  2. the n server-local roots of a partition run a reduce-broadcast over n
     one-hop trees: each of them is the root of one n-th of the partition and is
     linked directly to the other n - 1 roots;
  3. every server-local root broadcasts the result over its local tree.

Readings where the paper is silent:
  * servers whose local packings split the payload differently: the partitions
    are the common refinement of the servers' weighted splits, so inside one
    partition every server uses exactly one of its trees;
  * which root owns which n-th of a partition: the i-th smallest root id owns
    the i-th piece (pieces equal up to the 4-element alignment);
  * folding order in phase 2: the owner adds the other roots' partial sums in
    ascending rank id, after its own phase-1 sum (phase 1 ends before phase 2
    starts), i.e. ((L_own + L_a) + L_b) + ... with a < b < ...;
  * a server's ranks are given in ascending global id, so that "children in
    ascending id" means the same thing locally and globally.

``three_phase_allreduce`` is the protocol written out phase by phase on whole
arrays.  ``compose`` states the same thing as one global tree per (partition,
piece): the owner's local tree with the other servers' local trees hanging off
the owner through their roots, those roots folded in last; ``three_phase_steps``
is the chunked step list over these trees.  The tests require the two to agree
bit for bit.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

from .execute import SUM, combine
from .graph import children_of
from .schedule import (ALLREDUCE, COPY, REDUCE, Step, _symbolic_replay, chunk_ranges,
                       emit_tree_steps, split_by_weight)


@dataclass(frozen=True)
class Server:
    ranks: Tuple[int, ...]                 # global id of local rank i, ascending
    roots: Tuple[int, ...]                 # per local tree: its root (local id)
    trees: Tuple[Tuple[int, ...], ...]     # per local tree: parent array (local ids, -1 at the root)
    weights: Tuple[float, ...]


@dataclass(frozen=True)
class GlobalTree:
    lo: int
    hi: int
    root: int
    parent: Tuple[int, ...]                # global ids
    late: frozenset                        # vertices attached to their parent in phase 2


def partitions(n: int, servers: Sequence[Server]) -> List[Tuple[int, int, Tuple[int, ...]]]:
    """(lo, hi, tree index per server) of the non-empty partitions of [0, n)."""
    splits = [split_by_weight(n, s.weights) for s in servers]
    cuts = sorted({b for sp in splits for b in sp})
    out = []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        sel = []
        for sp in splits:
            t = max(i for i in range(len(sp) - 1) if sp[i] <= lo and sp[i] < sp[i + 1])
            assert sp[t] <= lo and hi <= sp[t + 1]
            sel.append(t)
        out.append((lo, hi, tuple(sel)))
    return out


def pieces(lo: int, hi: int, n_servers: int) -> List[int]:
    """Boundaries of the n equal pieces of a partition (4-element alignment)."""
    return [lo + b for b in split_by_weight(hi - lo, [1.0] * n_servers)]


def three_phase_allreduce(x: Sequence[np.ndarray], servers: Sequence[Server],
                          redop: int = SUM) -> np.ndarray:
    """The value every rank ends with, phase by phase, in the inputs' dtype."""
    n = x[0].shape[0]
    is_int = x[0].dtype == np.int32
    xs = [a.view(np.uint32) if is_int else a for a in x]
    out = np.empty(n, xs[0].dtype)
    for lo, hi, sel in partitions(n, servers):
        # phase 1: every server-local root ends with its server's partial result
        partial: Dict[int, np.ndarray] = {}
        for srv, t in zip(servers, sel):
            ch = children_of(srv.trees[t])

            def S(v: int) -> np.ndarray:
                acc = xs[srv.ranks[v]][lo:hi].copy()
                for c in ch[v]:
                    acc = combine(acc, S(c), redop)
                return acc

            partial[srv.ranks[srv.roots[t]]] = S(srv.roots[t])
        # phase 2: one-hop reduce-broadcast among the roots, one piece per root
        root_ids = sorted(partial)
        cut = pieces(lo, hi, len(servers))
        for i, owner in enumerate(root_ids):
            a, b = cut[i] - lo, cut[i + 1] - lo
            acc = partial[owner][a:b].copy()
            for r in root_ids:
                if r != owner:
                    acc = combine(acc, partial[r][a:b], redop)
            out[cut[i]:cut[i + 1]] = acc
        # phase 3 hands out[lo:hi] to every rank of every server: nothing to compute
    return out.view(np.int32) if is_int else out


def compose(n: int, servers: Sequence[Server]) -> List[GlobalTree]:
    """One global tree per (partition, piece): see the module header."""
    k = sum(len(s.ranks) for s in servers)
    out: List[GlobalTree] = []
    for lo, hi, sel in partitions(n, servers):
        parent = [-2] * k
        root_ids = []
        for srv, t in zip(servers, sel):
            for v, p in enumerate(srv.trees[t]):
                parent[srv.ranks[v]] = srv.ranks[p] if p >= 0 else -1
            root_ids.append(srv.ranks[srv.roots[t]])
        root_ids.sort()
        cut = pieces(lo, hi, len(servers))
        for i, owner in enumerate(root_ids):
            if cut[i] == cut[i + 1]:
                continue
            par = list(parent)
            for r in root_ids:
                if r != owner:
                    par[r] = owner
            out.append(GlobalTree(cut[i], cut[i + 1], owner, tuple(par),
                                  frozenset(r for r in root_ids if r != owner)))
    return out


def ordered_children(parent: Sequence[int], late: frozenset) -> List[List[int]]:
    """Children in folding order: those of the local tree ascending, then the
    other servers' roots ascending."""
    ch = children_of(parent)
    return [[c for c in cs if c not in late] + [c for c in cs if c in late] for cs in ch]


def three_phase_steps(servers: Sequence[Server], n: int, chunk: int) -> List[Step]:
    """Chunked REDUCE / COPY steps of the whole protocol; ``tree`` numbers the
    global trees in ``compose`` order."""
    steps: List[Step] = []
    for t, g in enumerate(compose(n, servers)):
        emit_tree_steps(steps, t, g.root, g.parent, ordered_children(g.parent, g.late),
                        ALLREDUCE, g.lo, g.hi, chunk)
    return steps


def check_three_phase_steps(steps: Sequence[Step], servers: Sequence[Server], n: int,
                            chunk: int) -> None:
    """Structural checks on anyone's step list for the protocol: dependencies
    point backwards; per global tree the chunks tile its range once; per chunk
    there is one REDUCE and one COPY per tree arc; the symbolic replay ends, at
    every rank, with the owner's local sum followed by the other roots' sums."""
    k = sum(len(s.ranks) for s in servers)
    trees = compose(n, servers)
    for i, s in enumerate(steps):
        assert all(0 <= d < i for d in s.deps), f"step {i}: dependency not earlier"
        assert 0 <= s.src < k and 0 <= s.dst < k and s.src != s.dst
        assert 0 <= s.tree < len(trees)
    by_tc: Dict[Tuple[int, int], List[int]] = {}
    for i, s in enumerate(steps):
        by_tc.setdefault((s.tree, s.chunk), []).append(i)
    covered = 0
    for t, g in enumerate(trees):
        want = chunk_ranges(g.lo, g.hi, chunk)
        got = sorted({(steps[ix[0]].off, steps[ix[0]].len) for (tt, _), ix in by_tc.items() if tt == t})
        assert got == want, f"tree {t}: chunks {got[:3]}.. do not tile {want[:3]}.."
        covered += g.hi - g.lo
        arcs = sorted((g.parent[v], v) for v in range(k) if v != g.root)
        ch = ordered_children(g.parent, g.late)
        for (tt, c), ix in by_tc.items():
            if tt != t:
                continue
            off, ln = steps[ix[0]].off, steps[ix[0]].len
            assert all(steps[i].off == off and steps[i].len == ln for i in ix)
            copies = sorted((steps[i].src, steps[i].dst) for i in ix if steps[i].kind == COPY)
            reduces = sorted((steps[i].dst, steps[i].src) for i in ix if steps[i].kind == REDUCE)
            assert copies == arcs, f"tree {t} chunk {c}: COPY steps do not match the arcs"
            assert reduces == arcs, f"tree {t} chunk {c}: REDUCE steps do not match the arcs"
            _symbolic_replay(steps, ix, k, g.root, g.parent, ALLREDUCE, ch)
    assert covered == n


def hybrid_split(d_total: float, bw_pcie: float, bw_nvl: float, t_dpa: float) -> Tuple[float, float]:
    """Section 3.4: the amounts of data to send over the slow and over the fast
    class of links so that both finish together, the slow class paying the
    switch-over latency t_dpa first:
        d_pcie / bw_pcie + t_dpa = d_nvl / bw_nvl,   d_pcie + d_nvl = d_total.
    Reading: when the latency alone outweighs the gain (the formula turns
    negative) nothing goes over the slow class."""
    d_pcie = (d_total * bw_pcie - t_dpa * bw_pcie * bw_nvl) / (bw_pcie + bw_nvl)
    d_pcie = min(max(d_pcie, 0.0), d_total)
    return d_pcie, d_total - d_pcie
