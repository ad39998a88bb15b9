"""CPU oracle, part 3: from weighted trees to a chunked step list (paper
sections 3.3, 4.1, 4.2.1, 4.2.2).

TEST INFRASTRUCTURE ONLY (see oracle/graph.py).  Shares no code with the HIP
library's scheduler; the library's step list is checked with the validators at
the bottom of this file.

What the paper fixes:
  * the payload is split among the trees in proportion to their weights
    (section 4.1);
  * each tree's share is cut into chunks, the unit of transfer and of
    synchronisation: a node forwards a chunk only once it holds all of it
    (section 4.2.1);
  * Broadcast sends every chunk along every tree arc, root outwards;
    AllReduce first reduces towards the root over the reversed arcs, then
    broadcasts the result back over the same tree (section 3.3): 2(N-1)
    transfers per chunk on a tree of N vertices.

Readings where the paper is silent:
  * split boundaries: b_t = floor(n * (w_1+..+w_t) / W) rounded down to a
    multiple of ``align`` elements (4 = one 128-bit access) for 0 < t < T;
    b_0 = 0, b_T = n;
  * chunks have exactly C elements except a short last chunk per tree;
  * a node with several children folds them in ascending vertex id, one at a
    time, in place: parent <- parent + child.  This fixes the floating-point
    association order.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from fractions import Fraction
from typing import Dict, List, Optional, Sequence, Tuple

from .graph import children_of

REDUCE = 0  # dst[off:off+len] <- dst[off:off+len] + src[off:off+len]
COPY = 1    # dst[off:off+len] <- src[off:off+len]

BROADCAST = 0
ALLREDUCE = 1
REDUCE_TO_ROOT = 2   # the reduce phase alone: only the tree roots end with the result
ALLGATHER = 3        # every rank ends with the concatenation of all ranks' pieces
GATHER = 4           # only the tree roots do


@dataclass(frozen=True)
class Step:
    kind: int          # REDUCE or COPY
    tree: int
    chunk: int         # chunk index inside the tree's share
    src: int           # rank read
    dst: int           # rank written (and, for REDUCE, also read)
    off: int           # first element
    len: int           # number of elements
    deps: Tuple[int, ...]  # indices of earlier steps that must complete first


def split_by_weight(n: int, weights: Sequence[float], align: int = 4) -> List[int]:
    """Boundaries b_0..b_T of the per-tree shares of [0, n).  Exact rational
    arithmetic on the given weights."""
    fr = [Fraction(w) for w in weights]
    total = sum(fr)
    bounds = [0]
    acc = Fraction(0)
    for w in fr[:-1]:
        acc += w
        b = int(math.floor(n * acc / total))
        b -= b % align
        bounds.append(max(b, bounds[-1]))
    bounds.append(n)
    return bounds


def chunk_ranges(lo: int, hi: int, chunk: int) -> List[Tuple[int, int]]:
    """(offset, length) of the chunks tiling [lo, hi)."""
    if chunk <= 0:
        raise ValueError("chunk must be positive")
    return [(o, min(chunk, hi - o)) for o in range(lo, hi, chunk)]


def reduce_order(root: int, parent: Sequence[int], ch: Optional[List[List[int]]] = None) -> List[int]:
    """Non-root vertices, every vertex after all vertices of its subtree
    (post-order, children ascending unless ``ch`` gives another order): the
    order of the child->parent transfers of the reduce phase."""
    ch = children_of(parent) if ch is None else ch
    out: List[int] = []

    def visit(v: int) -> None:
        for c in ch[v]:
            visit(c)
        if v != root:
            out.append(v)

    visit(root)
    return out


def broadcast_order(root: int, parent: Sequence[int], ch: Optional[List[List[int]]] = None) -> List[int]:
    """Non-root vertices in breadth-first order from the root (children
    ascending unless ``ch`` gives another order): the order of the
    parent->child transfers."""
    ch = children_of(parent) if ch is None else ch
    out: List[int] = []
    frontier = [root]
    while frontier:
        nxt: List[int] = []
        for v in frontier:
            for c in ch[v]:
                out.append(c)
                nxt.append(c)
        frontier = nxt
    return out


def make_steps(roots: Sequence[int], trees: Sequence[Sequence[int]],
               weights: Sequence[float], op: int, n: int, chunk: int) -> List[Step]:
    """The whole step list: tree by tree, chunk by chunk, reduce phase then
    broadcast phase.  Dependencies name the steps that produce a step's inputs:

    REDUCE v->p waits for the REDUCE out of v's last child (v then holds the
    sum of its subtree, because siblings are chained) and for the REDUCE of
    p's previous child (in-place accumulation in ascending child order).
    COPY p->v waits for the COPY into p, or, when p is the root, for the last
    REDUCE into the root (none for a plain Broadcast)."""
    bounds = split_by_weight(n, weights)
    steps: List[Step] = []
    for t, (root, parent) in enumerate(zip(roots, trees)):
        emit_tree_steps(steps, t, root, parent, children_of(parent), op, bounds[t], bounds[t + 1], chunk)
    return steps


def emit_tree_steps(steps: List[Step], t: int, root: int, parent: Sequence[int],
                    ch: List[List[int]], op: int, lo: int, hi: int, chunk: int) -> None:
    """Append the steps of one tree on the range [lo, hi), chunk by chunk.  ``ch``
    lists every vertex's children in the order they are folded in."""
    for c, (off, ln) in enumerate(chunk_ranges(lo, hi, chunk)):
        red: Dict[int, int] = {}   # vertex -> index of its REDUCE-out step
        cp: Dict[int, int] = {}    # vertex -> index of the COPY into it
        if op in (ALLREDUCE, REDUCE_TO_ROOT):
            for v in reduce_order(root, parent, ch):
                p = parent[v]
                deps = []
                if ch[v]:
                    deps.append(red[ch[v][-1]])
                i = ch[p].index(v)
                if i > 0:
                    deps.append(red[ch[p][i - 1]])
                red[v] = len(steps)
                steps.append(Step(REDUCE, t, c, v, p, off, ln, tuple(deps)))
        for v in (broadcast_order(root, parent, ch) if op != REDUCE_TO_ROOT else []):
            p = parent[v]
            if p != root:
                deps = (cp[p],)
            elif op == ALLREDUCE:
                deps = (red[ch[root][-1]],)
            else:
                deps = ()
            cp[v] = len(steps)
            steps.append(Step(COPY, t, c, p, v, off, ln, deps))


# --------------------------------------------------------------------------
# Gather and AllGather (section 4.1 derives them from the collectives above: a
# gather runs a broadcast backwards, an all-gather is an all-reduce that only
# moves data)
# --------------------------------------------------------------------------
# Every rank buffer has n = k * m elements; rank j owns piece j = [j*m, (j+1)*m)
# and starts with it in place.  Each piece is split among the trees by weight
# like any payload, and tree t moves its share of piece j along its own edges:
#   * AllReduce without a reduction: what travels up to the root and back down
#     is the data itself, so piece j simply spreads from rank j over the
#     (undirected) tree, hop by hop, each rank forwarding a chunk once it has
#     all of it: a broadcast along the tree re-rooted at j;
#   * Gather: piece j climbs from rank j to the tree's root along the reverse of
#     the path Broadcast would use to reach j.
def reroot(parent: Sequence[int], new_root: int) -> Tuple[int, ...]:
    """The same undirected tree with every edge directed away from new_root."""
    k = len(parent)
    nbrs: List[List[int]] = [[] for _ in range(k)]
    for v, p in enumerate(parent):
        if p >= 0:
            nbrs[v].append(p)
            nbrs[p].append(v)
    out = [-2] * k
    out[new_root] = -1
    stack = [new_root]
    while stack:
        u = stack.pop()
        for v in nbrs[u]:
            if out[v] == -2:
                out[v] = u
                stack.append(v)
    return tuple(out)


def climb(parent: Sequence[int], j: int) -> Tuple[int, ...]:
    """Flow of piece j towards the root of ``parent``: j first, then its
    ancestors, each receiving from the one below; ranks off the path take no
    part (-2)."""
    out = [-2] * len(parent)
    out[j] = -1
    v = j
    while parent[v] >= 0:
        out[parent[v]] = v
        v = parent[v]
    return tuple(out)


def make_gather_steps(roots: Sequence[int], trees: Sequence[Sequence[int]],
                      weights: Sequence[float], op: int, n: int, chunk: int) -> List[Step]:
    """Step list of AllGather / Gather on buffers of n = k*m elements: only COPY
    steps; a COPY u->v of a piece's chunk waits for the COPY that brought that
    chunk into u (none when u owns the piece)."""
    k = len(trees[0])
    if n % k:
        raise ValueError("the buffer length must be a multiple of the number of ranks")
    m = n // k
    bounds = split_by_weight(m, weights)
    steps: List[Step] = []
    for t, (root, parent) in enumerate(zip(roots, trees)):
        for j in range(k):
            flow = reroot(parent, j) if op == ALLGATHER else climb(parent, j)
            lo, hi = j * m + bounds[t], j * m + bounds[t + 1]
            for c, (off, ln) in enumerate(chunk_ranges(lo, hi, chunk)):
                into: Dict[int, int] = {}
                for v in broadcast_order(j, [p if p >= 0 else -1 for p in flow]):
                    p = flow[v]
                    deps = (into[p],) if p != j else ()
                    into[v] = len(steps)
                    steps.append(Step(COPY, t, c, p, v, off, ln, deps))
    return steps


def check_gather_steps(steps: Sequence[Step], k: int, roots: Sequence[int],
                       trees: Sequence[Sequence[int]], weights: Sequence[float], op: int,
                       n: int, chunk: int) -> None:
    """For any scheduler's AllGather / Gather list: dependencies point backwards;
    per tree and piece the chunks tile the tree's share of the piece; every step
    is a COPY over a tree edge (either direction); replaying with symbolic
    contents, every step forwards a chunk its dependencies have delivered, and
    at the end every rank (AllGather) or the tree's root (Gather) holds piece
    j's data there, each rank having received it exactly once."""
    assert n % k == 0
    m = n // k
    bounds = split_by_weight(m, weights)
    for i, s in enumerate(steps):
        assert s.kind == COPY and all(0 <= d < i for d in s.deps)
    groups: Dict[Tuple[int, int, int], List[int]] = {}
    for i, s in enumerate(steps):
        groups.setdefault((s.tree, s.off // m if m else 0, s.chunk), []).append(i)
    for t, (root, parent) in enumerate(zip(roots, trees)):
        edges = {(parent[v], v) for v in range(k) if v != root} | {(v, parent[v]) for v in range(k) if v != root}
        for j in range(k):
            want = chunk_ranges(j * m + bounds[t], j * m + bounds[t + 1], chunk)
            if op == GATHER and j == root:
                want = []                          # the root's own piece is already in place
            got = sorted({(steps[ix[0]].off, steps[ix[0]].len) for (tt, jj, _), ix in groups.items()
                          if tt == t and jj == j})
            assert got == want, f"tree {t} piece {j}: chunks {got[:2]} do not tile {want[:2]}"
            for (tt, jj, c), ix in groups.items():
                if (tt, jj) != (t, j):
                    continue
                assert all((steps[i].off, steps[i].len) == (steps[ix[0]].off, steps[ix[0]].len) for i in ix), \
                    f"tree {t} piece {j} chunk {c}: steps disagree on the range"
                has = {j: -1}                      # rank -> step that delivered the chunk (-1: owner)
                closure: Dict[int, set] = {}
                for i in ix:
                    s = steps[i]
                    assert (s.src, s.dst) in edges, f"step {i} does not follow a tree edge"
                    cl = set()
                    for d in s.deps:
                        cl |= {d} | closure.get(d, set())
                    closure[i] = cl
                    assert s.src in has, f"step {i} forwards a chunk rank {s.src} does not hold"
                    assert has[s.src] == -1 or has[s.src] in cl, f"step {i} is not ordered after its input"
                    assert s.dst not in has, f"rank {s.dst} receives piece {j} twice"
                    has[s.dst] = i
                if op == ALLGATHER:
                    assert set(has) == set(range(k)), f"tree {t} piece {j} chunk {c}: not everywhere"
                else:
                    path = {j}
                    v = j
                    while parent[v] >= 0:
                        v = parent[v]
                        path.add(v)
                    assert set(has) == path, f"tree {t} piece {j} chunk {c}: {sorted(has)} is not the path to the root"


# --------------------------------------------------------------------------
# validators for ANY scheduler's step list
# --------------------------------------------------------------------------
def check_split(bounds: Sequence[int], n: int, weights: Sequence[float], align: int = 4) -> None:
    """Shares are contiguous, disjoint, cover [0, n) and are within one
    alignment unit of n * w_t / W."""
    T = len(weights)
    assert len(bounds) == T + 1 and bounds[0] == 0 and bounds[-1] == n
    W = sum(Fraction(w) for w in weights)
    for t in range(T):
        assert bounds[t] <= bounds[t + 1]
        if 0 < t:
            assert bounds[t] % align == 0 or bounds[t] == n
        ideal = n * Fraction(weights[t]) / W
        assert abs((bounds[t + 1] - bounds[t]) - ideal) < align + 1, (t, bounds, float(ideal))


def check_steps(steps: Sequence[Step], k: int, roots: Sequence[int],
                trees: Sequence[Sequence[int]], weights: Sequence[float], op: int,
                n: int, chunk: int) -> None:
    """Structural checks on a step list produced by anyone:
      * dependencies point backwards (hence the graph is acyclic);
      * per tree the chunks tile the tree's share exactly once;
      * per (tree, chunk): exactly one COPY per tree arc parent->child
        (Broadcast, AllReduce) and exactly one REDUCE per reversed arc
        child->parent (AllReduce, Reduce);
      * replaying the list in order with symbolic contents gives, at every
        rank, the tree-order sum over all ranks (AllReduce) or the root's
        value (Broadcast), or the tree-order sum at the root (Reduce), and every
        step reads only values its listed dependencies (transitively) made
        final."""
    bounds = split_by_weight(n, weights)
    for i, s in enumerate(steps):
        assert all(0 <= d < i for d in s.deps), f"step {i}: dependency not earlier"
        assert 0 <= s.src < k and 0 <= s.dst < k and s.src != s.dst
    by_tc: Dict[Tuple[int, int], List[int]] = {}
    for i, s in enumerate(steps):
        by_tc.setdefault((s.tree, s.chunk), []).append(i)
    for t, (root, parent) in enumerate(zip(roots, trees)):
        want = chunk_ranges(bounds[t], bounds[t + 1], chunk)
        got = sorted({(steps[ix[0]].off, steps[ix[0]].len) for (tt, _), ix in by_tc.items() if tt == t})
        assert got == want, f"tree {t}: chunks {got[:3]}.. do not tile {want[:3]}.."
        arcs = sorted((parent[v], v) for v in range(k) if v != root)
        for (tt, c), ix in by_tc.items():
            if tt != t:
                continue
            off, ln = steps[ix[0]].off, steps[ix[0]].len
            assert all(steps[i].off == off and steps[i].len == ln for i in ix)
            copies = sorted((steps[i].src, steps[i].dst) for i in ix if steps[i].kind == COPY)
            reduces = sorted((steps[i].dst, steps[i].src) for i in ix if steps[i].kind == REDUCE)
            assert copies == (arcs if op != REDUCE_TO_ROOT else []), \
                f"tree {t} chunk {c}: COPY steps do not match the tree arcs"
            assert reduces == (arcs if op != BROADCAST else []), \
                f"tree {t} chunk {c}: REDUCE steps do not match the reversed tree arcs"
            _symbolic_replay(steps, ix, k, root, parent, op)


def _tree_order_expr(v: int, ch: List[List[int]]):
    """Nested tuple standing for ((x_v + S(c1)) + S(c2)) + ..."""
    e = ("x", v)
    for c in ch[v]:
        e = ("+", e, _tree_order_expr(c, ch))
    return e


def _symbolic_replay(steps, idx, k, root, parent, op, ch=None) -> None:
    """Run one (tree, chunk)'s steps on symbolic values.  Each rank's cell holds
    (expression, index of the step that wrote it or -1).  A step may only read a
    cell whose writer is among its transitive dependencies, and may only
    overwrite a cell whose earlier readers are among them too.  ``ch``: the
    children in folding order when that is not ascending id."""
    ch = children_of(parent) if ch is None else ch
    val = [(("x", v), -1) for v in range(k)]
    readers: List[List[int]] = [[] for _ in range(k)]
    closure: Dict[int, set] = {}
    for i in idx:
        s = steps[i]
        cl = set()
        for d in s.deps:
            cl.add(d)
            cl |= closure.get(d, set())
        closure[i] = cl
        reads = [s.src] + ([s.dst] if s.kind == REDUCE else [])
        for r in reads:
            w = val[r][1]
            assert w == -1 or w in cl, f"step {i} reads rank {r} before step {w} is ordered"
        for rd in readers[s.dst]:
            assert rd in cl, f"step {i} overwrites rank {s.dst} while step {rd} may still read it"
        w = val[s.dst][1]
        assert w == -1 or w in cl, f"step {i} overwrites rank {s.dst} unordered with its writer {w}"
        if s.kind == REDUCE:
            val[s.dst] = (("+", val[s.dst][0], val[s.src][0]), i)
        else:
            val[s.dst] = (val[s.src][0], i)
        readers[s.dst] = []
        readers[s.src].append(i)
    want = _tree_order_expr(root, ch) if op != BROADCAST else ("x", root)
    for v in (range(k) if op != REDUCE_TO_ROOT else [root]):
        assert val[v][0] == want, f"rank {v} ends with {val[v][0]}, expected {want}"


def link_timeline(steps: Sequence[Step]) -> List[int]:
    """Start time of every step when each takes one time unit, starts once its
    dependencies are done, and a directed link (src, dst) carries one step at a
    time, serving the steps that use it in list order (what a stream per link
    does, sections 4.1 and 4.2.2)."""
    start: List[int] = []
    link_free: Dict[Tuple[int, int], int] = {}
    for s in steps:
        at = max([start[d] + 1 for d in s.deps] + [link_free.get((s.src, s.dst), 0)])
        start.append(at)
        link_free[(s.src, s.dst)] = at + 1
    return start


def pipeline_makespan(steps: Sequence[Step]) -> int:
    """Length, in unit chunk-transfer times, of the schedule under link_timeline.
    Used for the chunking claim of section 4.2.1 (h hops, c equal chunks:
    h + c - 1)."""
    start = link_timeline(steps)
    return max(start) + 1 if start else 0


def fair_order(steps: Sequence[Step]) -> List[Step]:
    """Section 4.2.2: where trees share a link a fair scheme sends one chunk of
    the first tree, then one chunk of the second, and so on.  The same steps
    with the chunks of all trees taking turns: chunk 0 of every tree, then chunk
    1 of every tree, ...; inside one (tree, chunk) the order is kept, so the
    dependencies (which never leave a (tree, chunk)) still point backwards."""
    order = sorted(range(len(steps)), key=lambda i: (steps[i].chunk, steps[i].tree, i))
    new_index = {old: new for new, old in enumerate(order)}
    return [Step(steps[i].kind, steps[i].tree, steps[i].chunk, steps[i].src, steps[i].dst, steps[i].off,
                 steps[i].len, tuple(new_index[d] for d in steps[i].deps)) for i in order]


def chunk_finish_times(steps: Sequence[Step]) -> Dict[Tuple[int, int], int]:
    """(tree, chunk) -> time at which the last step of that chunk is done, under
    link_timeline."""
    start = link_timeline(steps)
    out: Dict[Tuple[int, int], int] = {}
    for s, at in zip(steps, start):
        key = (s.tree, s.chunk)
        out[key] = max(out.get(key, 0), at + 1)
    return out


def longest_idle_gap(steps: Sequence[Step], link: Tuple[int, int]) -> int:
    """The longest time a link sits idle between two steps it carries (or before
    its first one), under link_timeline: the "gap in the forwarding pipeline" an
    unfair order opens downstream of a shared link (section 4.2.2)."""
    times = sorted(at for s, at in zip(steps, link_timeline(steps)) if (s.src, s.dst) == link)
    gaps = [times[0]] + [b - a - 1 for a, b in zip(times, times[1:])] if times else [0]
    return max(gaps)
