"""CPU oracle, part 4: what the collectives compute.

TEST INFRASTRUCTURE ONLY (see oracle/graph.py).  Shares no code with the HIP
library.

Broadcast and integer AllReduce have plain definitions (every rank ends with
the root's data / with the wrap-around sum of all ranks), written out below.
Floating-point AllReduce is the real-number sum evaluated in one specific
association order, the one the method's reduce phase produces (paper sections
3.3 and 4.1): inside tree t's share, S(v) = ((x_v + S(c_1)) + S(c_2)) + ... over
v's children in ascending id, and every rank ends with S(root_t).  It is given
twice: as that recursion (``tree_order_allreduce``) and as the literal
execution of a step list (``run_steps``); the tests require the two to agree
bit for bit.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from .graph import children_of
from .schedule import COPY, REDUCE, Step, split_by_weight

# Reduction operators (the paper's section 4.1 names min and max next to the sum
# and refers to "all the reduction functions" of the library it mirrors).
SUM, PROD, MIN, MAX = 0, 1, 2, 3


def _total_order_key(bits: np.ndarray) -> np.ndarray:
    """float32 bit patterns -> int32 keys whose signed order is the IEEE total
    order of the floats (-0 below +0); the map is its own inverse."""
    i = bits.view(np.int32)
    return i ^ ((i >> 31) & np.int32(0x7FFFFFFF))


def combine(a: np.ndarray, b: np.ndarray, redop: int) -> np.ndarray:
    """a (+) b element-wise.  a and b are float32, or uint32 views of int32 data.
    SUM/PROD: one rounded IEEE operation (float) or wrap-around modulo 2^32
    (integer).  MIN/MAX: the smaller/larger under the IEEE total order for
    floats (so the result does not depend on operand order even for signed
    zeros), signed comparison for integers."""
    if redop == SUM:
        return a + b
    if redop == PROD:
        return a * b
    if a.dtype == np.float32:
        ka, kb = _total_order_key(a.view(np.uint32)), _total_order_key(b.view(np.uint32))
        k = np.minimum(ka, kb) if redop == MIN else np.maximum(ka, kb)
        return _total_order_key(k.view(np.uint32)).view(np.float32)
    sa, sb = a.view(np.int32), b.view(np.int32)
    return (np.minimum(sa, sb) if redop == MIN else np.maximum(sa, sb)).view(np.uint32)


def run_steps(bufs: List[np.ndarray], steps: Sequence[Step],
              order: Optional[Sequence[int]] = None, redop: int = SUM) -> None:
    """Execute the step list in place on the rank buffers (1-D arrays of one
    dtype, float32 or int32).  ``order`` is any topological order of the steps
    (default: list order).  float32 adds round to nearest even once per add;
    int32 adds wrap modulo 2^32; other operators: see ``combine``."""
    is_int = bufs[0].dtype == np.int32
    views = [b.view(np.uint32) for b in bufs] if is_int else bufs
    for i in (range(len(steps)) if order is None else order):
        s = steps[i]
        a, b = s.off, s.off + s.len
        if s.kind == REDUCE:
            views[s.dst][a:b] = combine(views[s.dst][a:b], views[s.src][a:b], redop)
        elif s.kind == COPY:
            views[s.dst][a:b] = views[s.src][a:b]
        else:
            raise ValueError(s.kind)


def tree_order_allreduce(x: Sequence[np.ndarray], roots: Sequence[int],
                         trees: Sequence[Sequence[int]], weights: Sequence[float],
                         redop: int = SUM) -> np.ndarray:
    """The AllReduce result (identical at every rank) by the recursion over
    each tree, in the inputs' own dtype.  No chunks, no steps.  (For Reduce it
    is what the root of each tree ends with on that tree's share.)"""
    n = x[0].shape[0]
    is_int = x[0].dtype == np.int32
    xs = [a.view(np.uint32) if is_int else a for a in x]
    out = np.empty(n, xs[0].dtype)
    bounds = split_by_weight(n, weights)
    for t, (root, parent) in enumerate(zip(roots, trees)):
        lo, hi = bounds[t], bounds[t + 1]
        ch = children_of(parent)

        def S(v: int) -> np.ndarray:
            acc = xs[v][lo:hi].copy()
            for c in ch[v]:
                acc = combine(acc, S(c), redop)
            return acc

        out[lo:hi] = S(root)
    return out.view(np.int32) if is_int else out


def allreduce_int32_definition(x: Sequence[np.ndarray]) -> np.ndarray:
    """sum over ranks modulo 2^32, reinterpreted as int32."""
    acc = np.zeros(x[0].shape[0], np.uint64)
    for a in x:
        acc += a.view(np.uint32)
    return (acc & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.int32)


def reduce_definition(x: Sequence[np.ndarray], redop: int) -> np.ndarray:
    """Order-free operators written out as plain definitions: int32 SUM and PROD
    modulo 2^32 in unbounded Python-width arithmetic, MIN and MAX as the
    element-wise extreme (IEEE total order for float32).  float32 SUM and PROD
    have no order-free definition and are refused."""
    is_int = x[0].dtype == np.int32
    if redop in (MIN, MAX):
        if is_int:
            st = np.stack(x)
            return st.min(axis=0) if redop == MIN else st.max(axis=0)
        keys = np.stack([_total_order_key(a.view(np.uint32)) for a in x])
        k = keys.min(axis=0) if redop == MIN else keys.max(axis=0)
        return _total_order_key(k.view(np.uint32)).view(np.float32)
    if not is_int:
        raise ValueError("float32 sum/product depend on the association order")
    if redop == SUM:
        return allreduce_int32_definition(x)
    acc = np.ones(x[0].shape[0], np.uint64)
    for a in x:
        acc = (acc * a.view(np.uint32).astype(np.uint64)) & np.uint64(0xFFFFFFFF)
    return acc.astype(np.uint32).view(np.int32)


def allreduce_exact_f64(x: Sequence[np.ndarray]) -> np.ndarray:
    """Sum over ranks in float64 (k <= 16 float32 addends of similar magnitude:
    error far below one float32 ulp); the order-free yardstick for the
    recursive-summation error bound."""
    acc = np.zeros(x[0].shape[0], np.float64)
    for a in x:
        acc += a.astype(np.float64)
    return acc


def broadcast_definition(x: Sequence[np.ndarray], roots: Sequence[int],
                         weights: Sequence[float]) -> np.ndarray:
    """Every rank ends with the data of the tree roots: tree t's share comes
    from roots[t] (one common root in the ordinary case)."""
    n = x[0].shape[0]
    out = np.empty_like(x[0])
    bounds = split_by_weight(n, weights)
    for t, r in enumerate(roots):
        out[bounds[t]:bounds[t + 1]] = x[r][bounds[t]:bounds[t + 1]]
    return out


def random_topological_order(steps: Sequence[Step], seed: int) -> List[int]:
    """A uniformly shuffled order that still respects every dependency."""
    rng = np.random.default_rng(seed)
    n = len(steps)
    waiting = [len(s.deps) for s in steps]
    users: List[List[int]] = [[] for _ in range(n)]
    for i, s in enumerate(steps):
        for d in s.deps:
            users[d].append(i)
    ready = [i for i in range(n) if waiting[i] == 0]
    out: List[int] = []
    while ready:
        j = int(rng.integers(len(ready)))
        ready[j], ready[-1] = ready[-1], ready[j]
        i = ready.pop()
        out.append(i)
        for u in users[i]:
            waiting[u] -= 1
            if waiting[u] == 0:
                ready.append(u)
    assert len(out) == n
    return out


def allgather_definition(x: Sequence[np.ndarray]) -> np.ndarray:
    """Concatenation of the pieces: with k buffers of k*m elements, piece j is
    x[j][j*m:(j+1)*m]."""
    k = len(x)
    m = x[0].shape[0] // k
    return np.concatenate([x[j][j * m:(j + 1) * m] for j in range(k)])
