"""Seeded synthetic inputs: interconnect topologies and rank payloads.

This module is shared by the CPU oracle's tests, the GPU parity tests and the
benchmark.  It holds no arithmetic of the method itself (no packing, no
splitting, no reduction): it only describes graphs and draws random payloads.

Topologies are returned as ``Topology`` records: ``k`` vertices and arrays
``src``, ``dst``, ``cap`` of directed arcs (a bidirectional link is two arcs),
the graph model of the paper's section 3.1.

Payloads come from a counter-style recipe: block ``b`` of rank ``r`` under seed
``s`` is drawn from ``numpy.random.default_rng([s, r, b])`` in blocks of
``BLOCK`` elements, so any slice can be regenerated without holding the rest.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterable, List, Sequence, Tuple

import numpy as np

BLOCK = 1 << 20  # elements per independently seeded block


# --------------------------------------------------------------------------
# topologies
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Topology:
    k: int
    src: np.ndarray  # int32 [m]
    dst: np.ndarray  # int32 [m]
    cap: np.ndarray  # float64 [m]
    name: str = ""

    @property
    def m(self) -> int:
        return int(self.src.shape[0])

    def arcs(self) -> List[Tuple[int, int, float]]:
        return [(int(u), int(v), float(c)) for u, v, c in zip(self.src, self.dst, self.cap)]


def _from_links(k: int, links: Iterable[Tuple[int, int, float]], name: str) -> Topology:
    """Each undirected link (a, b, c) becomes arcs a->b and b->a of capacity c."""
    src, dst, cap = [], [], []
    for a, b, c in links:
        src += [a, b]
        dst += [b, a]
        cap += [c, c]
    return Topology(k, np.asarray(src, np.int32), np.asarray(dst, np.int32),
                    np.asarray(cap, np.float64), name)


def complete_graph(k: int, cap: float = 1.0) -> Topology:
    """Fully connected k-vertex graph (also the model of a non-blocking switch)."""
    links = [(a, b, cap) for a in range(k) for b in range(a + 1, k)]
    return _from_links(k, links, f"K{k}")


def chain(k: int, cap: float = 1.0) -> Topology:
    """0 - 1 - ... - (k-1), the depth-test topology of the paper's section 2.2."""
    return _from_links(k, [(i, i + 1, cap) for i in range(k - 1)], f"chain{k}")


def star(k: int, center: int = 0, cap: float = 1.0) -> Topology:
    """One centre linked to every other vertex (fan-in / fan-out test)."""
    return _from_links(k, [(center, i, cap) for i in range(k) if i != center], f"star{k}")


def ring(k: int, cap: float = 1.0) -> Topology:
    return _from_links(k, [(i, (i + 1) % k, cap) for i in range(k)], f"ring{k}")


def cube_mesh_links(doubled: bool) -> List[Tuple[int, int, float]]:
    """Hybrid cube-mesh on 8 vertices: {0..3} and {4..7} all-to-all, i <-> i+4.

    ``doubled`` gives capacity 2 to links 0-1, 2-3, 4-5, 6-7 and i <-> i+4 (six
    link-units into every vertex, as on the second-generation server the paper
    describes in its figure of the hybrid mesh-cube topology); otherwise every
    link has capacity 1.
    """
    links = []
    for base in (0, 4):
        for a in range(base, base + 4):
            for b in range(a + 1, base + 4):
                two = doubled and (a, b) in ((0, 1), (2, 3), (4, 5), (6, 7))
                links.append((a, b, 2.0 if two else 1.0))
    for i in range(4):
        links.append((i, i + 4, 2.0 if doubled else 1.0))
    return links


def hybrid_cube_mesh(doubled: bool = False) -> Topology:
    return _from_links(8, cube_mesh_links(doubled),
                       "cube_mesh_doubled" if doubled else "cube_mesh")


def dgx1v() -> Topology:
    """The 8-GPU second-generation server with its actual link multiplicities:
    the hybrid cube-mesh's 16 links, eight of them doubled (0-3, 0-4, 1-2, 1-5,
    2-3, 4-7, 5-6, 6-7), six link-units per GPU.  The paper's text does not list
    which links are doubled (its figure is not available); this assignment
    reproduces the paper's count of 46 distinct connected 3- to 8-GPU
    allocations, which ``hybrid_cube_mesh(doubled=True)`` (22) does not."""
    two = [(0, 3), (0, 4), (1, 2), (1, 5), (2, 3), (4, 7), (5, 6), (6, 7)]
    one = [(0, 1), (0, 2), (1, 3), (2, 6), (3, 7), (4, 5), (4, 6), (5, 7)]
    return _from_links(8, [(a, b, 2.0) for a, b in two] + [(a, b, 1.0) for a, b in one], "dgx1v")


def connected_allocations(top: Topology, sizes: Sequence[int] = (3, 4, 5, 6, 7, 8)) -> List[Tuple[int, ...]]:
    """All vertex subsets of the given sizes whose induced sub-topology is connected."""
    import itertools
    linked = {(int(u), int(v)) for u, v in zip(top.src, top.dst)}
    out = []
    for size in sizes:
        for sub in itertools.combinations(range(top.k), size):
            seen, stack = {sub[0]}, [sub[0]]
            while stack:
                x = stack.pop()
                for y in sub:
                    if y not in seen and (x, y) in linked:
                        seen.add(y)
                        stack.append(y)
            if len(seen) == size:
                out.append(sub)
    return out


def distinct_allocations(top: Topology, subsets: Sequence[Tuple[int, ...]]) -> List[Tuple[int, ...]]:
    """One subset (the first in the given order) of every class of subsets that
    are equal up to relabelling (same links with the same capacities): the
    class is named by the smallest capacity matrix over all vertex orders
    (brute force, <= 8 vertices)."""
    import itertools
    cap = {(int(u), int(v)): float(c) for u, v, c in zip(top.src, top.dst, top.cap)}
    forms = {}
    for sub in subsets:
        best = None
        for perm in itertools.permutations(sub):
            key = tuple(cap.get((perm[i], perm[j]), 0.0) for i in range(len(sub)) for j in range(i + 1, len(sub)))
            if best is None or key < best:
                best = key
        forms.setdefault((len(sub), best), sub)
    return list(forms.values())


def count_distinct_allocations(top: Topology, subsets: Sequence[Tuple[int, ...]]) -> int:
    """Number of subsets up to relabelling."""
    return len(distinct_allocations(top, subsets))


def induced(top: Topology, ranks: Sequence[int]) -> Topology:
    """Sub-topology on ``ranks`` (a fragmented allocation); vertices renumbered
    0..len(ranks)-1 in the order given."""
    pos = {int(r): i for i, r in enumerate(ranks)}
    keep = [i for i in range(top.m) if int(top.src[i]) in pos and int(top.dst[i]) in pos]
    src = np.asarray([pos[int(top.src[i])] for i in keep], np.int32)
    dst = np.asarray([pos[int(top.dst[i])] for i in keep], np.int32)
    cap = np.asarray([top.cap[i] for i in keep], np.float64)
    return Topology(len(ranks), src, dst, cap,
                    f"{top.name}[{','.join(str(r) for r in ranks)}]")


def random_digraph(k: int, p: float, seed: int, int_caps: bool = True,
                   max_cap: int = 3) -> Topology:
    """Random directed graph guaranteed connected from vertex 0: a random
    out-tree from 0 plus each other arc with probability p."""
    rng = np.random.default_rng([seed, k])
    arcs = {}
    order = list(rng.permutation(np.arange(1, k)))
    placed = [0]
    for v in order:
        u = placed[int(rng.integers(len(placed)))]
        arcs[(u, int(v))] = None
        placed.append(int(v))
    for u in range(k):
        for v in range(k):
            if u != v and rng.random() < p:
                arcs[(u, v)] = None
    src, dst, cap = [], [], []
    for (u, v) in sorted(arcs):
        src.append(u)
        dst.append(v)
        cap.append(float(rng.integers(1, max_cap + 1)) if int_caps
                   else float(rng.uniform(0.25, max_cap)))
    return Topology(k, np.asarray(src, np.int32), np.asarray(dst, np.int32),
                    np.asarray(cap, np.float64), f"rand{k}_{seed}")


# --------------------------------------------------------------------------
# payloads
# --------------------------------------------------------------------------
def payload_block(seed: int, rank: int, block: int, dist: str, dtype: str,
                  scale: float = 1.0, count: int = BLOCK) -> np.ndarray:
    """One seeded block of ``count`` (<= BLOCK) elements.

    dist: "uniform" (U[-scale, scale]), "normal" (N(0, sigma=scale)),
          "int" (full-range int32, exercises wrap-around).
    """
    rng = np.random.default_rng([seed, rank, block])
    if dtype == "int32":
        if dist != "int":
            raise ValueError("int32 payloads use dist='int'")
        return rng.integers(-(1 << 31), 1 << 31, size=count, dtype=np.int64).astype(np.int32)
    if dtype != "fp32":
        raise ValueError(dtype)
    if dist == "uniform":
        return ((rng.random(count, dtype=np.float32) * 2.0 - 1.0) * np.float32(scale)).astype(np.float32)
    if dist == "normal":
        return (rng.standard_normal(count, dtype=np.float32) * np.float32(scale)).astype(np.float32)
    raise ValueError(dist)


def payload(seed: int, rank: int, n: int, dist: str, dtype: str, scale: float = 1.0,
            start: int = 0) -> np.ndarray:
    """Elements [start, start+n) of rank ``rank``'s payload."""
    out = np.empty(n, np.int32 if dtype == "int32" else np.float32)
    pos = start
    end = start + n
    while pos < end:
        b = pos // BLOCK
        lo = pos - b * BLOCK
        take = min(end - pos, BLOCK - lo)
        blk = payload_block(seed, rank, b, dist, dtype, scale)
        out[pos - start:pos - start + take] = blk[lo:lo + take]
        pos += take
    return out


def bucket_sizes(total_elems: int = 138_000_000, n_buckets: int = 16, seed: int = 0,
                 lo_bytes: int = 64 << 10, hi_bytes: int = 400 << 20) -> List[int]:
    """Per-layer gradient buckets: byte sizes log-uniform in [lo, hi], rescaled to
    sum to total, clamped to the range, rounded to 4 elements, remainder to the
    largest bucket.  Returns element counts (fp32/int32)."""
    rng = np.random.default_rng([seed, 4040])
    b = np.exp(rng.uniform(np.log(lo_bytes), np.log(hi_bytes), n_buckets))
    b = b * (total_elems * 4.0 / b.sum())
    b = np.clip(b, lo_bytes, hi_bytes)
    e = (np.floor(b / 16.0).astype(np.int64)) * 4
    e[int(np.argmax(e))] += total_elems - int(e.sum())
    assert int(e.sum()) == total_elems and (e > 0).all()
    return [int(x) for x in e]


# --------------------------------------------------------------------------
# counter-based payloads: the same values from NumPy (any slice, on the host)
# and from torch (whole buffers, generated where they live)
# --------------------------------------------------------------------------
_M31 = (1 << 31) - 1


def _mix_numpy(seed: int, rank: int, idx: np.ndarray) -> np.ndarray:
    """31-bit hash of (seed, rank, element index); int64 arithmetic that never
    overflows (every product stays below 2^62), so NumPy and torch agree."""
    x = (idx.astype(np.int64) ^ np.int64((seed * 7919 + rank * 104729 + 12345) & _M31)) & _M31
    for mul, shift in ((1103515245, 13), (214013, 11), (69069, 15)):
        x = (x * np.int64(mul) + np.int64(12345)) & _M31
        x = x ^ (x >> shift)
    hi = (idx.astype(np.int64) >> 31) & _M31          # indices beyond 2^31 still differ
    x = ((x ^ hi) * np.int64(48271) + np.int64(11)) & _M31
    return x ^ (x >> 16)


def hash_payload(seed: int, rank: int, start: int, n: int, dtype: str) -> np.ndarray:
    """Elements [start, start+n): fp32 uniform on the grid k*2^-23 - 1 in [-1, 1),
    or int32 (31-bit hash shifted into the sign bit so that sums wrap)."""
    h = _mix_numpy(seed, rank, np.arange(start, start + n, dtype=np.int64))
    if dtype == "fp32":
        return ((h >> 7).astype(np.float32) * np.float32(2.0 ** -23) - np.float32(1.0)).astype(np.float32)
    if dtype == "int32":
        return ((h << 1) & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
    raise ValueError(dtype)


def hash_payload_torch(seed: int, rank: int, n: int, dtype: str, device, block: int = 1 << 24):
    """The same values as hash_payload(seed, rank, 0, n, dtype), generated by
    torch element-wise integer ops on `device` in blocks."""
    import torch
    out = torch.empty(n, dtype=torch.float32 if dtype == "fp32" else torch.int32, device=device)
    key = (seed * 7919 + rank * 104729 + 12345) & _M31
    for lo in range(0, n, block):
        hi_ = min(n, lo + block)
        idx = torch.arange(lo, hi_, dtype=torch.int64, device=device)
        x = (idx ^ key) & _M31
        for mul, shift in ((1103515245, 13), (214013, 11), (69069, 15)):
            x = (x * mul + 12345) & _M31
            x = x ^ (x >> shift)
        x = ((x ^ ((idx >> 31) & _M31)) * 48271 + 11) & _M31
        x = x ^ (x >> 16)
        if dtype == "fp32":
            out[lo:hi_] = (x >> 7).to(torch.float32) * (2.0 ** -23) - 1.0
        else:
            v = (x << 1) & 0xFFFFFFFF
            out[lo:hi_] = torch.where(v >= (1 << 31), v - (1 << 32), v).to(torch.int32)
    return out
