"""Pins for oracle/schedule.py.  CPU only."""
import dataclasses
from fractions import Fraction

import numpy as np
import pytest

import synth_inputs as si
from oracle import graph as og
from oracle import packing as op
from oracle import schedule as osch


def trees_for(top, root=0):
    g = og.Digraph.from_topology(top)
    return op.pack_trees(g, root)


# ---- weighted split -----------------------------------------------------------
def test_split_paper_example(paper_pins):
    """1000 MB over six equal trees: 166 MB each (section 3.2.1)."""
    n = int(paper_pins["split_total_MB"]) * 10**6 // 4
    b = osch.split_by_weight(n, [1.0] * 6)
    osch.check_split(b, n, [1.0] * 6)
    for t in range(6):
        assert (b[t + 1] - b[t]) * 4 // 10**6 == int(paper_pins["split_per_tree_MB"])


def test_split_k4_shares():
    b = osch.split_by_weight(1 << 20, [1.0, 1.0, 1.0])
    assert [b[i + 1] - b[i] for i in range(3)] == [349524, 349524, 349528]


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 17, 1000, 4099, 1 << 20])
@pytest.mark.parametrize("w", [[1.0], [1.0, 1.0], [0.5, 0.25, 0.25], [2.0, 1.0, 1.0, 0.5], [1 / 16] * 16])
def test_split_covers_exactly_once_and_is_proportional(n, w):
    b = osch.split_by_weight(n, w)
    osch.check_split(b, n, w)
    cover = np.zeros(n, np.int32)
    for t in range(len(w)):
        cover[b[t]:b[t + 1]] += 1
    assert (cover == 1).all()
    assert all(x % 4 == 0 for x in b[:-1])


def test_chunks_tile_each_share_exactly_once():
    for lo, hi, c in [(0, 10, 3), (8, 8, 4), (4, 100, 4), (0, 7, 100), (12, 13, 1)]:
        r = osch.chunk_ranges(lo, hi, c)
        cover = np.zeros(hi, np.int32)
        for off, ln in r:
            assert 0 < ln <= c
            cover[off:off + ln] += 1
        assert (cover[lo:hi] == 1).all() and (cover[:lo] == 0).all()
        assert all(ln == c for _, ln in r[:-1])
    with pytest.raises(ValueError):
        osch.chunk_ranges(0, 4, 0)


# ---- step list ----------------------------------------------------------------------
CASES = [
    (si.complete_graph(4), 0, 1 << 12, 1 << 9),
    (si.hybrid_cube_mesh(), 0, 40_004, 4096),
    (si.hybrid_cube_mesh(doubled=True), 3, 10_001, 512),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (2, 3, 5, 6, 7)), 0, 9_999, 1000),
    (si.chain(5), 2, 1000, 64),
    (si.star(6, 1), 1, 1000, 300),
]


@pytest.mark.parametrize("top,root,n,chunk", CASES)
@pytest.mark.parametrize("coll", [osch.ALLREDUCE, osch.BROADCAST])
def test_step_list_passes_validators_and_counts(top, root, n, chunk, coll, paper_pins):
    roots, trees, w = trees_for(top, root)
    steps = osch.make_steps(roots, trees, w, coll, n, chunk)
    osch.check_steps(steps, top.k, roots, trees, w, coll, n, chunk)
    # 2(N-1) transfers per chunk per tree for AllReduce, N-1 for Broadcast (section 3.3)
    assert paper_pins["allreduce_transfers_per_tree"] == "2*(N-1)"
    per = {}
    for s in steps:
        per[(s.tree, s.chunk)] = per.get((s.tree, s.chunk), 0) + 1
    want = (2 if coll == osch.ALLREDUCE else 1) * (top.k - 1)
    assert set(per.values()) == {want}
    b = osch.split_by_weight(n, w)
    n_chunks = sum(len(osch.chunk_ranges(b[t], b[t + 1], chunk)) for t in range(len(trees)))
    assert len(per) == n_chunks
    assert all(len(s.deps) <= 2 for s in steps)


def test_headline_step_count():
    roots, trees, w = trees_for(si.hybrid_cube_mesh(), 0)
    assert len(trees) == 4 and w == [1.0] * 4
    steps = osch.make_steps(roots, trees, w, osch.ALLREDUCE, 1 << 26, 1 << 18)
    assert len(steps) == 4 * 64 * 14


def test_one_hop_star_schedule():
    g = og.Digraph.from_topology(si.complete_graph(16))
    roots, trees, w = op.one_hop_stars(g)
    n, c = 16 * 4096, 1024
    steps = osch.make_steps(roots, trees, w, osch.ALLREDUCE, n, c)
    osch.check_steps(steps, 16, roots, trees, w, osch.ALLREDUCE, n, c)
    assert len(steps) == 16 * 4 * 30


# ---- planted mistakes must be caught ----------------------------------------------------
def _mutate(steps, i, **kw):
    out = list(steps)
    out[i] = dataclasses.replace(out[i], **kw)
    return out


def test_validators_catch_planted_mistakes():
    top = si.hybrid_cube_mesh()
    roots, trees, w = trees_for(top, 0)
    n, c = 8192, 1024
    steps = osch.make_steps(roots, trees, w, osch.ALLREDUCE, n, c)
    args = (top.k, roots, trees, w, osch.ALLREDUCE, n, c)
    osch.check_steps(steps, *args)
    # a dropped dependency
    i = next(i for i, s in enumerate(steps) if s.kind == osch.REDUCE and len(s.deps) == 2)
    with pytest.raises(AssertionError):
        osch.check_steps(_mutate(steps, i, deps=steps[i].deps[:1]), *args)
    with pytest.raises(AssertionError):
        osch.check_steps(_mutate(steps, i, deps=steps[i].deps[1:]), *args)
    # a COPY released before the root has the full sum
    j = next(i for i, s in enumerate(steps) if s.kind == osch.COPY)
    with pytest.raises(AssertionError):
        osch.check_steps(_mutate(steps, j, deps=()), *args)
    # transposed operands
    with pytest.raises(AssertionError):
        osch.check_steps(_mutate(steps, i, src=steps[i].dst, dst=steps[i].src), *args)
    # wrong offset / short length
    with pytest.raises(AssertionError):
        osch.check_steps(_mutate(steps, i, off=steps[i].off + 4), *args)
    with pytest.raises(AssertionError):
        osch.check_steps(_mutate(steps, i, len=steps[i].len - 1), *args)
    # a missing step
    with pytest.raises(AssertionError):
        osch.check_steps(steps[:-1], *args)
    # forward dependency
    with pytest.raises(AssertionError):
        osch.check_steps(_mutate(steps, 0, deps=(5,)), *args)
    # children folded in the wrong order: swap two sibling REDUCEs of one chunk
    sib = [(a, b) for a in range(14) for b in range(a + 1, 14)
           if steps[a].kind == steps[b].kind == osch.REDUCE and steps[a].dst == steps[b].dst]
    assert sib
    a, b = sib[0]
    wrong = list(steps)
    wrong[a] = dataclasses.replace(steps[b], deps=steps[a].deps)
    wrong[b] = dataclasses.replace(steps[a], deps=steps[b].deps)
    with pytest.raises(AssertionError):
        osch.check_steps(wrong, *args)


# ---- chunking shortens the pipeline (section 4.2.1) ----------------------------------------
def test_two_chunks_on_a_four_gpu_chain_save_a_third(paper_pins):
    gpus = int(paper_pins["chain_gpus"])
    chunks = int(paper_pins["chain_chunks"])
    saved = Fraction(paper_pins["chain_time_saved"])
    parent = tuple([-1] + list(range(gpus - 1)))
    n = 1 << 12
    one = osch.make_steps([0], [parent], [1.0], osch.BROADCAST, n, n)
    many = osch.make_steps([0], [parent], [1.0], osch.BROADCAST, n, n // chunks)
    t_one = osch.pipeline_makespan(one) * Fraction(1)
    t_many = osch.pipeline_makespan(many) * Fraction(1, chunks)
    assert 1 - t_many / t_one == saved


@pytest.mark.parametrize("hops,chunks", [(1, 1), (3, 1), (3, 2), (7, 16), (5, 64)])
def test_chain_makespan_is_hops_plus_chunks_minus_one(hops, chunks):
    parent = tuple([-1] + list(range(hops)))
    steps = osch.make_steps([0], [parent], [1.0], osch.BROADCAST, 64 * chunks, 64)
    assert osch.pipeline_makespan(steps) == hops + chunks - 1
    steps = osch.make_steps([0], [parent], [1.0], osch.ALLREDUCE, 64 * chunks, 64)
    assert osch.pipeline_makespan(steps) == 2 * hops + chunks - 1


# ---- Gather and AllGather (section 4.1) -----------------------------------------------------
def test_reroot_and_climb():
    parent = (-1, 0, 0, 2, 2)            # 0 -> {1, 2}, 2 -> {3, 4}
    assert osch.reroot(parent, 0) == parent
    assert osch.reroot(parent, 3) == (2, 0, 3, -1, 2)
    assert osch.reroot(osch.reroot(parent, 4), 0) == parent
    assert osch.climb(parent, 3) == (2, -2, 3, -1, -2)
    assert osch.climb(parent, 0) == (-1, -2, -2, -2, -2)


GATHER_CASES = [(si.hybrid_cube_mesh(), 0, 8 * 1001, 300), (si.complete_graph(4), 2, 4 * 64, 64),
                (si.chain(5), 1, 5 * 777, 100), (si.star(6, 0), 0, 6 * 10, 4)]


@pytest.mark.parametrize("top,root,n,chunk", GATHER_CASES)
def test_allgather_steps(top, root, n, chunk):
    roots, trees, w = trees_for(top, root)
    k = top.k
    steps = osch.make_gather_steps(roots, trees, w, osch.ALLGATHER, n, chunk)
    osch.check_gather_steps(steps, k, roots, trees, w, osch.ALLGATHER, n, chunk)
    # every rank other than the owner receives every piece once: k(k-1) copies per tree and chunk position
    m = n // k
    b = osch.split_by_weight(m, w)
    per_piece_chunks = sum(len(osch.chunk_ranges(b[t], b[t + 1], chunk)) for t in range(len(trees)))
    assert len(steps) == k * (k - 1) * per_piece_chunks
    # "AllReduce without a reduction": the directed edges in use are the tree's edges in both directions
    for t, (r, parent) in enumerate(zip(roots, trees)):
        used = {(s.src, s.dst) for s in steps if s.tree == t}
        arcs = {(parent[v], v) for v in range(k) if v != r}
        assert used == arcs | {(b_, a) for (a, b_) in arcs}


@pytest.mark.parametrize("top,root,n,chunk", GATHER_CASES)
def test_gather_is_the_inverse_of_broadcast(top, root, n, chunk):
    roots, trees, w = trees_for(top, root)
    k = top.k
    steps = osch.make_gather_steps(roots, trees, w, osch.GATHER, n, chunk)
    osch.check_gather_steps(steps, k, roots, trees, w, osch.GATHER, n, chunk)
    bc = osch.make_steps(roots, trees, w, osch.BROADCAST, n // k, chunk)
    for t in range(len(trees)):
        assert {(s.dst, s.src) for s in steps if s.tree == t} == {(s.src, s.dst) for s in bc if s.tree == t}
    # piece j makes depth(j) hops
    for t, (r, parent) in enumerate(zip(roots, trees)):
        for j in range(k):
            depth, v = 0, j
            while parent[v] >= 0:
                v, depth = parent[v], depth + 1
            hops = {(s.src, s.dst) for s in steps if s.tree == t and s.off // (n // k) == j}
            assert len(hops) == depth


def test_gather_validators_catch_planted_mistakes():
    top = si.hybrid_cube_mesh()
    roots, trees, w = trees_for(top, 0)
    n, c = 8 * 512, 128
    steps = osch.make_gather_steps(roots, trees, w, osch.ALLGATHER, n, c)
    args = (8, roots, trees, w, osch.ALLGATHER, n, c)
    osch.check_gather_steps(steps, *args)
    i = next(i for i, s in enumerate(steps) if s.deps)
    for bad in (_mutate(steps, i, deps=()), _mutate(steps, i, src=steps[i].dst, dst=steps[i].src),
                _mutate(steps, i, off=steps[i].off + 4), steps[:-1], _mutate(steps, i, kind=osch.REDUCE)):
        with pytest.raises(AssertionError):
            osch.check_gather_steps(bad, *args)
    with pytest.raises(ValueError):
        osch.make_gather_steps(roots, trees, w, osch.ALLGATHER, 8 * 512 + 1, c)
