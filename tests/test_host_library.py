"""Host-side logic of the HIP library through its C ABI (no GPU, no kernels):
tree packing and scheduling, judged by the oracle's validators."""
import os
import re

import numpy as np
import pytest

import paper_1910_04940_amd as bl
import synth_inputs as si
from oracle import graph as og
from oracle import packing as op
from oracle import schedule as osch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def pack(top, root, **kw):
    return bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, root, **kw)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "blink.h")).read()
    declared = set(re.findall(r"\b(blink_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 19
    from paper_1910_04940_amd import binding
    lib = binding.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(binding.EXPORTS)


# ---- packing ---------------------------------------------------------------------
PACK_CASES = [
    (si.complete_graph(4), 0),
    (si.complete_graph(8), 5),
    (si.hybrid_cube_mesh(), 0),
    (si.hybrid_cube_mesh(), 6),
    (si.hybrid_cube_mesh(doubled=True), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 4)), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (2, 3, 5, 6, 7)), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 3, 4, 5, 7)), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (1, 4, 5, 6)), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (2, 3, 6, 7)), 0),
    (si.chain(7, 2.0), 3),
    (si.star(6, 2), 2),
    (si.ring(6), 0),
]


@pytest.mark.parametrize("top,root", PACK_CASES)
def test_integer_graphs_reach_the_min_root_cut_with_few_trees(top, root):
    g = og.Digraph.from_topology(top)
    lam = og.min_root_cut(g, root)
    trees = pack(top, root)
    roots, parents, w = trees.as_lists()
    rate = op.check_packing(g, roots, parents, w)
    assert rate == pytest.approx(trees.rate)
    assert rate == lam                      # Edmonds: integral capacities pack exactly
    assert trees.count <= lam               # no more trees than units of rate
    assert all(r == root for r in roots)


def test_dgx1v_graph_gives_six_unit_trees(paper_pins):
    trees = pack(si.hybrid_cube_mesh(doubled=True), 0)
    assert trees.count == int(paper_pins["dgx1v_pruned_tree_count"])
    assert all(w == float(paper_pins["dgx1v_pruned_tree_rate"]) for w in trees.as_lists()[2])


@pytest.mark.parametrize("seed", range(10))
def test_random_fractional_graphs_feasible_and_near_optimal(seed):
    top = si.random_digraph(5 + seed % 4, 0.45, 500 + seed, int_caps=False)
    g = og.Digraph.from_topology(top)
    lam = og.min_root_cut(g, 0)
    eps, tol = 0.05, 0.05
    trees = pack(top, 0, eps=eps, prune_tol=tol)
    roots, parents, w = trees.as_lists()
    rate = op.check_packing(g, roots, parents, w)
    assert rate <= lam + 1e-9
    assert rate >= (1 - tol) * (1 - 2 * eps) * lam
    # a vertex of the packing polytope over MWU's trees: at most one tree per arc
    assert trees.count <= g.m


@pytest.mark.parametrize("seed", range(40))
def test_fractional_capacities_still_give_few_trees(seed):
    """Capacities on no common grid: MWU spreads the rate over thousands of trees;
    what comes back must be a handful (never more than there are arcs) at a rate
    within the tolerance."""
    k = 4 + seed % 13
    top = si.random_digraph(k, 0.3 + 0.05 * (seed % 8), 4000 + seed, int_caps=False)
    g = og.Digraph.from_topology(top)
    try:
        trees = pack(top, 0)
    except bl.BlinkError as e:
        assert e.status == bl.BLINK_EDISCONNECTED
        return
    roots, parents, w = trees.as_lists()
    rate = op.check_packing(g, roots, parents, w)
    assert trees.count <= min(g.m, 40)
    if k <= 12:
        lam = og.min_root_cut(g, 0)
        assert (1 - 0.05) * (1 - 2 * 0.05) * lam <= rate <= lam + 1e-9


@pytest.mark.parametrize("seed", range(80))
def test_random_integer_graphs_reach_the_cut_exactly(seed):
    """Edmonds: with integer capacities an integral packing of value min root cut
    exists; the pruned packing must find one (300 of 300 random graphs did)."""
    k = 3 + seed % 10
    top = si.random_digraph(k, 0.35 + 0.05 * (seed % 7), 9000 + seed, int_caps=True)
    g = og.Digraph.from_topology(top)
    lam = og.min_root_cut(g, 0)
    if lam <= 0:
        with pytest.raises(bl.BlinkError) as e:
            pack(top, 0)
        assert e.value.status == bl.BLINK_EDISCONNECTED
        return
    trees = pack(top, 0)
    roots, parents, w = trees.as_lists()
    assert op.check_packing(g, roots, parents, w) == pytest.approx(lam, abs=1e-9)
    assert all(abs(x - round(x)) < 1e-12 for x in w)        # unit-grid weights
    assert sum(round(x) for x in w) == lam and trees.count <= lam


def test_parallel_arcs_add_up():
    src = np.array([0, 0, 1, 1], np.int32)
    dst = np.array([1, 1, 0, 0], np.int32)
    cap = np.array([1.0, 1.0, 1.0, 1.0])
    trees = bl.blink_pack_trees(2, src, dst, cap, 0)
    assert trees.count == 1 and trees.rate == 2.0


def test_one_hop_trees_for_switch_topologies():
    top = si.complete_graph(16)
    trees = pack(top, bl.BLINK_ROOT_ANY)
    roots, parents, w = trees.as_lists()
    oroots, otrees, ow = op.one_hop_stars(og.Digraph.from_topology(top))
    assert roots == oroots and parents == otrees and w == ow
    with pytest.raises(bl.BlinkError) as e:
        pack(si.chain(4), bl.BLINK_ROOT_ANY)
    assert e.value.status == bl.BLINK_EINVAL


def test_pack_error_codes():
    top = si.complete_graph(4)
    bad = [
        dict(k=1), dict(k=17), dict(root=4), dict(root=-2), dict(eps=0.0), dict(eps=0.9),
        dict(prune_tol=1.0), dict(prune_tol=-0.1),
    ]
    for kw in bad:
        args = dict(k=top.k, src=top.src, dst=top.dst, cap=top.cap, root=0, eps=0.05, prune_tol=0.05)
        args.update(kw)
        with pytest.raises(bl.BlinkError) as e:
            bl.blink_pack_trees(**args)
        assert e.value.status == bl.BLINK_EINVAL, kw
    for src, dst, cap in [([0, 5], [1, 0], [1, 1]), ([0, 1], [1, 1], [1, 1]), ([0, 1], [1, 0], [1, 0]),
                          ([0, 1], [1, 0], [1, -1]), ([0, 1], [1, 0], [1, float("nan")])]:
        with pytest.raises(bl.BlinkError) as e:
            bl.blink_pack_trees(2, src, dst, cap, 0)
        assert e.value.status == bl.BLINK_EINVAL
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_pack_trees(3, [0, 2], [1, 1], [1.0, 1.0], 0)       # vertex 2 unreachable
    assert e.value.status == bl.BLINK_EDISCONNECTED
    assert "unreachable" in bl.strerror(bl.BLINK_EDISCONNECTED)


def test_small_eps_neither_hangs_nor_loses_the_rate():
    """The start length of section 3.2's arcs, (1+eps)((1+eps)m)^(-1/eps), is below
    the smallest double for eps of a few thousandths; the packing must still end
    and reach the min root cut.  An eps that would take tens of millions of rounds
    is refused at once."""
    import time
    top = si.hybrid_cube_mesh()
    assert (1.004 * len(top.src)) ** (-1 / 0.004) == 0.0          # the underflow in question
    t0 = time.time()
    trees = pack(top, 0, eps=0.004)
    assert time.time() - t0 < 60
    assert abs(trees.rate - 4.0) < 1e-9 and trees.count == 4
    roots, parents, w = trees.as_lists()
    assert op.check_packing(og.Digraph.from_topology(top), roots, parents, w) == 4.0
    k16 = si.complete_graph(16)
    t0 = time.time()
    with pytest.raises(bl.BlinkError) as e:
        pack(k16, 0, eps=0.001)
    assert e.value.status == bl.BLINK_EINVAL and time.time() - t0 < 1
    assert abs(pack(k16, 0, eps=0.2).rate - 15.0) < 1e-9


def test_trees_from_arrays_round_trip_and_rejects_non_trees():
    roots, parents, w = op.pack_trees(og.Digraph.from_topology(si.hybrid_cube_mesh()), 0)
    t = bl.blink_trees_from_arrays(8, roots, parents, w)
    assert t.as_lists() == (roots, parents, w) and t.k == 8 and t.rate == sum(w)
    for bad in [(-1, 2, 1), (-1, 0, 3), (0, 0, 1), (-1, -1, 0)]:
        with pytest.raises(bl.BlinkError):
            bl.blink_trees_from_arrays(3, [0], [bad], [1.0])
    with pytest.raises(bl.BlinkError):
        bl.blink_trees_from_arrays(3, [0], [(-1, 0, 1)], [0.0])


# ---- schedule ------------------------------------------------------------------------
def to_oracle_steps(sched):
    return [osch.Step(int(s["kind"]), int(s["tree"]), int(s["chunk"]), int(s["src"]), int(s["dst"]),
                      int(s["off"]), int(s["len"]), tuple(int(d) for d in s["deps"][:int(s["n_deps"])]))
            for s in sched.steps()]


SCHED_CASES = [
    (si.complete_graph(4), 0, 1 << 20, 1 << 16),
    (si.hybrid_cube_mesh(), 0, 300_001, 8192),
    (si.hybrid_cube_mesh(doubled=True), 2, 77_777, 5000),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (2, 3, 5, 6, 7)), 0, 65_536, 65_536),
    (si.chain(6), 0, 10_000, 999),
    (si.star(5, 3), 3, 1000, 64),
    (si.complete_graph(4), 0, 3, 64),
]


@pytest.mark.parametrize("top,root,n,chunk", SCHED_CASES)
@pytest.mark.parametrize("coll", [bl.BLINK_OP_ALLREDUCE, bl.BLINK_OP_BROADCAST, bl.BLINK_OP_REDUCE])
@pytest.mark.parametrize("fusion", [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE])
def test_schedule_passes_oracle_validators(top, root, n, chunk, coll, fusion):
    trees = pack(top, root)
    roots, parents, w = trees.as_lists()
    sched = bl.blink_make_schedule(trees, coll, n, chunk, fusion)
    assert sched.bounds() == osch.split_by_weight(n, w)
    steps = to_oracle_steps(sched)
    ocoll = {bl.BLINK_OP_ALLREDUCE: osch.ALLREDUCE, bl.BLINK_OP_BROADCAST: osch.BROADCAST,
             bl.BLINK_OP_REDUCE: osch.REDUCE_TO_ROOT}[coll]
    osch.check_steps(steps, top.k, roots, parents, w, ocoll, n, chunk)
    assert len(steps) == len(osch.make_steps(roots, parents, w, ocoll, n, chunk))
    # analytic traffic of the three fusion levels (4-byte elements)
    k = top.k
    if fusion == bl.BLINK_FUSE_EDGE:
        per = {bl.BLINK_OP_ALLREDUCE: 20 * (k - 1), bl.BLINK_OP_BROADCAST: 8 * (k - 1),
               bl.BLINK_OP_REDUCE: 12 * (k - 1)}[coll]
        assert sched.traffic_bytes == per * n and sched.num_stages == len(steps)
    if fusion == bl.BLINK_FUSE_TREE:
        per = {bl.BLINK_OP_ALLREDUCE: 8 * k, bl.BLINK_OP_BROADCAST: 4 * k, bl.BLINK_OP_REDUCE: 4 * k + 4}[coll]
        assert sched.traffic_bytes == per * n
        assert sched.num_stages == len({(s.tree, s.chunk) for s in steps})
    if fusion == bl.BLINK_FUSE_NODE and coll != bl.BLINK_OP_REDUCE:
        b = sched.bounds()
        want = 0
        for t, parent in enumerate(parents):
            internal = len({p for p in parent if p >= 0})
            per = 4 * (2 * (k - 1) + 3 * internal - 1) if coll == bl.BLINK_OP_ALLREDUCE else 4 * (internal + k - 1)
            want += per * (b[t + 1] - b[t])
        assert sched.traffic_bytes == want


def test_trees_advance_together_in_the_step_order():
    """Fair interleaving (section 4.2.2): in execution order the chunk any tree
    works on is never further from another tree's than the pipeline is deep,
    counted in batches of chunks (tests/test_fair_order.py holds the order to
    the finer properties)."""
    trees = pack(si.hybrid_cube_mesh(), 0)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_BROADCAST, 1 << 22, 1 << 16, bl.BLINK_FUSE_EDGE)
    seen = {}
    for s in sched.steps():
        seen[int(s["tree"])] = int(s["chunk"])
        if len(seen) == trees.count:
            assert max(seen.values()) - min(seen.values()) <= 5 * sched.batch   # tree height 4: five levels in flight
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_BROADCAST, 1 << 22, 1 << 16, bl.BLINK_FUSE_TREE)
    # fully fused: stage i belongs to tree i mod T
    assert sched.num_stages == trees.count * 16


@pytest.mark.parametrize("weights", [[1.0, 1.0, 1.0], [0.3, 0.7], [1e-9, 1.0, 3.0], [0.1] * 7,
                                     [2.0 ** -40, 2.0 ** 40], [1 / 3, 1 / 7, 1 / 11, 0.5]])
@pytest.mark.parametrize("n", [0, 1, 5, 4096, 1_000_003, (1 << 40) + 12345])
def test_exact_weighted_split_matches_rational_arithmetic(weights, n):
    T = len(weights)
    parents = [(-1, 0)] * T
    trees = bl.blink_trees_from_arrays(2, [0] * T, parents, weights)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_BROADCAST, n, 1 << 30, bl.BLINK_FUSE_TREE)
    b = sched.bounds()
    assert b == osch.split_by_weight(n, weights)
    osch.check_split(b, n, weights)


def test_schedule_error_codes():
    trees = pack(si.complete_graph(4), 0)
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 100, 0)
    assert e.value.status == bl.BLINK_EINVAL
    with pytest.raises(bl.BlinkError):
        bl.blink_make_schedule(trees, 7, 100, 10)
    with pytest.raises(bl.BlinkError):
        bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 100, 10, 9)
    stars = pack(si.complete_graph(4), bl.BLINK_ROOT_ANY)
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_make_schedule(stars, bl.BLINK_OP_BROADCAST, 100, 10)   # several roots
    assert e.value.status == bl.BLINK_EMISMATCH
    empty = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 0, 64)
    assert empty.num_steps == 0 and empty.num_stages == 0 and empty.traffic_bytes == 0


def test_chunk_lengths_at_the_32_bit_limit():
    """A chunk's length travels in 32 bits.  A chunk size beyond that is fine as
    long as no share is that long (it then means "one chunk per tree"), an error
    otherwise; payloads beyond 2^32 elements work with ordinary chunks."""
    trees = pack(si.complete_graph(4), 0)
    one = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 1000, 1 << 40, bl.BLINK_FUSE_EDGE)
    assert one.num_steps == 3 * 6                       # one chunk per tree
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 1 << 33, 1 << 33)
    assert e.value.status == bl.BLINK_EINVAL
    big = bl.blink_make_schedule(trees, bl.BLINK_OP_BROADCAST, (1 << 33) + 5, 1 << 28, bl.BLINK_FUSE_TREE)
    assert big.bounds()[-1] == (1 << 33) + 5
    steps = big.steps()
    assert int(steps["off"].max()) + int(steps["len"][np.argmax(steps["off"])]) == (1 << 33) + 5
    assert int(steps["len"].astype(np.uint64).sum()) == 3 * ((1 << 33) + 5)      # 3 arcs per tree


# ---- Gather and AllGather -----------------------------------------------------------------
GATHER_SCHED_CASES = [
    (si.hybrid_cube_mesh(), 0, 8 * 10_001, 3000),
    (si.complete_graph(4), 1, 4 * 4096, 1024),
    (si.chain(6), 2, 6 * 500, 64),
    (si.hybrid_cube_mesh(doubled=True), 5, 8 * 999, 1 << 20),
]


@pytest.mark.parametrize("top,root,n,chunk", GATHER_SCHED_CASES)
@pytest.mark.parametrize("coll", [bl.BLINK_OP_ALLGATHER, bl.BLINK_OP_GATHER])
@pytest.mark.parametrize("fusion", [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE])
def test_gather_schedules_pass_oracle_validators(top, root, n, chunk, coll, fusion):
    trees = pack(top, root)
    roots, parents, w = trees.as_lists()
    k = top.k
    sched = bl.blink_make_schedule(trees, coll, n, chunk, fusion)
    assert sched.bounds() == osch.split_by_weight(n // k, w)
    steps = to_oracle_steps(sched)
    ocoll = osch.ALLGATHER if coll == bl.BLINK_OP_ALLGATHER else osch.GATHER
    osch.check_gather_steps(steps, k, roots, parents, w, ocoll, n, chunk)
    assert len(steps) == len(osch.make_gather_steps(roots, parents, w, ocoll, n, chunk))
    if coll == bl.BLINK_OP_ALLGATHER:
        # every piece reaches the k-1 other ranks: per-edge it is read and written once per hop,
        # fully fused it is read once and written k-1 times
        per_piece = {bl.BLINK_FUSE_EDGE: 8 * (k - 1), bl.BLINK_FUSE_TREE: 4 * k}.get(fusion)
        if per_piece:
            assert sched.traffic_bytes == per_piece * n
    elif fusion == bl.BLINK_FUSE_TREE:
        # Gather fused: every piece but the root's goes to the root in one hop
        assert sched.traffic_bytes == 8 * (n - n // k)


def test_gather_needs_a_multiple_of_k():
    trees = pack(si.complete_graph(4), 0)
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_make_schedule(trees, bl.BLINK_OP_ALLGATHER, 4 * 100 + 2, 64)
    assert e.value.status == bl.BLINK_EINVAL


def test_sweep_switch_takes_zero_or_one():
    """blink_schedule_set_sweep: host-side state only, no GPU needed."""
    from paper_1910_04940_amd import binding
    top = si.hybrid_cube_mesh()
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 1 << 16, 1 << 12, bl.BLINK_FUSE_TREE)
    sched.set_sweep(False)
    sched.set_sweep(True)
    lib = binding.lib()
    assert lib.blink_schedule_set_sweep(sched._h, 2) == bl.BLINK_EINVAL
    assert lib.blink_schedule_set_sweep(sched._h, -1) == bl.BLINK_EINVAL
    assert lib.blink_schedule_set_sweep(None, 1) == bl.BLINK_EINVAL


def test_kernel_switch_takes_zero_to_three():
    """blink_schedule_set_kernel: automatic, or one of the three ways a schedule
    can be served; host-side state only."""
    from paper_1910_04940_amd import binding
    top = si.hybrid_cube_mesh()
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 1 << 16, 1 << 12, bl.BLINK_FUSE_TREE)
    for way in (0, 1, 2, 3, 0):
        sched.set_kernel(way)
    assert sched.last_kernel == 0                        # nothing has run yet
    lib = binding.lib()
    assert lib.blink_schedule_set_kernel(sched._h, 4) == bl.BLINK_EINVAL
    assert lib.blink_schedule_set_kernel(sched._h, -1) == bl.BLINK_EINVAL
    assert lib.blink_schedule_set_kernel(None, 1) == bl.BLINK_EINVAL
