"""Pins for oracle/multiserver.py: the three-phase protocol across servers
(paper section 3.5) and the two-link-class split (section 3.4).  CPU only."""
import dataclasses

import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox
from oracle import graph as og
from oracle import multiserver as om
from oracle import packing as op
from oracle import schedule as osch


def server(top, ranks, root=0):
    """A server whose local ranks (in `top`'s numbering) get the global ids `ranks`."""
    roots, trees, w = op.pack_trees(og.Digraph.from_topology(top), root)
    return om.Server(tuple(ranks), tuple(roots), tuple(tuple(t) for t in trees), tuple(w))


def three_plus_five(interleaved=False):
    """The paper's multi-server experiment: 3 GPUs of one server and 5 of another
    (fragments of the doubled-link cube-mesh)."""
    mesh = si.hybrid_cube_mesh(doubled=True)
    a, b = si.induced(mesh, (0, 1, 4)), si.induced(mesh, (2, 3, 5, 6, 7))
    if interleaved:
        return [server(a, (0, 2, 5)), server(b, (1, 3, 4, 6, 7), root=2)]
    return [server(a, (0, 1, 2)), server(b, (3, 4, 5, 6, 7))]


def two_full(roots=(0, 0)):
    mesh = si.hybrid_cube_mesh()
    return [server(mesh, range(0, 8), roots[0]), server(mesh, range(8, 16), roots[1])]


def three_servers():
    """Three servers with 2, 3 and 1 trees: their splits do not line up."""
    return [server(si.ring(3), (0, 3, 6)), server(si.complete_graph(4), (1, 2, 7, 8), root=1),
            server(si.chain(2), (4, 5), root=1)]


LAYOUTS = {"3+5": three_plus_five, "3+5 interleaved": lambda: three_plus_five(True),
           "8+8": two_full, "ring3+K4+chain2": three_servers}


def inputs(k, n, dtype, seed):
    dist = "int" if dtype == "int32" else "uniform"
    return [si.payload(seed, r, n, dist, dtype) for r in range(k)]


def k_of(servers):
    return sum(len(s.ranks) for s in servers)


# ---- the data result ----------------------------------------------------------
@pytest.mark.parametrize("layout", LAYOUTS)
def test_int32_result_is_the_wraparound_sum_of_all_ranks(layout):
    servers = LAYOUTS[layout]()
    x = inputs(k_of(servers), 10_007, "int32", seed=3)
    assert np.array_equal(om.three_phase_allreduce(x, servers), ox.allreduce_int32_definition(x))


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("redop", [ox.MIN, ox.MAX])
def test_order_free_operators_equal_their_definition(layout, redop):
    servers = LAYOUTS[layout]()
    for dtype in ("int32", "fp32"):
        x = inputs(k_of(servers), 4_099, dtype, seed=4)
        got = om.three_phase_allreduce(x, servers, redop)
        assert np.array_equal(got.view(np.uint32), ox.reduce_definition(x, redop).view(np.uint32))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_fp32_result_is_within_the_recursive_summation_bound(layout):
    servers = LAYOUTS[layout]()
    k = k_of(servers)
    x = inputs(k, 20_011, "fp32", seed=5)
    got = om.three_phase_allreduce(x, servers).astype(np.float64)
    bound = (k - 1) * 2.0**-24 * np.sum([np.abs(a.astype(np.float64)) for a in x], axis=0)
    assert (np.abs(got - ox.allreduce_exact_f64(x)) <= bound * (1 + 1e-9)).all()


def test_one_server_is_the_plain_tree_allreduce():
    srv = server(si.hybrid_cube_mesh(), range(8), root=5)
    x = inputs(8, 9_001, "fp32", seed=6)
    want = ox.tree_order_allreduce(x, srv.roots, srv.trees, srv.weights)
    assert np.array_equal(om.three_phase_allreduce(x, [srv]).view(np.uint32), want.view(np.uint32))


def test_one_rank_per_server_is_the_one_hop_allreduce_of_a_switch():
    """n servers of one GPU each: only phase 2 is left, which is section 3.5's
    own description of the switch case (n one-hop trees, one n-th each)."""
    n_srv = 6
    servers = [om.Server((i,), (0,), ((-1,),), (1.0,)) for i in range(n_srv)]
    roots, trees, w = op.one_hop_stars(og.Digraph.from_topology(si.complete_graph(n_srv)))
    x = inputs(n_srv, 6_007, "fp32", seed=7)
    want = ox.tree_order_allreduce(x, roots, trees, w)
    assert np.array_equal(om.three_phase_allreduce(x, servers).view(np.uint32), want.view(np.uint32))


def test_two_by_two_fold_order_written_out():
    """Servers {0,1} and {2,3}, local roots 1 and 2: rank 1 owns the first half
    and ends with (x1 + x0) + (x2 + x3); rank 2 owns the second half and ends
    with (x2 + x3) + (x1 + x0)."""
    servers = [om.Server((0, 1), (1,), ((1, -1),), (1.0,)), om.Server((2, 3), (0,), ((-1, 0),), (1.0,))]
    x = inputs(4, 64, "fp32", seed=8)
    got = om.three_phase_allreduce(x, servers)
    a, b = x[1] + x[0], x[2] + x[3]
    assert np.array_equal(got[:32], (a + b)[:32])
    assert np.array_equal(got[32:], (b + a)[32:])


# ---- partitions and the composed trees ----------------------------------------
def test_partitions_follow_the_number_of_local_trees():
    """Section 3.5 / its figure: two servers with four local trees each give four
    partitions, each cut in two for the cross-server phase."""
    servers = two_full()
    assert [len(s.trees) for s in servers] == [4, 4]
    n = 1 << 20
    parts = om.partitions(n, servers)
    assert [(lo, hi) for lo, hi, _ in parts] == [(i << 18, (i + 1) << 18) for i in range(4)]
    assert [sel for _, _, sel in parts] == [(t, t) for t in range(4)]
    trees = om.compose(n, servers)
    assert len(trees) == 8 and all(g.hi - g.lo == 1 << 17 for g in trees)


def test_partitions_refine_unequal_splits():
    servers = three_servers()
    assert [len(s.trees) for s in servers] == [2, 3, 1]
    n = 12_000
    parts = om.partitions(n, servers)
    assert [(lo, hi) for lo, hi, _ in parts] == [(0, 4000), (4000, 6000), (6000, 8000), (8000, 12000)]
    assert [sel for _, _, sel in parts] == [(0, 0, 0), (0, 1, 0), (1, 1, 0), (1, 2, 0)]
    assert sum(g.hi - g.lo for g in om.compose(n, servers)) == n


@pytest.mark.parametrize("layout", LAYOUTS)
def test_composed_trees_span_all_ranks_and_cross_servers_only_at_the_roots(layout):
    servers = LAYOUTS[layout]()
    k = k_of(servers)
    home = {g: i for i, s in enumerate(servers) for g in s.ranks}
    anywhere = og.Digraph.from_topology(si.complete_graph(k))
    for g in om.compose(50_000, servers):
        assert og.is_spanning_arborescence(anywhere, g.root, g.parent)
        crossing = [(g.parent[v], v) for v in range(k) if v != g.root and home[v] != home[g.parent[v]]]
        # n - 1 one-hop links, all into the owner, from the other servers' roots
        assert len(crossing) == len(servers) - 1
        assert all(p == g.root for p, _ in crossing) and {v for _, v in crossing} == set(g.late)


# ---- the step list ------------------------------------------------------------
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("dtype", ["fp32", "int32"])
def test_step_list_reproduces_the_phase_by_phase_result_bitwise(layout, dtype):
    servers = LAYOUTS[layout]()
    k, n, chunk = k_of(servers), 30_011, 1024
    x = inputs(k, n, dtype, seed=9)
    want = om.three_phase_allreduce(x, servers)
    steps = om.three_phase_steps(servers, n, chunk)
    om.check_three_phase_steps(steps, servers, n, chunk)
    for order in (None, ox.random_topological_order(steps, 1), ox.random_topological_order(steps, 2)):
        bufs = [a.copy() for a in x]
        ox.run_steps(bufs, steps, order)
        for b in bufs:
            assert np.array_equal(b.view(np.uint32), want.view(np.uint32))


def test_step_count_is_two_transfers_per_arc_and_chunk():
    servers = three_plus_five()
    n, chunk = 40_000, 1000
    steps = om.three_phase_steps(servers, n, chunk)
    chunks = sum(len(osch.chunk_ranges(g.lo, g.hi, chunk)) for g in om.compose(n, servers))
    assert len(steps) == chunks * 2 * (8 - 1)


def _mutations(steps, servers, n):
    late_fold = next(i for i, s in enumerate(steps)
                     if s.kind == osch.REDUCE and s.src in om.compose(n, servers)[s.tree].late)
    yield "dropped step", steps[:5] + steps[6:]
    yield "cross-server sum no longer waits for the local one", \
        steps[:late_fold] + [dataclasses.replace(steps[late_fold], deps=steps[late_fold].deps[:1])] + \
        steps[late_fold + 1:]
    yield "wrong source", [dataclasses.replace(steps[0], src=(steps[0].src + 1) % 8
                                               if (steps[0].src + 1) % 8 != steps[0].dst
                                               else (steps[0].src + 2) % 8)] + steps[1:]
    yield "shifted range", [dataclasses.replace(steps[0], off=steps[0].off + 4)] + steps[1:]


def test_validator_rejects_planted_mistakes():
    servers = three_plus_five()
    n, chunk = 20_000, 4096
    steps = om.three_phase_steps(servers, n, chunk)
    om.check_three_phase_steps(steps, servers, n, chunk)
    for name, bad in _mutations(steps, servers, n):
        with pytest.raises(AssertionError):
            om.check_three_phase_steps(bad, servers, n, chunk)
            pytest.fail(f"not caught: {name}")


def test_validator_rejects_remote_roots_folded_before_local_children():
    """Ascending-id folding everywhere would put a remote root with a small id
    ahead of the owner's own children: a different floating-point result."""
    servers = three_plus_five(interleaved=True)
    n, chunk = 8_000, 8_000
    wrong = []
    for t, g in enumerate(om.compose(n, servers)):
        osch.emit_tree_steps(wrong, t, g.root, g.parent, og.children_of(g.parent), osch.ALLREDUCE,
                             g.lo, g.hi, chunk)
    assert wrong != om.three_phase_steps(servers, n, chunk)
    with pytest.raises(AssertionError):
        om.check_three_phase_steps(wrong, servers, n, chunk)


# ---- the split between two classes of links (section 3.4) ---------------------
@pytest.mark.parametrize("d,bp,bn,t", [(500e6, 10e9, 60e9, 1e-4), (1e9, 8e9, 25e9, 0.0),
                                       (64e6, 12e9, 120e9, 2e-4)])
def test_split_makes_both_classes_finish_together(d, bp, bn, t):
    dp, dn = om.hybrid_split(d, bp, bn, t)
    assert dp > 0 and dn > 0 and dp + dn == pytest.approx(d, rel=1e-15)
    assert dp / bp + t == pytest.approx(dn / bn, rel=1e-12)


def test_split_without_latency_is_proportional_to_bandwidth():
    dp, dn = om.hybrid_split(700.0, 10.0, 25.0, 0.0)
    assert dp == pytest.approx(200.0) and dn == pytest.approx(500.0)


def test_split_minimises_the_completion_time_by_brute_force():
    d, bp, bn, t = 1000.0, 3.0, 17.0, 4.0
    grid = np.linspace(0.0, d, 200_001)
    finish = np.maximum(np.where(grid > 0, grid / bp + t, 0.0), (d - grid) / bn)
    dp, _ = om.hybrid_split(d, bp, bn, t)
    assert abs(grid[np.argmin(finish)] - dp) <= d / 200_000
    # the slow class is left idle once its latency exceeds the whole fast transfer
    assert om.hybrid_split(d, bp, bn, d / bn + 1.0) == (0.0, d)
    grid_finish = np.maximum(np.where(grid > 0, grid / bp + d / bn + 1.0, 0.0), (d - grid) / bn)
    assert np.argmin(grid_finish) == 0
