"""Pins for oracle/graph.py: closed forms, theorems and library routines the
brute-force code must reproduce.  CPU only."""
import itertools

import numpy as np
import pytest
import scipy.optimize
import scipy.sparse
import scipy.sparse.csgraph

import synth_inputs as si
from oracle import graph as og


def G(top):
    return og.Digraph.from_topology(top)


# ---- counting arborescences -------------------------------------------------
@pytest.mark.parametrize("n", [2, 3, 4, 5, 6])
def test_complete_graph_has_n_pow_n_minus_2_trees(n, paper_pins):
    # the paper's count for the complete graph (section 3.1): n^(n-2) per root
    assert paper_pins["complete_graph_tree_count"] == "n^(n-2)"
    g = G(si.complete_graph(n))
    want = n ** (n - 2)
    assert og.count_arborescences_matrix_tree(g, 0) == want
    assert len(og.enumerate_arborescences(g, 0)) == want


def test_enumeration_matches_matrix_tree_on_cube_mesh():
    g = G(si.hybrid_cube_mesh())
    trees = og.enumerate_arborescences(g, 0)
    assert len(trees) == og.count_arborescences_matrix_tree(g, 0)
    assert len(set(trees)) == len(trees)
    assert all(og.is_spanning_arborescence(g, 0, t) for t in trees[::97])


@pytest.mark.parametrize("seed", range(6))
def test_enumeration_matches_matrix_tree_random(seed):
    g = G(si.random_digraph(5 + seed % 2, 0.4, seed))
    for root in (0, g.k - 1):
        assert len(og.enumerate_arborescences(g, root)) == og.count_arborescences_matrix_tree(g, root)


def test_is_spanning_arborescence_rejects_bad_trees():
    g = G(si.chain(4))
    assert og.is_spanning_arborescence(g, 0, (-1, 0, 1, 2))
    assert not og.is_spanning_arborescence(g, 0, (-1, 0, 0, 2))      # arc 0->2 absent
    assert not og.is_spanning_arborescence(g, 0, (-1, 2, 1, 2))      # 1<->2 cycle
    assert not og.is_spanning_arborescence(g, 0, (1, 0, 1, 2))       # root has a parent
    assert not og.is_spanning_arborescence(g, 0, (-1, 0, 1))         # wrong length


# ---- min root cut -------------------------------------------------------------
def test_min_root_cut_closed_forms():
    assert og.min_root_cut(G(si.complete_graph(4)), 0) == 3
    assert og.min_root_cut(G(si.complete_graph(8)), 3) == 7
    assert og.min_root_cut(G(si.complete_graph(16)), 0) == 15
    for r in range(8):
        assert og.min_root_cut(G(si.hybrid_cube_mesh()), r) == 4
        assert og.min_root_cut(G(si.hybrid_cube_mesh(doubled=True)), r) == 6
    assert og.min_root_cut(G(si.chain(5, 2.5)), 0) == 2.5
    assert og.min_root_cut(G(si.star(6, 2, 0.75)), 2) == 0.75
    assert og.min_root_cut(G(si.ring(5)), 0) == 2


def test_min_root_cut_fragmented_allocations():
    d = si.hybrid_cube_mesh(doubled=True)
    want = {(0, 1, 4): 2, (2, 3, 5, 6, 7): 2, (0, 1, 3, 4, 5, 7): 4, (1, 4, 5, 6): 2, (2, 3, 6, 7): 4}
    for ranks, rate in want.items():
        assert og.min_root_cut(G(si.induced(d, ranks)), 0) == rate, ranks


def _maxflow_rate(top, root):
    """min over targets of max-flow(root -> target) with scipy's routine."""
    g = G(top)
    cap = np.zeros((g.k, g.k), np.int32)
    for (u, v, c) in g.arcs:
        cap[u, v] = int(c)
    m = scipy.sparse.csr_matrix(cap)
    return min(scipy.sparse.csgraph.maximum_flow(m, root, t).flow_value
               for t in range(g.k) if t != root)


@pytest.mark.parametrize("seed", range(8))
def test_min_root_cut_equals_min_over_targets_of_max_flow(seed):
    top = si.random_digraph(4 + seed % 4, 0.35, 100 + seed)
    for root in range(top.k):
        g = G(top)
        if not all(g.reachable_from(root)):
            continue
        assert og.min_root_cut(g, root) == _maxflow_rate(top, root)


def test_min_root_cut_zero_when_unreachable():
    g = og.Digraph(3, [(0, 1, 1.0), (2, 1, 1.0)])
    assert og.min_root_cut(g, 0) == 0.0


# ---- Edmonds: packing value equals the min root cut ----------------------------
@pytest.mark.parametrize("top,root", [
    (si.complete_graph(4), 0),
    (si.complete_graph(3, 2.0), 1),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 4)), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (1, 4, 5, 6)), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (2, 3, 6, 7)), 2),
    (si.random_digraph(5, 0.5, 7), 0),
    (si.random_digraph(5, 0.6, 8), 0),
    (si.ring(5), 0),
])
def test_exhaustive_integral_packing_equals_min_root_cut(top, root):
    g = G(top)
    assert og.max_integral_packing_exhaustive(g, root) == og.min_root_cut(g, root)


def _lp_packing_rate(g, root):
    """Packing LP of section 3.1 over ALL arborescences, solved by scipy."""
    trees = og.enumerate_arborescences(g, root)
    arcs = sorted(g.cap)
    A = np.zeros((len(arcs), len(trees)))
    pos = {a: i for i, a in enumerate(arcs)}
    for j, t in enumerate(trees):
        for a in og.tree_arcs(root, t):
            A[pos[a], j] = 1.0
    res = scipy.optimize.linprog(-np.ones(len(trees)), A_ub=A,
                                 b_ub=np.array([g.cap[a] for a in arcs]), bounds=(0, None))
    assert res.status == 0
    return -res.fun


@pytest.mark.parametrize("seed", range(5))
def test_fractional_packing_lp_equals_min_root_cut(seed):
    g = G(si.random_digraph(5, 0.5, 200 + seed, int_caps=False))
    assert _lp_packing_rate(g, 0) == pytest.approx(og.min_root_cut(g, 0), rel=1e-7)


def test_children_sorted_and_tree_arcs():
    parent = (-1, 3, 0, 0, 3)
    assert og.children_of(parent) == [[2, 3], [], [], [1, 4], []]
    assert sorted(og.tree_arcs(0, parent)) == [(0, 2), (0, 3), (3, 1), (3, 4)]
