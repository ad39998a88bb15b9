"""Pins for oracle/packing.py.  CPU only."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import graph as og
from oracle import packing as op


def G(top):
    return og.Digraph.from_topology(top)


# ---- minimum arborescence against brute force ---------------------------------
@pytest.mark.parametrize("seed", range(12))
def test_min_arborescence_matches_exhaustive_minimum(seed):
    top = si.random_digraph(4 + seed % 3, 0.5, 300 + seed)
    g = G(top)
    rng = np.random.default_rng(seed)
    # few distinct lengths so that ties and contractions of cycles both occur
    lengths = rng.integers(1, 4, size=g.m).astype(float)
    arcs = [(u, v, lengths[i]) for i, (u, v, _) in enumerate(g.arcs)]
    for root in range(g.k):
        idx = op.min_arborescence(g.k, arcs, root)
        trees = og.enumerate_arborescences(g, root)
        if not trees:
            assert idx is None
            continue
        cost = {(u, v): w for (u, v, w) in arcs}
        best = min(sum(cost[a] for a in og.tree_arcs(root, t)) for t in trees)
        parent = op._parents_from_arcs(g.k, g.arcs, idx, root)
        assert og.is_spanning_arborescence(g, root, parent)
        assert sum(arcs[i][2] for i in idx) == best


def test_min_arborescence_unreachable_vertex():
    assert op.min_arborescence(3, [(0, 1, 1.0), (2, 1, 1.0)], 0) is None


# ---- MWU: feasible, near-optimal ------------------------------------------------
@pytest.mark.parametrize("top,root,eps", [
    (si.complete_graph(4), 0, 0.1),
    (si.hybrid_cube_mesh(), 0, 0.1),
    (si.hybrid_cube_mesh(), 5, 0.1),
    (si.hybrid_cube_mesh(doubled=True), 0, 0.1),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (2, 3, 5, 6, 7)), 0, 0.1),
    (si.random_digraph(6, 0.5, 11, int_caps=False), 0, 0.1),
    (si.random_digraph(7, 0.4, 12, int_caps=False), 0, 0.2),
    (si.chain(6, 1.5), 0, 0.1),
])
def test_mwu_is_feasible_and_within_guarantee(top, root, eps):
    g = G(top)
    trees, w = op.mwu_pack(g, root, eps)
    assert len(set(trees)) == len(trees)
    rate = op.check_packing(g, [root] * len(trees), trees, w)
    lam = og.min_root_cut(g, root)
    assert rate <= lam + 1e-9
    assert rate >= (1 - 2 * eps) * lam


def test_mwu_rejects_disconnected():
    with pytest.raises(ValueError):
        op.mwu_pack(og.Digraph(3, [(0, 1, 1.0), (2, 1, 1.0)]), 0)


# ---- pruning ---------------------------------------------------------------------
def test_dgx1v_graph_prunes_to_six_unit_trees(paper_pins):
    """The paper's worked example (section 3.2.1): MWU returns many trees with
    small fractional weights, the integer program leaves 6 trees of rate 1.0."""
    g = G(si.hybrid_cube_mesh(doubled=True))
    trees, w = op.mwu_pack(g, 0, 0.1)
    assert len(trees) > 20 and min(w) < 0.05       # "no bound on the number of trees"
    roots, trees, w = op.pack_trees(g, 0, 0.1, 0.05)
    op.check_packing(g, roots, trees, w)
    assert len(trees) == int(paper_pins["dgx1v_pruned_tree_count"])
    assert w == [float(paper_pins["dgx1v_pruned_tree_rate"])] * len(trees)


@pytest.mark.parametrize("top,root", [
    (si.complete_graph(4), 0),
    (si.hybrid_cube_mesh(), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 4)), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 3, 4, 5, 7)), 0),
    (si.random_digraph(6, 0.5, 21, int_caps=False), 0),
])
def test_pruned_packing_within_tolerance_and_smaller(top, root):
    g = G(top)
    mt, mw = op.mwu_pack(g, root, 0.1)
    roots, trees, w = op.pack_trees(g, root, 0.1, 0.05)
    rate = op.check_packing(g, roots, trees, w)
    assert rate >= 0.95 * sum(mw) - 1e-9
    assert rate <= og.min_root_cut(g, root) + 1e-9
    assert len(trees) <= len(mt)


def test_chain_of_capacity_two_is_one_tree_of_weight_two():
    g = G(si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 4)))
    roots, trees, w = op.pack_trees(g, 0)
    assert len(trees) == 1 and w == [2.0]


def test_grid_program_is_exact_on_a_small_case():
    """Against exhaustive search over ALL arborescences of K4."""
    g = G(si.complete_graph(4))
    allt = og.enumerate_arborescences(g, 0)
    x, rate = op.grid_max_packing(g, 0, allt, 1.0)
    assert rate == og.max_integral_packing_exhaustive(g, 0, allt) == 3
    x, rate = op.grid_max_packing(g, 0, allt[:1], 0.5)   # one candidate only
    assert rate == 1.0 and x == [2]


# ---- one-hop trees for switch topologies -------------------------------------------
def test_one_hop_stars(paper_pins):
    assert paper_pins["switch_tree_count"] == "m" and paper_pins["switch_share_per_root"] == "1/m"
    m = 16
    g = G(si.complete_graph(m))
    roots, trees, w = op.one_hop_stars(g)
    assert roots == list(range(m)) and len(trees) == m
    assert w == [1.0 / m] * m
    for r, t in zip(roots, trees):
        assert og.is_spanning_arborescence(g, r, t)
        assert all(t[v] == r for v in range(m) if v != r)
    op.check_packing(g, roots, trees, w)
    with pytest.raises(ValueError):
        op.one_hop_stars(G(si.chain(4)))


# ---- the validator itself must catch planted mistakes --------------------------------
def test_check_packing_catches_overload_and_bad_tree():
    g = G(si.complete_graph(4))
    t = (-1, 0, 0, 0)
    op.check_packing(g, [0], [t], [1.0])
    with pytest.raises(AssertionError):
        op.check_packing(g, [0], [t], [1.5])
    with pytest.raises(AssertionError):
        op.check_packing(g, [0, 0], [t, (-1, 0, 1, 0)], [0.6, 0.6])   # arc 0->1 carries 1.2
    with pytest.raises(AssertionError):
        op.check_packing(G(si.chain(4)), [0], [t], [1.0])
    with pytest.raises(AssertionError):
        op.check_packing(g, [0], [t], [0.0])
