"""Every connected 3- to 8-GPU allocation of the two 8-GPU servers the paper
evaluates (its sections 2.1 and 5.2): the topology encodings reproduce the
paper's counts of distinct allocations, and the library's packer reaches the
optimal rate on each of them.  CPU only."""
import pytest

import paper_1910_04940_amd as bl
import synth_inputs as si
from oracle import graph as og
from oracle import packing as op


def test_counts_of_distinct_allocations_match_the_paper(paper_pins):
    p100 = si.hybrid_cube_mesh()
    v100 = si.dgx1v()
    assert si.count_distinct_allocations(p100, si.connected_allocations(p100)) == \
        int(paper_pins["distinct_allocations_first_generation"])
    assert si.count_distinct_allocations(v100, si.connected_allocations(v100)) == \
        int(paper_pins["distinct_allocations_second_generation"])
    # six link-units per GPU on the second generation, four on the first
    for v in range(8):
        assert sum(c for (u, w, c) in v100.arcs() if w == v) == 6
        assert sum(c for (u, w, c) in p100.arcs() if w == v) == 4


def test_full_second_generation_server_packs_six_unit_trees(paper_pins):
    top = si.dgx1v()
    for root in range(8):
        assert og.min_root_cut(og.Digraph.from_topology(top), root) == 6
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
    assert trees.count == int(paper_pins["dgx1v_pruned_tree_count"])
    assert all(w == float(paper_pins["dgx1v_pruned_tree_rate"]) for w in trees.as_lists()[2])
    roots, parents, w = op.pack_trees(og.Digraph.from_topology(top), 0)       # the oracle's packer too
    assert len(parents) == 6 and w == [1.0] * 6


@pytest.mark.parametrize("name", ["first_generation", "second_generation"])
def test_every_connected_allocation_is_packed_at_its_optimal_rate(name):
    full = si.hybrid_cube_mesh() if name == "first_generation" else si.dgx1v()
    subsets = si.connected_allocations(full)
    assert len(subsets) > 150
    for sub in subsets:
        top = si.induced(full, sub)
        g = og.Digraph.from_topology(top)
        lam = og.min_root_cut(g, 0)
        trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
        roots, parents, w = trees.as_lists()
        rate = op.check_packing(g, roots, parents, w)
        assert rate == lam, (sub, rate, lam)            # integer capacities: exactly the min root cut
        assert trees.count <= lam, (sub, trees.count, lam)
