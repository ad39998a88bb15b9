"""Pins for oracle/execute.py: plain definitions, closed cases, error bounds and
invariances.  CPU only."""
import dataclasses

import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox
from oracle import graph as og
from oracle import packing as op
from oracle import schedule as osch


def make(top, root=0, stars=False):
    g = og.Digraph.from_topology(top)
    return op.one_hop_stars(g) if stars else op.pack_trees(g, root)


def inputs(k, n, dtype, seed=0, dist=None, scale=1.0):
    dist = dist or ("int" if dtype == "int32" else "uniform")
    return [si.payload(seed, r, n, dist, dtype, scale) for r in range(k)]


CASES = [
    (si.complete_graph(4), 0, False, 10_007, 1024),
    (si.hybrid_cube_mesh(), 0, False, 33_333, 4096),
    (si.hybrid_cube_mesh(doubled=True), 6, False, 20_000, 777),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 3, 4, 5, 7)), 0, False, 12_345, 2048),
    (si.complete_graph(16), 0, True, 16_400, 256),
    (si.chain(7), 3, False, 5_000, 512),
]


@pytest.mark.parametrize("top,root,stars,n,chunk", CASES)
def test_int32_allreduce_equals_wraparound_sum(top, root, stars, n, chunk):
    roots, trees, w = make(top, root, stars)
    x = inputs(top.k, n, "int32", seed=1)
    want = ox.allreduce_int32_definition(x)
    # wrap-around must actually occur in the data for the pin to bite
    assert (np.abs(np.sum([a.astype(np.int64) for a in x], axis=0)) > 2**31).any()
    bufs = [a.copy() for a in x]
    ox.run_steps(bufs, osch.make_steps(roots, trees, w, osch.ALLREDUCE, n, chunk))
    for b in bufs:
        assert np.array_equal(b, want)
    assert np.array_equal(ox.tree_order_allreduce(x, roots, trees, w), want)


@pytest.mark.parametrize("top,root,stars,n,chunk", CASES)
def test_fp32_steps_equal_tree_recursion_bitwise_and_meet_error_bound(top, root, stars, n, chunk):
    roots, trees, w = make(top, root, stars)
    x = inputs(top.k, n, "fp32", seed=2)
    bufs = [a.copy() for a in x]
    steps = osch.make_steps(roots, trees, w, osch.ALLREDUCE, n, chunk)
    ox.run_steps(bufs, steps)
    rec = ox.tree_order_allreduce(x, roots, trees, w)
    for b in bufs:
        assert np.array_equal(b.view(np.uint32), rec.view(np.uint32))
    # recursive-summation bound against the float64 sum
    exact = ox.allreduce_exact_f64(x)
    bound = (top.k - 1) * 2.0**-24 * np.sum([np.abs(a.astype(np.float64)) for a in x], axis=0)
    assert (np.abs(bufs[0].astype(np.float64) - exact) <= bound * (1 + 1e-6)).all()
    # the association order matters: a different order differs somewhere
    flat = x[0].copy()
    for a in x[1:]:
        flat = flat + a
    if top.k > 3 and not stars:
        assert not np.array_equal(flat, rec)


def test_fp32_invariant_under_chunk_size_and_step_order():
    top = si.hybrid_cube_mesh()
    roots, trees, w = make(top)
    n = 50_001
    x = inputs(8, n, "fp32", seed=3, dist="normal", scale=1e-2)
    ref = None
    for chunk in (n, 8192, 1000, 64):
        steps = osch.make_steps(roots, trees, w, osch.ALLREDUCE, n, chunk)
        for order in (None, ox.random_topological_order(steps, 7), ox.random_topological_order(steps, 8)):
            bufs = [a.copy() for a in x]
            ox.run_steps(bufs, steps, order)
            if ref is None:
                ref = bufs[0].copy()
            for b in bufs:
                assert np.array_equal(b.view(np.uint32), ref.view(np.uint32))


def test_two_ranks_is_a_single_rounded_add():
    top = si.chain(2)
    roots, trees, w = make(top)
    x = inputs(2, 4097, "fp32", seed=4)
    bufs = [a.copy() for a in x]
    ox.run_steps(bufs, osch.make_steps(roots, trees, w, osch.ALLREDUCE, 4097, 1000))
    assert np.array_equal(bufs[0], x[0] + x[1]) and np.array_equal(bufs[1], x[0] + x[1])


def test_chain_is_a_running_sum_from_the_far_end():
    k, n = 6, 3000
    parent = tuple([-1] + list(range(k - 1)))       # 0 -> 1 -> ... -> 5
    x = inputs(k, n, "fp32", seed=5)
    bufs = [a.copy() for a in x]
    ox.run_steps(bufs, osch.make_steps([0], [parent], [1.0], osch.ALLREDUCE, n, 512))
    # element by element, in Python, with explicit float32 roundings
    for j in range(0, n, 37):
        acc = np.float32(x[k - 1][j])
        for r in range(k - 2, -1, -1):
            acc = np.float32(np.float32(x[r][j]) + acc)
        assert bufs[0][j] == acc and bufs[k - 1][j] == acc


def test_tiny_tree_by_hand():
    """Root 0 with children 1 and 2; 2 has child 3.  S = (x0 + x1) + (x2 + x3)."""
    parent = (-1, 0, 0, 2)
    x = [np.array([v], np.float32) for v in (1e8, 1.0, -1e8, 3.0)]
    bufs = [a.copy() for a in x]
    ox.run_steps(bufs, osch.make_steps([0], [parent], [1.0], osch.ALLREDUCE, 1, 1))
    want = np.float32(np.float32(np.float32(1e8) + np.float32(1.0)) + np.float32(np.float32(-1e8) + np.float32(3.0)))
    assert want == 0.0      # both small addends are absorbed in this association order
    assert all(b[0] == want for b in bufs)
    # a left-to-right sum would give 3.0: the tree order is observable
    assert np.float32(np.float32(np.float32(1e8) + np.float32(1.0)) + np.float32(-1e8)) + np.float32(3.0) == 3.0


@pytest.mark.parametrize("top,root,n,chunk", [
    (si.hybrid_cube_mesh(), 0, 70_001, 8192),
    (si.complete_graph(4), 2, 999, 100),
    (si.chain(5), 4, 4096, 4096),
])
def test_broadcast_equals_root_buffer(top, root, n, chunk):
    roots, trees, w = make(top, root)
    x = inputs(top.k, n, "fp32", seed=6, dist="normal")
    bufs = [a.copy() for a in x]
    steps = osch.make_steps(roots, trees, w, osch.BROADCAST, n, chunk)
    ox.run_steps(bufs, steps, ox.random_topological_order(steps, 1))
    want = ox.broadcast_definition(x, roots, w)
    assert np.array_equal(want, x[root])
    for b in bufs:
        assert b.tobytes() == x[root].tobytes()


def test_empty_payload_is_a_no_op():
    roots, trees, w = make(si.complete_graph(4))
    steps = osch.make_steps(roots, trees, w, osch.ALLREDUCE, 0, 64)
    assert steps == []
    bufs = [np.zeros(0, np.float32) for _ in range(4)]
    ox.run_steps(bufs, steps)


def test_a_dropped_dependency_changes_some_valid_looking_execution():
    """Sanity of the random-order harness: if a REDUCE loses its dependency on
    its child's subtree, some order compatible with the (broken) list gives a
    wrong sum."""
    top = si.chain(4)
    parent = (-1, 0, 1, 2)
    n = 64
    x = inputs(4, n, "int32", seed=9)
    steps = osch.make_steps([0], [parent], [1.0], osch.ALLREDUCE, n, n)
    i = next(i for i, s in enumerate(steps) if s.kind == osch.REDUCE and s.deps)
    broken = list(steps)
    broken[i] = dataclasses.replace(steps[i], deps=())
    want = ox.allreduce_int32_definition(x)
    wrong = 0
    for seed in range(20):
        bufs = [a.copy() for a in x]
        ox.run_steps(bufs, broken, ox.random_topological_order(broken, seed))
        wrong += not np.array_equal(bufs[0], want)
    assert wrong > 0


# ---- other reduction operators and the Reduce collective --------------------------------
@pytest.mark.parametrize("redop", [ox.PROD, ox.MIN, ox.MAX])
@pytest.mark.parametrize("dtype", ["int32", "fp32"])
def test_other_operators_against_plain_definitions(redop, dtype):
    top = si.hybrid_cube_mesh()
    roots, trees, w = make(top)
    n, chunk = 20_001, 3000
    x = inputs(8, n, dtype, seed=12)
    if dtype == "fp32":
        x[3][::7] = -0.0
        x[5][::7] = 0.0          # signed zeros: MIN must give -0, MAX +0, whatever the order
    bufs = [a.copy() for a in x]
    steps = osch.make_steps(roots, trees, w, osch.ALLREDUCE, n, chunk)
    ox.run_steps(bufs, steps, ox.random_topological_order(steps, 3), redop=redop)
    rec = ox.tree_order_allreduce(x, roots, trees, w, redop)
    for b in bufs:
        assert b.tobytes() == rec.tobytes()
    if redop in (ox.MIN, ox.MAX) or dtype == "int32":
        assert rec.tobytes() == ox.reduce_definition(x, redop).tobytes()
    if redop in (ox.MIN, ox.MAX):
        # element by element against Python's min/max on a sample
        st = np.stack(x)
        for j in range(0, n, 501):
            col = [v.item() for v in st[:, j]]
            assert rec[j] == (min(col) if redop == ox.MIN else max(col))
        if dtype == "fp32":
            col = np.stack([a[::7] for a in x])
            only_zeros_extreme = (col.min(axis=0) == 0) if redop == ox.MIN else (col.max(axis=0) == 0)
            sign = np.signbit(rec[::7][only_zeros_extreme])
            assert sign.all() if redop == ox.MIN else (~sign).all()
    else:
        # float product: within k-1 roundings of the float64 product
        if dtype == "fp32":
            exact = np.prod(np.stack(x).astype(np.float64), axis=0)
            assert np.allclose(rec.astype(np.float64), exact, rtol=8 * 2.0 ** -24, atol=1e-45)


def test_int32_product_wraps():
    x = [np.array([65537, -3, 7], np.int32), np.array([65537, 5, -7], np.int32)]
    got = ox.reduce_definition(x, ox.PROD)
    assert got.tolist() == [(65537 * 65537) % (1 << 32) - 0 if (65537 * 65537) % (1 << 32) < (1 << 31)
                            else (65537 * 65537) % (1 << 32) - (1 << 32), -15, -49]
    assert ox.combine(x[0].view(np.uint32), x[1].view(np.uint32), ox.PROD).view(np.int32).tolist() == got.tolist()


@pytest.mark.parametrize("top,root", [(si.hybrid_cube_mesh(), 0), (si.chain(5), 2), (si.complete_graph(4), 1)])
def test_reduce_to_root(top, root):
    roots, trees, w = make(top, root)
    n, chunk = 9_999, 1024
    x = inputs(top.k, n, "fp32", seed=13)
    bufs = [a.copy() for a in x]
    steps = osch.make_steps(roots, trees, w, osch.REDUCE_TO_ROOT, n, chunk)
    osch.check_steps(steps, top.k, roots, trees, w, osch.REDUCE_TO_ROOT, n, chunk)
    assert all(s.kind == osch.REDUCE for s in steps)
    ox.run_steps(bufs, steps, ox.random_topological_order(steps, 2))
    want = ox.tree_order_allreduce(x, roots, trees, w)
    assert bufs[root].tobytes() == want.tobytes()
    # leaves are untouched by a Reduce
    ch = og.children_of(trees[0])
    leaves_everywhere = [v for v in range(top.k) if all(not og.children_of(t)[v] for t in trees)]
    for v in leaves_everywhere:
        assert bufs[v].tobytes() == x[v].tobytes()


# ---- Gather and AllGather -------------------------------------------------------------------
@pytest.mark.parametrize("top,root", [(si.hybrid_cube_mesh(), 0), (si.chain(5), 2), (si.complete_graph(4), 1)])
@pytest.mark.parametrize("dtype", ["int32", "fp32"])
def test_allgather_equals_concatenation_and_zero_padded_allreduce(top, root, dtype):
    roots, trees, w = make(top, root)
    k = top.k
    m, chunk = 1003, 200
    n = k * m
    x = inputs(k, n, dtype, seed=14)
    want = ox.allgather_definition(x)
    bufs = [a.copy() for a in x]
    steps = osch.make_gather_steps(roots, trees, w, osch.ALLGATHER, n, chunk)
    ox.run_steps(bufs, steps, ox.random_topological_order(steps, 4))
    for b in bufs:
        assert b.tobytes() == want.tobytes()
    # the paper's description: an AllReduce whose reduction has nothing to do
    padded = []
    for j in range(k):
        z = np.zeros(n, x[0].dtype)
        z[j * m:(j + 1) * m] = x[j][j * m:(j + 1) * m]
        padded.append(z)
    ox.run_steps(padded, osch.make_steps(roots, trees, w, osch.ALLREDUCE, n, chunk))
    assert np.array_equal(padded[0], want)          # values (a stored -0.0 would come back as +0.0)


@pytest.mark.parametrize("top,root", [(si.hybrid_cube_mesh(), 3), (si.star(5, 2), 2)])
def test_gather_collects_at_the_root(top, root):
    roots, trees, w = make(top, root)
    k = top.k
    n, chunk = k * 500, 64
    x = inputs(k, n, "fp32", seed=15)
    bufs = [a.copy() for a in x]
    steps = osch.make_gather_steps(roots, trees, w, osch.GATHER, n, chunk)
    ox.run_steps(bufs, steps, ox.random_topological_order(steps, 5))
    assert bufs[root].tobytes() == ox.allgather_definition(x).tobytes()
