"""The kernel's passes ("stages") of every fusion level, checked and replayed on
the CPU: the stage records the library exports are interpreted here with NumPy,
in a random order that respects their dependencies, and must reproduce the
oracle's result bit for bit.  A race check requires every pair of stages that
touch the same elements of the same rank, one of them writing, to be ordered by
the dependencies.  No GPU."""
import numpy as np
import pytest

import paper_1910_04940_amd as bl
import synth_inputs as si
from oracle import execute as ox
from oracle import multiserver as om

from test_host_multiserver import LAYOUT_NAMES, make

FUSIONS = [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE]
LD, ADD, ST = 0, 1, 2


def pack(top, root):
    return bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, root)


def topological_order(stages, seed):
    rng = np.random.default_rng(seed)
    n = len(stages)
    waiting = [int(s["n_dep"]) for s in stages]
    users = [[] for _ in range(n)]
    for i, s in enumerate(stages):
        for d in s["deps"][:int(s["n_dep"])]:
            assert 0 <= d < i, f"stage {i}: dependency {d} is not earlier"
            users[int(d)].append(i)
    ready = [i for i in range(n) if waiting[i] == 0]
    order = []
    while ready:
        j = int(rng.integers(len(ready)))
        ready[j], ready[-1] = ready[-1], ready[j]
        i = ready.pop()
        order.append(i)
        for u in users[i]:
            waiting[u] -= 1
            if waiting[u] == 0:
                ready.append(u)
    assert len(order) == n
    return order


def run_stages(bufs, stages, order, redop=ox.SUM):
    """Interpret the stage records on float32 arrays, or uint32 views of int32 data."""
    for i in order:
        s = stages[i]
        a, b = int(s["off"]), int(s["off"]) + int(s["len"])
        slots = [bufs[int(r)][a:b].copy() for r in s["load_rank"][:int(s["n_load"])]]
        acc = None
        for code in s["op"][:int(s["n_op"])]:
            kind, slot = int(code) >> 6, int(code) & 63
            if kind == LD:
                acc = slots[slot].copy()
            elif kind == ADD:
                acc = ox.combine(acc, slots[slot], redop)
            else:
                assert kind == ST
                slots[slot] = acc.copy()
        # the same stage as a stack program (what the streaming kernel runs):
        # every stage has one, and it gives the same bits
        assert 1 <= int(s["seq_depth"]) <= max(1, int(s["n_load"]) // 2), "stage without a stack program"
        stack, deepest = [], 0
        for j in range(int(s["n_load"])):
            x = bufs[int(s["seq_rank"][j])][a:b]
            code = int(s["seq_code"][j])
            if code & 1:
                stack.append(x.copy())
            else:
                stack[-1] = ox.combine(stack[-1], x, redop)
            deepest = max(deepest, len(stack))
            for _ in range(code >> 1):
                top = stack.pop()
                stack[-1] = ox.combine(stack[-1], top, redop)
        assert len(stack) == 1 and deepest == int(s["seq_depth"])
        assert sorted(int(r) for r in s["seq_rank"][:int(s["n_load"])]) == \
            sorted(int(r) for r in s["load_rank"][:int(s["n_load"])])
        assert np.array_equal(stack[0].view(np.uint32), acc.view(np.uint32))
        for r in s["store_rank"][:int(s["n_store"])]:
            bufs[int(r)][a:b] = acc


def check_no_unordered_conflicts(stages):
    """Stages of different (flow, chunk) work on disjoint element ranges; inside
    one, any two that conflict on a rank must be ordered by the dependencies."""
    groups = {}
    for i, s in enumerate(stages):
        groups.setdefault((int(s["flow"]), int(s["chunk"])), []).append(i)
    spans = sorted((int(stages[ix[0]]["off"]), int(stages[ix[0]]["off"]) + int(stages[ix[0]]["len"])) for ix in groups.values())
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:])), "chunks of different trees overlap"
    closure = {}
    for i, s in enumerate(stages):
        cl = set()
        for d in s["deps"][:int(s["n_dep"])]:
            cl.add(int(d))
            cl |= closure[int(d)]
        closure[i] = cl
    for ix in groups.values():
        assert len({(int(stages[i]["off"]), int(stages[i]["len"])) for i in ix}) == 1
        rw = [(set(map(int, stages[i]["load_rank"][:int(stages[i]["n_load"])])),
               set(map(int, stages[i]["store_rank"][:int(stages[i]["n_store"])]))) for i in ix]
        for a in range(len(ix)):
            for b in range(a + 1, len(ix)):
                (ra, wa), (rb, wb) = rw[a], rw[b]
                if wa & (rb | wb) or wb & ra:
                    assert ix[a] in closure[ix[b]], f"stages {ix[a]} and {ix[b]} conflict but are not ordered"


def as_views(x):
    return [a.view(np.uint32) if a.dtype == np.int32 else a for a in x]


CASES = [
    (si.complete_graph(4), 0, 10_007, 1024),
    (si.hybrid_cube_mesh(), 0, 33_333, 4096),
    (si.hybrid_cube_mesh(doubled=True), 6, 20_000, 777),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 3, 4, 5, 7)), 0, 12_345, 2048),
    (si.complete_graph(16), bl.BLINK_ROOT_ANY, 16_400, 256),
    (si.chain(7), 3, 5_000, 512),
    (si.star(6, 2), 2, 3_001, 64),
]


@pytest.mark.parametrize("top,root,n,chunk", CASES)
@pytest.mark.parametrize("fusion", FUSIONS)
@pytest.mark.parametrize("dtype", ["fp32", "int32"])
def test_allreduce_stages_replayed_on_the_cpu(top, root, n, chunk, fusion, dtype):
    trees = pack(top, root)
    roots, parents, w = trees.as_lists()
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    stages = sched.stages()
    assert len(stages) == sched.num_stages
    check_no_unordered_conflicts(stages)
    x = [si.payload(3, r, n, "int" if dtype == "int32" else "uniform", dtype) for r in range(top.k)]
    want = ox.tree_order_allreduce(x, roots, parents, w)
    for redop in ((ox.SUM,) if dtype == "int32" else (ox.SUM, ox.MAX)):
        bufs = as_views([a.copy() for a in x])
        run_stages(bufs, stages, topological_order(stages, 7), redop)
        ref = want if redop == ox.SUM else ox.reduce_definition(x, redop)
        for b in bufs:
            assert np.array_equal(b.view(np.uint32), ref.view(np.uint32))
    # bytes moved, as the stage records say, equal what the library reports
    moved = sum(int(s["len"]) * 4 * (int(s["n_load"]) + int(s["n_store"])) for s in stages)
    assert moved == sched.traffic_bytes


@pytest.mark.parametrize("top,root,n,chunk", CASES[:4] + CASES[5:])
@pytest.mark.parametrize("fusion", FUSIONS)
def test_broadcast_and_reduce_stages_replayed_on_the_cpu(top, root, n, chunk, fusion):
    trees = pack(top, root)
    roots, parents, w = trees.as_lists()
    x = [si.payload(4, r, n, "uniform", "fp32") for r in range(top.k)]
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_BROADCAST, n, chunk, fusion)
    stages = sched.stages()
    check_no_unordered_conflicts(stages)
    bufs = [a.copy() for a in x]
    run_stages(bufs, stages, topological_order(stages, 8))
    want = ox.broadcast_definition(x, roots, w)
    assert all(np.array_equal(b.view(np.uint32), want.view(np.uint32)) for b in bufs)

    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_REDUCE, n, chunk, fusion)
    stages = sched.stages()
    check_no_unordered_conflicts(stages)
    bufs = [a.copy() for a in x]
    run_stages(bufs, stages, topological_order(stages, 9))
    want = ox.tree_order_allreduce(x, roots, parents, w)
    b = sched.bounds()
    for t, r in enumerate(roots):
        assert np.array_equal(bufs[r][b[t]:b[t + 1]].view(np.uint32), want[b[t]:b[t + 1]].view(np.uint32))


@pytest.mark.parametrize("top,root", [(si.hybrid_cube_mesh(), 0), (si.chain(5), 2),
                                      (si.complete_graph(16), bl.BLINK_ROOT_ANY)])
@pytest.mark.parametrize("fusion", FUSIONS)
def test_gather_stages_replayed_on_the_cpu(top, root, fusion):
    k = top.k
    n, chunk = k * 1_250, 512
    trees = pack(top, root)
    roots, _, _ = trees.as_lists()
    x = [si.payload(5, r, n, "int", "int32") for r in range(k)]
    want = ox.allgather_definition(x)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLGATHER, n, chunk, fusion)
    stages = sched.stages()
    check_no_unordered_conflicts(stages)
    bufs = as_views([a.copy() for a in x])
    run_stages(bufs, stages, topological_order(stages, 10))
    assert all(np.array_equal(b, want.view(np.uint32)) for b in bufs)
    if len(set(roots)) == 1:
        sched = bl.blink_make_schedule(trees, bl.BLINK_OP_GATHER, n, chunk, fusion)
        stages = sched.stages()
        check_no_unordered_conflicts(stages)
        bufs = as_views([a.copy() for a in x])
        run_stages(bufs, stages, topological_order(stages, 11))
        assert np.array_equal(bufs[roots[0]], want.view(np.uint32))


@pytest.mark.parametrize("layout", LAYOUT_NAMES)
@pytest.mark.parametrize("fusion", FUSIONS)
def test_multi_server_stages_replayed_on_the_cpu(layout, fusion):
    n, chunk = 20_011, 2048
    sched, servers = make(layout, n, chunk, fusion)
    k = sum(len(s.ranks) for s in servers)
    stages = sched.stages()
    check_no_unordered_conflicts(stages)
    x = [si.payload(6, r, n, "uniform", "fp32") for r in range(k)]
    want = om.three_phase_allreduce(x, servers)
    bufs = [a.copy() for a in x]
    run_stages(bufs, stages, topological_order(stages, 12))
    for b in bufs:
        assert np.array_equal(b.view(np.uint32), want.view(np.uint32))


def test_the_race_check_catches_a_dropped_dependency():
    top = si.chain(4)
    sched = bl.blink_make_schedule(pack(top, 0), bl.BLINK_OP_ALLREDUCE, 4_096, 1_024, bl.BLINK_FUSE_EDGE)
    stages = sched.stages().copy()
    check_no_unordered_conflicts(stages)
    victim = next(i for i, s in enumerate(stages) if int(s["n_dep"]) > 0)
    stages[victim]["n_dep"] = 0
    with pytest.raises(AssertionError):
        check_no_unordered_conflicts(stages)


def test_stack_programs_of_deep_and_random_trees():
    """Depth of the stack program: a caterpillar whose every second child is the
    next internal node needs one accumulator per level (k / 2 of them), which is
    the worst case; random trees stay within n_load / 2 and replay correctly."""
    k = 16
    parent = [-1] + [0] * (k - 1)
    # vertex 0: children 1 (leaf) and 2; vertex 2: children 3 (leaf) and 4; ...
    for v in range(1, k):
        parent[v] = v - 1 if v % 2 == 1 else v - 2
    trees = bl.blink_trees_from_arrays(k, [0], [parent], [1.0])
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 4096, 1024, bl.BLINK_FUSE_TREE)
    stages = sched.stages()
    assert int(stages[0]["seq_depth"]) == k // 2
    x = [si.payload(8, r, 4096, "uniform", "fp32") for r in range(k)]
    want = ox.tree_order_allreduce(x, [0], [tuple(parent)], [1.0])
    bufs = [a.copy() for a in x]
    run_stages(bufs, stages, list(range(len(stages))))
    assert all(np.array_equal(b.view(np.uint32), want.view(np.uint32)) for b in bufs)
    rng = np.random.default_rng(5)
    for _ in range(40):
        k = int(rng.integers(2, 17))
        order = rng.permutation(k)
        parent = [0] * k
        parent[order[0]] = -1
        for i in range(1, k):
            parent[order[i]] = int(order[rng.integers(0, i)])
        root = int(order[0])
        trees = bl.blink_trees_from_arrays(k, [root], [parent], [1.0])
        for fusion in FUSIONS:
            sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 1000, 256, fusion)
            stages = sched.stages()
            x = [si.payload(9, r, 1000, "uniform", "fp32") for r in range(k)]
            want = ox.tree_order_allreduce(x, [root], [tuple(parent)], [1.0])
            bufs = [a.copy() for a in x]
            run_stages(bufs, stages, topological_order(stages, 3))
            assert all(np.array_equal(b.view(np.uint32), want.view(np.uint32)) for b in bufs)
