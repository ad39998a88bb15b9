"""Fair sharing of the machine among the trees (paper section 4.2.2): where trees
pass through the same link, one chunk of the first is sent, then one chunk of
the second, and so on, instead of one tree running ahead and the others being
"arbitrarily delayed", which "introduces gaps in the forwarding pipeline".

The oracle states the scheme (oracle.schedule.fair_order) and a model to judge
orders by (link_timeline: unit-time steps, one step per directed link at a
time, served in list order).  Its numbers on the section's own example are
pinned to values derived by hand below.  The library's two orderings are then
held to the same properties: the public step list (per-edge program) and the
order in which the kernel hands out tiles (whole-tree program).  No GPU."""
import numpy as np
import pytest

import paper_1910_04940_amd as bl
import synth_inputs as si
from oracle import schedule as osch

# The example of section 4.2.2: two trees that both start at GPU1 and share the
# link GPU1 -> GPU2 as their first hop, then part ways.  0-based, 4 vertices:
#   tree 0: 0 -> 1 -> 2 -> 3        tree 1: 0 -> 1 -> 3 -> 2
ROOTS = [0, 0]
PARENTS = [(-1, 0, 1, 2), (-1, 0, 3, 1)]
WEIGHTS = [0.5, 0.5]
CHUNKS = 8
CHUNK = 1024
N = 2 * CHUNKS * CHUNK


def tree_major_steps():
    steps = osch.make_steps(ROOTS, PARENTS, WEIGHTS, osch.BROADCAST, N, CHUNK)
    assert [s.tree for s in steps] == sorted(s.tree for s in steps)        # the oracle emits tree by tree
    return steps


def test_oracle_fair_order_on_the_papers_example_matches_hand_derived_times():
    unfair = tree_major_steps()
    fair = osch.fair_order(unfair)
    assert sorted((s.tree, s.chunk, s.src, s.dst, s.off, s.len) for s in fair) == \
        sorted((s.tree, s.chunk, s.src, s.dst, s.off, s.len) for s in unfair)
    osch.check_steps(fair, 4, ROOTS, PARENTS, WEIGHTS, osch.BROADCAST, N, CHUNK)
    # The shared link 0 -> 1 carries 2 * CHUNKS chunks, one per time unit, whatever
    # the order; the last one then has two more hops to go: both orders end at
    # 2 * CHUNKS + 2.  (In this model fairness does not shorten the whole; it
    # bounds how long any one tree is held up.)
    assert osch.pipeline_makespan(unfair) == 2 * CHUNKS + 2 == 18
    assert osch.pipeline_makespan(fair) == 2 * CHUNKS + 2
    assert osch.pipeline_makespan(fair) <= osch.pipeline_makespan(unfair)
    # Tree-major: tree 1's chunk j enters the shared link at CHUNKS + j and is done
    # 3 hops later; its own link 1 -> 3 sits idle for CHUNKS + 1 units first.
    done = osch.chunk_finish_times(unfair)
    assert [done[(0, j)] for j in range(CHUNKS)] == [j + 3 for j in range(CHUNKS)]
    assert [done[(1, j)] for j in range(CHUNKS)] == [CHUNKS + j + 3 for j in range(CHUNKS)]
    assert osch.longest_idle_gap(unfair, (1, 3)) == CHUNKS + 1 == 9
    # Fair: the trees alternate on the shared link, tree 0 at even times, tree 1
    # at odd ones; every chunk is done 3 hops after it entered; no link of either
    # tree waits more than one unit between chunks (two before its first).
    done = osch.chunk_finish_times(fair)
    assert [done[(0, j)] for j in range(CHUNKS)] == [2 * j + 3 for j in range(CHUNKS)]
    assert [done[(1, j)] for j in range(CHUNKS)] == [2 * j + 4 for j in range(CHUNKS)]
    for link in ((1, 2), (2, 3), (1, 3), (3, 2)):
        assert osch.longest_idle_gap(fair, link) <= 3
    assert osch.longest_idle_gap(fair, (1, 3)) == 2
    # no tree is ever more than one chunk ahead of the other
    for j in range(CHUNKS):
        assert abs(done[(0, j)] - done[(1, j)]) == 1


def test_a_planted_unfair_order_is_told_apart():
    """The properties above must separate the two orders (else they pin nothing)."""
    unfair = tree_major_steps()
    done = osch.chunk_finish_times(unfair)
    assert max(abs(done[(0, j)] - done[(1, j)]) for j in range(CHUNKS)) == CHUNKS
    assert osch.longest_idle_gap(unfair, (1, 3)) > 3


def as_oracle_steps(arr):
    return [osch.Step(int(s["kind"]), int(s["tree"]), int(s["chunk"]), int(s["src"]), int(s["dst"]), int(s["off"]),
                      int(s["len"]), tuple(int(d) for d in s["deps"][:int(s["n_deps"])])) for s in arr]


def test_library_step_list_on_the_papers_example_is_fair():
    trees = bl.blink_trees_from_arrays(4, ROOTS, PARENTS, WEIGHTS)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_BROADCAST, N, CHUNK, bl.BLINK_FUSE_EDGE)
    steps = as_oracle_steps(sched.steps())
    osch.check_steps(steps, 4, ROOTS, PARENTS, WEIGHTS, osch.BROADCAST, N, CHUNK)
    done = osch.chunk_finish_times(steps)
    assert osch.pipeline_makespan(steps) == 2 * CHUNKS + 2
    for j in range(CHUNKS):
        assert abs(done[(0, j)] - done[(1, j)]) <= 1
    for link in ((1, 2), (2, 3), (1, 3), (3, 2)):
        assert osch.longest_idle_gap(steps, link) <= 3
    # on the shared link the trees alternate chunk by chunk
    shared = [(s.chunk, s.tree) for s in steps if (s.src, s.dst) == (0, 1)]
    assert shared == [(j, t) for j in range(CHUNKS) for t in (0, 1)]


@pytest.mark.parametrize("coll", [bl.BLINK_OP_BROADCAST, bl.BLINK_OP_ALLREDUCE])
def test_library_step_list_shares_every_link_chunk_by_chunk(coll):
    """On every directed link, among transfers at the same position in their
    trees, no tree sends a chunk of the next batch before every tree using that
    link there has sent its chunks of this one, and inside a batch the trees
    alternate chunk by chunk wherever they are at the same stage of their
    pipelines (a batch is blink_schedule_batch chunks: 1 unless the schedule has
    many small chunks)."""
    for top, root in ((si.hybrid_cube_mesh(), 0), (si.hybrid_cube_mesh(True), 3), (si.complete_graph(8), 2)):
        trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, root)
        roots, parents, w = trees.as_lists()
        n = trees.count * 6 * 512
        sched = bl.blink_make_schedule(trees, coll, n, 512, bl.BLINK_FUSE_EDGE)
        steps = sched.steps()
        batch = sched.batch
        assert 1 <= batch <= 6
        depth = []
        for p in parents:
            d = [0] * top.k
            for v in range(top.k):
                u, c = v, 0
                while p[u] >= 0:
                    u, c = p[u], c + 1
                d[v] = c
            depth.append(d)
        per_link = {}
        for s in steps:
            t = int(s["tree"])
            level = depth[t][int(s["dst"])] if int(s["kind"]) == bl.BLINK_STEP_COPY else -depth[t][int(s["src"])]
            per_link.setdefault((int(s["src"]), int(s["dst"]), level), []).append((int(s["chunk"]), t))
        shared = 0
        for key, seq in per_link.items():
            by_batch = [(c // batch, t) for c, t in seq]
            assert [b for b, _ in by_batch] == sorted(b for b, _ in by_batch), f"link {key}: {seq[:8]}"
            for t in {t for _, t in seq}:
                own = [c for c, tt in seq if tt == t]
                assert own == sorted(own), f"link {key}, tree {t}: its own chunks out of order"
            shared += len({t for _, t in seq}) > 1
        if top.name.startswith("hybrid") and coll == bl.BLINK_OP_BROADCAST and root == 0:
            assert shared > 0, "the cube-mesh trees from one root do share first-hop links"


def test_tile_order_of_the_whole_tree_program_walks_across_the_trees():
    """The kernel hands out tickets in ascending order; where no stage waits for
    another, ticket -> (stage, tile) goes tile by tile across the trees: the
    finest form of taking turns.  This is the function the kernels call."""
    top = si.hybrid_cube_mesh()
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
    T = trees.count
    n, chunk, tile = (1 << 22) + 40, 1 << 18, 2048
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_TREE)
    stages = sched.stages()
    stage, tl = sched.tickets(tile)
    real = tl >= 0
    # every (stage, tile) with elements in it exactly once, none missing
    want = set()
    for i, s in enumerate(stages):
        off, ln = int(s["off"]), int(s["len"])
        for b in range(off // tile, (off + ln + tile - 1) // tile):
            want.add((i, b - off // tile))
    got = list(zip(stage[real].tolist(), tl[real].tolist()))
    assert len(got) == len(set(got)) and set(got) == want
    # consecutive tickets go to consecutive trees, the tile index moves on once per round
    tree_of = np.array([int(s["tree"]) for s in stages])[stage]
    per_round = T
    full = (len(stage) // per_round) * per_round
    rounds = tree_of[:full].reshape(-1, per_round)
    assert all(sorted(r.tolist()) == list(range(T)) for r in rounds), "a round of tickets visits every tree once"
    first = np.flatnonzero(tl[:per_round * 8:per_round] >= 0)
    assert tl[0] == 0 and tl[per_round] == 1 and len(first) == 8
    # no tree is ever more than one tile ahead of another within a chunk position
    seen = {}
    for t_idx, (sg, ti) in enumerate(zip(stage.tolist(), tl.tolist())):
        c = int(stages[sg]["chunk"])
        seen.setdefault(c, {})[int(stages[sg]["tree"])] = ti
        if len(seen[c]) == T and min(seen[c].values()) >= 0:
            assert max(seen[c].values()) - min(seen[c].values()) <= 1


def test_tile_order_keeps_stages_together_where_that_is_the_rule():
    """Stages that wait for one another follow the execution order itself; so do
    whole-tree stages that read more than 8 ranks (too many request streams at a
    time otherwise)."""
    top = si.complete_graph(16)
    trees = bl.blink_pack_trees(16, top.src, top.dst, top.cap, bl.BLINK_ROOT_ANY)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 16 * 8192, 4096, bl.BLINK_FUSE_TREE)
    stage, tl = sched.tickets(1024)
    assert stage.tolist() == sorted(stage.tolist())
    cm = si.hybrid_cube_mesh()
    trees = bl.blink_pack_trees(8, cm.src, cm.dst, cm.cap, 0)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 1 << 16, 1 << 12, bl.BLINK_FUSE_EDGE)
    stage, tl = sched.tickets(1024)
    assert stage.tolist() == sorted(stage.tolist())
    with pytest.raises(bl.BlinkError):
        sched.tickets(1000)


@pytest.mark.parametrize("seed", range(40))
def test_tickets_of_random_schedules_cover_every_tile_exactly_once(seed):
    """Random trees, weights, sizes, chunk and tile sizes, every fusion level:
    the tickets that stand for something are exactly the (stage, tile) pairs
    that hold elements; and the last group of stages gets no more rounds of
    tickets than its largest stage has tiles."""
    from test_random_schedules import random_case
    rng = np.random.default_rng([81, seed])
    k, roots, parents, w, _, _ = random_case(3000 + seed, same_root=False)
    n = int(rng.integers(1, 400_000))
    chunk = int(rng.integers(1, 60_000))
    tile = 1 << int(rng.integers(8, 13))
    fusion = [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE][seed % 3]
    trees = bl.blink_trees_from_arrays(k, roots, parents, w)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    stages = sched.stages()
    stage, tl = sched.tickets(tile)
    real = tl >= 0
    want = set()
    for i, s in enumerate(stages):
        off, ln = int(s["off"]), int(s["len"])
        for b in range(off // tile, (off + ln + tile - 1) // tile):
            want.add((i, b - off // tile))
    got = list(zip(stage[real].tolist(), tl[real].tolist()))
    assert len(got) == len(set(got)) and set(got) == want
    if len(stage):
        # the last ticket's round is one some stage of its group needs
        last_stage = int(stage[-1])
        group = set(stage[np.flatnonzero(stage == last_stage)[0]:].tolist())
        last_round = max(t for s_, t in want if s_ in group)
        assert sum(1 for s_, t in zip(stage.tolist(), tl.tolist()) if s_ in group and t == last_round) >= 1
