"""Randomised differential tests: random spanning trees, weights, payload and
chunk sizes through the library's scheduler, judged by the oracle's validators
and by replaying the library's step list on the CPU.  Seeded; no GPU."""
import numpy as np
import pytest

import paper_1910_04940_amd as bl
import synth_inputs as si
from oracle import execute as ox
from oracle import schedule as osch

from test_host_library import to_oracle_steps

OPS = {bl.BLINK_OP_ALLREDUCE: osch.ALLREDUCE, bl.BLINK_OP_BROADCAST: osch.BROADCAST,
       bl.BLINK_OP_REDUCE: osch.REDUCE_TO_ROOT}


def random_case(seed, same_root):
    rng = np.random.default_rng([77, seed])
    k = int(rng.integers(2, 17))
    T = int(rng.integers(1, 6))
    roots, parents = [], []
    root0 = int(rng.integers(k))
    for _ in range(T):
        root = root0 if same_root else int(rng.integers(k))
        order = [root] + [int(v) for v in rng.permutation([v for v in range(k) if v != root])]
        parent = [-1] * k
        for i in range(1, k):     # attach every vertex to a random earlier one: a random arborescence
            parent[order[i]] = order[int(rng.integers(i))]
        roots.append(root)
        parents.append(tuple(parent))
    weights = [float(w) for w in np.exp(rng.uniform(-6, 6, T))]
    n = int(rng.choice([0, 1, 3, 4, 17, 255, 1024, int(rng.integers(1, 6000))]))
    chunk = int(rng.choice([1, 4, 7, 64, 1000, 4096, int(rng.integers(1, 3000))]))
    return k, roots, parents, weights, n, chunk


@pytest.mark.parametrize("seed", range(60))
def test_random_trees_schedule_and_replay(seed):
    op = [bl.BLINK_OP_ALLREDUCE, bl.BLINK_OP_BROADCAST, bl.BLINK_OP_REDUCE][seed % 3]
    fusion = [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE][(seed // 3) % 3]
    k, roots, parents, w, n, chunk = random_case(seed, same_root=op == bl.BLINK_OP_BROADCAST)
    trees = bl.blink_trees_from_arrays(k, roots, parents, w)
    sched = bl.blink_make_schedule(trees, op, n, chunk, fusion)
    assert sched.bounds() == osch.split_by_weight(n, w)
    osch.check_split(sched.bounds(), n, w)
    steps = to_oracle_steps(sched)
    osch.check_steps(steps, k, roots, parents, w, OPS[op], n, chunk)
    assert len(steps) == len(osch.make_steps(roots, parents, w, OPS[op], n, chunk))
    # replay on data, in a shuffled topological order
    x = [si.payload(seed, r, n, "uniform", "fp32") for r in range(k)]
    bufs = [a.copy() for a in x]
    ox.run_steps(bufs, steps, ox.random_topological_order(steps, seed))
    b = sched.bounds()
    if op == bl.BLINK_OP_BROADCAST:
        want = ox.broadcast_definition(x, roots, w)
        assert all(np.array_equal(g.view(np.uint32), want.view(np.uint32)) for g in bufs)
    else:
        want = ox.tree_order_allreduce(x, roots, parents, w)
        holders = range(k) if op == bl.BLINK_OP_ALLREDUCE else None
        for t, r in enumerate(roots):
            for v in (holders if holders is not None else [r]):
                assert np.array_equal(bufs[v][b[t]:b[t + 1]].view(np.uint32), want[b[t]:b[t + 1]].view(np.uint32))
