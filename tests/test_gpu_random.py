"""GPU parity on random spanning trees, weights, payload and chunk sizes (the
cases of tests/test_random_schedules.py, larger payloads), through the C ABI."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox

from test_gpu_parity import bl, dev, stream, to_dev, torch  # noqa: F401
from test_random_schedules import random_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(45))
def test_random_trees_on_the_gpu(dev, seed):
    op = [bl.BLINK_OP_ALLREDUCE, bl.BLINK_OP_BROADCAST, bl.BLINK_OP_REDUCE][seed % 3]
    fusion = [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE][(seed // 3) % 3]
    dtype = ["fp32", "int32"][(seed // 9) % 2]
    k, roots, parents, w, n, chunk = random_case(seed, same_root=op == bl.BLINK_OP_BROADCAST)
    rng = np.random.default_rng([78, seed])
    n = n * int(rng.integers(1, 60)) + int(rng.integers(0, 4))        # up to ~350 k elements, ragged
    chunk = chunk * int(rng.integers(1, 40))
    trees = bl.blink_trees_from_arrays(k, roots, parents, w)
    sched = bl.blink_make_schedule(trees, op, n, chunk, fusion)
    x = [si.payload(seed, r, n, "int" if dtype == "int32" else "uniform", dtype) for r in range(k)]
    bufs = to_dev(x, dev)
    code = bl.BLINK_INT32 if dtype == "int32" else bl.BLINK_FP32
    print(f"seed {seed}: k={k} T={len(roots)} n={n} chunk={chunk} op={op} fusion={fusion} {dtype}", flush=True)
    if op == bl.BLINK_OP_ALLREDUCE:
        bl.blink_allreduce(bufs, n, code, sched, stream())
    elif op == bl.BLINK_OP_BROADCAST:
        bl.blink_broadcast(bufs, n, code, sched, stream())
    else:
        bl.blink_reduce(bufs, n, code, bl.BLINK_SUM, sched, stream())
    torch.cuda.synchronize()
    got = [b.cpu().numpy() for b in bufs]
    b = sched.bounds()
    if op == bl.BLINK_OP_BROADCAST:
        want = ox.broadcast_definition(x, roots, w)
        assert all(g.tobytes() == want.tobytes() for g in got)
        return
    want = ox.tree_order_allreduce(x, roots, parents, w)
    if dtype == "int32":
        assert np.array_equal(want, ox.allreduce_int32_definition(x))
    for t, r in enumerate(roots):
        for v in (range(k) if op == bl.BLINK_OP_ALLREDUCE else [r]):
            assert got[v][b[t]:b[t + 1]].tobytes() == want[b[t]:b[t + 1]].tobytes(), (t, v)


@pytest.mark.parametrize("seed", [2, 6, 16, 24, 34])
@pytest.mark.parametrize("fusion", [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE])
def test_many_unevenly_weighted_trees_from_real_valued_capacities(dev, seed, fusion):
    """Random digraphs with real-valued capacities: the packer returns a dozen or
    more trees with uneven weights, hence many flows with ragged shares."""
    k = 8 + seed % 9
    top = si.random_digraph(k, 0.5, 4000 + seed, int_caps=False)
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
    roots, parents, w = trees.as_lists()
    assert trees.count >= 8
    n, chunk = 400_003, 9_000
    x = [si.payload(seed, r, n, "uniform", "fp32") for r in range(k)]
    want = ox.tree_order_allreduce(x, roots, parents, w)
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    print(f"seed {seed}: k={k} T={trees.count} fusion={fusion}", flush=True)
    bl.blink_allreduce(bufs, n, bl.BLINK_FP32, sched, stream())
    torch.cuda.synchronize()
    for b in bufs:
        assert b.cpu().numpy().tobytes() == want.tobytes()
