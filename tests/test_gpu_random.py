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


def streaming_case(seed):
    """Random trees on a payload large enough for the streaming launch (about
    1 GiB of traffic), ragged, in views that start a random distance past a
    1 KiB boundary: the same distance for all ranks, or one of its own each."""
    k, roots, parents, w, _, _ = random_case(1000 + seed, same_root=False)
    rng = np.random.default_rng([79, seed])
    n = (1 << 27) // k + int(rng.integers(0, 5000))
    chunk = int(rng.integers(50_000, 2_000_000))
    if seed % 3 == 0:
        past = [0] * k
    elif seed % 3 == 1:
        past = [16 * int(rng.integers(0, 64))] * k
    else:
        past = [16 * int(v) for v in rng.integers(0, 64, k)]
    return k, roots, parents, w, n, chunk, past


@pytest.mark.parametrize("seed", range(8))
def test_random_trees_at_streaming_size_over_three_calls(dev, seed):
    """Any of the three ways, three calls in place (the second goes through the tiles
    backwards): after call c every rank holds the oracle's sum times k^(c-1),
    modulo 2^32, and no byte outside the views has changed."""
    k, roots, parents, w, n, chunk, past = streaming_case(seed)
    kernel = 1 + seed % 3      # a way the schedule does not have falls back to the first
    trees = bl.blink_trees_from_arrays(k, roots, parents, w)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_TREE)
    sched.set_kernel(kernel)
    x = [si.payload(200 + seed, r, n, "int", "int32") for r in range(k)]
    stride = n + 4096
    slab = torch.zeros(k * stride + 1024, dtype=torch.int32, device=dev)
    assert slab.data_ptr() % 1024 == 0
    bufs = []
    for r in range(k):
        first = r * stride + (-(r * stride) % 256) + past[r] // 4
        bufs.append(slab[first:first + n])
        assert bufs[r].data_ptr() % 1024 == past[r]
        bufs[r].copy_(torch.from_numpy(x[r]))
    print(f"seed {seed}: k={k} T={len(roots)} n={n} chunk={chunk} past={past} kernel={kernel}", flush=True)
    want = ox.allreduce_int32_definition(x).view(np.uint32).astype(np.uint64)
    for call in range(3):
        bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream())
        torch.cuda.synchronize()
        expect = ((want * np.uint64(pow(k, call, 1 << 32))) & np.uint64(0xFFFFFFFF)).astype(np.uint32)
        for r in range(k):
            assert np.array_equal(bufs[r].cpu().numpy().view(np.uint32), expect), (call, r, sched.last_kernel)
    assert sched.status()[0] == bl.BLINK_OK
    for b in bufs:
        b.zero_()
    assert int(torch.count_nonzero(slab)) == 0, "bytes outside the rank buffers were written"
