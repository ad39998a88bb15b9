"""The two kernels that can run a whole-tree sum at streaming size (the
ticket-drawing kernel with loads staged through registers, and the streaming
kernel with loads straight into LDS and the stage computed as a stack program),
each forced in turn, and the automatic choice between them: all against the
oracle, bit for bit.  Sizes are large enough that the schedules stream (below
that size both choices run the small-payload kernel)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1910_04940_amd as bl  # noqa: E402


def _dev():
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    return dev, torch.cuda.current_stream().cuda_stream


def _deep_tree(k):
    """Every second child is the next internal vertex: the stack program needs
    k / 2 accumulators."""
    parent = [-1] + [0] * (k - 1)
    for v in range(1, k):
        parent[v] = v - 1 if v % 2 == 1 else v - 2
    return parent


CASES = [
    # topology, root, elements per rank (ragged, and not a multiple of 4), chunk
    ("cube", 0, (1 << 24) + 4_099, 1 << 18),
    ("cube2-6", 0, 13_000_003, 250_001),          # chunks that do not start on 16-byte boundaries
    ("k16", bl.BLINK_ROOT_ANY, (1 << 23) + 12, 1 << 20),
    ("k2", 1, (1 << 26) + 1, 1 << 20),
    ("chain5", 2, 30_000_002, 1 << 19),
    ("deep8", 0, (1 << 24) + 7, 1 << 18),          # 4 accumulators: the most the streaming kernel takes
    ("deep12", 0, 9_000_001, 1 << 18),             # 6 accumulators: only the ticket-drawing kernel can run it
]


def _trees(name, root):
    if name.startswith("deep"):
        k = int(name[4:])
        return k, bl.blink_trees_from_arrays(k, [0], [_deep_tree(k)], [1.0])
    top = {"cube": si.hybrid_cube_mesh, "k16": lambda: si.complete_graph(16), "k2": lambda: si.complete_graph(2),
           "cube2-6": lambda: si.induced(si.hybrid_cube_mesh(True), (0, 1, 3, 4, 5, 7)),
           "chain5": lambda: si.chain(5)}[name]()
    return top.k, bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, root)


@pytest.mark.parametrize("kernel", [1, 2, 3])
@pytest.mark.parametrize("name,root,n,chunk", CASES)
def test_each_kernel_against_the_oracle(name, root, n, chunk, kernel):
    dev, stream = _dev()
    k, trees = _trees(name, root)
    roots, parents, w = trees.as_lists()
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_TREE)
    sched.set_kernel(kernel)
    for dtype, code in (("int32", bl.BLINK_INT32), ("fp32", bl.BLINK_FP32)):
        x = [si.hash_payload(21, r, 0, n, dtype) for r in range(k)]
        want = ox.tree_order_allreduce(x, roots, parents, w)
        if dtype == "int32":
            assert np.array_equal(want, ox.allreduce_int32_definition(x))
        bufs = [torch.from_numpy(a).to(dev) for a in x]
        bl.blink_allreduce(bufs, n, code, sched, stream)
        torch.cuda.synchronize()
        one_tree = name.startswith("deep") or name in ("k2", "chain5")
        expected_kernel = 1 if (name == "deep12" or (kernel == 3 and (one_tree or name == "k16"))) else kernel
        assert sched.last_kernel == expected_kernel
        for r, b in enumerate(bufs):
            got = b.cpu().numpy()
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (name, dtype, kernel, r)
        del bufs


@pytest.mark.parametrize("coll", ["reduce", "broadcast"])
def test_streaming_kernel_on_reduce_and_broadcast(coll):
    dev, stream = _dev()
    top = si.hybrid_cube_mesh()
    n, chunk, k = (1 << 25) + 8, 1 << 18, 8
    trees = bl.blink_pack_trees(k, top.src, top.dst, top.cap, 0)
    roots, parents, w = trees.as_lists()
    x = [si.hash_payload(22, r, 0, n, "int32") for r in range(k)]
    bufs = [torch.from_numpy(a).to(dev) for a in x]
    if coll == "reduce":
        sched = bl.blink_make_schedule(trees, bl.BLINK_OP_REDUCE, n, chunk, bl.BLINK_FUSE_TREE)
        sched.set_kernel(2)
        bl.blink_reduce(bufs, n, bl.BLINK_INT32, bl.BLINK_SUM, sched, stream)
        torch.cuda.synchronize()
        assert sched.last_kernel == 2
        assert np.array_equal(bufs[0].cpu().numpy(), ox.allreduce_int32_definition(x))
        for r in range(1, k):
            assert np.array_equal(bufs[r].cpu().numpy(), x[r])
        # another operator than the sum runs on the ticket-drawing kernel, whatever was asked for
        bufs = [torch.from_numpy(a).to(dev) for a in x]
        bl.blink_reduce(bufs, n, bl.BLINK_INT32, bl.BLINK_MAX, sched, stream)
        torch.cuda.synchronize()
        assert sched.last_kernel == 1
        assert np.array_equal(bufs[0].cpu().numpy(), np.maximum.reduce(x))
    else:
        sched = bl.blink_make_schedule(trees, bl.BLINK_OP_BROADCAST, n, chunk, bl.BLINK_FUSE_TREE)
        sched.set_kernel(2)
        bl.blink_broadcast(bufs, n, bl.BLINK_INT32, sched, stream)
        torch.cuda.synchronize()
        assert sched.last_kernel == 2
        for b in bufs:
            assert np.array_equal(b.cpu().numpy(), x[0])


def test_automatic_choice_times_every_way_and_settles():
    dev, stream = _dev()
    top = si.hybrid_cube_mesh()
    n, chunk, k = 1 << 24, 1 << 18, 8
    trees = bl.blink_pack_trees(k, top.src, top.dst, top.cap, 0)
    roots, parents, w = trees.as_lists()
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_TREE)
    x = [si.hash_payload(23, r, 0, n, "int32") for r in range(k)]
    want = ox.allreduce_int32_definition(x)
    seen = []
    for call in range(16):
        bufs = [torch.from_numpy(a).to(dev) for a in x]
        bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream)
        seen.append(sched.last_kernel)
        torch.cuda.synchronize()
        for b in bufs:
            assert np.array_equal(b.cpu().numpy(), want), call
    # the timed calls go round the three ways (either kernel, and the first with
    # the trees taking turns chunk by chunk), then one of them serves
    assert seen[:12] == [1, 2, 3] * 4
    assert len(set(seen[12:])) == 1 and seen[12] in (1, 2, 3)
    # one tree: nothing to take turns, two ways
    one = bl.blink_trees_from_arrays(k, [0], [_deep_tree(k)], [1.0])
    sched = bl.blink_make_schedule(one, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_TREE)
    seen = []
    for call in range(10):
        bufs = [torch.from_numpy(a).to(dev) for a in x]
        bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream)
        seen.append(sched.last_kernel)
        torch.cuda.synchronize()
        assert np.array_equal(bufs[k - 1].cpu().numpy(), want), call
    assert seen[:8] == [1, 2] * 4 and len(set(seen[8:])) == 1 and seen[8] in (1, 2)
    # a small payload is not worth a trial
    m = 1 << 12
    small = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, m, 1 << 10, bl.BLINK_FUSE_TREE)
    bufs = [torch.zeros(m, dtype=torch.int32, device=dev) for _ in range(k)]
    for _ in range(3):
        bl.blink_allreduce(bufs, m, bl.BLINK_INT32, small, stream)
        assert small.last_kernel == 1
    torch.cuda.synchronize()


@pytest.mark.parametrize("kernel", [1, 2, 3])
def test_alternating_sweep_gives_the_same_bits_as_forward_calls(kernel):
    """Every other call on a dependency-free schedule goes through the tiles
    backwards (the default); with that switched off all go forwards.  Four calls
    in a row, ragged size: the same bits after every call, and the oracle's."""
    dev, stream = _dev()
    top = si.hybrid_cube_mesh()
    n, chunk, k = (1 << 24) + 1_027, 250_001, 8
    trees = bl.blink_pack_trees(k, top.src, top.dst, top.cap, 0)
    roots, parents, w = trees.as_lists()
    x = [si.hash_payload(29, r, 0, n, "fp32") for r in range(k)]
    results = {}
    for alternate in (True, False):
        sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_TREE)
        sched.set_kernel(kernel)
        sched.set_sweep(alternate)
        bufs = [torch.from_numpy(a).to(dev) for a in x]
        after = []
        for _ in range(4):
            bl.blink_allreduce(bufs, n, bl.BLINK_FP32, sched, stream)
            torch.cuda.synchronize()
            assert sched.last_kernel == kernel
            after.append([b.cpu().numpy().view(np.uint32).copy() for b in bufs])
        results[alternate] = after
    want = [a.copy() for a in x]
    for call in range(4):
        summed = ox.tree_order_allreduce(want, roots, parents, w)
        want = [summed.copy() for _ in range(k)]
        for r in range(k):
            assert np.array_equal(results[True][call][r], results[False][call][r]), (call, r)
            assert np.array_equal(results[True][call][r], summed.view(np.uint32)), (call, r)


@pytest.mark.parametrize("kernel", [1, 2, 3])
@pytest.mark.parametrize("past", [(16,) * 8, (512,) * 8, (1008,) * 8, (0, 16, 32, 48, 512, 528, 1008, 64)])
def test_rank_buffers_that_do_not_start_on_1k_boundaries(kernel, past):
    """Rank buffers that are views into larger ones.  Where all of them start
    the same distance past a 1 KiB boundary the library moves its tile grid by
    that distance; where they differ it does not.  Same bits as the oracle in
    both cases, over three calls (the second goes through the tiles backwards)."""
    dev, stream = _dev()
    top = si.hybrid_cube_mesh()
    n, chunk, k = (1 << 24) + 2_051, 1 << 18, 8
    trees = bl.blink_pack_trees(k, top.src, top.dst, top.cap, 0)
    roots, parents, w = trees.as_lists()
    x = [si.hash_payload(31, r, 0, n, "int32") for r in range(k)]
    stride = n + 4096
    slab = torch.zeros(k * stride + 1024, dtype=torch.int32, device=dev)
    assert slab.data_ptr() % 1024 == 0
    bufs = []
    for r in range(k):
        first = r * stride + (-(r * stride) % 256) + past[r] // 4      # elements; 256 elements = 1 KiB
        bufs.append(slab[first:first + n])
        assert bufs[r].data_ptr() % 1024 == past[r]
        bufs[r].copy_(torch.from_numpy(x[r]))
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_TREE)
    sched.set_kernel(kernel)
    want = ox.allreduce_int32_definition(x).view(np.uint32).astype(np.uint64)
    for call in range(3):
        bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream)
        torch.cuda.synchronize()
        assert sched.last_kernel == kernel
        expect = ((want * np.uint64(pow(8, call, 1 << 32))) & np.uint64(0xFFFFFFFF)).astype(np.uint32)
        for r in range(k):
            assert np.array_equal(bufs[r].cpu().numpy().view(np.uint32), expect), (call, r)
    # nothing outside the views was written
    for b in bufs:
        b.zero_()
    assert int(torch.count_nonzero(slab)) == 0, "bytes outside the rank buffers were written"


@pytest.mark.parametrize("n", [1_500_003, 2_713_001, 4_200_005, 6_000_002])
def test_payloads_whose_tickets_are_dealt_out_in_several_rounds(n):
    """Between the smallest payloads (one ticket per wave) and the streaming
    sizes the tickets are dealt out over every wave that fits, two to five each,
    on the 16-column kernel with two waves per SIMD.  Two calls in place, both
    element types, against the oracle."""
    dev, stream = _dev()
    top = si.hybrid_cube_mesh()
    k, chunk = 8, 1 << 18
    trees = bl.blink_pack_trees(k, top.src, top.dst, top.cap, 0)
    roots, parents, w = trees.as_lists()
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_TREE)
    for dtype, code in (("int32", bl.BLINK_INT32), ("fp32", bl.BLINK_FP32)):
        x = [si.hash_payload(41, r, 0, n, dtype) for r in range(k)]
        bufs = [torch.from_numpy(a).to(dev) for a in x]
        want = x
        for call in range(2):
            bl.blink_allreduce(bufs, n, code, sched, stream)
            torch.cuda.synchronize()
            summed = ox.tree_order_allreduce(want, roots, parents, w)
            want = [summed.copy() for _ in range(k)]
            for r, b in enumerate(bufs):
                assert np.array_equal(b.cpu().numpy().view(np.uint32), summed.view(np.uint32)), (dtype, call, r)
    assert sched.last_kernel == 1
    assert sched.status()[0] == bl.BLINK_OK
