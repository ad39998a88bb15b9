"""blink_allreduce_noalloc (the entry point for callers that cannot allocate)
against blink_allreduce, through the C ABI: same inputs, same schedule, results
compared bit for bit (int32 and fp32; the fp32 bar of at most 1e-6 relative is
implied by equality), and against the CPU oracle.  Calls come in pairs on one
stream without a synchronisation in between, the second on a smaller input, and
use the device block all such calls share."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox
from oracle import schedule as osch

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1910_04940_amd as bl  # noqa: E402

FUSIONS = [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE]


def _setup():
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    return dev, torch.cuda.current_stream().cuda_stream


def _case(top, root, n, chunk, dtype, fusion, seed):
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, root)
    roots, parents, w = trees.as_lists()
    x = [si.payload(seed, r, n, "int" if dtype == "int32" else "uniform", dtype) for r in range(top.k)]
    want = [a.copy() for a in x]
    ox.run_steps(want, osch.make_steps(roots, parents, w, osch.ALLREDUCE, n, chunk))
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    return x, want, sched


@pytest.mark.parametrize("dtype", ["int32", "fp32"])
@pytest.mark.parametrize("fusion", FUSIONS)
def test_two_calls_in_a_row_second_smaller(dtype, fusion):
    dev, stream = _setup()
    code = bl.BLINK_INT32 if dtype == "int32" else bl.BLINK_FP32
    big = _case(si.hybrid_cube_mesh(), 0, (1 << 20) + 12, 1 << 16, dtype, fusion, 11)
    small = _case(si.complete_graph(4), 1, 300_001, 1 << 13, dtype, fusion, 12)
    for round_no in range(2):                      # the second round finds the block holding the other tables
        got = []
        for x, want, sched in (big, small):
            bufs = [torch.from_numpy(a).to(dev) for a in x]
            bl.blink_allreduce_noalloc(bufs, len(x[0]), code, sched, stream)
            got.append(bufs)
        torch.cuda.synchronize()
        for (x, want, sched), bufs in zip((big, small), got):
            ref = [torch.from_numpy(a).to(dev) for a in x]
            bl.blink_allreduce(ref, len(x[0]), code, sched, stream)      # the existing entry point
            torch.cuda.synchronize()
            for r, (b, rb, wv) in enumerate(zip(bufs, ref, want)):
                g, e = b.cpu().numpy(), rb.cpu().numpy()
                assert np.array_equal(g.view(np.uint32), e.view(np.uint32)), (round_no, r, "vs blink_allreduce")
                assert np.array_equal(g.view(np.uint32), wv.view(np.uint32)), (round_no, r, "vs oracle")
            assert sched.status()[0] == bl.BLINK_OK


def test_repeated_calls_on_one_schedule_and_mixing_with_the_allocating_entry_point():
    dev, stream = _setup()
    x, want, sched = _case(si.hybrid_cube_mesh(), 0, 1 << 18, 1 << 14, "int32", bl.BLINK_FUSE_EDGE, 13)
    total = [a.copy() for a in x]
    bufs = [torch.from_numpy(a).to(dev) for a in x]
    trees = bl.blink_pack_trees(8, *[getattr(si.hybrid_cube_mesh(), f) for f in ("src", "dst", "cap")], 0)
    roots, parents, w = trees.as_lists()
    steps = osch.make_steps(roots, parents, w, osch.ALLREDUCE, 1 << 18, 1 << 14)
    for i in range(6):                             # in place: each call works on the previous result
        if i % 3 == 2:
            bl.blink_allreduce(bufs, 1 << 18, bl.BLINK_INT32, sched, stream)
        else:
            bl.blink_allreduce_noalloc(bufs, 1 << 18, bl.BLINK_INT32, sched, stream)
        ox.run_steps(total, steps)
    torch.cuda.synchronize()
    for b, wv in zip(bufs, total):
        assert np.array_equal(b.cpu().numpy(), wv)
    assert sched.status()[0] == bl.BLINK_OK


def test_a_schedule_beyond_the_block_is_refused_and_nothing_runs():
    dev, stream = _setup()
    top = si.hybrid_cube_mesh()
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
    n = 1 << 20
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, 1 << 10, bl.BLINK_FUSE_EDGE)
    assert sched.num_stages * 312 > (4 << 20)
    bufs = [torch.full((n,), r + 1, dtype=torch.int32, device=dev) for r in range(top.k)]
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_allreduce_noalloc(bufs, n, bl.BLINK_INT32, sched, stream)
    assert e.value.status == bl.BLINK_ELIMIT
    torch.cuda.synchronize()
    for r, b in enumerate(bufs):
        assert int(b.min()) == r + 1 and int(b.max()) == r + 1
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream)          # the allocating entry point takes it
    torch.cuda.synchronize()
    assert int(bufs[3].min()) == 36 and int(bufs[3].max()) == 36


def test_arguments_are_checked_like_blink_allreduce():
    dev, stream = _setup()
    x, want, sched = _case(si.complete_graph(4), 0, 4096, 1024, "int32", bl.BLINK_FUSE_TREE, 14)
    bufs = [torch.from_numpy(a).to(dev) for a in x]
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_allreduce_noalloc(bufs[:3], 4096, bl.BLINK_INT32, sched, stream)
    assert e.value.status == bl.BLINK_EMISMATCH
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_allreduce_noalloc([bufs[0], bufs[0], bufs[1], bufs[2]], 4096, bl.BLINK_INT32, sched, stream)
    assert e.value.status == bl.BLINK_EINVAL
