"""HIP graphs and the library, through the C ABI.  A call of blink_allreduce
carries its number on the schedule, which a replay would repeat: on a capturing
stream it is refused and records nothing.  blink_allreduce_noalloc starts every
call from cleared counters and allocates nothing: recorded once, it must give
the eager result on every replay (bit for bit, int32 and fp32), with eager work
of the program between the replays."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox
from oracle import schedule as osch

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1910_04940_amd as bl  # noqa: E402

FUSIONS = [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE]


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
def test_a_recorded_noalloc_call_gives_the_eager_result_on_every_replay(dtype, fusion):
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    code = bl.BLINK_INT32 if dtype == "int32" else bl.BLINK_FP32
    n = (1 << 20) + 12
    x, want, sched = _case(si.hybrid_cube_mesh(), 0, n, 1 << 16, dtype, fusion, 21)
    other_x, other_want, other = _case(si.complete_graph(4), 1, 300_001, 1 << 13, dtype, fusion, 22)
    src = [torch.from_numpy(a).to(dev) for a in x]
    bufs = [b.clone() for b in src]
    main = torch.cuda.current_stream()
    # once beforehand: the tables go into the block, the launch is planned
    bl.blink_allreduce_noalloc(bufs, n, code, sched, main.cuda_stream)
    torch.cuda.synchronize()
    for b, wv in zip(bufs, want):
        assert np.array_equal(b.cpu().numpy().view(np.uint32), wv.view(np.uint32))

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        bl.blink_allreduce_noalloc(bufs, n, code, sched, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()

    for replay in range(4):
        # the program's own eager work between replays: the inputs go back, and
        # another schedule runs through the allocating entry point
        for b, s0 in zip(bufs, src):
            b.copy_(s0)
        ob = [torch.from_numpy(a).to(dev) for a in other_x]
        bl.blink_allreduce(ob, len(other_x[0]), code, other, main.cuda_stream)
        torch.cuda.synchronize()
        assert np.array_equal(ob[2].cpu().numpy().view(np.uint32), other_want[2].view(np.uint32))
        graph.replay()
        torch.cuda.synchronize()
        for r, (b, wv) in enumerate(zip(bufs, want)):
            assert np.array_equal(b.cpu().numpy().view(np.uint32), wv.view(np.uint32)), (replay, r)
        assert sched.status()[0] == bl.BLINK_OK


def test_a_capturing_stream_refuses_what_a_replay_could_not_repeat():
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    n = 1 << 16
    x, want, sched = _case(si.complete_graph(4), 0, n, 1 << 13, "int32", bl.BLINK_FUSE_TREE, 23)
    _, _, stranger = _case(si.complete_graph(4), 2, n, 1 << 12, "int32", bl.BLINK_FUSE_EDGE, 24)
    src = [torch.from_numpy(a).to(dev) for a in x]
    bufs = [b.clone() for b in src]
    bl.blink_allreduce_noalloc(bufs, n, bl.BLINK_INT32, sched, torch.cuda.current_stream().cuda_stream)
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for b, s0 in zip(bufs, src):
        b.copy_(s0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        stream = torch.cuda.current_stream().cuda_stream
        with pytest.raises(bl.BlinkError) as e:          # numbered call: not recordable
            bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream)
        assert e.value.status == bl.BLINK_EINVAL
        with pytest.raises(bl.BlinkError) as e:          # its tables are not in the block: it would have to wait and copy
            bl.blink_allreduce_noalloc(bufs, n, bl.BLINK_INT32, stranger, stream)
        assert e.value.status == bl.BLINK_EINVAL
        bl.blink_allreduce_noalloc(bufs, n, bl.BLINK_INT32, sched, stream)
    torch.cuda.synchronize()
    for b, s0 in zip(bufs, src):                          # recording ran nothing
        assert torch.equal(b, s0)
    graph.replay()
    torch.cuda.synchronize()
    for b, wv in zip(bufs, want):
        assert np.array_equal(b.cpu().numpy(), wv)
    # the refusals consumed no call number: the schedule goes on eagerly
    for b, s0 in zip(bufs, src):
        b.copy_(s0)
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for b, wv in zip(bufs, want):
        assert np.array_equal(b.cpu().numpy(), wv)
    assert sched.status()[0] == bl.BLINK_OK
