"""The give-up path of a stage's wait for another stage, and recovery from it.

The per-edge program hands chunks from stage to stage through counters of
finished tiles (the paper's event per chunk, section 4.1).  A wait that can
never end is forced from the host: one call is counted as made without being
launched, so the next call's stages wait for progress nobody produces.  Every
wave runs into the (tiny) wait limit, records what it waited for and leaves;
the kernel ends normally.  Nothing here faults or hangs the GPU."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox
from oracle import schedule as osch

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1910_04940_amd as bl  # noqa: E402


@pytest.mark.parametrize("fusion", [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE])
@pytest.mark.parametrize("n,chunk", [(1 << 16, 1 << 12), (1 << 22, 1 << 16)])
def test_abandoned_wait_is_reported_and_reset_recovers(fusion, n, chunk):
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream().cuda_stream
    top = si.hybrid_cube_mesh()
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
    roots, parents, w = trees.as_lists()
    steps = osch.make_steps(roots, parents, w, osch.ALLREDUCE, n, chunk)
    x = [si.payload(7, r, n, "int", "int32") for r in range(top.k)]
    want = [a.copy() for a in x]
    ox.run_steps(want, steps)

    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    st, rec = sched.status()
    assert st == bl.BLINK_OK and rec["state"] == 0 and rec["stage"] == -1     # never ran

    # a healthy call
    bufs = [torch.from_numpy(a).to(dev) for a in x]
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream)
    st, rec = sched.status()
    assert st == bl.BLINK_OK and rec["state"] == 0
    for b, wv in zip(bufs, want):
        assert np.array_equal(b.cpu().numpy(), wv)

    # the host counts a call that never ran; the next one cannot complete its waits
    sched.set_wait_limit(2000)
    sched.test_skip_call()
    bufs = [torch.from_numpy(a).to(dev) for a in x]
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream)
    st, rec = sched.status()                       # waits for the kernel, which ends by itself
    assert st == bl.BLINK_ESTUCK and rec["state"] == 1
    stages = sched.stages()
    assert 0 <= rec["stage"] < len(stages) and 0 <= rec["awaited_stage"] < rec["stage"]
    assert rec["awaited_stage"] in [int(d) for d in stages[rec["stage"]]["deps"][:stages[rec["stage"]]["n_dep"]]]
    assert rec["seen"] < rec["wanted"]
    assert rec["call"] == 3                        # 1 ran, 2 was skipped
    assert rec["wanted"] % 3 == 0 and rec["seen"] <= rec["wanted"] // 3 * 2

    # until the reset, calls on the schedule leave the buffers alone and the record stays
    bufs = [torch.from_numpy(a).to(dev) for a in x]
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream)
    st2, rec2 = sched.status()
    assert st2 == bl.BLINK_ESTUCK and rec2 == rec
    for b, a in zip(bufs, x):
        assert np.array_equal(b.cpu().numpy(), a)

    # reset: as new
    sched.reset()
    sched.set_wait_limit(0)
    st, rec = sched.status()
    assert st == bl.BLINK_OK and rec["state"] == 0
    for _ in range(2):
        bufs = [torch.from_numpy(a).to(dev) for a in x]
        bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream)
        torch.cuda.synchronize()
        for b, wv in zip(bufs, want):
            assert np.array_equal(b.cpu().numpy(), wv)
    assert sched.status()[0] == bl.BLINK_OK


def test_status_of_a_dependency_free_schedule_stays_ok():
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    top = si.complete_graph(4)
    trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
    n = 1 << 18
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, 1 << 14, bl.BLINK_FUSE_TREE)
    bufs = [torch.zeros(n, dtype=torch.int32, device=dev) for _ in range(4)]
    sched.test_skip_call()        # no stage waits for another: a skipped call number changes nothing
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, torch.cuda.current_stream().cuda_stream)
    assert sched.status()[0] == bl.BLINK_OK
