"""Every distinct connected 3- to 8-GPU allocation of the two 8-GPU servers of
the paper's evaluation (section 5.2: 14 on the first generation, 46 on the
second) through the whole path on the GPU: blink_pack_trees on the induced
topology, blink_make_schedule, blink_allreduce, against the oracle executing
the same trees step by step.  Per-edge and whole-tree programs, int32 (bit
exact) and fp32 (bit exact, hence within the 1e-6 bar), a ragged payload."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox
from oracle import schedule as osch

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1910_04940_amd as bl  # noqa: E402


def representatives(name):
    full = si.hybrid_cube_mesh() if name == "first_generation" else si.dgx1v()
    return full, si.distinct_allocations(full, si.connected_allocations(full))


@pytest.mark.parametrize("name,count", [("first_generation", 14), ("second_generation", 46)])
def test_allreduce_on_every_distinct_allocation(name, count):
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream().cuda_stream
    full, reps = representatives(name)
    assert len(reps) == count
    n, chunk = 200_003, 8_192
    uneven = 0
    for sub in reps:
        top = si.induced(full, sub)
        trees = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
        roots, parents, w = trees.as_lists()
        uneven += len(set(w)) > 1
        steps = osch.make_steps(roots, parents, w, osch.ALLREDUCE, n, chunk)
        for dtype, code in (("int32", bl.BLINK_INT32), ("fp32", bl.BLINK_FP32)):
            x = [si.payload(41, r, n, "int" if dtype == "int32" else "normal", dtype, 1e-2) for r in range(top.k)]
            want = [a.copy() for a in x]
            ox.run_steps(want, steps)
            if dtype == "int32":
                assert np.array_equal(want[0], ox.allreduce_int32_definition(x))
            for fusion in (bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_TREE):
                sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
                bufs = [torch.from_numpy(a).to(dev) for a in x]
                bl.blink_allreduce(bufs, n, code, sched, stream)
                torch.cuda.synchronize()
                for r, (b, wv) in enumerate(zip(bufs, want)):
                    got = b.cpu().numpy()
                    assert np.array_equal(got.view(np.uint32), wv.view(np.uint32)), (sub, dtype, fusion, r)
                assert sched.status()[0] == bl.BLINK_OK
    if name == "second_generation":
        assert uneven > 0, "some allocations of the doubled-link server pack trees of unequal weight"
