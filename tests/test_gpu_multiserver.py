"""Parity of the HIP path with the CPU oracle on the multi-server AllReduce
(paper section 3.5), through the C ABI: the k ranks of all servers are k HBM
buffers on the one GPU."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox
from oracle import multiserver as om

from test_gpu_parity import FUSIONS, assert_fp32_close_and_equal, bl, dev, stream, to_dev, torch  # noqa: F401
from test_host_multiserver import LAYOUT_NAMES, make

pytestmark = pytest.mark.gpu


def run(dev, sched, x, dtype, redop=bl.BLINK_SUM):
    bufs = to_dev(x, dev)
    code = bl.BLINK_INT32 if dtype == "int32" else bl.BLINK_FP32
    if redop == bl.BLINK_SUM:
        bl.blink_allreduce(bufs, x[0].shape[0], code, sched, stream())
    else:
        bl.blink_allreduce_op(bufs, x[0].shape[0], code, redop, sched, stream())
    torch.cuda.synchronize()
    return [b.cpu().numpy() for b in bufs]


@pytest.mark.parametrize("layout", LAYOUT_NAMES)
@pytest.mark.parametrize("fusion", FUSIONS)
@pytest.mark.parametrize("dtype", ["int32", "fp32"])
@pytest.mark.parametrize("n,chunk", [(200_003, 4096), (1 << 20, 1 << 16), (13, 256)])
def test_three_phase_allreduce_matches_the_oracle(dev, layout, fusion, dtype, n, chunk):
    sched, servers = make(layout, n, chunk, fusion)
    k = sum(len(s.ranks) for s in servers)
    x = [si.payload(21, r, n, "int" if dtype == "int32" else "uniform", dtype) for r in range(k)]
    want = om.three_phase_allreduce(x, servers)
    if dtype == "int32":
        assert np.array_equal(want, ox.allreduce_int32_definition(x))
    for r, g in enumerate(run(dev, sched, x, dtype)):
        label = f"{layout} n={n} chunk={chunk} {dtype} fusion={fusion} rank={r}"
        if dtype == "fp32":
            assert_fp32_close_and_equal(g, want, label)
        else:
            assert np.array_equal(g, want), label


@pytest.mark.parametrize("fusion", FUSIONS)
@pytest.mark.parametrize("redop,oredop", [(bl.BLINK_MAX, ox.MAX), (bl.BLINK_PROD, ox.PROD)])
def test_other_operators_across_servers(dev, fusion, redop, oredop):
    n, chunk = 100_003, 8192
    sched, servers = make("3+5 interleaved", n, chunk, fusion)
    x = [si.payload(22, r, n, "uniform", "fp32", 1.5) for r in range(8)]
    want = om.three_phase_allreduce(x, servers, oredop)
    for g in run(dev, sched, x, "fp32", redop):
        assert np.array_equal(g.view(np.uint32), want.view(np.uint32))


def test_repeated_calls_and_a_large_payload_on_two_full_servers(dev):
    """16 ranks, 16 Mi elements each, twice on the same schedule: the second
    call reduces the first call's results."""
    n, chunk = 1 << 24, 1 << 18
    sched, servers = make("8+8", n, chunk, bl.BLINK_FUSE_TREE)
    x = [si.payload(23, r, n, "int", "int32") for r in range(16)]
    bufs = to_dev(x, dev)
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream())
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream())
    torch.cuda.synchronize()
    once = ox.allreduce_int32_definition(x)
    twice = ox.allreduce_int32_definition([once] * 16)
    for b in bufs:
        assert np.array_equal(b.cpu().numpy(), twice)


def test_two_tree_sets_on_a_split_payload(dev):
    """Section 3.4 end to end: one set of trees per class of links (here a chain
    standing in for the slow class, the packed cube-mesh trees for the fast one),
    the payload cut where blink_hybrid_split says, each part reduced along its
    own trees by a call on offset pointers."""
    n, chunk, k = 3_000_000, 1 << 16, 8
    d_slow, d_fast = bl.blink_hybrid_split(n * 4.0, 10e9, 100e9, 20e-6)
    want_slow, _ = om.hybrid_split(n * 4.0, 10e9, 100e9, 20e-6)
    assert d_slow == pytest.approx(want_slow) and d_slow + d_fast == pytest.approx(n * 4.0)
    cut = int(d_slow // 16) * 4                       # elements, on a 16-byte boundary
    assert 0 < cut < n
    slow_top, fast_top = si.chain(8), si.hybrid_cube_mesh()
    slow = bl.blink_pack_trees(k, slow_top.src, slow_top.dst, slow_top.cap, 0)
    fast = bl.blink_pack_trees(k, fast_top.src, fast_top.dst, fast_top.cap, 0)
    x = [si.payload(24, r, n, "uniform", "fp32") for r in range(k)]
    bufs = to_dev(x, dev)
    s1 = bl.blink_make_schedule(slow, bl.BLINK_OP_ALLREDUCE, cut, chunk, bl.BLINK_FUSE_TREE)
    s2 = bl.blink_make_schedule(fast, bl.BLINK_OP_ALLREDUCE, n - cut, chunk, bl.BLINK_FUSE_TREE)
    bl.blink_allreduce([b[:cut] for b in bufs], cut, bl.BLINK_FP32, s1, stream())
    bl.blink_allreduce([b[cut:] for b in bufs], n - cut, bl.BLINK_FP32, s2, stream())
    torch.cuda.synchronize()
    want = np.concatenate([ox.tree_order_allreduce([a[:cut] for a in x], *slow.as_lists()),
                           ox.tree_order_allreduce([a[cut:] for a in x], *fast.as_lists())])
    for r, b in enumerate(bufs):
        assert_fp32_close_and_equal(b.cpu().numpy(), want, f"rank {r}")
