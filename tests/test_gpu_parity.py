"""GPU parity: the HIP library through its C ABI against the CPU oracle, element
by element on the same seeded inputs.  Bars: int32 and Broadcast bit-exact; fp32
AllReduce max relative error <= 1e-6 against the oracle summing in the same tree
order (0 is expected and also asserted)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import execute as ox
from oracle import graph as og
from oracle import packing as op
from oracle import schedule as osch

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_1910_04940_amd as bl  # noqa: E402

FUSIONS = [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE]
FP32_REL_TOL = 1e-6


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the GPU"
    d = torch.device("cuda:0")
    torch.cuda.set_device(d)
    return d


def pack(top, root):
    return bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, root)


def to_dev(arrs, dev):
    return [torch.from_numpy(a).to(dev) for a in arrs]


def stream():
    return torch.cuda.current_stream().cuda_stream


def assert_fp32_close_and_equal(got, want, label):
    denom = np.maximum(np.abs(want), np.finfo(np.float32).tiny)
    rel = np.max(np.abs(got.astype(np.float64) - want.astype(np.float64)) / denom) if want.size else 0.0
    assert rel <= FP32_REL_TOL, f"{label}: max relative error {rel}"
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{label}: not bit-identical"


def run_allreduce_case(dev, top, root, n, chunk, dtype, fusion, seed, dist=None, scale=1.0,
                       launch=None, calls=1):
    trees = pack(top, root)
    roots, parents, w = trees.as_lists()
    dist = dist or ("int" if dtype == "int32" else "uniform")
    x = [si.payload(seed, r, n, dist, dtype, scale) for r in range(top.k)]
    want = [a.copy() for a in x]
    steps = osch.make_steps(roots, parents, w, osch.ALLREDUCE, n, chunk)
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    if launch:
        sched.set_launch(*launch)
    code = bl.BLINK_INT32 if dtype == "int32" else bl.BLINK_FP32
    for _ in range(calls):
        bl.blink_allreduce(bufs, n, code, sched, stream())
        ox.run_steps(want, steps)
    torch.cuda.synchronize()
    for r, (b, wv) in enumerate(zip(bufs, want)):
        got = b.cpu().numpy()
        label = f"{top.name} n={n} chunk={chunk} {dtype} fusion={fusion} rank={r}"
        if dtype == "int32":
            assert np.array_equal(got, wv), label
        else:
            assert_fp32_close_and_equal(got, wv, label)
    if dtype == "int32" and calls == 1:
        assert np.array_equal(want[0], ox.allreduce_int32_definition(x))


TOPOLOGIES = [
    (si.complete_graph(4), 0),
    (si.hybrid_cube_mesh(), 0),
    (si.hybrid_cube_mesh(doubled=True), 5),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 4)), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (2, 3, 5, 6, 7)), 0),
    (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 3, 4, 5, 7)), 0),
    (si.chain(8), 0),
    (si.star(7, 3), 3),
    (si.complete_graph(2), 1),
]


@pytest.mark.parametrize("top,root", TOPOLOGIES)
@pytest.mark.parametrize("fusion", FUSIONS)
@pytest.mark.parametrize("dtype", ["int32", "fp32"])
def test_allreduce_matches_oracle(dev, top, root, fusion, dtype):
    # several tiles per chunk, several chunks per tree, a ragged tail (n % 4 != 0)
    run_allreduce_case(dev, top, root, n=300_003, chunk=20_000, dtype=dtype, fusion=fusion, seed=11)


@pytest.mark.parametrize("fusion", FUSIONS)
def test_config_k4_1m_fp32_chunk_64k(dev, fusion):
    run_allreduce_case(dev, si.complete_graph(4), 0, n=1 << 20, chunk=1 << 16, dtype="fp32",
                       fusion=fusion, seed=0)
    run_allreduce_case(dev, si.complete_graph(4), 0, n=1 << 20, chunk=1 << 16, dtype="int32",
                       fusion=fusion, seed=0)


@pytest.mark.parametrize("n,chunk", [(1, 64), (3, 64), (4, 4), (5, 4), (17, 8), (1023, 1 << 20),
                                     (4096, 1000), (4100, 1001), (100_000, 7), (8191, 8192),
                                     (2048 * 8 + 4, 2048)])
@pytest.mark.parametrize("fusion", FUSIONS)
def test_small_ragged_and_misaligned_sizes(dev, n, chunk, fusion):
    if chunk == 7 and n > 20_000:
        n = 20_000      # element-wise path: keep the run short
    for dtype in ("int32", "fp32"):
        run_allreduce_case(dev, si.hybrid_cube_mesh(), 0, n=n, chunk=chunk, dtype=dtype,
                           fusion=fusion, seed=n)


@pytest.mark.parametrize("fusion", FUSIONS)
def test_sixteen_rank_switch_one_hop_trees(dev, fusion):
    top = si.complete_graph(16)
    run_allreduce_case(dev, top, bl.BLINK_ROOT_ANY, n=16 * 5000 + 2, chunk=1024, dtype="fp32",
                       fusion=fusion, seed=5)
    run_allreduce_case(dev, top, bl.BLINK_ROOT_ANY, n=16 * 5000 + 2, chunk=1024, dtype="int32",
                       fusion=fusion, seed=5)
    run_allreduce_case(dev, top, 0, n=50_000, chunk=4096, dtype="fp32", fusion=fusion, seed=6)


@pytest.mark.parametrize("fusion", FUSIONS)
@pytest.mark.parametrize("launch", [(1, 256), (1, 4096), (0, 512), (2, 0), (16, 1024), (0, 65536), (3, 16384)])
def test_launch_shapes_and_repeated_calls_on_one_schedule(dev, fusion, launch):
    top = si.hybrid_cube_mesh()
    run_allreduce_case(dev, top, 0, n=200_000, chunk=16_384, dtype="int32", fusion=fusion,
                       seed=21, launch=launch, calls=3)
    run_allreduce_case(dev, top, 0, n=200_000, chunk=16_384, dtype="fp32", fusion=fusion,
                       seed=22, dist="normal", scale=1e-3, launch=launch, calls=3)


def test_gradient_like_values_and_denormals(dev):
    # tiny magnitudes: subnormal partial sums must not be flushed
    top = si.hybrid_cube_mesh()
    run_allreduce_case(dev, top, 0, n=65_536, chunk=8192, dtype="fp32", fusion=bl.BLINK_FUSE_TREE,
                       seed=31, dist="normal", scale=1e-39)
    run_allreduce_case(dev, top, 0, n=65_536, chunk=8192, dtype="fp32", fusion=bl.BLINK_FUSE_EDGE,
                       seed=31, dist="normal", scale=1e-39)


@pytest.mark.parametrize("fusion", FUSIONS)
def test_oracle_packed_trees_injected(dev, fusion):
    """Trees chosen by the oracle's own packer, handed to the library as arrays."""
    top = si.hybrid_cube_mesh(doubled=True)
    roots, parents, w = op.pack_trees(og.Digraph.from_topology(top), 0)
    trees = bl.blink_trees_from_arrays(top.k, roots, parents, w)
    n, chunk = 123_457, 10_000
    x = [si.payload(41, r, n, "uniform", "fp32") for r in range(top.k)]
    want = [a.copy() for a in x]
    ox.run_steps(want, osch.make_steps(roots, parents, w, osch.ALLREDUCE, n, chunk))
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    bl.blink_allreduce(bufs, n, bl.BLINK_FP32, sched, stream())
    torch.cuda.synchronize()
    for b in bufs:
        assert_fp32_close_and_equal(b.cpu().numpy(), want[0], "injected trees")
    assert np.array_equal(want[0], ox.tree_order_allreduce(x, roots, parents, w))


def test_uneven_weights(dev):
    parents = [(-1, 0, 0, 1), (-1, 0, 1, 2), (-1, 3, 0, 0)]
    w = [0.5, 1.25, 0.3]
    trees = bl.blink_trees_from_arrays(4, [0, 0, 0], parents, w)
    n, chunk = 99_999, 4096
    for fusion in FUSIONS:
        x = [si.payload(51, r, n, "uniform", "fp32") for r in range(4)]
        want = [a.copy() for a in x]
        ox.run_steps(want, osch.make_steps([0, 0, 0], parents, w, osch.ALLREDUCE, n, chunk))
        bufs = to_dev(x, dev)
        sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
        bl.blink_allreduce(bufs, n, bl.BLINK_FP32, sched, stream())
        torch.cuda.synchronize()
        for b in bufs:
            assert_fp32_close_and_equal(b.cpu().numpy(), want[0], f"uneven weights fusion {fusion}")


# The paper's micro-benchmark shapes (section 2.2): depth (chains) and breadth
# (fan-in / fan-out up to 3) are among TOPOLOGIES; here the two with several
# flows through one node.  Ranks 0 and 1 send, 2 is the centre, 3 and 4 receive.
PAPER_SHAPES = {
    # two trees through the centre: both inputs are folded at rank 2, one tree
    # delivers to rank 3 first, the other to rank 4 first
    "multi-input multi-output": ([3, 4], [(2, 2, 3, -1, 3), (2, 2, 4, 4, -1)], [1.0, 1.0]),
    # two reduce-and-forward chains 0 -> 1 -> 2 and 4 -> 3 -> 2 merging at the centre
    "multi-chain aggregation": ([2], [(1, 2, -1, 2, 3)], [1.0]),
    # fan-in and fan-out of three at one node
    "fan of three": ([0], [(-1, 0, 0, 0, 1)], [1.0]),
}


@pytest.mark.parametrize("shape", PAPER_SHAPES)
@pytest.mark.parametrize("fusion", FUSIONS)
@pytest.mark.parametrize("dtype", ["int32", "fp32"])
def test_micro_benchmark_tree_shapes_of_the_paper(dev, shape, fusion, dtype):
    roots, parents, w = PAPER_SHAPES[shape]
    trees = bl.blink_trees_from_arrays(5, roots, parents, w)
    n, chunk = 250_003, 16_384
    x = [si.payload(61, r, n, "int" if dtype == "int32" else "uniform", dtype) for r in range(5)]
    want = ox.tree_order_allreduce(x, roots, parents, w)
    if dtype == "int32":
        assert np.array_equal(want, ox.allreduce_int32_definition(x))
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    bl.blink_allreduce(bufs, n, bl.BLINK_INT32 if dtype == "int32" else bl.BLINK_FP32, sched, stream())
    torch.cuda.synchronize()
    for b in bufs:
        assert b.cpu().numpy().tobytes() == want.tobytes(), shape


# ---- Broadcast -----------------------------------------------------------------------
@pytest.mark.parametrize("top,root", [(si.hybrid_cube_mesh(), 0), (si.complete_graph(4), 2),
                                      (si.chain(6), 5), (si.hybrid_cube_mesh(doubled=True), 3)])
@pytest.mark.parametrize("fusion", FUSIONS)
def test_broadcast_equals_root(dev, top, root, fusion):
    n, chunk = 262_147, 16_384
    trees = pack(top, root)
    roots, parents, w = trees.as_lists()
    x = [si.payload(61, r, n, "normal", "fp32") for r in range(top.k)]
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_BROADCAST, n, chunk, fusion)
    bl.blink_broadcast(bufs, n, bl.BLINK_FP32, sched, stream())
    torch.cuda.synchronize()
    want = ox.broadcast_definition(x, roots, w)
    for b in bufs:
        assert b.cpu().numpy().tobytes() == want.tobytes()
    # int32 payloads through the same path
    xi = [si.payload(62, r, n, "int", "int32") for r in range(top.k)]
    bufs = to_dev(xi, dev)
    bl.blink_broadcast(bufs, n, bl.BLINK_INT32, sched, stream())
    torch.cuda.synchronize()
    for b in bufs:
        assert np.array_equal(b.cpu().numpy(), xi[root])


# ---- edge cases and errors ---------------------------------------------------------------
def test_empty_payload_is_a_no_op(dev):
    trees = pack(si.complete_graph(4), 0)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, 0, 64)
    bufs = [torch.zeros(4, device=dev) for _ in range(4)]
    bl.blink_allreduce(bufs, 0, bl.BLINK_FP32, sched, stream())
    bl.blink_allreduce([0, 0, 0, 0], 0, bl.BLINK_FP32, sched, stream())   # null pointers are not looked at
    torch.cuda.synchronize()


def test_untouched_memory_beyond_n(dev):
    """The kernel writes elements [0, n) only."""
    top = si.complete_graph(4)
    n = 10_001
    trees = pack(top, 0)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, 2048)
    bufs = [torch.full((n + 64,), 7.0, device=dev) for _ in range(4)]
    bl.blink_allreduce(bufs, n, bl.BLINK_FP32, sched, stream())
    torch.cuda.synchronize()
    for b in bufs:
        assert (b[n:] == 7.0).all() and (b[:n] == 28.0).all()


def test_call_errors(dev):
    top = si.complete_graph(4)
    n = 4096
    trees = pack(top, 0)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, 1024)
    bufs = [torch.zeros(n + 4, device=dev) for _ in range(4)]

    def status(fn, *a):
        with pytest.raises(bl.BlinkError) as e:
            fn(*a)
        return e.value.status

    assert status(bl.blink_allreduce, bufs[:3], n, bl.BLINK_FP32, sched, stream()) == bl.BLINK_EMISMATCH
    assert status(bl.blink_allreduce, bufs, n - 1, bl.BLINK_FP32, sched, stream()) == bl.BLINK_EMISMATCH
    assert status(bl.blink_broadcast, bufs, n, bl.BLINK_FP32, sched, stream()) == bl.BLINK_EMISMATCH
    assert status(bl.blink_allreduce, bufs, n, 5, sched, stream()) == bl.BLINK_EINVAL
    mis = [bufs[0].data_ptr() + 4] + [b.data_ptr() for b in bufs[1:]]
    assert status(bl.blink_allreduce, mis, n, bl.BLINK_FP32, sched, stream()) == bl.BLINK_EINVAL
    ovl = [bufs[0].data_ptr(), bufs[0].data_ptr() + 16] + [b.data_ptr() for b in bufs[2:]]
    assert status(bl.blink_allreduce, ovl, n, bl.BLINK_FP32, sched, stream()) == bl.BLINK_EINVAL
    null = [0] + [b.data_ptr() for b in bufs[1:]]
    assert status(bl.blink_allreduce, null, n, bl.BLINK_FP32, sched, stream()) == bl.BLINK_EINVAL
    for bad_tile in (3, 128, 131072, 768):
        assert status(sched.set_launch, 0, bad_tile) == bl.BLINK_EINVAL
    assert status(sched.set_launch, -1, 0) == bl.BLINK_EINVAL
    # the schedule still works after all those refusals
    bl.blink_allreduce(bufs, n, bl.BLINK_FP32, sched, stream())
    torch.cuda.synchronize()


def test_non_default_stream(dev):
    top = si.hybrid_cube_mesh()
    n, chunk = 150_000, 8192
    trees = pack(top, 0)
    roots, parents, w = trees.as_lists()
    x = [si.payload(71, r, n, "int", "int32") for r in range(8)]
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, bl.BLINK_FUSE_EDGE)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, s.cuda_stream)
    s.synchronize()
    want = ox.allreduce_int32_definition(x)
    for b in bufs:
        assert np.array_equal(b.cpu().numpy(), want)


# ---- other reduction operators and the Reduce collective -----------------------------------
REDOPS = {"prod": (bl.BLINK_PROD, ox.PROD), "min": (bl.BLINK_MIN, ox.MIN), "max": (bl.BLINK_MAX, ox.MAX),
          "sum": (bl.BLINK_SUM, ox.SUM)}


@pytest.mark.parametrize("redop", ["prod", "min", "max"])
@pytest.mark.parametrize("fusion", FUSIONS)
@pytest.mark.parametrize("dtype", ["int32", "fp32"])
def test_allreduce_with_other_operators(dev, redop, fusion, dtype):
    top = si.hybrid_cube_mesh()
    n, chunk = 150_003, 16_384
    trees = pack(top, 0)
    roots, parents, w = trees.as_lists()
    if dtype == "fp32":
        # products of 8 numbers near 1 neither overflow nor vanish; signed zeros for min / max
        x = [(si.payload(81, r, n, "uniform", "fp32") * np.float32(0.5) + np.float32(1.0)).astype(np.float32)
             for r in range(8)]
        if redop != "prod":
            x = [si.payload(81, r, n, "uniform", "fp32") for r in range(8)]
            x[2][::5] = -0.0
            x[6][::5] = 0.0
            for r in (0, 1, 3, 4, 5, 7):
                x[r][::5] = np.float32(0.0) if redop == "min" else np.float32(-0.0)
    else:
        x = [si.payload(82, r, n, "int", "int32") for r in range(8)]
    want = [a.copy() for a in x]
    ox.run_steps(want, osch.make_steps(roots, parents, w, osch.ALLREDUCE, n, chunk), redop=REDOPS[redop][1])
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    code = bl.BLINK_INT32 if dtype == "int32" else bl.BLINK_FP32
    bl.blink_allreduce_op(bufs, n, code, REDOPS[redop][0], sched, stream())
    torch.cuda.synchronize()
    for r, b in enumerate(bufs):
        assert b.cpu().numpy().tobytes() == want[r].tobytes(), f"{redop} {dtype} fusion {fusion} rank {r}"
    if redop != "prod" or dtype == "int32":
        assert want[0].tobytes() == ox.reduce_definition(x, REDOPS[redop][1]).tobytes()


@pytest.mark.parametrize("top,root", [(si.hybrid_cube_mesh(), 0), (si.chain(6), 3), (si.complete_graph(16), bl.BLINK_ROOT_ANY)])
@pytest.mark.parametrize("fusion", FUSIONS)
@pytest.mark.parametrize("redop", ["sum", "max"])
def test_reduce_to_the_roots(dev, top, root, fusion, redop):
    n, chunk = 120_002, 8_192
    trees = pack(top, root)
    roots, parents, w = trees.as_lists()
    x = [si.payload(91, r, n, "uniform", "fp32") for r in range(top.k)]
    want = ox.tree_order_allreduce(x, roots, parents, w, REDOPS[redop][1])
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_REDUCE, n, chunk, fusion)
    bl.blink_reduce(bufs, n, bl.BLINK_FP32, REDOPS[redop][0], sched, stream())
    torch.cuda.synchronize()
    b = sched.bounds()
    for t, r in enumerate(roots):                      # tree t's share ends up at tree t's root
        got = bufs[r][b[t]:b[t + 1]].cpu().numpy()
        assert got.tobytes() == want[b[t]:b[t + 1]].tobytes(), f"tree {t} root {r}"
    # a schedule made for Reduce cannot run an AllReduce
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_allreduce(bufs, n, bl.BLINK_FP32, sched, stream())
    assert e.value.status == bl.BLINK_EMISMATCH
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_reduce(bufs, n, bl.BLINK_FP32, 9, sched, stream())
    assert e.value.status == bl.BLINK_EINVAL


# ---- Gather and AllGather ---------------------------------------------------------------------
@pytest.mark.parametrize("top,root", [(si.hybrid_cube_mesh(), 0), (si.chain(5), 2),
                                      (si.complete_graph(16), bl.BLINK_ROOT_ANY),
                                      (si.induced(si.hybrid_cube_mesh(doubled=True), (0, 1, 3, 4, 5, 7)), 0)])
@pytest.mark.parametrize("fusion", FUSIONS)
def test_allgather_equals_concatenation(dev, top, root, fusion):
    k = top.k
    m, chunk = 20_003, 4096          # piece length not a multiple of 4: pieces start off 16-byte boundaries
    n = k * m
    trees = pack(top, root)
    x = [si.payload(95, r, n, "int", "int32") for r in range(k)]
    want = ox.allgather_definition(x)
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLGATHER, n, chunk, fusion)
    bl.blink_allgather(bufs, n, bl.BLINK_INT32, sched, stream())
    torch.cuda.synchronize()
    for r, b in enumerate(bufs):
        assert np.array_equal(b.cpu().numpy(), want), f"rank {r}"
    # float payloads take the same path (bit copy, -0.0 and all)
    xf = [si.payload(96, r, n, "normal", "fp32") for r in range(k)]
    xf[1][m:2 * m:3] = -0.0
    bufs = to_dev(xf, dev)
    bl.blink_allgather(bufs, n, bl.BLINK_FP32, sched, stream())
    torch.cuda.synchronize()
    wantf = ox.allgather_definition(xf)
    for b in bufs:
        assert b.cpu().numpy().tobytes() == wantf.tobytes()


@pytest.mark.parametrize("top,root", [(si.hybrid_cube_mesh(), 3), (si.star(6, 1), 1), (si.chain(4), 0)])
@pytest.mark.parametrize("fusion", FUSIONS)
def test_gather_collects_at_the_root(dev, top, root, fusion):
    k = top.k
    m, chunk = 16_384, 2048
    n = k * m
    trees = pack(top, root)
    x = [si.payload(97, r, n, "uniform", "fp32") for r in range(k)]
    bufs = to_dev(x, dev)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_GATHER, n, chunk, fusion)
    bl.blink_gather(bufs, n, bl.BLINK_FP32, sched, stream())
    torch.cuda.synchronize()
    assert bufs[root].cpu().numpy().tobytes() == ox.allgather_definition(x).tobytes()
    # nobody's own piece is disturbed
    for r in range(k):
        assert np.array_equal(bufs[r][r * m:(r + 1) * m].cpu().numpy(), x[r][r * m:(r + 1) * m])


# ---- many hand-overs ---------------------------------------------------------------
@pytest.mark.parametrize("fusion", [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE])
def test_many_hand_overs_between_waves_stay_exact(dev, fusion):
    """Small chunks on a deep tree: tens of thousands of chunk hand-overs between
    waves on different XCDs per call, 60 calls in a row on one schedule.  int32,
    so every element has a closed form: the sum times k^(calls-1) modulo 2^32."""
    top = si.chain(8)
    n, chunk, k = 1 << 21, 1 << 10, 8
    trees = pack(top, 0)
    sched = bl.blink_make_schedule(trees, bl.BLINK_OP_ALLREDUCE, n, chunk, fusion)
    assert sched.num_stages >= 2048 * 8
    x = [si.hash_payload(17, r, 0, n, "int32") for r in range(k)]
    bufs = to_dev(x, dev)
    first = ox.allreduce_int32_definition(x).view(np.uint32).astype(np.uint64)
    calls = 0
    for burst in (1, 9, 20, 30):
        for _ in range(burst):
            bl.blink_allreduce(bufs, n, bl.BLINK_INT32, sched, stream())
        calls += burst
        torch.cuda.synchronize()
        want = (first * np.uint64(pow(k, calls - 1, 1 << 32))) & np.uint64(0xFFFFFFFF)
        for r in (0, 3, 7):
            got = bufs[r].cpu().numpy().view(np.uint32).astype(np.uint64)
            assert np.array_equal(got, want), f"after {calls} calls, rank {r}"
