"""Host side of the multi-server AllReduce (paper section 3.5) and of the
two-link-class split (section 3.4) through the C ABI, judged by the oracle.
No GPU."""
import numpy as np
import pytest

import paper_1910_04940_amd as bl
import synth_inputs as si
from oracle import execute as ox
from oracle import multiserver as om
from oracle import schedule as osch

FUSIONS = [bl.BLINK_FUSE_EDGE, bl.BLINK_FUSE_NODE, bl.BLINK_FUSE_TREE]


def lib_server(top, ranks, root=0):
    """(library trees, rank list, oracle Server built from those same trees)."""
    if top is None:
        return None, tuple(ranks), om.Server(tuple(ranks), (0,), ((-1,),), (1.0,))
    t = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, root)
    roots, parents, w = t.as_lists()
    return t, tuple(ranks), om.Server(tuple(ranks), tuple(roots), tuple(tuple(p) for p in parents), tuple(w))


def layouts():
    mesh2 = si.hybrid_cube_mesh(doubled=True)
    a, b = si.induced(mesh2, (0, 1, 4)), si.induced(mesh2, (2, 3, 5, 6, 7))
    return {
        "3+5": [lib_server(a, (0, 1, 2)), lib_server(b, (3, 4, 5, 6, 7))],
        "3+5 interleaved": [lib_server(a, (0, 2, 5)), lib_server(b, (1, 3, 4, 6, 7), root=2)],
        "8+8": [lib_server(si.hybrid_cube_mesh(), range(0, 8)), lib_server(si.hybrid_cube_mesh(), range(8, 16), 3)],
        "ring3+K4+chain2+single": [lib_server(si.ring(3), (0, 3, 6)), lib_server(si.complete_graph(4), (1, 2, 7, 8), 1),
                                   lib_server(si.chain(2), (4, 5), 1), lib_server(None, (9,))],
        "four singles": [lib_server(None, (i,)) for i in range(4)],
    }


LAYOUT_NAMES = list(layouts())


def make(layout, n, chunk, fusion):
    servers = layouts()[layout]
    sched = bl.blink_make_schedule_servers([s[0] for s in servers], [s[1] for s in servers], n, chunk, fusion)
    return sched, [s[2] for s in servers]


def to_oracle_steps(sched):
    return [osch.Step(int(s["kind"]), int(s["tree"]), int(s["chunk"]), int(s["src"]), int(s["dst"]),
                      int(s["off"]), int(s["len"]), tuple(int(d) for d in s["deps"][:int(s["n_deps"])]))
            for s in sched.steps()]


@pytest.mark.parametrize("layout", LAYOUT_NAMES)
@pytest.mark.parametrize("fusion", FUSIONS)
@pytest.mark.parametrize("n,chunk", [(30_011, 1024), (1 << 18, 1 << 14), (7, 64)])
def test_schedule_passes_the_oracle_validator(layout, fusion, n, chunk):
    sched, servers = make(layout, n, chunk, fusion)
    trees = om.compose(n, servers)
    assert sched.num_trees == len(trees)
    assert sched.bounds() == [g.lo for g in trees] + [n]
    steps = to_oracle_steps(sched)
    om.check_three_phase_steps(steps, servers, n, chunk)
    assert len(steps) == len(om.three_phase_steps(servers, n, chunk))
    k = sum(len(s.ranks) for s in servers)
    if fusion == bl.BLINK_FUSE_TREE:
        assert sched.traffic_bytes == 8 * k * n
    if fusion == bl.BLINK_FUSE_EDGE:
        assert sched.traffic_bytes == 20 * (k - 1) * n


@pytest.mark.parametrize("layout", LAYOUT_NAMES)
@pytest.mark.parametrize("dtype", ["fp32", "int32"])
def test_library_step_list_replayed_on_the_cpu_gives_the_protocol_result(layout, dtype):
    n, chunk = 20_011, 2048
    sched, servers = make(layout, n, chunk, bl.BLINK_FUSE_EDGE)
    k = sum(len(s.ranks) for s in servers)
    x = [si.payload(11, r, n, "int" if dtype == "int32" else "uniform", dtype) for r in range(k)]
    want = om.three_phase_allreduce(x, servers)
    steps = to_oracle_steps(sched)
    bufs = [a.copy() for a in x]
    ox.run_steps(bufs, steps, ox.random_topological_order(steps, 5))
    for b in bufs:
        assert np.array_equal(b.view(np.uint32), want.view(np.uint32))


def test_error_codes():
    top = si.complete_graph(3)
    t = bl.blink_pack_trees(top.k, top.src, top.dst, top.cap, 0)
    ok = ([t, t], [(0, 1, 2), (3, 4, 5)])
    bl.blink_make_schedule_servers(*ok, 1000, 64)
    for local, ranks in [
        ([t, t], [(0, 1, 2), (2, 3, 4)]),        # an id twice
        ([t, t], [(0, 1, 2), (3, 4, 6)]),        # not a permutation of 0..k-1
        ([t, t], [(0, 2, 1), (3, 4, 5)]),        # not ascending inside a server
        ([t] * 6, [tuple(range(3 * i, 3 * i + 3)) for i in range(6)]),  # more than 16 ranks
        ([None], [(0,)]),                        # fewer than two ranks
    ]:
        with pytest.raises(bl.BlinkError) as e:
            bl.blink_make_schedule_servers(local, ranks, 1000, 64)
        assert e.value.status == bl.BLINK_EINVAL
    with pytest.raises(bl.BlinkError):
        bl.blink_make_schedule_servers(*ok, 1000, 0)
    with pytest.raises(bl.BlinkError):
        bl.blink_make_schedule_servers(*ok, 1000, 64, 7)
    assert bl.blink_make_schedule_servers(*ok, 0, 64).num_steps == 0


# ---- section 3.4 ---------------------------------------------------------------------
@pytest.mark.parametrize("d,bs,bf,t", [(500e6, 10e9, 60e9, 1e-4), (1e9, 8e9, 25e9, 0.0),
                                       (64e6, 12e9, 120e9, 2e-4), (1e5, 10e9, 60e9, 1e-3), (0.0, 1.0, 2.0, 0.5)])
def test_hybrid_split_matches_the_oracle(d, bs, bf, t):
    got = bl.blink_hybrid_split(d, bs, bf, t)
    want = om.hybrid_split(d, bs, bf, t)
    assert got == pytest.approx(want, rel=1e-12, abs=1e-9)
    assert got[0] + got[1] == pytest.approx(d)


@pytest.mark.parametrize("args", [(-1.0, 1, 1, 0), (1.0, 0, 1, 0), (1.0, 1, -2, 0), (1.0, 1, 1, -1e-3),
                                  (float("nan"), 1, 1, 0), (1.0, float("inf"), 1, 0)])
def test_hybrid_split_rejects_meaningless_arguments(args):
    with pytest.raises(bl.BlinkError) as e:
        bl.blink_hybrid_split(*args)
    assert e.value.status == bl.BLINK_EINVAL
