#!/usr/bin/env python3
"""Benchmark of the packed-tree collectives hot path on one MI355X.

Default (--config headline): a "step" is one blink_allreduce call over the
headline workload: 8 virtual ranks (8 HBM buffers on the one GPU) on the
unit-capacity hybrid cube-mesh, 67,108,864 fp32 per rank (256 MiB), 4 packed
unit-weight trees, 1 MiB chunks.  --config 1, 2, 3a, 3b, 3c, 4, 5 run the other
benchmark configurations the same way (see CONFIGS); in configuration 4 a step
is the 16 bucket calls back to back.  Inputs are resident in HBM before the
timed region; schedules are built once outside it (the paper reuses its
generated code across iterations).

Prints ONE JSON line.  value = algorithm GB/s = per-rank payload bytes / time.
"""
import argparse
import hashlib
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "AllReduce alg GB/s + achieved HBM GB/s vs peak, 8 ranks, 256 MB fp32"
HBM_PEAK_GBS = 8000.0
# Per call the input of step i+1 is the output of step i (in place), so values grow
# by a factor k per step; buffers are restored from a pristine copy before they
# could overflow.  The restore is a plain device copy inside the timed bracket
# (it only makes the reported number slightly pessimistic) and is counted.
MAX_STEPS_BETWEEN_RESTORES = 32
RANK_PAD_BYTES = 68 * 1024   # extra distance between consecutive rank buffers (see main)
ORACLE_SAMPLE_TOTAL = 1 << 29   # the CPU baseline runs on at most this many elements over all ranks

# name -> (what, topology, ranks kept (None = all), root, collective, elements per rank,
#          chunk bytes, value distribution, scale)
CONFIGS = {
    "headline": ("8 ranks, hybrid cube-mesh, 256 MiB fp32 per rank",
                 "cube", None, 0, "allreduce", 1 << 26, 1 << 20, "uniform", 1.0),
    "1": ("4 ranks, complete graph, 1 Mi fp32 per rank, 64 Ki-element chunks; reported: the CPU oracle's seconds",
          "k4", None, 0, "allreduce", 1 << 20, 4 << 16, "uniform", 1.0),
    "2": ("Broadcast from rank 0, 8 ranks, hybrid cube-mesh, 64 MiB fp32 N(0,1)",
          "cube", None, 0, "broadcast", 1 << 24, 1 << 20, "normal", 1.0),
    "3a": ("3-rank fragment {0,1,4} of the cube-mesh with doubled links, 25.6 M fp32 per rank N(0,1e-2)",
           "cube2", (0, 1, 4), 0, "allreduce", 25_600_000, 1 << 20, "normal", 1e-2),
    "3b": ("5-rank fragment {2,3,5,6,7} of the cube-mesh with doubled links, 25.6 M fp32 per rank N(0,1e-2)",
           "cube2", (2, 3, 5, 6, 7), 0, "allreduce", 25_600_000, 1 << 20, "normal", 1e-2),
    "3c": ("6-rank fragment {0,1,3,4,5,7} of the cube-mesh with doubled links, 25.6 M fp32 per rank N(0,1e-2)",
           "cube2", (0, 1, 3, 4, 5, 7), 0, "allreduce", 25_600_000, 1 << 20, "normal", 1e-2),
    "4": ("8 ranks, hybrid cube-mesh, 138 M fp32 in 16 buckets (log-uniform 64 KiB - 400 MiB), one call per bucket, "
          "N(0,1e-3); a step is the 16 calls back to back",
          "cube", None, 0, "allreduce", 138_000_000, 1 << 20, "normal", 1e-3),
    "5": ("16 ranks, fully connected switch topology, one-hop trees, 256 Mi fp32 per rank (1 GiB), 4 MiB chunks",
          "k16", None, -1, "allreduce", 1 << 28, 4 << 20, "hash", 1.0),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", choices=sorted(CONFIGS), default="headline",
                    help="benchmark configuration (default: the headline workload)")
    ap.add_argument("--fusion", choices=["edge", "node", "tree"], default="tree")
    ap.add_argument("--progress", action="store_true", help="say on stderr what is being done (for slow, profiled runs)")
    ap.add_argument("--sweep", choices=["alternate", "forward"], default="alternate",
                    help="alternate (the library's default): every other call goes through the payload backwards, "
                         "starting on what the call before it left in the 256 MiB memory-side cache; "
                         "forward: every call goes forwards and streams past that cache")
    ap.add_argument("--collective", choices=["allreduce", "broadcast"], default=None,
                    help="override the configuration's collective")
    ap.add_argument("--chunk-bytes", type=int, default=0, help="override the configuration's chunk size")
    ap.add_argument("--elems", type=int, default=0, help="override the configuration's elements per rank")
    ap.add_argument("--dtype", choices=["fp32", "int32"], default="fp32")
    ap.add_argument("--tile-elems", type=int, default=0,
                    help="elements per ticket (power of two in 256..65536; 0 = library default)")
    ap.add_argument("--wg-per-cu", type=int, default=0)
    ap.add_argument("--rank-pad-bytes", type=int, default=None,
                    help="the rank buffers are carved from one allocation, consecutive ones this "
                         "many bytes further apart than the payload (multiple of 16; default: "
                         f"{RANK_PAD_BYTES} for the headline, else one allocation per buffer)")
    ap.add_argument("--separate-buffers", action="store_true",
                    help="one allocation per rank buffer (whatever distances the allocator gives)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of the benchmark, run a plain device copy of known size "
                         "(reference for scaling the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def calibrate_copy(steps):
    """A plain 1 GiB device-to-device copy (torch's copy kernel), `steps` times:
    reads 2^30 bytes and writes 2^30 bytes per launch."""
    import torch
    torch.cuda.set_device(0)
    nbytes = 1 << 30
    src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").uniform_(-1, 1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    print(json.dumps({"calibration": "plain copy", "read_bytes_per_launch": nbytes,
                      "write_bytes_per_launch": nbytes, "launches": steps, "ms_per_launch": ms,
                      "GB/s": 2 * nbytes / ms / 1e6}))


def kernel_sources_digest():
    """Identifies the kernels a measurement belongs to: a digest of the device
    sources and of the launcher."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1910_04940_amd", "csrc")
    for name in ("kernel.hpp", "stream.hpp", "exec.hip", "schedule.hpp"):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def traffic_from_profiles(name):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
    if a committed summary under profiles/ carries it AND was measured on the
    kernels as they are now (the summary records the digest of the kernel
    sources it was taken on); else None."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, None
    value, digest = None, None
    for line in open(path):
        if line.startswith("hbm_bytes_per_launch:"):
            value = float(line.split(":", 1)[1].split()[0])
        if line.startswith("kernel_sources_digest:"):
            digest = line.split(":", 1)[1].strip()
    if value is None or digest != kernel_sources_digest():
        return None, digest
    return value, digest


def make_topology(si, name, keep):
    top = {"cube": si.hybrid_cube_mesh, "cube2": lambda: si.hybrid_cube_mesh(True),
           "k4": lambda: si.complete_graph(4), "k16": lambda: si.complete_graph(16)}[name]()
    return si.induced(top, keep) if keep else top


def host_payload(si, seed, rank, n, dist, dtype, scale, start=0):
    if dtype == "int32":
        return si.hash_payload(seed, rank, start, n, "int32") if dist == "hash" else \
            si.payload(seed, rank, n, "int", "int32", start=start)
    if dist == "hash":
        return si.hash_payload(seed, rank, start, n, "fp32")
    return si.payload(seed, rank, n, dist, "fp32", scale, start=start)


def cpu_baseline(si, trees_lists, k, n, chunk, collective, dist, scale):
    """The oracle as it stands, timed on the host: literal step-list execution in
    NumPy float32, one pass over the workload, or over its first
    ORACLE_SAMPLE_TOTAL / k elements per rank when it is larger (same trees, same
    chunk size)."""
    from oracle import execute as ox
    from oracle import schedule as osch

    roots, parents, weights = trees_lists
    m = min(n, ORACLE_SAMPLE_TOTAL // k)
    steps = osch.make_steps(roots, parents, weights,
                            osch.ALLREDUCE if collective == "allreduce" else osch.BROADCAST, m, chunk)
    bufs = [host_payload(si, 0, r, m, dist, "fp32", scale) for r in range(k)]
    t0 = time.perf_counter()
    ox.run_steps(bufs, steps)
    dt = time.perf_counter() - t0
    what = "full workload" if m == n else f"the first {m} of {n} elements per rank"
    return {"value": m * 4 / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{what}, one pass: {k} ranks x {m} fp32, {len(steps)} steps, {dt:.2f} s; "
                      f"NumPy elementwise ops are single-threaded (host has {os.cpu_count()} logical "
                      f"CPUs, {len(os.sched_getaffinity(0))} usable)",
            "seconds": dt}


def check_against_oracle(si, np, bufs, trees_lists, bounds, k, n, collective, dist, scale):
    """Sampled slices of the device result against the oracle's tree-order sum
    (broadcast: against the root's values), bit for bit.  Every slice lies inside
    one tree's share; slices sit at both ends of every share and at seeded
    random places."""
    from oracle import execute as ox

    roots, parents, weights = trees_lists
    width = 1 << 16
    rng = np.random.default_rng(17)
    starts = {0, max(0, n - width)}
    for b in bounds[1:-1]:
        starts |= {max(0, b - width), b}
    starts |= {int(s) for s in rng.integers(0, max(1, n - width), 16)}
    checked = 0
    for a in sorted(starts):
        t = max(i for i in range(len(roots)) if bounds[i] <= a)
        m = min(width, bounds[t + 1] - a, n - a)
        if m <= 0:
            continue
        xs = [host_payload(si, 0, r, m, dist, "fp32", scale, start=a) for r in range(k)]
        want = xs[roots[t]] if collective == "broadcast" else \
            ox.tree_order_allreduce(xs, [roots[t]], [parents[t]], [1.0])
        for r in (0, k - 1):
            got = bufs[r][a:a + m].cpu().numpy()
            if not np.array_equal(got.view(np.uint32), want.view(np.uint32)):
                return False, checked
        checked += m
    return True, checked


def git_head():
    try:
        return subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True,
                              text=True, timeout=10).stdout.strip() or None
    except Exception:
        return None


def main():
    args = parse()

    def say(what):
        if args.progress:
            print(f"bench.py: {what}", file=sys.stderr, flush=True)
    if args.calibrate_copy:
        calibrate_copy(args.steps)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the k ranks are k HBM buffers on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1910_04940_amd as bl
    import synth_inputs as si

    what, top_name, keep, root, collective, n, chunk_bytes, dist, scale = CONFIGS[args.config]
    collective = args.collective or collective
    n = args.elems or n
    chunk_bytes = args.chunk_bytes or chunk_bytes
    headline_layout = args.config == "headline"
    if args.dtype == "int32":
        dist = "hash" if dist == "hash" else "int"

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    top = make_topology(si, top_name, keep)
    k = top.k
    chunk = chunk_bytes // 4
    fusion = {"edge": bl.BLINK_FUSE_EDGE, "node": bl.BLINK_FUSE_NODE, "tree": bl.BLINK_FUSE_TREE}[args.fusion]
    dtype = bl.BLINK_FP32 if args.dtype == "fp32" else bl.BLINK_INT32
    broadcast = collective == "broadcast"
    op = bl.BLINK_OP_BROADCAST if broadcast else bl.BLINK_OP_ALLREDUCE

    trees = bl.blink_pack_trees(k, top.src, top.dst, top.cap, bl.BLINK_ROOT_ANY if root < 0 else root)
    trees_lists = trees.as_lists()
    # configuration 4: one schedule and one set of buffers per bucket; all others: one call per step
    sizes = si.bucket_sizes() if args.config == "4" else [n]
    scheds = [bl.blink_make_schedule(trees, op, m, chunk, fusion) for m in sizes]
    if args.tile_elems or args.wg_per_cu:
        for s in scheds:
            s.set_launch(args.wg_per_cu, args.tile_elems)
    for s in scheds:
        s.set_sweep(args.sweep == "alternate")

    # Inputs from the shared seeded recipe, resident in HBM before anything is
    # timed.  Rank buffers whose distances are large powers of two put equal
    # offsets of all ranks on the same HBM channel and bank; the headline run
    # therefore carves its buffers from one allocation, a small odd-ish
    # distance further apart than the payload (--rank-pad-bytes 0 and
    # --separate-buffers measure the other placements).
    pad = args.rank_pad_bytes
    if pad is None and headline_layout and not args.separate_buffers:
        pad = RANK_PAD_BYTES
    tdtype = torch.float32 if args.dtype == "fp32" else torch.int32
    calls = []          # per call of a step: (schedule, buffers, pristine copies, elements)
    offset = 0
    for m, sched in zip(sizes, scheds):
        if dist == "hash":
            pristine = []
            for r in range(k):
                pristine.append(si.hash_payload_torch(0, r, m, args.dtype, dev))
                say(f"payload of rank {r} generated")
        else:
            pristine = [torch.from_numpy(host_payload(si, 0, r, m, dist, args.dtype, scale, start=offset)).to(dev)
                        for r in range(k)]
        if pad is None or args.separate_buffers:
            bufs = [torch.empty_like(p) for p in pristine]
            layout = "one allocation per rank buffer"
        else:
            if pad % 16 or pad < 0:
                sys.exit("bench.py: --rank-pad-bytes must be a non-negative multiple of 16")
            # every rank buffer starts on a 4 KiB boundary, as buffers handed out
            # by an allocator do, whatever the payload size (a buffer that starts
            # 16 bytes off a 1 KiB boundary costs the kernel a fifth of its
            # throughput)
            stride = -(-(m + pad // 4) // 1024) * 1024
            slab = torch.empty(k * stride, dtype=tdtype, device=dev)
            bufs = [slab[r * stride: r * stride + m] for r in range(k)]
            layout = f"one allocation, rank buffers {m * 4} + {stride * 4 - m * 4} bytes apart"
        calls.append((sched, bufs, pristine, m))
        offset += m if args.config == "4" else 0
    stream = torch.cuda.current_stream()
    run = bl.blink_broadcast if broadcast else bl.blink_allreduce

    def restore():
        for _, bufs, pristine, _ in calls:
            for b, p in zip(bufs, pristine):
                b.copy_(p)

    def step():
        for sched, bufs, _, m in calls:
            run(bufs, m, dtype, sched, stream.cuda_stream)

    # Set-up, outside warm-up and timing like the building of the schedules: the
    # library spends a schedule's first thirteen calls at most choosing among the
    # ways it can serve it (twelve timed calls, then one that waits for them).
    SETUP_CALLS = 13
    say("inputs are on the device")
    restore()
    if args.progress:
        torch.cuda.synchronize()
        say("inputs restored")
    for i in range(SETUP_CALLS):
        step()
        if args.progress:           # slow, profiled runs: say where they are, call by call
            torch.cuda.synchronize()
            say(f"set-up call {i + 1} of {SETUP_CALLS} done")
    torch.cuda.synchronize()
    say("set-up calls done")
    since_restore = 0
    restore()
    for _ in range(args.warmup):
        if since_restore == MAX_STEPS_BETWEEN_RESTORES:
            restore()
            since_restore = 0
        step()
        since_restore += 1
    restore()
    since_restore = 0
    restores = 0
    torch.cuda.synchronize()
    say("warm-up done")

    # Kernel time with HIP events on the launch stream.  Launches follow one another
    # without a gap while the stream has work queued, so the average duration of a
    # launch is taken over runs of consecutive steps (first event of the run to the
    # last); an event pair around every single step would add the few microseconds
    # between a record and the launch next to it to each, which is a tenth of the
    # smaller configurations' kernels.  A run ends where the inputs are restored.
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    run_starts = []      # (event, index of the run's first step)
    t0 = time.perf_counter()
    for i in range(args.steps):
        if since_restore == MAX_STEPS_BETWEEN_RESTORES:
            restore()
            restores += 1
            since_restore = 0
        if i == 0 or since_restore == 0:
            ev = torch.cuda.Event(enable_timing=True)
            ev.record(stream)
            run_starts.append((ev, i))
        step()
        ends[i].record(stream)
        since_restore += 1
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    firsts = {first: ev for ev, first in run_starts}
    kernel_ms = [(firsts[i] if i in firsts else ends[i - 1]).elapsed_time(ends[i]) for i in range(args.steps)]
    avg_kernel_ms = sum(kernel_ms) / args.steps      # per step: all the step's launches together

    total = sum(sizes)
    ms_per_step = wall * 1e3 / args.steps
    value = total * 4 / (ms_per_step * 1e-3) / 1e9

    per_elem = ({"edge": 8 * (k - 1), "node": None, "tree": 4 * k} if broadcast else
                {"edge": 20 * (k - 1), "node": None, "tree": 8 * k})[args.fusion]
    alg_bytes = sum(s.traffic_bytes for s in scheds)      # == per_elem * n for edge and tree
    if per_elem is not None:
        assert alg_bytes == per_elem * total
    achieved = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9
    prof_name = (f"blink_consume_{collective}_cube8_{n * 4 >> 20}MiB_{args.fusion}.txt" if args.config == "headline"
                 else f"config{args.config}_{collective}_{args.fusion}.txt")
    say("timed steps done")
    traffic, traffic_digest = traffic_from_profiles(prof_name)
    roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS,
                "traffic": traffic,
                "traffic_source": (f"profiles/{prof_name}, measured on kernel sources {traffic_digest}"
                                   if traffic is not None else
                                   "none: no rocprofv3 counter summary under profiles/ for this workload was "
                                   "taken on the kernel sources as they are now"),
                "kernel_sources_digest": kernel_sources_digest(),
                "algorithmic_bytes_per_launch": alg_bytes,
                "launches_per_step": len(calls),
                "bytes_per_element": alg_bytes / total,
                "accounting": {"edge": "per-edge: every tree edge is a transfer between two rank buffers, "
                                       "20(k-1) B/elt (broadcast: 8(k-1))",
                               "node": "per-node: one pass per fan-in and per fan-out",
                               "tree": "staged minimum: every rank buffer read once and written once, 8k B/elt "
                                       "(broadcast: the root read once, the others written once, 4k)"}[args.fusion],
                "kernel": "blink_stream / blink_consume", "avg_kernel_ms": avg_kernel_ms,
                "median_kernel_ms": sorted(kernel_ms)[len(kernel_ms) // 2],
                "min_kernel_ms": min(kernel_ms)}
    if traffic is not None:   # the counters' bytes over this run's kernel time
        roofline["traffic_rate_GBs"] = traffic / (avg_kernel_ms * 1e-3) / 1e9

    metric = METRIC if args.config == "headline" else \
        f"{'Broadcast' if broadcast else 'AllReduce'} alg GB/s + achieved HBM GB/s vs peak, configuration {args.config}"
    out = {
        "metric": metric, "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if args.dtype == "fp32" else "i32",
        "data": "synthetic",
        "config": {"workload": f"configuration {args.config}: " + ("Broadcast from rank 0" if broadcast else "AllReduce") +
                               f", {what}; {k} virtual ranks (HBM buffers on one GPU), {trees.count} packed trees of "
                               f"rate {trees.rate:g}, {total} {args.dtype} per rank, {chunk_bytes} B chunks, seed 0",
                   "ranks": k, "elements_per_rank": total, "chunk_bytes": chunk_bytes,
                   "calls_per_step": len(calls), "trees": trees.count, "fusion": args.fusion, "layout": layout,
                   "stages": sum(s.num_stages for s in scheds),
                   "steps_in_schedule": sum(s.num_steps for s in scheds),
                   "restores_in_timed_region": restores, "setup_calls_per_schedule": SETUP_CALLS,
                   "sweep": args.sweep,
                   "kernel_serving": sorted({s.last_kernel for s in scheds}), "commit": git_head()},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline and args.dtype == "fp32":
        # leave the device with exactly one step applied to the pristine inputs
        restore()
        step()
        torch.cuda.synchronize()
        same, checked = True, 0
        off = 0
        for sched, bufs, _, m in calls:
            hdist = dist
            ok, c = check_against_oracle(
                _Shifted(si, off) if args.config == "4" else si, np, bufs, trees_lists, sched.bounds(), k, m,
                collective, hdist, scale)
            same, checked = same and ok, checked + c
            off += m
        out["config"]["matches_oracle_bitwise"] = same
        out["config"]["elements_checked_against_oracle"] = checked
        m = max(sizes)
        out["cpu_baseline"] = cpu_baseline(si, trees_lists, k, m, chunk, collective, dist, scale)
        if args.config == "4":
            out["cpu_baseline"]["sample"] = "the largest bucket; " + out["cpu_baseline"]["sample"]
        if args.config == "1":
            out["config"]["cpu_oracle_seconds"] = out["cpu_baseline"]["seconds"]
        if not same:
            print("bench.py: GPU result differs from the oracle", file=sys.stderr)
            print(json.dumps(out))
            sys.exit(1)
    print(json.dumps(out))


class _Shifted:
    """synth_inputs with every payload request moved `shift` elements on: bucket
    j of configuration 4 holds elements [shift_j, shift_j + m_j) of the 138 M."""

    def __init__(self, si, shift):
        self._si, self._shift = si, shift

    def payload(self, seed, rank, n, dist, dtype, scale=1.0, start=0):
        return self._si.payload(seed, rank, n, dist, dtype, scale, start=start + self._shift)

    def hash_payload(self, seed, rank, start, n, dtype):
        return self._si.hash_payload(seed, rank, start + self._shift, n, dtype)


if __name__ == "__main__":
    main()
