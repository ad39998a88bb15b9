"""ctypes binding of libblink.so: the same names as include/blink.h, argument
marshalling only.  Every step of the method runs inside the library.

The library must have been built (``python -m paper_1910_04940_amd.build`` or
``__graft_entry__.build()``); loading fails loudly otherwise.  There is no CPU
fallback.
"""
from __future__ import annotations

import ctypes as C
import importlib.util
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libblink.so")

BLINK_MAX_RANKS = 16
BLINK_ROOT_ANY = -1
BLINK_OK, BLINK_EINVAL, BLINK_EDISCONNECTED, BLINK_ENOMEM, BLINK_EMISMATCH, BLINK_EHIP, BLINK_ESTUCK, BLINK_ELIMIT = range(8)
BLINK_INT32, BLINK_FP32 = 0, 1
BLINK_OP_BROADCAST, BLINK_OP_ALLREDUCE, BLINK_OP_REDUCE, BLINK_OP_ALLGATHER, BLINK_OP_GATHER = 0, 1, 2, 3, 4
BLINK_SUM, BLINK_PROD, BLINK_MIN, BLINK_MAX = 0, 1, 2, 3
BLINK_STEP_REDUCE, BLINK_STEP_COPY = 0, 1
BLINK_FUSE_EDGE, BLINK_FUSE_NODE, BLINK_FUSE_TREE = 0, 1, 2

# numpy mirror of blink_step_t
STEP_DTYPE = np.dtype([("kind", "<i4"), ("tree", "<i4"), ("chunk", "<i4"), ("src", "<i4"),
                       ("dst", "<i4"), ("n_deps", "<i4"), ("deps", "<i4", (2,)),
                       ("off", "<u8"), ("len", "<u8")], align=True)

# numpy mirror of blink_progress_t
PROGRESS_DTYPE = np.dtype([("state", "<i4"), ("stage", "<i4"), ("awaited_stage", "<i4"), ("reserved", "<i4"),
                           ("seen", "<u8"), ("wanted", "<u8"), ("call", "<u8")], align=True)

# numpy mirror of blink_stage_t
STAGE_DTYPE = np.dtype([("off", "<u8"), ("len", "<u4"), ("tree", "<i4"), ("chunk", "<i4"), ("flow", "<i4"),
                        ("n_load", "u1"), ("n_op", "u1"), ("n_store", "u1"), ("n_dep", "u1"),
                        ("load_rank", "u1", (16,)), ("store_rank", "u1", (16,)), ("op", "u1", (40,)),
                        ("deps", "<i4", (8,)), ("seq_rank", "u1", (16,)), ("seq_code", "u1", (16,)),
                        ("seq_depth", "u1"), ("reserved", "u1", (3,))], align=True)

EXPORTS = [
    "blink_pack_trees", "blink_trees_from_arrays", "blink_trees_count", "blink_trees_k",
    "blink_trees_rate", "blink_trees_get", "blink_trees_free", "blink_make_schedule",
    "blink_schedule_num_steps", "blink_schedule_num_stages", "blink_schedule_num_trees",
    "blink_schedule_get_steps", "blink_schedule_get_bounds", "blink_schedule_traffic_bytes",
    "blink_schedule_free", "blink_allreduce", "blink_broadcast", "blink_schedule_set_launch",
    "blink_allreduce_op", "blink_reduce", "blink_allgather", "blink_gather", "blink_strerror",
    "blink_miad_create", "blink_miad_chunk", "blink_miad_steady", "blink_miad_report",
    "blink_miad_free", "blink_make_schedule_servers", "blink_hybrid_split",
    "blink_schedule_get_stages", "blink_schedule_status", "blink_schedule_reset",
    "blink_schedule_set_wait_limit", "blink_schedule_test_skip_call", "blink_allreduce_noalloc",
    "blink_schedule_set_kernel", "blink_schedule_last_kernel", "blink_schedule_set_sweep", "blink_schedule_get_tickets", "blink_schedule_batch",
]


class BlinkError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_lib = None
_hip = None


def _load_hip_runtime() -> None:
    """libblink.so leaves the HIP entry points undefined so that it binds to the
    one HIP runtime of the process.  PyTorch wheels bundle their own
    libamdhip64; device memory and streams come from PyTorch, so that copy is
    the one to share.  Without PyTorch the system ROCm runtime is used."""
    global _hip
    if _hip is not None:
        return
    candidates = []
    spec = importlib.util.find_spec("torch")
    if spec is not None and spec.origin:
        candidates.append(os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so"))
    candidates += ["/opt/rocm/lib/libamdhip64.so", "libamdhip64.so"]
    errors = []
    for path in candidates:
        if os.path.isabs(path) and not os.path.exists(path):
            continue
        try:
            _hip = C.CDLL(path, mode=C.RTLD_GLOBAL)
            return
        except OSError as e:  # try the next candidate
            errors.append(f"{path}: {e}")
    raise ImportError("no HIP runtime could be loaded: " + "; ".join(errors))


def lib() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first "
                          "(python -m paper_1910_04940_amd.build); there is no fallback path")
    _load_hip_runtime()
    L = C.CDLL(LIB_PATH)
    i32p, f64p, vp = C.POINTER(C.c_int32), C.POINTER(C.c_double), C.c_void_p
    L.blink_pack_trees.argtypes = [C.c_int, C.c_int, i32p, i32p, f64p, C.c_int, C.c_double,
                                   C.c_double, C.POINTER(vp)]
    L.blink_trees_from_arrays.argtypes = [C.c_int, C.c_int, i32p, i32p, f64p, C.POINTER(vp)]
    L.blink_trees_count.argtypes = [vp]
    L.blink_trees_k.argtypes = [vp]
    L.blink_trees_rate.argtypes = [vp]
    L.blink_trees_rate.restype = C.c_double
    L.blink_trees_get.argtypes = [vp, C.c_int, i32p, i32p, f64p]
    L.blink_trees_free.argtypes = [vp]
    L.blink_trees_free.restype = None
    L.blink_make_schedule.argtypes = [vp, C.c_int, C.c_size_t, C.c_size_t, C.c_int, C.POINTER(vp)]
    L.blink_make_schedule_servers.argtypes = [C.c_int, C.POINTER(vp), C.POINTER(C.c_int32), C.c_size_t,
                                              C.c_size_t, C.c_int, C.POINTER(vp)]
    L.blink_hybrid_split.argtypes = [C.c_double] * 4 + [C.POINTER(C.c_double)] * 2
    L.blink_schedule_num_steps.argtypes = [vp]
    L.blink_schedule_num_steps.restype = C.c_size_t
    L.blink_schedule_get_stages.argtypes = [vp, vp]
    L.blink_schedule_num_stages.argtypes = [vp]
    L.blink_schedule_num_stages.restype = C.c_size_t
    L.blink_schedule_num_trees.argtypes = [vp]
    L.blink_schedule_batch.argtypes = [vp]
    L.blink_schedule_batch.restype = C.c_uint64
    L.blink_schedule_get_steps.argtypes = [vp, vp]
    L.blink_schedule_get_bounds.argtypes = [vp, C.POINTER(C.c_uint64)]
    L.blink_schedule_traffic_bytes.argtypes = [vp]
    L.blink_schedule_traffic_bytes.restype = C.c_uint64
    L.blink_schedule_free.argtypes = [vp]
    L.blink_schedule_free.restype = None
    for name in ("blink_allreduce", "blink_broadcast", "blink_allgather", "blink_gather", "blink_allreduce_noalloc"):
        getattr(L, name).argtypes = [C.POINTER(vp), C.c_int, C.c_size_t, C.c_int, vp, vp]
    for name in ("blink_allreduce_op", "blink_reduce"):
        getattr(L, name).argtypes = [C.POINTER(vp), C.c_int, C.c_size_t, C.c_int, C.c_int, vp, vp]
    L.blink_schedule_set_launch.argtypes = [vp, C.c_int, C.c_int]
    L.blink_schedule_status.argtypes = [vp, vp]
    L.blink_schedule_reset.argtypes = [vp]
    L.blink_schedule_set_wait_limit.argtypes = [vp, C.c_uint64]
    L.blink_schedule_test_skip_call.argtypes = [vp]
    L.blink_schedule_set_kernel.argtypes = [vp, C.c_int]
    L.blink_schedule_get_tickets.argtypes = [vp, C.c_uint32, C.POINTER(C.c_uint64), vp, vp]
    L.blink_schedule_last_kernel.argtypes = [vp]
    L.blink_schedule_set_sweep.argtypes = [vp, C.c_int]
    L.blink_miad_create.argtypes = [C.c_size_t, C.c_double, C.c_size_t, C.c_size_t, C.c_size_t,
                                    C.c_double, C.POINTER(vp)]
    L.blink_miad_chunk.argtypes = [vp]
    L.blink_miad_chunk.restype = C.c_size_t
    L.blink_miad_steady.argtypes = [vp]
    L.blink_miad_report.argtypes = [vp, C.c_double]
    L.blink_miad_free.argtypes = [vp]
    L.blink_miad_free.restype = None
    L.blink_strerror.argtypes = [C.c_int]
    L.blink_strerror.restype = C.c_char_p
    _lib = L
    return L


def strerror(status: int) -> str:
    return lib().blink_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != BLINK_OK:
        raise BlinkError(status, where)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


class Trees:
    """Owns a blink_trees_t handle."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.blink_trees_free(self._h)
            self._h = None

    @property
    def count(self) -> int:
        return lib().blink_trees_count(self._h)

    @property
    def k(self) -> int:
        return lib().blink_trees_k(self._h)

    @property
    def rate(self) -> float:
        return lib().blink_trees_rate(self._h)

    def get(self, t: int) -> Tuple[int, Tuple[int, ...], float]:
        root = C.c_int32()
        weight = C.c_double()
        parent = np.empty(self.k, np.int32)
        _check(lib().blink_trees_get(self._h, t, C.byref(root), _ptr(parent, C.c_int32),
                                     C.byref(weight)), "blink_trees_get")
        return int(root.value), tuple(int(x) for x in parent), float(weight.value)

    def as_lists(self):
        """(roots, parent tuples, weights)."""
        items = [self.get(t) for t in range(self.count)]
        return [r for r, _, _ in items], [p for _, p, _ in items], [w for _, _, w in items]


def blink_pack_trees(k: int, src, dst, cap, root: int, eps: float = 0.05,
                     prune_tol: float = 0.05) -> Trees:
    src, dst = _i32(src), _i32(dst)
    cap = np.ascontiguousarray(cap, dtype=np.float64)
    if not (src.shape == dst.shape == cap.shape and src.ndim == 1):
        raise ValueError("src, dst, cap must be 1-D arrays of one length")
    out = C.c_void_p()
    _check(lib().blink_pack_trees(k, src.shape[0], _ptr(src, C.c_int32), _ptr(dst, C.c_int32),
                                  _ptr(cap, C.c_double), root, eps, prune_tol, C.byref(out)),
           "blink_pack_trees")
    return Trees(out.value)


def blink_trees_from_arrays(k: int, roots, parents, weights) -> Trees:
    roots = _i32(roots)
    parents = _i32(parents).reshape(-1)
    weights = np.ascontiguousarray(weights, dtype=np.float64)
    T = roots.shape[0]
    if parents.shape[0] != T * k or weights.shape[0] != T:
        raise ValueError("parents must be T*k, weights T")
    out = C.c_void_p()
    _check(lib().blink_trees_from_arrays(k, T, _ptr(roots, C.c_int32), _ptr(parents, C.c_int32),
                                         _ptr(weights, C.c_double), C.byref(out)),
           "blink_trees_from_arrays")
    return Trees(out.value)


class Schedule:
    """Owns a blink_schedule_t handle."""

    def __init__(self, handle: int, k: int, n: int, op: int):
        self._h = C.c_void_p(handle)
        self.k, self.n, self.op = k, n, op

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.blink_schedule_free(self._h)
            self._h = None

    @property
    def num_steps(self) -> int:
        return lib().blink_schedule_num_steps(self._h)

    @property
    def num_stages(self) -> int:
        return lib().blink_schedule_num_stages(self._h)

    @property
    def num_trees(self) -> int:
        return lib().blink_schedule_num_trees(self._h)

    @property
    def batch(self) -> int:
        return lib().blink_schedule_batch(self._h)

    @property
    def traffic_bytes(self) -> int:
        return lib().blink_schedule_traffic_bytes(self._h)

    def steps(self) -> np.ndarray:
        out = np.zeros(self.num_steps, STEP_DTYPE)
        _check(lib().blink_schedule_get_steps(self._h, out.ctypes.data), "blink_schedule_get_steps")
        return out

    def stages(self) -> np.ndarray:
        out = np.zeros(self.num_stages, STAGE_DTYPE)
        _check(lib().blink_schedule_get_stages(self._h, out.ctypes.data), "blink_schedule_get_stages")
        return out

    def bounds(self) -> List[int]:
        out = np.zeros(self.num_trees + 1, np.uint64)
        _check(lib().blink_schedule_get_bounds(self._h, _ptr(out, C.c_uint64)),
               "blink_schedule_get_bounds")
        return [int(x) for x in out]

    def set_launch(self, wg_per_cu: int = 0, tile_elems: int = 0) -> None:
        _check(lib().blink_schedule_set_launch(self._h, wg_per_cu, tile_elems), "blink_schedule_set_launch")

    def tickets(self, tile_elems: int) -> Tuple[np.ndarray, np.ndarray]:
        """(stage, tile) per ticket, in the order the kernel hands them out."""
        n = C.c_uint64()
        _check(lib().blink_schedule_get_tickets(self._h, tile_elems, C.byref(n), None, None), "blink_schedule_get_tickets")
        stage, tile = np.zeros(n.value, np.int32), np.zeros(n.value, np.int32)
        _check(lib().blink_schedule_get_tickets(self._h, tile_elems, C.byref(n), stage.ctypes.data, tile.ctypes.data),
               "blink_schedule_get_tickets")
        return stage, tile

    def set_kernel(self, kernel: int) -> None:
        """0 = the library times the ways it can serve this schedule and keeps the
        fastest; 1 = ticket-drawing kernel, 2 = streaming kernel, 3 = ticket-drawing
        kernel with the trees taking turns chunk by chunk (see blink.h)."""
        _check(lib().blink_schedule_set_kernel(self._h, kernel), "blink_schedule_set_kernel")

    def set_sweep(self, alternate: bool) -> None:
        _check(lib().blink_schedule_set_sweep(self._h, 1 if alternate else 0), "blink_schedule_set_sweep")

    @property
    def last_kernel(self) -> int:
        """The way the latest call on this schedule ran (1, 2 or 3; 0 before the first)."""
        return lib().blink_schedule_last_kernel(self._h)

    def status(self) -> Tuple[int, dict]:
        """(status code, blink_progress_t as a dict); waits for the device."""
        out = np.zeros(1, PROGRESS_DTYPE)
        st = lib().blink_schedule_status(self._h, out.ctypes.data)
        if st not in (BLINK_OK, BLINK_ESTUCK):
            raise BlinkError(st, "blink_schedule_status")
        return st, {name: int(out[0][name]) for name in PROGRESS_DTYPE.names}

    def reset(self) -> None:
        _check(lib().blink_schedule_reset(self._h), "blink_schedule_reset")

    def set_wait_limit(self, microseconds: int) -> None:
        _check(lib().blink_schedule_set_wait_limit(self._h, microseconds), "blink_schedule_set_wait_limit")

    def test_skip_call(self) -> None:
        _check(lib().blink_schedule_test_skip_call(self._h), "blink_schedule_test_skip_call")


def blink_make_schedule(trees: Trees, op: int, n_elems: int, chunk_elems: int,
                        fusion: int = BLINK_FUSE_TREE) -> Schedule:
    out = C.c_void_p()
    _check(lib().blink_make_schedule(trees._h, op, n_elems, chunk_elems, fusion, C.byref(out)),
           "blink_make_schedule")
    return Schedule(out.value, trees.k, n_elems, op)


def blink_make_schedule_servers(local: Sequence[Optional[Trees]], ranks: Sequence[Sequence[int]],
                                n_elems: int, chunk_elems: int,
                                fusion: int = BLINK_FUSE_TREE) -> Schedule:
    """local[s]: server s's trees (None for a one-rank server); ranks[s]: the
    global ids of its local ranks, ascending."""
    if len(local) != len(ranks):
        raise ValueError("one rank list per server")
    for t, r in zip(local, ranks):
        if len(r) != (t.k if t is not None else 1):
            raise ValueError("a server's rank list must have one id per local rank")
    handles = (C.c_void_p * len(local))(*[t._h if t is not None else None for t in local])
    flat = np.ascontiguousarray([g for r in ranks for g in r], dtype=np.int32)
    out = C.c_void_p()
    _check(lib().blink_make_schedule_servers(len(local), handles, _ptr(flat, C.c_int32), n_elems,
                                             chunk_elems, fusion, C.byref(out)),
           "blink_make_schedule_servers")
    return Schedule(out.value, len(flat), n_elems, BLINK_OP_ALLREDUCE)


def blink_hybrid_split(d_total: float, bw_slow: float, bw_fast: float, t_switch: float):
    a, b = C.c_double(), C.c_double()
    _check(lib().blink_hybrid_split(d_total, bw_slow, bw_fast, t_switch, C.byref(a), C.byref(b)),
           "blink_hybrid_split")
    return a.value, b.value


def _pointers(bufs: Sequence) -> "C.Array":
    vals = [int(b.data_ptr()) if hasattr(b, "data_ptr") else int(b) for b in bufs]
    return (C.c_void_p * len(vals))(*vals)


def blink_allreduce(bufs: Sequence, n_elems: int, dtype: int, schedule: Schedule, stream: int = 0) -> None:
    """bufs: k device pointers (ints) or objects with .data_ptr(); stream: hipStream_t as int."""
    arr = _pointers(bufs)
    _check(lib().blink_allreduce(arr, len(bufs), n_elems, dtype, schedule._h, C.c_void_p(stream)),
           "blink_allreduce")


def blink_allreduce_noalloc(bufs: Sequence, n_elems: int, dtype: int, schedule: Schedule, stream: int = 0) -> None:
    """blink_allreduce on the library's static device block: the call allocates nothing."""
    arr = _pointers(bufs)
    _check(lib().blink_allreduce_noalloc(arr, len(bufs), n_elems, dtype, schedule._h, C.c_void_p(stream)),
           "blink_allreduce_noalloc")


def blink_broadcast(bufs: Sequence, n_elems: int, dtype: int, schedule: Schedule, stream: int = 0) -> None:
    arr = _pointers(bufs)
    _check(lib().blink_broadcast(arr, len(bufs), n_elems, dtype, schedule._h, C.c_void_p(stream)),
           "blink_broadcast")


def blink_allgather(bufs: Sequence, n_elems: int, dtype: int, schedule: Schedule, stream: int = 0) -> None:
    arr = _pointers(bufs)
    _check(lib().blink_allgather(arr, len(bufs), n_elems, dtype, schedule._h, C.c_void_p(stream)),
           "blink_allgather")


def blink_gather(bufs: Sequence, n_elems: int, dtype: int, schedule: Schedule, stream: int = 0) -> None:
    arr = _pointers(bufs)
    _check(lib().blink_gather(arr, len(bufs), n_elems, dtype, schedule._h, C.c_void_p(stream)),
           "blink_gather")


def blink_allreduce_op(bufs: Sequence, n_elems: int, dtype: int, redop: int, schedule: Schedule,
                       stream: int = 0) -> None:
    arr = _pointers(bufs)
    _check(lib().blink_allreduce_op(arr, len(bufs), n_elems, dtype, redop, schedule._h,
                                    C.c_void_p(stream)), "blink_allreduce_op")


def blink_reduce(bufs: Sequence, n_elems: int, dtype: int, redop: int, schedule: Schedule,
                 stream: int = 0) -> None:
    arr = _pointers(bufs)
    _check(lib().blink_reduce(arr, len(bufs), n_elems, dtype, redop, schedule._h, C.c_void_p(stream)),
           "blink_reduce")


class Miad:
    """Owns a blink_miad_t handle (chunk-size search, paper section 4.2.1)."""

    def __init__(self, initial_chunk: int, factor: float = 2.0, step: int = 0, lo: int = 1,
                 hi: int = 1 << 40, rel_tol: float = 0.0):
        out = C.c_void_p()
        _check(lib().blink_miad_create(initial_chunk, factor, step or initial_chunk, lo, hi, rel_tol,
                                       C.byref(out)), "blink_miad_create")
        self._h = out

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.blink_miad_free(self._h)
            self._h = None

    @property
    def chunk(self) -> int:
        return lib().blink_miad_chunk(self._h)

    @property
    def steady(self) -> bool:
        return bool(lib().blink_miad_steady(self._h))

    def report(self, throughput: float) -> None:
        _check(lib().blink_miad_report(self._h, throughput), "blink_miad_report")
