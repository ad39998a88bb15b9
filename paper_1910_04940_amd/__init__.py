"""Packed-spanning-tree Broadcast / AllReduce for one MI355X (HIP library + thin binding)."""
from .binding import (  # noqa: F401
    BLINK_EDISCONNECTED, BLINK_EHIP, BLINK_ESTUCK, BLINK_ELIMIT, BLINK_EINVAL, BLINK_EMISMATCH, BLINK_ENOMEM, BLINK_FP32,
    BLINK_FUSE_EDGE, BLINK_FUSE_NODE, BLINK_FUSE_TREE, BLINK_INT32, BLINK_MAX_RANKS, BLINK_OK,
    BLINK_MAX, BLINK_MIN, BLINK_OP_ALLGATHER, BLINK_OP_ALLREDUCE, BLINK_OP_BROADCAST, BLINK_OP_GATHER, BLINK_OP_REDUCE, BLINK_PROD, BLINK_ROOT_ANY, BLINK_SUM, BLINK_STEP_COPY, BLINK_STEP_REDUCE,
    BlinkError, Miad, Schedule, Trees, blink_allgather, blink_allreduce, blink_allreduce_noalloc, blink_allreduce_op, blink_broadcast, blink_gather, blink_hybrid_split,
    blink_make_schedule, blink_make_schedule_servers, blink_reduce,
    blink_pack_trees, blink_trees_from_arrays, strerror,
)
