/*
 * blink.h - C ABI of the packed-spanning-tree collectives for one MI355X.
 *
 * The k "ranks" of a collective are k separate device (HBM) buffers on the
 * current HIP device.  A collective is prepared in two host-side steps and then
 * executed by one persistent gfx950 kernel:
 *
 *   blink_pack_trees     topology graph -> weighted spanning trees
 *                        (paper sections 3.1, 3.2, 3.2.1, 3.5)
 *   blink_make_schedule  trees + payload size + chunk size -> step list
 *                        (paper sections 3.3, 4.1, 4.2.1, 4.2.2)
 *   blink_broadcast /    run the step list on k device buffers, asynchronously
 *   blink_allreduce      on a HIP stream (paper sections 3.3, 4.1)
 *   blink_miad_*         pick the chunk size over the first iterations of a job
 *                        (paper section 4.2.1)
 *   blink_make_schedule_servers / blink_hybrid_split
 *                        several servers, two classes of links (sections 3.5, 3.4)
 *
 * Conventions
 *   - Every function that can fail returns blink_status_t; results come back
 *     through pointer arguments.  No exception crosses this boundary.
 *   - "host" / "device" in a parameter comment says where the pointed-to memory
 *     must live.
 *   - Handles (blink_trees_t, blink_schedule_t) are owned by the library and
 *     released with the matching *_free.  The caller owns every buffer it
 *     passes in; the library never frees or reallocates caller memory.
 *   - A schedule keeps device-side progress counters: it may be used by many
 *     calls one after another on ONE stream at a time.  Two calls that overlap
 *     in time on the same schedule race (stages of one may then wait for
 *     progress the other consumed; such a wait is bounded, see
 *     blink_schedule_status).  Every launch carries the number of
 *     the call on its schedule, so a call cannot be recorded into a HIP graph
 *     (a replay would repeat a number): on a capturing stream every collective
 *     but blink_allreduce_noalloc returns BLINK_EINVAL and records nothing.
 *   - At most BLINK_MAX_RANKS ranks.
 */
#ifndef BLINK_H
#define BLINK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BLINK_MAX_RANKS 16
/* root argument of blink_pack_trees for switch-like (fully connected)
 * topologies: one one-hop tree per rank, rank i the root of tree i, each tree
 * carrying 1/k of the data (paper section 3.5). */
#define BLINK_ROOT_ANY (-1)

typedef enum {
    BLINK_OK = 0,
    BLINK_EINVAL = 1,        /* bad argument (null pointer, k < 2, bad vertex id, capacity <= 0, chunk 0, misaligned buffer ...) */
    BLINK_EDISCONNECTED = 2, /* some vertex cannot be reached from the root: rate 0 */
    BLINK_ENOMEM = 3,        /* host or device allocation failed */
    BLINK_EMISMATCH = 4,     /* schedule does not fit the call (k, n, collective) */
    BLINK_EHIP = 5,          /* a HIP runtime call failed (no device, launch error) */
    BLINK_ESTUCK = 6,        /* a stage gave up waiting for another one (see blink_schedule_status) */
    BLINK_ELIMIT = 7         /* the schedule does not fit the fixed device block of blink_allreduce_noalloc */
} blink_status_t;

typedef enum { BLINK_INT32 = 0, BLINK_FP32 = 1 } blink_dtype_t;
/* Collectives (paper section 4.1).  REDUCE is the reduce phase of AllReduce on
 * its own: afterwards only the root of each tree holds the result (on that
 * tree's share); what the other ranks' buffers hold is unspecified. */
/* ALLGATHER and GATHER work on buffers of n_elems = k * m elements in which rank
 * j owns piece j = [j*m, (j+1)*m) and starts with it in place: afterwards every
 * rank (ALLGATHER) or the root of each tree (GATHER, on that tree's share of
 * every piece) holds all k pieces.  Section 4.1 derives both from the
 * collectives above: a gather runs a broadcast backwards, an all-gather is an
 * all-reduce that only moves data.  Here every piece is split among the trees
 * by weight; a tree moves its share of piece j hop by hop along its own edges,
 * away from rank j in every direction (ALLGATHER) or up to its root (GATHER). */
typedef enum {
    BLINK_OP_BROADCAST = 0, BLINK_OP_ALLREDUCE = 1, BLINK_OP_REDUCE = 2,
    BLINK_OP_ALLGATHER = 3, BLINK_OP_GATHER = 4
} blink_op_t;
/* Reduction operators (section 4.1 names min and max next to the sum).  SUM and
 * PROD: one IEEE operation per step for fp32, wrap-around modulo 2^32 for
 * int32.  MIN and MAX: signed comparison for int32; for fp32 the smaller /
 * larger under the IEEE total order (-0 below +0), so the result does not
 * depend on the order of the operands. */
typedef enum { BLINK_SUM = 0, BLINK_PROD = 1, BLINK_MIN = 2, BLINK_MAX = 3 } blink_redop_t;
typedef enum { BLINK_STEP_REDUCE = 0, BLINK_STEP_COPY = 1 } blink_step_kind_t;

/* How many tree-edge transfers one wavefront carries a tile through before the
 * data returns to HBM.  The result is bit-identical for all three.
 *   EDGE  one transfer per step, as the paper issues them: a REDUCE reads both
 *         rank buffers and writes the parent's, a COPY reads the parent's and
 *         writes the child's; steps of one chunk hand over through device-side
 *         completion counters.
 *   NODE  the fan-in of one tree node (own data + all children) is one pass and
 *         its fan-out (to all children) another; counters between nodes.  This
 *         is what one GPU would do locally if every rank were its own GPU.
 *   TREE  a tile is carried through all transfers of its tree at once: every
 *         rank buffer is read once and written once; partial sums stay in LDS.
 */
typedef enum { BLINK_FUSE_EDGE = 0, BLINK_FUSE_NODE = 1, BLINK_FUSE_TREE = 2 } blink_fusion_t;

typedef struct blink_trees blink_trees_t;
typedef struct blink_schedule blink_schedule_t;

/* One transfer over one tree edge for one chunk (paper section 4.1).
 * REDUCE: dst[off, off+len) <- dst[off, off+len) + src[off, off+len)
 * COPY:   dst[off, off+len) <- src[off, off+len)
 * deps[0..n_deps) are indices of earlier steps of the list that must have
 * completed before this one may start (the chunk-granular "event" of the
 * paper). */
typedef struct {
    int32_t kind;    /* blink_step_kind_t */
    int32_t tree;
    int32_t chunk;   /* index of the chunk inside the tree's share */
    int32_t src;     /* rank read */
    int32_t dst;     /* rank written */
    int32_t n_deps;  /* 0..2 */
    int32_t deps[2];
    uint64_t off;    /* first element */
    uint64_t len;    /* elements */
} blink_step_t;

/* One pass of the kernel over a chunk ("stage"): what blink_schedule_get_stages
 * reports, so that a schedule can be checked, or replayed on the host, without
 * a GPU.  For every element of [off, off + len): slot i <- rank load_rank[i]
 * (i < n_load); then the n_op micro-operations in order, each (kind << 6) | slot
 * with kind 0: acc <- slot, 1: acc <- acc (+) slot, 2: slot <- acc; finally acc
 * is stored to every rank in store_rank[0 .. n_store).  deps: indices of the
 * earlier stages all of which must have finished on their whole chunk first.
 * seq_*: the same computation as a program for a stack of accumulators (what the
 * streaming kernel runs): for i < n_load in turn, rank seq_rank[i] either starts
 * a new accumulator on top of the stack (seq_code[i] & 1) or is combined into
 * the top one; then seq_code[i] >> 1 times the top accumulator is combined into
 * the one below it and dropped.  One accumulator is left: the result.
 * seq_depth: the accumulators needed; 0 when the stage has no such form. */
#define BLINK_STAGE_MAX_OPS 40
#define BLINK_STAGE_MAX_DEPS 8
typedef struct {
    uint64_t off;
    uint32_t len;
    int32_t tree;    /* the packed tree the stage belongs to */
    int32_t chunk;   /* chunk index inside its flow's range */
    int32_t flow;    /* one tree carrying one contiguous range in one direction;
                        the gathers have several per tree (one per piece) */
    uint8_t n_load, n_op, n_store, n_dep;
    uint8_t load_rank[BLINK_MAX_RANKS];
    uint8_t store_rank[BLINK_MAX_RANKS];
    uint8_t op[BLINK_STAGE_MAX_OPS];
    int32_t deps[BLINK_STAGE_MAX_DEPS];
    uint8_t seq_rank[BLINK_MAX_RANKS];
    uint8_t seq_code[BLINK_MAX_RANKS];
    uint8_t seq_depth;
    uint8_t reserved[3];
} blink_stage_t;

/* ---- tree packing (host only; no GPU needed) ------------------------------ */

/* Pack spanning trees into a capacitated directed graph (section 3.1): k
 * vertices, m arcs src[i] -> dst[i] of capacity cap[i] > 0 (all three: host
 * arrays of length m; a bidirectional link is two arcs; parallel arcs add up).
 * root in [0,k): multiplicative-weight-update fractional packing of
 * arborescences rooted there (section 3.2, accuracy eps in (0, 0.5]; the
 * rounds needed grow like m ln m / eps^2, and an eps for which that estimate
 * exceeds 5e7 (eps of 0.005 or less on 240 arcs, below 0.0015 on 32) is refused
 * with BLINK_EINVAL instead of running for minutes), then
 * reduced to few trees (section 3.2.1) accepting a rate loss of at most
 * prune_tol in [0,1) against the MWU rate.  root == BLINK_ROOT_ANY: k one-hop
 * trees (section 3.5); needs every arc i->j to be present, else BLINK_EINVAL.
 * *out receives a new handle.  BLINK_EDISCONNECTED if a vertex is unreachable. */
blink_status_t blink_pack_trees(int k, int m, const int32_t* src, const int32_t* dst,
                                const double* cap, int root, double eps, double prune_tol,
                                blink_trees_t** out);

/* Wrap caller-chosen trees: roots[T], parent[T*k] (parent[t*k+v] is v's
 * predecessor in tree t, -1 for the root), weight[T] > 0; host arrays.  Every
 * tree must be a spanning arborescence of the complete graph on k vertices
 * (no topology is checked here). */
blink_status_t blink_trees_from_arrays(int k, int T, const int32_t* roots, const int32_t* parent,
                                       const double* weight, blink_trees_t** out);

int blink_trees_count(const blink_trees_t* trees);  /* T; -1 for a null handle */
int blink_trees_k(const blink_trees_t* trees);      /* k; -1 for a null handle */
double blink_trees_rate(const blink_trees_t* trees); /* sum of the weights */
/* Tree t: *root, parent[k] (host, caller-allocated), *weight.  Any of the
 * three output pointers may be null. */
blink_status_t blink_trees_get(const blink_trees_t* trees, int t, int32_t* root,
                               int32_t* parent, double* weight);
void blink_trees_free(blink_trees_t* trees);

/* ---- schedule (host only; no GPU needed) ------------------------------------ */

/* Split [0, n_elems) among the trees in proportion to their weights (section
 * 4.1): share boundaries are floor(n * prefix_weight / total_weight) rounded
 * down to a multiple of 4 elements, exact in rational arithmetic.  Cut every
 * share into chunks of chunk_elems (last one short, section 4.2.1).  Emit, per
 * tree and chunk, one COPY per tree arc (Broadcast, AllReduce) and one REDUCE
 * per reversed arc before them (AllReduce, Reduce; section 3.3), with their
 * dependencies, ordered so that all
 * trees advance together, one chunk of each in turn (section 4.2.2).
 * A node folds its children in ascending rank id (this fixes the fp32
 * association order).  The reduce phase uses every tree arc backwards: like the
 * paper (section 3.3) this takes links to be bidirectional; no topology is
 * consulted here.  Broadcast needs all trees to share one root, else
 * BLINK_EMISMATCH.  n_elems == 0 gives an empty, valid schedule. */
blink_status_t blink_make_schedule(const blink_trees_t* trees, blink_op_t op, size_t n_elems,
                                   size_t chunk_elems, blink_fusion_t fusion,
                                   blink_schedule_t** out);

/* AllReduce across n_servers servers, each with its own packed local trees
 * (section 3.5, the three-phase protocol): inside every server the root of a
 * tree reduces its partition of the payload over that tree; the server-local
 * roots of a partition then run a one-hop reduce-broadcast among themselves,
 * each of them owning one n-th of the partition; every root finally broadcasts
 * over its local tree.
 *   local[n_servers] (host): each server's trees; null for a server with one rank.
 *   ranks (host): for server 0, 1, .. in turn, the global rank id of each of its
 *       local ranks, strictly ascending inside a server; together a permutation
 *       of 0 .. k-1, k = total number of ranks <= BLINK_MAX_RANKS.
 * Partitions are the common refinement of the servers' weighted splits, so
 * that one tree per server serves a partition; the i-th smallest root id owns
 * the i-th of the n equal pieces (4-element alignment) of a partition and adds
 * the other roots' partial sums in ascending id after its own local sum.
 * The result is a schedule for BLINK_OP_ALLREDUCE on k ranks (run it with
 * blink_allreduce / blink_allreduce_op); its "trees" are the (partition,
 * piece) pairs with non-empty range, in payload order.  The local handles are
 * not retained. */
blink_status_t blink_make_schedule_servers(int n_servers, const blink_trees_t* const* local,
                                           const int32_t* ranks, size_t n_elems,
                                           size_t chunk_elems, blink_fusion_t fusion,
                                           blink_schedule_t** out);

/* Split of d_total between a slow and a fast class of links (section 3.4, the
 * PCIe / NVLink case) so that both finish together when the slow class first
 * pays the switch-over latency t_switch:
 *   d_slow / bw_slow + t_switch = d_fast / bw_fast,  d_slow + d_fast = d_total.
 * d_slow is clamped to [0, d_total] (nothing goes over the slow class when the
 * latency outweighs it).  Units are the caller's (bytes, bytes/s, s).
 * BLINK_EINVAL for non-positive bandwidths, negative sizes or latencies, or
 * null outputs. */
blink_status_t blink_hybrid_split(double d_total, double bw_slow, double bw_fast, double t_switch,
                                  double* d_slow, double* d_fast);

size_t blink_schedule_num_steps(const blink_schedule_t* s);   /* tree-edge transfers */
size_t blink_schedule_num_stages(const blink_schedule_t* s);  /* passes the kernel makes (== steps for EDGE) */
int blink_schedule_num_trees(const blink_schedule_t* s);
/* Chunks of a tree that share a time slot of the step list.  The list is ordered
 * by time slots of a fully pipelined execution in which the chunks advance from
 * one tree level to the next in batches of this many; inside a slot the trees
 * take turns chunk by chunk (section 4.2.2).  1 for short schedules; more where
 * the kernel's waves would otherwise outrun the dependencies (many small chunks). */
uint64_t blink_schedule_batch(const blink_schedule_t* s);
/* out[num_steps] (host, caller-allocated): the step list in execution order. */
blink_status_t blink_schedule_get_steps(const blink_schedule_t* s, blink_step_t* out);
/* out[num_stages] (host, caller-allocated): the kernel's passes in the order
 * in which their tickets are handed out (a topological order of the deps). */
blink_status_t blink_schedule_get_stages(const blink_schedule_t* s, blink_stage_t* out);
/* The order in which the kernel hands out its work when a tile has tile_elems
 * elements (a power of two in [256, 65536]; the library's own choice depends on
 * the device): ticket t is tile tile[t] of stage stage[t] (an index into
 * blink_schedule_get_stages; tile i of a stage covers the stage's elements in
 * block (off / tile_elems + i) of the payload's tile_elems-element blocks), or
 * tile[t] == -1 for a ticket that stands for nothing (stages shorter than the
 * longest one).  Wavefronts take tickets in ascending order.  Where the order
 * is free (no stage waits for another) the tickets walk tile by tile across the
 * trees (section 4.2.2: trees sharing the machine take turns) unless a stage
 * reads more than 8 ranks (the library may also serve a schedule chunk by chunk
 * where it measured that to be faster, see blink_schedule_set_kernel), calls may
 * go through this list in alternating
 * directions (blink_schedule_set_sweep), and for rank buffers that all start the
 * same distance past a 1 KiB boundary the blocks are counted from that boundary.
 * *n_tickets receives the count; stage and tile (host, caller-allocated, that
 * many entries) may both be null to ask for the count. */
blink_status_t blink_schedule_get_tickets(const blink_schedule_t* s, uint32_t tile_elems, uint64_t* n_tickets,
                                          int32_t* stage, int32_t* tile);
/* out[T+1] (host): share boundaries b_0 = 0 .. b_T = n_elems. */
blink_status_t blink_schedule_get_bounds(const blink_schedule_t* s, uint64_t* out);
/* Bytes the kernel reads plus writes in rank buffers for one call with 4-byte
 * elements, by construction of the stages (no cache effects). */
uint64_t blink_schedule_traffic_bytes(const blink_schedule_t* s);
void blink_schedule_free(blink_schedule_t* s);

/* ---- execution (needs the GPU) -------------------------------------------------- */

/* bufs: HOST array of k DEVICE pointers; each buffer holds at least n_elems
 * 4-byte elements, is 16-byte aligned and overlaps no other.  In place.
 * (Performance only: a wave moves 1 KiB per access and wants it to start on a
 * 1 KiB boundary in memory.  Buffers that all start the same distance past such
 * a boundary (allocations, equal offsets into larger buffers) get that at any
 * distance; buffers that differ in it lose up to a quarter of the throughput
 * when the differences are odd multiples of 16 bytes, a twentieth at multiples
 * of 128.  Some distances between the buffers put equal offsets of all ranks on
 * the same HBM channel; the kernel spreads its accesses so that this costs at
 * most a sixth, on few distances.)
 * The call enqueues one kernel on `stream` (a hipStream_t passed as void*;
 * null = the default stream) and returns without waiting; when the stream
 * reaches the end of that kernel every bufs[i] holds the result:
 *   allreduce: element j of every rank = sum over ranks of element j, added in
 *              the order fixed by the tree that owns j (int32: modulo 2^32);
 *   broadcast: every rank = the root's buffer.
 * k, n_elems and the collective must be those the schedule was made for
 * (BLINK_EMISMATCH otherwise).  With n_elems == 0 the call does nothing and
 * does not look at the entries of bufs (they may be null).  The first call
 * on a schedule also allocates and fills its small device-side tables
 * (synchronously). */
blink_status_t blink_allreduce(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                               blink_schedule_t* s, void* stream);
blink_status_t blink_broadcast(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                               blink_schedule_t* s, void* stream);
/* AllReduce with another operator (blink_allreduce is this with BLINK_SUM), and
 * Reduce: the schedule must have been made for BLINK_OP_REDUCE; on completion
 * the root of each tree holds, on that tree's share, the reduction over all
 * ranks in tree order. */
blink_status_t blink_allreduce_op(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                                  blink_redop_t redop, blink_schedule_t* s, void* stream);
blink_status_t blink_reduce(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                            blink_redop_t redop, blink_schedule_t* s, void* stream);
/* AllGather / Gather; the schedule must have been made for BLINK_OP_ALLGATHER /
 * BLINK_OP_GATHER with the same n_elems (a multiple of k, else
 * blink_make_schedule returns BLINK_EINVAL).  For these two collectives
 * blink_schedule_get_bounds returns the split of one piece (n_elems / k). */
blink_status_t blink_allgather(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                               blink_schedule_t* s, void* stream);
blink_status_t blink_gather(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                            blink_schedule_t* s, void* stream);

/* blink_allreduce for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same result bit for bit; the call itself never allocates or frees
 * device or host memory.  The schedule's device-side tables and progress
 * counters do not go into an allocation of the schedule's own but into a block
 * of fixed size that is part of the library's device image (4 MiB, held by
 * every GPU the library has run on until the process ends).  Limit: the
 * schedule's block, 256 bytes + 312 bytes per stage (blink_schedule_num_stages)
 * + 124 bytes per distinct stage shape + 4 KiB, must fit into it, which allows
 * about 13,000 stages (the per-edge program of 8 ranks x 256 MiB in 1 MiB
 * chunks has 3,584); BLINK_ELIMIT otherwise, and nothing is launched.
 * All calls of this function on one GPU share the block, whichever schedule
 * they use: calls that overlap in time on one GPU race.  Each call clears the
 * counters it needs on `stream` before its kernel.  When the block last held
 * another schedule's tables the call first waits for `stream` and copies its own
 * in synchronously; a capturing stream can record neither, so there the call
 * returns BLINK_EINVAL and records nothing: make one call on the schedule before
 * the capture.  A recorded call starts from cleared counters like any other and
 * may be replayed any number of times, as long as the block still holds its
 * schedule's tables at every replay (no call of this function on another
 * schedule in between: the replay would run on the other's tables).
 * blink_schedule_status reports on
 * the block the latest call of the schedule used.  blink_allreduce and the other
 * entry points are unaffected and may be mixed with this one on one schedule. */
blink_status_t blink_allreduce_noalloc(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                                       blink_schedule_t* s, void* stream);

/* Launch shape override for tuning: waves per compute unit (0 = automatic) and
 * elements per tile, the unit of work a wave draws at a time (0 = automatic;
 * else a power of two in [256, 65536]).  Changing the tile size waits for the
 * device and restarts the schedule's progress counters.  Applies to later
 * calls on this schedule. */
blink_status_t blink_schedule_set_launch(blink_schedule_t* s, int wg_per_cu, int tile_elems);
/* A schedule whose stages do not wait for one another (whole-tree fusion) can
 * be served in up to three ways at streaming sizes; they give the same bits.
 * 1 = the ticket-drawing kernel with loads staged through registers; 2 = the
 * streaming kernel with loads straight into LDS (sums only, stages within its
 * limits); 3 = the ticket-drawing kernel with the trees taking turns chunk by
 * chunk (section 4.2.2 at the paper's own granularity) instead of tile by tile
 * (several trees only).  kernel: 0 = automatic: the first calls of at least
 * 64 MiB of traffic go round the ways the schedule has, four times each (eight
 * or twelve calls), timed with events on the caller's stream; the call after
 * them waits for them, and the fastest way serves from then on
 * (blink_allreduce_noalloc takes no part in the timing and uses way 1);
 * 1, 2, 3 = that way, or way 1 where the schedule does not have it.
 * blink_schedule_last_kernel: the way the latest call ran (0 before the first
 * call). */
blink_status_t blink_schedule_set_kernel(blink_schedule_t* s, int kernel);
int blink_schedule_last_kernel(const blink_schedule_t* s);
/* The order in which a call works through the payload is free where no stage
 * waits for another (whole-tree fusion).  alternate = 1 (the default): the
 * second, fourth, ... call on such a schedule goes through the tiles backwards
 * and results are written with a policy that lets them stay in the GPU's
 * 256 MiB memory-side cache, so a call on the buffers of the call before it
 * (training iterations without much else in between, benchmark loops) starts
 * on data that is still there.  alternate = 0: every call goes forwards and
 * streams its stores past the cache.  Same bits either way; schedules with
 * dependencies and blink_allreduce_noalloc always go forwards. */
blink_status_t blink_schedule_set_sweep(blink_schedule_t* s, int alternate);

/* What became of the calls made on a schedule so far.  In the per-edge and
 * per-node programs a stage waits, chunk by chunk, for the stages it depends on
 * (section 4.1: an event per chunk).  Such a wait is bounded: after the wait
 * limit (default 5 s) the waiting wavefront records what it waited for and
 * leaves the kernel, every other wait of that call then ends as well, the
 * kernel finishes normally, and later calls on the schedule do nothing until
 * blink_schedule_reset.  The rank buffers of an abandoned call hold partial
 * results.  Nothing but a bug (or two calls overlapping on one schedule) makes
 * a wait that long. */
typedef struct {
    int32_t state;          /* 0: every call so far ran to completion; 1: a wait was abandoned */
    int32_t stage;          /* index (blink_schedule_get_stages order) of the stage that gave up; -1 if none */
    int32_t awaited_stage;  /* the stage it waited for; -1 if none */
    int32_t reserved;
    uint64_t seen;          /* finished tiles the awaited stage had counted, over all calls */
    uint64_t wanted;        /* the count it had to reach */
    uint64_t call;          /* number of the call on this schedule (1 = first) */
} blink_progress_t;
/* Waits for the device (hipDeviceSynchronize), then fills *out (host).
 * BLINK_OK if state == 0, BLINK_ESTUCK otherwise. */
blink_status_t blink_schedule_status(blink_schedule_t* s, blink_progress_t* out);
/* Waits for the device, then clears the progress counters and the status
 * record: the schedule is as after blink_make_schedule (launch overrides are
 * kept). */
blink_status_t blink_schedule_reset(blink_schedule_t* s);
/* Wait limit in microseconds for later calls (0 = the default). */
blink_status_t blink_schedule_set_wait_limit(blink_schedule_t* s, uint64_t microseconds);
/* For tests of the give-up path only: counts one call as made without
 * launching it.  The stages of the next call then wait for progress that never
 * comes, the waits run into the limit, and the call ends as described above. */
blink_status_t blink_schedule_test_skip_call(blink_schedule_t* s);

/* ---- chunk-size selection across iterations (host only) ---------------------- */

/* Multiplicative-increase, additive-decrease search for the chunk size (paper
 * section 4.2.1): start at initial_chunk; multiply by factor (> 1) from one
 * iteration to the next while the reported throughput rises by more than
 * rel_tol (>= 0, relative); at the first measurement that does not, subtract
 * step (>= 1) per iteration while that still raises the throughput; then stay
 * at the best chunk measured.  Chunks are kept inside [lo, hi] (elements, lo >=
 * 1).  Usage per iteration: make a schedule with blink_miad_chunk(), run and
 * time the collective, blink_miad_report(throughput, any unit); stop tuning
 * once blink_miad_steady() is non-zero (further reports change nothing). */
typedef struct blink_miad blink_miad_t;
blink_status_t blink_miad_create(size_t initial_chunk, double factor, size_t step, size_t lo,
                                 size_t hi, double rel_tol, blink_miad_t** out);
size_t blink_miad_chunk(const blink_miad_t* m);   /* chunk for the next iteration; 0 for a null handle */
int blink_miad_steady(const blink_miad_t* m);     /* 1 once the search has ended */
blink_status_t blink_miad_report(blink_miad_t* m, double throughput);
void blink_miad_free(blink_miad_t* m);

const char* blink_strerror(blink_status_t st);

#ifdef __cplusplus
}
#endif
#endif /* BLINK_H */
