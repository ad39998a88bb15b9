// The device side: one persistent gfx950 kernel that consumes the stage list of
// all trees concurrently (paper sections 3.3, 4.1, 4.2.1, 4.2.2).  The kernel is a
// template; kernel_{f32,i32}_{many,stream}.hip instantiate it for the two element
// types and the two column budgets (four translation units, so that they compile
// side by side), exec.hip holds the launcher.
//
// A workgroup is ONE 64-lane wavefront: nothing in the kernel needs a
// workgroup barrier, and a wave that waits for a dependency holds up nobody
// else.  Work unit: (stage instance, tile).  Waves draw units from ticket
// counters in the schedule's execution order, so every unit a wave might have
// to wait for has already been drawn by a running wave, or is about to be (see
// the kernel's loop): waiting can never deadlock, whatever the grid size.
//
// A tile (256..65536 elements, chosen per schedule) is cut into sub-tiles; a
// sub-tile of a stage is processed in three phases by the 64 lanes, each owning
// U 128-bit columns, where U is as large as the stage allows under a budget of
// 32 columns in registers and LDS (a stage that reads 8 ranks gets U = 4, a
// plain copy the maximum, 16), so that every wave keeps up to 32 KiB of loads
// in flight whatever the stage looks like (16 columns for small payloads):
//   1. load the sub-tile from every rank the stage reads; all loads are issued
//      before the first is consumed, then parked in per-lane LDS slots;
//   2. run the stage's micro-program (acc = slot / acc += slot / slot = acc)
//      over the slots: this is where the tree's summation order is applied,
//      with partial sums staged in LDS instead of going back to HBM;
//   3. store acc to every rank the stage writes.
// LDS slots are private to a lane (lane l only touches column l).
//
// Chunk-granular hand-over (the paper's per-chunk event): a stage instance has
// a 64-bit counter of finished tiles.  Counters are never reset; call number e
// on a schedule waits for e * tiles.  Data handed from stage to stage travels
// with system-scope cache policy (see blink_consume), the counters with
// agent-scope atomics.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstddef>
#include <cstdio>
#include <type_traits>
#include <vector>

#include "schedule.hpp"
#include "state.hpp"

namespace blink {

constexpr int kLanes = 64;        // one wavefront per workgroup
// 128-bit columns a lane holds in registers (and LDS slots) at once = ranks
// read x U: 32 (32 KiB of LDS per wave) for payloads large enough to stream,
// which run fastest with few waves that each keep many bytes in flight
// (measured on 8 x 256 MiB, against 16 columns and one more wave per CU:
// whole-tree stages 0.690 -> 0.680 ms, per-node stages 1.35 -> 1.19 ms,
// per-edge stages 1.52 -> 1.41 ms); 16 where every wave that fits is wanted
// (small payloads).
constexpr int kColumnsMany = 16;
constexpr int kColumnsStream = 32;
constexpr unsigned kMinTile = kLanes * 4;   // elements: one column per lane
constexpr unsigned kMaxTile = 65536;        // elements
// One ticket counter sustains roughly 80 draws per microsecond.  A ticket of a
// dependency-free schedule, which draws from one counter, should therefore move
// about this many bytes (6 TB/s are then 47 draws per microsecond).
constexpr unsigned kTicketBytes = 128 * 1024;
// Progress counters sit 256 bytes apart: the few counters that are hot at any
// moment then live in different cache lines and memory channels, so thousands
// of polling waves do not pile up on one of them.
constexpr int kCounterStride = 32;  // in 8-byte words
// Tickets can be dealt from several counters ("queues"), ticket t from queue
// t mod n: one counter sustains ~83 fetch-adds per microsecond however many
// waves ask, n counters in different memory channels n times that (measured:
// 540 per microsecond with 8, 1040 with 16).  Schedules whose stages wait for
// one another use 4 queues and half-size tickets (per-edge AllReduce on
// 8 x 256 MiB: 1.336 -> 1.277 ms, per-node 1.169 -> 1.125 ms).  Dependency-free
// streaming keeps ONE queue: there the single counter is no bottleneck at
// kTicketBytes per ticket, and strictly ordered tickets are as fast as anything
// tried with more queues and smaller tiles (0.6826 vs 0.6824 ms).
constexpr int kMaxQueues = 16;
constexpr unsigned kQueuesHandOver = 4;
constexpr unsigned kTicketBytesHandOver = 64 * 1024;
// The status record at the head of a schedule's device block, 64-bit words.
// Word kStatusState is 0 while all is well.  A wave whose wait for another stage
// outlasts the limit makes it 1 (the first such wave wins), fills in the other
// words and leaves; from then on every wave that looks leaves too, and every
// later launch on the block returns at once, until the host clears the record.
enum : int {
    kStatusState = 0,    // 0 = ok, 1 = a wait was abandoned
    kStatusStage = 1,    // the stage instance that waited
    kStatusAwaited = 2,  // the instance it waited for
    kStatusSeen = 3,     // finished tiles that instance had counted
    kStatusWanted = 4,   // finished tiles it had to reach
    kStatusCall = 5,     // number of the call on its schedule
    kStatusWords = 32,   // the record takes one 256-byte line of its own
};
// The steady counter the waits are timed with ticks at 100 MHz.
constexpr unsigned long long kTicksPerMicrosecond = 100;
constexpr unsigned long long kDefaultWaitMicroseconds = 5000000;  // 5 s: generous; only a bug waits that long

struct KParams {
    void* buf[BLINK_MAX_RANKS];
    const StageTmpl* tmpl;
    const StageInst* inst;
    unsigned long long* done;
    unsigned long long* ticket;
    unsigned long long* status;          // the status record (kStatus* words)
    unsigned long long wait_ticks;       // longest wait for another stage, in ticks of the steady counter
    unsigned long long ticket_base[kMaxQueues];  // value of each queue's counter when this call starts
    unsigned n_queues;
    unsigned long long n_items;
    unsigned long long static_items;  // tickets below this are dealt round-robin, without the counter
    unsigned long long epoch;
    unsigned tiles_per_chunk;
    unsigned tile_shift;  // a tile is 2^tile_shift elements
    unsigned redop;       // blink_redop_t
    unsigned group;  // consecutive instances whose tiles are handed out in turn (1 = instance by instance)
    unsigned max_naps;  // longest pause between two looks at a dependency, in units of ~0.2 us
    unsigned reverse;   // tickets walk the tiles from the last to the first (schedules without dependencies only)
    unsigned grid_shift;  // elements by which the tile grid is moved down (schedules without dependencies only)
    unsigned n_inst;      // stage instances (n_items is less than n_inst * tiles_per_chunk where the last group has fewer tiles)
};

// Address spaces: the kernel arguments and the schedule tables are never
// written by the kernel, so they are read through the constant address space,
// which lets wave-uniform reads use the scalar unit.
#define BLINK_CONST __attribute__((address_space(4)))
using ConstParams = const BLINK_CONST KParams*;
using ConstTmpl = const BLINK_CONST StageTmpl*;
using ConstInst = const BLINK_CONST StageInst*;

typedef float F4 __attribute__((ext_vector_type(4)));
typedef unsigned U4 __attribute__((ext_vector_type(4)));  // one 128-bit access, as raw bits

// Element-wise a (+) b on raw bits; `op` is wave-uniform.  fp32 SUM / PROD: one
// IEEE operation per element (round to nearest even, subnormals kept).  int32
// SUM / PROD: unsigned arithmetic, i.e. wrap-around modulo 2^32 without
// signed-overflow UB.  MIN / MAX: signed comparison for int32; for fp32 the
// bits are mapped to keys whose signed order is the IEEE total order (-0 below
// +0; the map is its own inverse), so min and max commute bit for bit.
template <typename T>
__device__ __forceinline__ unsigned combine1(unsigned op, unsigned a, unsigned b);
template <>
__device__ __forceinline__ unsigned combine1<float>(unsigned op, unsigned a, unsigned b) {
    if (op == BLINK_SUM)
        return __builtin_bit_cast(unsigned, __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b));
    if (op == BLINK_PROD)
        return __builtin_bit_cast(unsigned, __builtin_bit_cast(float, a) * __builtin_bit_cast(float, b));
    const int ka = static_cast<int>(a) ^ ((static_cast<int>(a) >> 31) & 0x7fffffff);
    const int kb = static_cast<int>(b) ^ ((static_cast<int>(b) >> 31) & 0x7fffffff);
    const int k = op == BLINK_MIN ? min(ka, kb) : max(ka, kb);
    return static_cast<unsigned>(k ^ ((k >> 31) & 0x7fffffff));
}
template <>
__device__ __forceinline__ unsigned combine1<unsigned>(unsigned op, unsigned a, unsigned b) {
    if (op == BLINK_SUM) return a + b;
    if (op == BLINK_PROD) return a * b;
    const int sa = static_cast<int>(a), sb = static_cast<int>(b);
    return static_cast<unsigned>(op == BLINK_MIN ? min(sa, sb) : max(sa, sb));
}
template <typename T>
__device__ __forceinline__ U4 combine4(unsigned op, U4 a, U4 b) {
    if (op == BLINK_SUM) {  // the common case, kept free of per-element selects
        if constexpr (std::is_same<T, float>::value)
            return __builtin_bit_cast(U4, __builtin_bit_cast(F4, a) + __builtin_bit_cast(F4, b));
        else
            return a + b;
    }
    U4 r;
    r.x = combine1<T>(op, a.x, b.x);
    r.y = combine1<T>(op, a.y, b.y);
    r.z = combine1<T>(op, a.z, b.z);
    r.w = combine1<T>(op, a.w, b.w);
    return r;
}

// Byte `field_offset + i` of a stage template, fetched as part of a 32-bit word
// so that the scalar unit can do it.
__device__ __forceinline__ unsigned tmpl_byte(ConstTmpl st, unsigned byte_index) {
    const BLINK_CONST uint32_t* w = reinterpret_cast<const BLINK_CONST uint32_t*>(st);
    return (w[byte_index >> 2] >> ((byte_index & 3u) * 8u)) & 0xffu;
}
#define BLINK_TMPL(st, field, i) tmpl_byte(st, static_cast<unsigned>(offsetof(StageTmpl, field)) + (i))

// Rank buffers are accessed through buffer descriptors that cover exactly the
// bytes still to be processed: lanes past the end read zeros and their stores
// are dropped by the hardware range check, so ragged ends need no branches.
// The cache-policy bits of each access are chosen per kernel flavour (below).
constexpr int kRawDword3 = 0x00020000;  // raw 32-bit data format, no swizzle (gfx9 family)
constexpr int kPolicyDefault = 0;
constexpr int kPolicyStream = 2;        // nt: streamed once, do not keep in cache
constexpr int kPolicyThrough = 16;      // sc1: agent scope, stores written through
constexpr int kPolicySystem = 17;       // sc0 sc1: bypass / write through every cache level

// Kernel flavours: the cache policy of rank-buffer loads and stores.
enum Flavour : int {
    kHandOver = 0,    // stages hand chunks over to one another (see blink_consume)
    kBalanced = 1,    // streaming, about as many bytes read as written
    kWriteHeavy = 2,  // streaming, at least twice as many bytes written as read
    kReadHeavy = 3,   // streaming, at least twice as many bytes read as written
};
// Measured on 8 x 256 MiB, fp32 (load policy, store policy -> ms):
//   AllReduce  (nt, nt) 0.676  (nt, nt sc1) 0.668  (default, nt sc1) 0.688  (nt, sc1) 0.676
//   Reduce     (nt, nt) 0.411  (nt, sc1) 0.383     (default, any) 0.44-0.46
//   Broadcast  (nt, nt) 0.383  (default, nt sc1) 0.297  (default, nt) 0.304
//   per-edge AllReduce  (sc0 sc1, sc0 sc1) 1.417  (sc0 sc1 nt, sc0 sc1) 1.337  nt on stores 1.65-1.72
template <int FLAVOUR>
struct Policy {
    static constexpr int kLoad = FLAVOUR == kHandOver ? (kPolicySystem | kPolicyStream)
                                 : (FLAVOUR == kWriteHeavy ? kPolicyDefault : kPolicyStream);
    static constexpr int kStore = FLAVOUR == kHandOver     ? kPolicySystem
                                  : FLAVOUR == kWriteHeavy ? (kPolicyStream | kPolicyThrough)
                                  : FLAVOUR == kReadHeavy  ? kPolicyThrough
                                                           : kPolicyStream;
};

// The rank buffers' addresses live in a vector register pair, lane r holding rank
// r's (loaded once per wave): a rank's pointer is then one readlane away instead
// of a scalar load that depends on another scalar load (the rank's number from
// the stage's table), twice per rank and sub-tile.
struct RankTable {
    unsigned lo, hi;
};
__device__ __forceinline__ RankTable load_rank_table(ConstParams p, int lane) {
    const unsigned long long mine = reinterpret_cast<unsigned long long>(p->buf[lane & (BLINK_MAX_RANKS - 1)]);
    return {static_cast<unsigned>(mine), static_cast<unsigned>(mine >> 32)};
}
__device__ __forceinline__ unsigned long long rank_base(RankTable t, unsigned rank) {
    const unsigned lo = __builtin_amdgcn_readlane(t.lo, rank);
    const unsigned hi = __builtin_amdgcn_readlane(t.hi, rank);
    return (static_cast<unsigned long long>(hi) << 32) | lo;
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rank_window(RankTable t, unsigned rank,
                                                              unsigned long long byte_off, unsigned bytes) {
    char* base = reinterpret_cast<char*>(rank_base(t, rank) + byte_off);
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, static_cast<int>(bytes), kRawDword3);
}

// The micro-program of a stage over the LDS slots of one sub-tile, U columns per
// lane.  All LDS reads of an operation are issued before the first is used, and
// the sum, by far the most common operator, has a loop of its own: with the
// operator dispatched per column inside one loop the compiler emitted a chain
// of branches and a full wait after every single column read.
// The operations come off a shift register that holds the whole program
// (fetched with two wide scalar loads per tile), not from memory one by one.
template <typename T, int U, bool SUM>
__device__ __forceinline__ void run_program(U4* __restrict__ slots, const unsigned long long (&prog)[5], int n_op,
                                            unsigned redop, int lane, U4 (&acc)[U]) {
    unsigned long long q0 = prog[0], q1 = prog[1], q2 = prog[2], q3 = prog[3], q4 = prog[4];
    for (int o = 0; o < n_op; ++o) {
        const unsigned code = static_cast<unsigned>(q0) & 0xffu;
        q0 = (q0 >> 8) | (q1 << 56);
        q1 = (q1 >> 8) | (q2 << 56);
        q2 = (q2 >> 8) | (q3 << 56);
        q3 = (q3 >> 8) | (q4 << 56);
        q4 >>= 8;
        U4* sl = slots + (code & 63u) * (U * kLanes) + lane;
        const unsigned kind = code >> 6;
        if (kind == OP_ST) {
#pragma unroll
            for (int u = 0; u < U; ++u) sl[u * kLanes] = acc[u];
            continue;
        }
        U4 in[U];
#pragma unroll
        for (int u = 0; u < U; ++u) in[u] = sl[u * kLanes];
        if (kind == OP_LD) {
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] = in[u];
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (!SUM)
                    acc[u] = combine4<T>(redop, acc[u], in[u]);
                else if constexpr (std::is_same<T, float>::value)
                    acc[u] = __builtin_bit_cast(U4, __builtin_bit_cast(F4, acc[u]) + __builtin_bit_cast(F4, in[u]));
                else
                    acc[u] = acc[u] + in[u];
            }
        }
    }
}

// Phases 1-3 over `bytes` bytes (a multiple of 16) at byte_off for a stage that
// reads N ranks, U columns per lane and sub-tile.
//
// The U columns of a sub-tile are not neighbours: with n sub-tiles to the tile,
// sub-tile s takes columns s, s + n, s + 2n, ... (a column is one 16-byte access
// per lane, 1 KiB).  All ranks are read at the same offsets at the same time,
// and rank buffers an unlucky distance apart put equal offsets of all of them
// on the same memory channel: neighbouring columns then make one burst of
// N * U KiB into a single channel, spread columns several smaller ones into
// different channels (measured with a standalone probe, 6 ranks x 128 MiB,
// buffers 4 KiB or 68 KiB more than their size apart: 0.68 -> 0.80 of the HBM
// peak; 5 ranks: 0.72 -> 0.78; buffers exactly their size apart: 0.80 -> 0.79).
// Columns past the end of a ragged tile fall outside the window: such loads
// return zeros and such stores are dropped.
template <typename T, int N, int U, int LD, int ST>
__device__ __forceinline__ void run_vec(U4* __restrict__ slots, ConstParams p, RankTable ranks, ConstTmpl st,
                                        unsigned long long byte_off, unsigned bytes, int lane) {
    constexpr unsigned kSubBytes = kLanes * U * 16;
    const unsigned redop = p->redop;
    const int n_op = BLINK_TMPL(st, n_op, 0);
    const int n_store = BLINK_TMPL(st, n_store, 0);
    const BLINK_CONST uint32_t* w = reinterpret_cast<const BLINK_CONST uint32_t*>(st);
    constexpr unsigned kOpWord = offsetof(StageTmpl, op) / 4;
    static_assert(offsetof(StageTmpl, op) % 8 == 0 && kMaxOps == 40, "the micro-program is fetched as five 64-bit words");
    unsigned long long prog[5];
#pragma unroll
    for (int q = 0; q < 5; ++q)
        prog[q] = static_cast<unsigned long long>(w[kOpWord + 2 * q]) |
                  (static_cast<unsigned long long>(w[kOpWord + 2 * q + 1]) << 32);
    const unsigned n_sub = (bytes + kSubBytes - 1) / kSubBytes;
    for (unsigned sub = 0; sub < n_sub; ++sub) {
        // phase 1: issue every load, then park the values in LDS
        U4 r[N][U];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const __amdgpu_buffer_rsrc_t win = rank_window(ranks, BLINK_TMPL(st, load_rank, i), byte_off, bytes);
#pragma unroll
            for (int u = 0; u < U; ++u)
                r[i][u] = __builtin_amdgcn_raw_buffer_load_b128(win, ((u * n_sub + sub) * kLanes + lane) * 16, 0, LD);
        }
#pragma unroll
        for (int i = 0; i < N; ++i)
#pragma unroll
            for (int u = 0; u < U; ++u) slots[(i * U + u) * kLanes + lane] = r[i][u];
        // phase 2: the stage's micro-program
        U4 acc[U];
        if (redop == BLINK_SUM)
            run_program<T, U, true>(slots, prog, n_op, redop, lane, acc);
        else
            run_program<T, U, false>(slots, prog, n_op, redop, lane, acc);
        // phase 3: stores
        for (int j = 0; j < n_store; ++j) {
            const __amdgpu_buffer_rsrc_t win = rank_window(ranks, BLINK_TMPL(st, store_rank, j), byte_off, bytes);
#pragma unroll
            for (int u = 0; u < U; ++u)
                __builtin_amdgcn_raw_buffer_store_b128(acc[u], win, ((u * n_sub + sub) * kLanes + lane) * 16, 0, ST);
        }
    }
}

// Pick U for a stage that reads N ranks: the largest power of two (at most 16)
// with N * U <= COLS that does not exceed the tile (cols = tile columns per lane).
template <typename T, int N, int COLS, int LD, int ST>
__device__ __forceinline__ void run_vec_n(U4* __restrict__ slots, ConstParams p, RankTable ranks, ConstTmpl st,
                                          unsigned long long byte_off, unsigned bytes, unsigned cols, int lane) {
    constexpr int kFit = COLS / N;
    constexpr int kBudget = kFit >= 16 ? 16 : (kFit >= 8 ? 8 : (kFit >= 4 ? 4 : (kFit >= 2 ? 2 : 1)));
    if constexpr (kBudget >= 16)
        if (cols >= 16) return run_vec<T, N, 16, LD, ST>(slots, p, ranks, st, byte_off, bytes, lane);
    if constexpr (kBudget >= 8)
        if (cols >= 8) return run_vec<T, N, 8, LD, ST>(slots, p, ranks, st, byte_off, bytes, lane);
    if constexpr (kBudget >= 4)
        if (cols >= 4) return run_vec<T, N, 4, LD, ST>(slots, p, ranks, st, byte_off, bytes, lane);
    if constexpr (kBudget >= 2)
        if (cols >= 2) return run_vec<T, N, 2, LD, ST>(slots, p, ranks, st, byte_off, bytes, lane);
    run_vec<T, N, 1, LD, ST>(slots, p, ranks, st, byte_off, bytes, lane);
}

template <typename T, int COLS, int LD, int ST>
__device__ __forceinline__ void run_vec_any(U4* __restrict__ slots, ConstParams p, RankTable ranks, ConstTmpl st,
                                            unsigned long long byte_off, unsigned bytes, unsigned cols, int lane) {
    switch (BLINK_TMPL(st, n_load, 0)) {
#define BLINK_CASE(N) case N: run_vec_n<T, N, COLS, LD, ST>(slots, p, ranks, st, byte_off, bytes, cols, lane); break;
        BLINK_CASE(1) BLINK_CASE(2) BLINK_CASE(3) BLINK_CASE(4) BLINK_CASE(5) BLINK_CASE(6)
        BLINK_CASE(7) BLINK_CASE(8) BLINK_CASE(9) BLINK_CASE(10) BLINK_CASE(11) BLINK_CASE(12)
        BLINK_CASE(13) BLINK_CASE(14) BLINK_CASE(15) BLINK_CASE(16)
#undef BLINK_CASE
        default: break;
    }
}

// The same for up to kLanes single 4-byte elements: the ragged end of a payload
// whose length is not a multiple of 4 elements, and chunks that do not start on
// a 16-byte boundary.  Slow path; one element per lane.
template <typename T, int LD, int ST>
__device__ __forceinline__ void run_scalar(unsigned* __restrict__ slots, ConstParams p, RankTable ranks, ConstTmpl st,
                                           unsigned long long byte_off, unsigned bytes, int lane) {
    const int n_load = BLINK_TMPL(st, n_load, 0);
    for (int i = 0; i < n_load; ++i) {
        const __amdgpu_buffer_rsrc_t win = rank_window(ranks, BLINK_TMPL(st, load_rank, i), byte_off, bytes);
        slots[i * kLanes + lane] = __builtin_amdgcn_raw_buffer_load_b32(win, lane * 4, 0, LD);
    }
    unsigned acc = 0;
    const unsigned redop = p->redop;
    const int n_op = BLINK_TMPL(st, n_op, 0);
    for (int o = 0; o < n_op; ++o) {
        const unsigned code = BLINK_TMPL(st, op, o);
        unsigned* sl = slots + (code & 63u) * kLanes + lane;
        const unsigned kind = code >> 6;
        if (kind == OP_LD)
            acc = *sl;
        else if (kind == OP_ADD)
            acc = combine1<T>(redop, acc, *sl);
        else
            *sl = acc;
    }
    const int n_store = BLINK_TMPL(st, n_store, 0);
    for (int j = 0; j < n_store; ++j) {
        const __amdgpu_buffer_rsrc_t win = rank_window(ranks, BLINK_TMPL(st, store_rank, j), byte_off, bytes);
        __builtin_amdgcn_raw_buffer_store_b32(acc, win, lane * 4, 0, ST);
    }
}

// T: element type (float, or unsigned for wrap-around int32).  FLAVOUR selects
// how data is exchanged between stages:
//   streaming flavours: the schedule has no stage that waits for another (TREE
//          fusion): streaming accesses with the policy measured best for the
//          schedule's mix of reads and writes, no fences;
//   kHandOver: stages hand chunks over to each other, possibly across XCDs whose
//          L2 caches are not coherent with one another: all rank-buffer accesses
//          use system-scope cache policy (loads bypass, stores write through;
//          the loads also carry the streaming hint, which changes no scope),
//          so the hand-over needs no L2 write-back or invalidate, only "my
//          stores have completed" before the counter is bumped.
// COLS: the column budget (LDS slots per lane).
// The kernel takes all 256 vector registers and 96 accumulation registers, so
// one wave per SIMD fits (4 per CU).  The 16-column variant, for payloads too
// small to keep the memory system busy with that, is held to half the register
// file (the second launch bound: two waves per SIMD; about 160 registers then
// live in per-lane scratch memory): twice the waves hide more latency than the
// spills cost (8 ranks x 4 trees, 1 M elements per rank 17.9 -> 15.4 us, 4.2 M
// 52.0 -> 45.7 us); three per SIMD lose again (4.2 M: 52.1 us), and where
// stages wait for one another the spills cost more than the waves bring.
// The by-value argument is only there to size the kernel-argument segment; it is
// read through the constant address space (see ConstParams).
template <typename T, int FLAVOUR, int COLS>
__global__ __launch_bounds__(kLanes, COLS == kColumnsMany && FLAVOUR != kHandOver ? 2 : 1) void blink_consume(
    const KParams) {
    __shared__ U4 slots[COLS * kLanes];  // 16 or 32 KiB: COLS columns per lane
    constexpr int LD = Policy<FLAVOUR>::kLoad;
    constexpr int ST = Policy<FLAVOUR>::kStore;
    const int lane = threadIdx.x;
    ConstParams p = (ConstParams)__builtin_amdgcn_kernarg_segment_ptr();
    const RankTable ranks = load_rank_table(p, lane);
    unsigned long long* const ticket = p->ticket;
    unsigned long long* const done = p->done;
    ConstTmpl const tmpl = reinterpret_cast<ConstTmpl>(reinterpret_cast<unsigned long long>(p->tmpl));
    ConstInst const inst = reinterpret_cast<ConstInst>(reinterpret_cast<unsigned long long>(p->inst));
    const unsigned long long n_items = p->n_items, epoch = p->epoch;
    const unsigned n_queues = p->n_queues;
    const unsigned tiles_per_chunk = p->tiles_per_chunk;
    const unsigned tile_shift = p->tile_shift;
    const unsigned tile_elems = 1u << tile_shift;
    const unsigned cols = min(tile_elems / kMinTile, static_cast<unsigned>(COLS));
    const unsigned group = p->group;
    const unsigned long long grid_shift = p->grid_shift;
    const unsigned n_inst = p->n_inst;

    // Lane-dependent regions.  readfirstlane needs lane 0 present, so the
    // compiler must never get the chance to let some lanes run ahead of lane 0
    // around the loop: a version with a lane-0 region at the tail of the loop
    // (completion signal) and one at its head (ticket draw) had the two merged
    // across the back edge and hung.  Hence the completion signal of a tile is
    // posted together with the next ticket draw, in ONE lane-0 region at the
    // head, and the back edges are wave-uniform.  The only other lane-dependent
    // region is the wait for dependencies in the middle of the body (lanes
    // below n_dep poll one counter each).  It cannot be merged with the region
    // at the head in either direction: between the two, on both sides, lies
    // wave-uniform code with effects of its own (the readfirstlane pair and the
    // ticket arithmetic after the head; the tile's loads and stores after the
    // wait), and the wait ends in a ballot over all lanes, which the lanes can
    // only reach together.  All other branches are wave-uniform.
    //
    // Small schedules without dependencies are dealt round-robin instead (wave w
    // takes tickets w, w + grid, ...; static_items == n_items): even several
    // counters are too slow when thousands of waves each want one small tile.
    //
    // Drawn tickets: ticket static_items + j * n_queues + q is the j-th of queue
    // q.  A wave starts on queue (its number mod n_queues), stays with it until
    // it is empty and then goes round the others, so every wave draws exactly
    // one ticket past the end of every queue.  The grid has at least n_queues
    // waves, so each queue has waves of its own; with dependencies this keeps
    // the schedule free of deadlock: take the first unfinished ticket t in
    // schedule order.  Everything it waits for is finished.  If t is drawn its
    // holder runs; if not, its queue is not empty, the queue's own waves hold
    // only earlier tickets of that queue, which are finished, so one of them
    // draws t next.
    //
    // A block whose status record is set (an earlier call gave up a wait, so its
    // counters no longer mean anything) is left alone.
    unsigned long long* const status = p->status;
    if (__hip_atomic_load(status + kStatusState, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    const unsigned long long static_items = p->static_items;
    unsigned long long next_static = blockIdx.x;
    unsigned queue = blockIdx.x % n_queues, empty_queues = 0;
    long long pending = -1;  // instance whose finished tile still has to be counted
    for (;;) {
        unsigned long long t;
        if (next_static < static_items) {
            t = next_static;
            next_static += gridDim.x;
        } else {
            if (static_items == n_items) break;  // fully dealt out: nothing left to draw
            unsigned long long raw = 0;
            if (lane == 0) {
                if (pending >= 0)
                    __hip_atomic_fetch_add(done + pending * kCounterStride, 1ull, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                raw = __hip_atomic_fetch_add(ticket + queue * kCounterStride, 1ull, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
            }
            pending = -1;
            const unsigned lo = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(raw));
            const unsigned hi = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(raw >> 32));
            const unsigned long long nth = ((static_cast<unsigned long long>(hi) << 32) | lo) - p->ticket_base[queue];
            t = static_items + nth * n_queues + queue;
            if (t >= n_items) {  // this queue is empty: on to the next, or done
                if (++empty_queues == n_queues) break;
                queue = queue + 1 == n_queues ? 0 : queue + 1;
                continue;
            }
        }
        if (t >= n_items) break;
        // Every other call on a schedule whose stages do not wait for one
        // another walks the tiles backwards: it starts where the call before it
        // ended, on what that call left in the memory-side cache.
        if (p->reverse) t = n_items - 1 - t;
        // ticket -> (instance, tile).  Within a group of `group` consecutive
        // instances (the trees' turns at one chunk position) tickets walk tile
        // by tile across the instances, so neighbouring waves work on all trees
        // at once (section 4.2.2); group == 1 keeps an instance's tiles together.
        unsigned ii, tile;
        ticket_to_tile(t, group, tiles_per_chunk, n_inst, &ii, &tile);
        ConstInst in = inst + ii;
        // Tiles lie on the absolute grid of tile_elems-element blocks of the
        // payload, so tile starts are 128-byte (indeed tile-size) aligned even
        // when a tree's share starts at an odd multiple of 16 bytes; the first
        // and last tile of an instance are the ragged ones.  Where the rank
        // buffers themselves all start the same distance past a 1 KiB boundary
        // the launcher moves the grid down by that distance (grid_shift
        // elements): tiles then start on such boundaries in memory, which is
        // what the 1 KiB accesses of a wave want (buffers 16 bytes past one:
        // 0.61 of the HBM peak against 0.77, 512 bytes: 0.77 against 0.81).
        const unsigned long long off = in->off, end = off + in->len;
        const unsigned long long block = ((off + grid_shift) >> tile_shift) + tile;
        const unsigned long long block_lo = block << tile_shift;  // on the moved grid
        const unsigned long long lo_e = block_lo > grid_shift ? max(off, block_lo - grid_shift) : off;
        const unsigned long long hi_e = min(end, block_lo + tile_elems - grid_shift);
        if (lo_e < hi_e) {  // instances have at most tiles_per_chunk tiles, some fewer
            const unsigned tlen = static_cast<unsigned>(hi_e - lo_e);
            ConstTmpl st = tmpl + in->tmpl;

            const int n_dep = in->n_dep;
            if (n_dep) {
                bool gave_up = false;
                if (lane < n_dep) {
                    const unsigned long long want =
                        epoch * (((end + tile_elems - 1) >> tile_shift) - (off >> tile_shift));
                    const unsigned long long* f = done + static_cast<long long>(in->dep[lane]) * kCounterStride;
                    // poll, backing off (up to ~0.8 us between looks for large
                    // schedules) so that waiting waves leave the memory system
                    // to the working ones.  Every 64th look also checks the
                    // clock and the status record: a wait that outlasts the
                    // limit, or any wait once another wave has given up, ends
                    // here, and the wave leaves the kernel.
                    const unsigned max_naps = p->max_naps;
                    unsigned naps = 1, looks = 0;
                    unsigned long long since = 0, seen;
                    while ((seen = __hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) < want) {
                        for (unsigned i = 0; i < naps; ++i) __builtin_amdgcn_s_sleep(8);
                        if (naps < max_naps) naps *= 2;
                        if ((++looks & 63u) != 0) continue;
                        const unsigned long long now = wall_clock64();
                        if (since == 0) since = now;
                        const bool late = now - since > p->wait_ticks;
                        if (late && __hip_atomic_exchange(status + kStatusState, 1ull, __ATOMIC_RELAXED,
                                                          __HIP_MEMORY_SCOPE_AGENT) == 0) {
                            status[kStatusStage] = ii;
                            status[kStatusAwaited] = static_cast<unsigned long long>(in->dep[lane]);
                            status[kStatusSeen] = seen;
                            status[kStatusWanted] = want;
                            status[kStatusCall] = epoch;
                        }
                        if (late || __hip_atomic_load(status + kStatusState, __ATOMIC_RELAXED,
                                                      __HIP_MEMORY_SCOPE_AGENT) != 0) {
                            gave_up = true;
                            break;
                        }
                    }
                }
                if (__builtin_amdgcn_ballot_w64(gave_up) != 0) break;  // wave-uniform: leave the kernel
                // orders the polls before the data loads; the loads themselves bypass the caches
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            }

            const unsigned long long e0 = lo_e;  // first element of the tile
            if ((e0 & 3ull) == 0) {
                const unsigned vec_bytes = (tlen >> 2) * 16u;
                if (vec_bytes) run_vec_any<T, COLS, LD, ST>(slots, p, ranks, st, e0 * 4ull, vec_bytes, cols, lane);
                const unsigned rem = tlen & 3u;  // only where the payload itself ends off a 16-byte boundary
                if (rem)
                    run_scalar<T, LD, ST>(reinterpret_cast<unsigned*>(slots), p, ranks, st, e0 * 4ull + vec_bytes,
                                          rem * 4u, lane);
            } else {
                // chunk size not a multiple of 4 elements: element-wise, slow but correct
                for (unsigned b = 0; b < tlen * 4u; b += kLanes * 4u)
                    run_scalar<T, LD, ST>(reinterpret_cast<unsigned*>(slots), p, ranks, st, e0 * 4ull + b,
                                          min(static_cast<unsigned>(kLanes) * 4u, tlen * 4u - b), lane);
            }

            if (BLINK_TMPL(st, signals, 0)) {
                // every store of this wave has reached memory before the counter moves
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_s_waitcnt(0);
                pending = ii;
            }
        }
    }
}

// ---- what the launcher sees ---------------------------------------------------------
using KernelFn = void (*)(const KParams);

template <typename T, int COLS>
KernelFn pick_kernel_of(int flavour) {
    switch (flavour) {
        case kHandOver: return blink_consume<T, kHandOver, COLS>;
        case kWriteHeavy: return blink_consume<T, kWriteHeavy, COLS>;
        case kReadHeavy: return blink_consume<T, kReadHeavy, COLS>;
        default: return blink_consume<T, kBalanced, COLS>;
    }
}

// The kernel for a flavour, per element type (float; wrap-around int32 added as
// unsigned) and column budget (many: kColumnsMany, stream: kColumnsStream).
// Each is defined in a translation unit of its own, so that the four compile
// side by side.
KernelFn kernel_f32_many(int flavour);
KernelFn kernel_f32_stream(int flavour, bool direct);
KernelFn kernel_i32_many(int flavour);
KernelFn kernel_i32_stream(int flavour, bool direct);

}  // namespace blink
