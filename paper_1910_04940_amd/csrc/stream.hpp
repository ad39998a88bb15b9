// The streaming kernel: the sum over schedules in which no stage waits for
// another (whole-tree fusion; paper sections 3.3, 4.1, 4.2.2), at payloads large
// enough to be bound by HBM.  Same work units, tickets and tile grid as
// blink_consume (kernel.hpp), which can run the same schedules; the launcher
// times both on a schedule's first calls and keeps the faster (exec.hip).
// blink_consume wins on most placements of the caller's buffers (8 ranks x
// 256 MiB: 6.05 against 5.65 TB/s); this kernel is the steadier one: where
// blink_consume drops to 4.4 TB/s (same shape at 2^25 elements with the ranks
// 68 KiB off a power of two apart) it still does 5.65.  How a wave works here:
//
//   * Two waves per compute unit, each with 64 KiB of loads in flight.  Loads
//     go from HBM straight into the wave's LDS slots (buffer_load ... lds): no
//     vector registers are tied up by data in flight and nothing has to be
//     copied into LDS afterwards.
//   * Everything a tile needs besides its data lives in scalar registers,
//     fetched with a few wide scalar loads: the stage's rank lists and its
//     program; the rank pointers sit in a vector register, lane r holding rank
//     r's, one readlane away.  No memory access per operation or per rank.
//   * The stage's computation runs as a stack program (see stack_program in
//     schedule.hpp): ranks are loaded in the order in which they are consumed,
//     rank i into LDS slot i, so every LDS address is a compile-time constant,
//     the reads of all ranks can be scheduled ahead of the arithmetic, partial
//     sums stay in registers (up to four accumulators).  The waits are written
//     per rank (vector memory operations complete in order, so rank i has
//     arrived once no more than the later ranks' loads are outstanding), but the
//     compiler puts a wait for ALL of the wave's vector memory operations in
//     front of the first LDS read that follows loads into LDS, whose
//     destinations it cannot tell apart: the sum starts when the last rank is in.
//   * The next ticket is drawn just before the tile's loads are issued and
//     resolved (instance, tile, stage shape) while they are in flight.
//
// What limits it (measured per 64 KiB sub-tile of an 8-rank stage, one wave per
// CU): issuing the 64 loads takes 2.8 us and the 64 stores 2.7 us, both at the
// pace at which HBM takes them; the sum itself 2.0 us, during which the wave has
// nothing in flight (most of it moves and selects: the compiler turns the
// uniform branches on the depth into selects over all accumulators).  A second
// wave per CU fills those gaps only in part.  Variants without these costs (LDS
// reads as assembly so that rank i really is consumed when it arrives; only the
// top accumulator in registers and the others parked in LDS; loads issued a
// sub-tile ahead into two LDS halves; the ticket drawn a tile ahead) were built
// and measured on the same machine: each made one wave per CU faster (8 ranks
// x 256 MiB: 0.51 -> 0.75 of the HBM peak) and two waves per CU, this kernel's
// launch, slower (0.73 -> 0.69; 6 ranks: 0.685 -> 0.65), because a lone wave is
// bound by its own instruction issue and two fast ones crowd the memory system;
// none beat blink_consume's 0.795, so the kernel stayed as it is.
#pragma once
#include <utility>

#include "kernel.hpp"

namespace blink {

constexpr int kColumnsDirect = 64;  // LDS slots per lane: 64 KiB per wave

using LdsPtr = __attribute__((address_space(3))) void*;

// Loads that write LDS: the explicit waits before the LDS reads
// (wait_vector_memory below) state what each read needs; the compiler adds a
// wait of its own for all vector memory operations before the first of them.

struct TicketSource {
    unsigned long long* counter;
    unsigned long long base, n_items, next_static;
    unsigned stride;
    bool dealt;  // all tickets are dealt round-robin, the counter is not used
    // Drawing a ticket is split in two so that the counter's answer can travel
    // while the wave issues loads.  With the counter every wave draws until it
    // gets a ticket >= n_items, hence exactly one past the end, which is what
    // the host adds to the base per wave.
    __device__ __forceinline__ unsigned long long begin_draw(int lane) {
        unsigned long long raw = 0;
        if (!dealt && lane == 0)
            raw = __hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return raw;
    }
    __device__ __forceinline__ unsigned long long end_draw(unsigned long long raw) {
        if (dealt) {
            const unsigned long long t = next_static;
            next_static += stride;
            return t;
        }
        const unsigned lo = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(raw));
        const unsigned hi = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(raw >> 32));
        return ((static_cast<unsigned long long>(hi) << 32) | lo) - base;
    }
    __device__ __forceinline__ unsigned long long draw(int lane) { return end_draw(begin_draw(lane)); }
};

// What a ticket resolves to, all of it wave-uniform (scalar registers): the
// tile's elements and its stage's shape.  tlen == 0: no ticket is left.
struct Tile {
    unsigned long long first;  // first element
    unsigned tlen;             // elements
    unsigned tmpl_index;
    unsigned n_load, n_op, n_store;
    uint32_t store_ranks[4];     // store_rank[16], one byte each
    uint32_t seq_ranks[4];       // seq_rank[16]: the ranks in the order the stage consumes them
    uint32_t seq_codes[4];       // seq_code[16]: (folds << 1) | push
};

struct Resolver {
    ConstTmpl tmpl;
    ConstInst inst;
    TicketSource tickets;
    unsigned tiles_per_chunk, tile_shift, group, n_inst;
    unsigned long long grid_shift;
    bool reverse;

    // ticket -> (instance, tile), as in blink_consume: tile by tile across the
    // trees' turns at one chunk position (section 4.2.2).  Tickets of instances
    // that have fewer tiles than the longest one are skipped (a fresh draw).
    __device__ __forceinline__ Tile resolve(unsigned long long t, int lane) {
        Tile out;
        out.tlen = 0;
        while (t < tickets.n_items) {
            unsigned ii, tile;
            // every other call walks the tiles backwards (see blink_consume)
            ticket_to_tile(reverse ? tickets.n_items - 1 - t : t, group, tiles_per_chunk, n_inst, &ii, &tile);
            ConstInst in = inst + ii;
            // the tile grid, moved down by grid_shift elements (see blink_consume)
            const unsigned long long off = in->off, end = off + in->len;
            const unsigned long long block = ((off + grid_shift) >> tile_shift) + tile;
            const unsigned long long block_lo = block << tile_shift;
            const unsigned long long lo_e = block_lo > grid_shift ? max(off, block_lo - grid_shift) : off;
            const unsigned long long hi_e = min(end, block_lo + (1ull << tile_shift) - grid_shift);
            if (lo_e < hi_e) {
                out.first = lo_e;
                out.tlen = static_cast<unsigned>(hi_e - lo_e);
                out.tmpl_index = in->tmpl;
                const BLINK_CONST uint32_t* w = reinterpret_cast<const BLINK_CONST uint32_t*>(tmpl + out.tmpl_index);
                static_assert(offsetof(StageTmpl, n_load) == 0 && offsetof(StageTmpl, n_op) == 1 &&
                                  offsetof(StageTmpl, n_store) == 2 && offsetof(StageTmpl, load_rank) == 8 &&
                                  offsetof(StageTmpl, store_rank) == 24 && offsetof(StageTmpl, op) == 40 &&
                                  kMaxOps == 40 && BLINK_MAX_RANKS == 16,
                              "the stage template is fetched as whole words");
                const uint32_t head = w[0];
                out.n_load = head & 0xffu;
                out.n_op = (head >> 8) & 0xffu;
                out.n_store = (head >> 16) & 0xffu;
                constexpr unsigned kStoreWord = offsetof(StageTmpl, store_rank) / 4,
                                   kSeqRankWord = offsetof(StageTmpl, seq_rank) / 4,
                                   kSeqCodeWord = offsetof(StageTmpl, seq_code) / 4;
                static_assert(offsetof(StageTmpl, seq_rank) % 4 == 0 && offsetof(StageTmpl, seq_code) % 4 == 0,
                              "the stack program is fetched as whole words");
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    out.store_ranks[q] = w[kStoreWord + q];
                    out.seq_ranks[q] = w[kSeqRankWord + q];
                    out.seq_codes[q] = w[kSeqCodeWord + q];
                }
                break;
            }
            t = tickets.draw(lane);
        }
        return out;
    }
};

// s_waitcnt vmcnt(n): at most n of this wave's vector memory operations are
// still outstanding (they complete in the order in which they were issued).
template <int N>
__device__ __forceinline__ void wait_vector_memory() {
    static_assert(N >= 0 && N <= 63, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
    asm volatile("" ::: "memory");  // no LDS read may be moved above the wait
}

// U columns of a lane as one value.  The accumulators are values of this type,
// not arrays: conditional updates of values stay in registers, whereas the
// compiler turns conditional updates of array levels selected by the depth into
// one run-time index, and the stack would live in memory.
template <int U>
struct Wide {
    typedef unsigned Bits __attribute__((ext_vector_type(4 * U)));
    typedef float Floats __attribute__((ext_vector_type(4 * U)));
};

template <typename T, int U>
__device__ __forceinline__ typename Wide<U>::Bits wide_sum(typename Wide<U>::Bits a, typename Wide<U>::Bits b) {
    if constexpr (std::is_same<T, float>::value)
        return __builtin_bit_cast(typename Wide<U>::Bits, __builtin_bit_cast(typename Wide<U>::Floats, a) +
                                                              __builtin_bit_cast(typename Wide<U>::Floats, b));
    else
        return a + b;
}

// The U columns of LDS slot `slot` that belong to this lane.
template <int U>
__device__ __forceinline__ typename Wide<U>::Bits read_slot(const U4* __restrict__ slots, int slot, int lane) {
    typename Wide<U>::Bits x;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const U4 v = slots[(slot * U + u) * kLanes + lane];
        x[4 * u] = v.x, x[4 * u + 1] = v.y, x[4 * u + 2] = v.z, x[4 * u + 3] = v.w;
    }
    return x;
}

// The stack program of a stage over the ranks in LDS slots 0 .. N-1 (slot i =
// the i-th rank consumed), U columns per lane, with the sum as the operator and
// up to D accumulators a0 (bottom) .. a3; `depth` (wave-uniform) is the index of
// the top one.  Registers cannot be indexed at run time: every operation
// branches, uniformly, on the depth.  The wait before rank i is for its own
// loads: the loads were the wave's last N * U vector memory operations (but for
// any issued after them, which only makes a wait longer than needed).
template <typename T, int N, int U, int D>
__device__ __forceinline__ void run_stack(const U4* __restrict__ slots, const uint32_t (&codes)[4], int lane,
                                          U4 (&result)[U]) {
    using W = typename Wide<U>::Bits;
    W a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    int depth = -1;
#define BLINK_STACK_STEP(I)                                                              \
    if constexpr (I < N) {                                                               \
        wait_vector_memory<(N - 1 - I) * U>();                                           \
        const W x = read_slot<U>(slots, I, lane);                                        \
        const unsigned code = (codes[I / 4] >> ((I & 3) * 8)) & 0xffu;                   \
        if (code & 1u) {                                                                 \
            ++depth;                                                                     \
            if (D == 1 || depth == 0) a0 = x;                                            \
            if (D > 1 && depth == 1) a1 = x;                                             \
            if (D > 2 && depth == 2) a2 = x;                                             \
            if (D > 3 && depth == 3) a3 = x;                                             \
        } else {                                                                         \
            if (D == 1 || depth == 0) a0 = wide_sum<T, U>(a0, x);                        \
            if (D > 1 && depth == 1) a1 = wide_sum<T, U>(a1, x);                         \
            if (D > 2 && depth == 2) a2 = wide_sum<T, U>(a2, x);                         \
            if (D > 3 && depth == 3) a3 = wide_sum<T, U>(a3, x);                         \
        }                                                                                \
        if (D > 1)                                                                       \
            for (unsigned f = code >> 1; f; --f) { /* the level below += the top level */ \
                if (depth == 1) a0 = wide_sum<T, U>(a0, a1);                             \
                if (D > 2 && depth == 2) a1 = wide_sum<T, U>(a1, a2);                    \
                if (D > 3 && depth == 3) a2 = wide_sum<T, U>(a2, a3);                    \
                --depth;                                                                 \
            }                                                                            \
    }
    BLINK_STACK_STEP(0) BLINK_STACK_STEP(1) BLINK_STACK_STEP(2) BLINK_STACK_STEP(3)
    BLINK_STACK_STEP(4) BLINK_STACK_STEP(5) BLINK_STACK_STEP(6) BLINK_STACK_STEP(7)
    BLINK_STACK_STEP(8) BLINK_STACK_STEP(9) BLINK_STACK_STEP(10) BLINK_STACK_STEP(11)
    BLINK_STACK_STEP(12) BLINK_STACK_STEP(13) BLINK_STACK_STEP(14) BLINK_STACK_STEP(15)
#undef BLINK_STACK_STEP
#pragma unroll
    for (int u = 0; u < U; ++u) {
        U4 v;
        v.x = a0[4 * u], v.y = a0[4 * u + 1], v.z = a0[4 * u + 2], v.w = a0[4 * u + 3];
        result[u] = v;
    }
}

// The 16-byte columns of one tile of a stage that reads N ranks: `bytes` bytes
// at element cur.first.  Draws and resolves the wave's next ticket while the
// tile's first loads are in flight, and returns it.
template <typename T, int N, int LD, int ST>
__device__ __forceinline__ Tile stream_tile(U4* __restrict__ slots, RankTable ranks,
                                            const Tile& cur, unsigned bytes, int lane, Resolver& res) {
    constexpr int U = N <= 4 ? 16 : (N <= 8 ? 8 : 4);  // N * U <= kColumnsDirect
    // a stack program over N ranks needs at most N / 2 accumulators; schedules
    // that need more than four do not come here (see the launcher)
    constexpr int D = N < 4 ? 1 : (N < 6 ? 2 : (N < 8 ? 3 : 4));
    constexpr unsigned kSubBytes = kLanes * U * 16;
    const unsigned long long byte_off = cur.first * 4ull;
    const int n_store = static_cast<int>(cur.n_store);
    Tile next;
    for (unsigned b = 0; b < bytes; b += kSubBytes) {
        const unsigned left = bytes - b;
        unsigned long long raw = 0;
        if (b == 0) raw = res.tickets.begin_draw(lane);
        // phase 1: every load of the sub-tile, straight into the LDS slots
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const unsigned rank = (cur.seq_ranks[i / 4] >> ((i & 3) * 8)) & 0xffu;
            const __amdgpu_buffer_rsrc_t win = __builtin_amdgcn_make_buffer_rsrc(
                reinterpret_cast<char*>(rank_base(ranks, rank) + byte_off + b), 0, static_cast<int>(left),
                kRawDword3);
#pragma unroll
            for (int u = 0; u < U; ++u)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(win, (LdsPtr)(slots + (i * U + u) * kLanes), 16,
                                                         (u * kLanes + lane) * 16, 0, 0, LD);
        }
        // The counter's answer arrives before the data (vector memory operations
        // complete in order); the next tile is resolved while the data travels.
        // The empty statement pins the answer's first use to this point of the
        // program: without it the compiler reads it, and waits for it, before
        // issuing the loads.
        if (b == 0) {
            unsigned raw_lo = static_cast<unsigned>(raw), raw_hi = static_cast<unsigned>(raw >> 32);
            asm volatile("" : "+v"(raw_lo), "+v"(raw_hi)::"memory");
            next = res.resolve(res.tickets.end_draw((static_cast<unsigned long long>(raw_hi) << 32) | raw_lo), lane);
        }
        // phase 2: the stage's stack program; rank i is awaited just before its turn
        U4 acc[U];
        run_stack<T, N, U, D>(slots, cur.seq_codes, lane, acc);
        // phase 3: stores.  The LDS reads above have all been consumed (their
        // values are in acc, which the stores take) before the next sub-tile's
        // loads, later in program order, overwrite the slots.
#pragma unroll
        for (int j = 0; j < BLINK_MAX_RANKS; ++j) {
            if (j < n_store) {
                const unsigned rank = (cur.store_ranks[j / 4] >> ((j & 3) * 8)) & 0xffu;
                const __amdgpu_buffer_rsrc_t win = __builtin_amdgcn_make_buffer_rsrc(
                    reinterpret_cast<char*>(rank_base(ranks, rank) + byte_off + b), 0,
                    static_cast<int>(left), kRawDword3);
#pragma unroll
                for (int u = 0; u < U; ++u)
                    __builtin_amdgcn_raw_buffer_store_b128(acc[u], win, (u * kLanes + lane) * 16, 0, ST);
            }
        }
    }
    return next;
}

template <typename T, int FLAVOUR>
__global__ __launch_bounds__(kLanes) void blink_stream(const KParams) {
    __shared__ U4 slots[kColumnsDirect * kLanes];
    constexpr int LD = Policy<FLAVOUR>::kLoad;
    constexpr int ST = Policy<FLAVOUR>::kStore;
    const int lane = threadIdx.x;
    ConstParams p = (ConstParams)__builtin_amdgcn_kernarg_segment_ptr();
    if (__hip_atomic_load(p->status + kStatusState, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    const RankTable ranks = load_rank_table(p, lane);

    Resolver res;
    res.tmpl = reinterpret_cast<ConstTmpl>(reinterpret_cast<unsigned long long>(p->tmpl));
    res.inst = reinterpret_cast<ConstInst>(reinterpret_cast<unsigned long long>(p->inst));
    res.tiles_per_chunk = p->tiles_per_chunk;
    res.tile_shift = p->tile_shift;
    res.group = p->group;
    res.reverse = p->reverse != 0;
    res.grid_shift = p->grid_shift;
    res.n_inst = p->n_inst;
    res.tickets.counter = p->ticket;
    res.tickets.base = p->ticket_base[0];
    res.tickets.n_items = p->n_items;
    res.tickets.next_static = blockIdx.x;
    res.tickets.stride = gridDim.x;
    res.tickets.dealt = p->static_items == p->n_items;

    Tile cur = res.resolve(res.tickets.draw(lane), lane);
    while (cur.tlen) {
        const bool aligned = (cur.first & 3ull) == 0;
        const unsigned vec_bytes = aligned ? (cur.tlen >> 2) * 16u : 0u;
        Tile next;
        bool resolved = false;
        if (vec_bytes) {
            resolved = true;
            switch (cur.n_load) {
#define BLINK_CASE(N) case N: next = stream_tile<T, N, LD, ST>(slots, ranks, cur, vec_bytes, lane, res); break;
                BLINK_CASE(1) BLINK_CASE(2) BLINK_CASE(3) BLINK_CASE(4) BLINK_CASE(5) BLINK_CASE(6)
                BLINK_CASE(7) BLINK_CASE(8) BLINK_CASE(9) BLINK_CASE(10) BLINK_CASE(11) BLINK_CASE(12)
                BLINK_CASE(13) BLINK_CASE(14) BLINK_CASE(15) BLINK_CASE(16)
#undef BLINK_CASE
                default: resolved = false; break;
            }
        }
        // what is not a whole 16-byte column: the end of a payload whose length
        // is no multiple of 4 elements, and tiles of chunks that do not start on
        // a 16-byte boundary.  Element-wise, slow, rare.
        ConstTmpl st = res.tmpl + cur.tmpl_index;
        if (aligned) {
            const unsigned rem = cur.tlen & 3u;
            if (rem)
                run_scalar<T, LD, ST>(reinterpret_cast<unsigned*>(slots), p, ranks, st, cur.first * 4ull + vec_bytes, rem * 4u,
                                      lane);
        } else {
            for (unsigned b = 0; b < cur.tlen * 4u; b += kLanes * 4u)
                run_scalar<T, LD, ST>(reinterpret_cast<unsigned*>(slots), p, ranks, st, cur.first * 4ull + b,
                                      min(static_cast<unsigned>(kLanes) * 4u, cur.tlen * 4u - b), lane);
        }
        if (!resolved) next = res.resolve(res.tickets.draw(lane), lane);
        cur = next;
    }
}

// The most accumulators the stack program of a stage that reads n_load ranks may
// need for blink_stream to run it (stream_tile's D).
inline int stream_stack_limit(int n_load) { return n_load < 4 ? 1 : (n_load < 6 ? 2 : (n_load < 8 ? 3 : 4)); }

// The kernel for a flavour on payloads that stream.  `direct`: the schedule has no
// dependencies, all its stages have stack programs within the limit and the
// operator is the sum (the one blink_stream is compiled for: every further
// operator would double its code); other calls (stages that hand chunks over to
// one another among them) run on blink_consume with its 32 columns.
template <typename T>
KernelFn pick_stream_kernel_of(int flavour, bool direct) {
    if (!direct) return pick_kernel_of<T, kColumnsStream>(flavour);
    switch (flavour) {
        case kWriteHeavy: return blink_stream<T, kWriteHeavy>;
        case kReadHeavy: return blink_stream<T, kReadHeavy>;
        default: return blink_stream<T, kBalanced>;
    }
}

}  // namespace blink
