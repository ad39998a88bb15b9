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
//     sums stay in registers (up to four accumulators), and rank i is consumed
//     as soon as ITS loads have arrived (vector memory operations complete in
//     order), while later ranks are still on their way.
//   * The next ticket is drawn just before the tile's loads are issued and
//     resolved (instance, tile, stage shape) while they are in flight.
//
// What limits it (measured per 64 KiB sub-tile of an 8-rank stage, one wave per
// CU): issuing the 64 loads takes 2.8 us and the 64 stores 2.7 us, both at the
// pace at which HBM takes them; the sum itself 2.0 us, during which the wave has
// nothing in flight.  A second wave per CU fills those gaps only in part.
#pragma once
#include <utility>

#include "kernel.hpp"

namespace blink {

constexpr int kColumnsDirect = 64;  // LDS slots per lane: 64 KiB per wave

// Accumulators a stage's stack program may have at a time: the top one in
// registers, the others parked in LDS.  A stage over N ranks needs at most N / 2.
constexpr int kStreamStackLevels = BLINK_MAX_RANKS / 2;

using LdsPtr = __attribute__((address_space(3))) void*;


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
    // The answer is taken out of its vector register on every path, the dealt
    // one included (the empty statement is a use the compiler cannot drop).  A
    // path on which the register may still be awaiting the counter costs more
    // than the wait it saves: wherever that register is written next, the
    // compiler first waits for all the wave's vector memory operations, and it
    // reuses the register in the middle of the tile loop.  (For the same reason
    // the answer is not kept across a tile to hide the counter's latency
    // altogether: under the tile body's register pressure the compiler moves it
    // to another register at once, which is a wait for it at once.)
    __device__ __forceinline__ unsigned long long end_draw(unsigned long long raw) {
        unsigned raw_lo = static_cast<unsigned>(raw), raw_hi = static_cast<unsigned>(raw >> 32);
        asm volatile("" : "+v"(raw_lo), "+v"(raw_hi)::"memory");
        const unsigned lo = __builtin_amdgcn_readfirstlane(raw_lo);
        const unsigned hi = __builtin_amdgcn_readfirstlane(raw_hi);
        if (dealt) {
            const unsigned long long t = next_static;
            next_static += stride;
            return t;
        }
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

    // ticket -> (instance, tile), as in blink_consume: tile by tile across the
    // trees' turns at one chunk position (section 4.2.2).  Tickets of instances
    // that have fewer tiles than the longest one are skipped (a fresh draw).
    __device__ __forceinline__ Tile resolve(unsigned long long t, int lane) {
        Tile out;
        out.tlen = 0;
        while (t < tickets.n_items) {
            unsigned ii, tile;
            ticket_to_tile(t, group, tiles_per_chunk, n_inst, &ii, &tile);
            ConstInst in = inst + ii;
            const unsigned long long off = in->off, end = off + in->len;
            const unsigned long long block = (off >> tile_shift) + tile;
            const unsigned long long lo_e = max(off, block << tile_shift);
            const unsigned long long hi_e = min(end, (block + 1) << tile_shift);
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

template <typename T>
__device__ __forceinline__ U4 column_sum(U4 a, U4 b) {
    if constexpr (std::is_same<T, float>::value)
        return __builtin_bit_cast(U4, __builtin_bit_cast(F4, a) + __builtin_bit_cast(F4, b));
    else
        return a + b;
}

// LDS access to a lane's U columns of one slot, as assembly.  `addr`: the LDS
// address of the lane's column 0 of the slot minus OFF bytes (columns are
// kLanes * 16 = 1024 bytes apart).
//
// Assembly because of what the compiler does with LDS reads it can see: it
// tracks loads that write LDS, cannot tell their destinations apart, and puts
// s_waitcnt vmcnt(0) in front of the first LDS read after them.  That wait
// covers every load of the sub-tile and the previous sub-tile's stores: the wave
// would start summing only once nothing of its own is in flight any more.  Here
// the wait before rank i's slot is the caller's (wait_vector_memory), for that
// rank's loads alone.  Each statement ends with lgkmcnt(0): what it read is an
// ordinary register value to the compiler, what it wrote is in LDS.
#define BLINK_LDS4(OPCODE, CONSTRAINT, B)                                                                     \
    asm volatile(OPCODE " %0, %4 offset:%5\n\t" OPCODE " %1, %4 offset:%6\n\t" OPCODE " %2, %4 offset:%7\n\t" \
                 OPCODE " %3, %4 offset:%8\n\ts_waitcnt lgkmcnt(0)"                                           \
                 : CONSTRAINT(v[B]), CONSTRAINT(v[B + 1]), CONSTRAINT(v[B + 2]), CONSTRAINT(v[B + 3])         \
                 : "v"(addr), "n"(OFF + (B) * 1024), "n"(OFF + (B + 1) * 1024), "n"(OFF + (B + 2) * 1024),    \
                   "n"(OFF + (B + 3) * 1024)                                                                  \
                 : "memory")
#define BLINK_LDS8(OPCODE, CONSTRAINT, B)                                                                     \
    asm volatile(OPCODE " %0, %8 offset:%9\n\t" OPCODE " %1, %8 offset:%10\n\t" OPCODE                        \
                        " %2, %8 offset:%11\n\t" OPCODE " %3, %8 offset:%12\n\t" OPCODE                       \
                        " %4, %8 offset:%13\n\t" OPCODE " %5, %8 offset:%14\n\t" OPCODE                       \
                        " %6, %8 offset:%15\n\t" OPCODE " %7, %8 offset:%16\n\ts_waitcnt lgkmcnt(0)"          \
                 : CONSTRAINT(v[B]), CONSTRAINT(v[B + 1]), CONSTRAINT(v[B + 2]), CONSTRAINT(v[B + 3]),        \
                   CONSTRAINT(v[B + 4]), CONSTRAINT(v[B + 5]), CONSTRAINT(v[B + 6]), CONSTRAINT(v[B + 7])     \
                 : "v"(addr), "n"(OFF + (B) * 1024), "n"(OFF + (B + 1) * 1024), "n"(OFF + (B + 2) * 1024),    \
                   "n"(OFF + (B + 3) * 1024), "n"(OFF + (B + 4) * 1024), "n"(OFF + (B + 5) * 1024),           \
                   "n"(OFF + (B + 6) * 1024), "n"(OFF + (B + 7) * 1024)                                       \
                 : "memory")
template <int U, int OFF>
__device__ __forceinline__ void lds_read(unsigned addr, U4 (&v)[U]) {
    static_assert(U == 4 || U == 8 || U == 16, "one statement per batch of four or eight columns");
    static_assert(OFF >= 0 && OFF + (U - 1) * 1024 < 65536, "the offset field has 16 bits");
    if constexpr (U == 4) {
        BLINK_LDS4("ds_read_b128", "=&v", 0);
    } else if constexpr (U == 8) {
        BLINK_LDS8("ds_read_b128", "=&v", 0);
    } else {
        BLINK_LDS8("ds_read_b128", "=&v", 0);
        BLINK_LDS8("ds_read_b128", "=&v", 8);
    }
}
#undef BLINK_LDS4
#undef BLINK_LDS8
// ds_write takes the address first, then the data: statements of their own.
#define BLINK_LDSW4(B)                                                                                      \
    asm volatile("ds_write_b128 %0, %1 offset:%5\n\tds_write_b128 %0, %2 offset:%6\n\t"                    \
                 "ds_write_b128 %0, %3 offset:%7\n\tds_write_b128 %0, %4 offset:%8\n\ts_waitcnt lgkmcnt(0)" \
                 :                                                                                          \
                 : "v"(addr), "v"(v[B]), "v"(v[B + 1]), "v"(v[B + 2]), "v"(v[B + 3]), "n"(OFF + (B) * 1024),  \
                   "n"(OFF + (B + 1) * 1024), "n"(OFF + (B + 2) * 1024), "n"(OFF + (B + 3) * 1024)           \
                 : "memory")
template <int U, int OFF>
__device__ __forceinline__ void lds_write(unsigned addr, const U4 (&v)[U]) {
    static_assert(U == 4 || U == 8 || U == 16, "one statement per batch of four columns");
    static_assert(OFF >= 0 && OFF + (U - 1) * 1024 < 65536, "the offset field has 16 bits");
    BLINK_LDSW4(0);
    if constexpr (U >= 8) BLINK_LDSW4(4);
    if constexpr (U == 16) {
        BLINK_LDSW4(8);
        BLINK_LDSW4(12);
    }
}
#undef BLINK_LDSW4

// The stack program of a stage over the ranks in LDS slots 0 .. N-1 (slot i =
// the i-th rank consumed, U columns per lane), with the sum as the operator.
// Only the top accumulator of the stack lives in registers.  A rank that starts
// a new accumulator first parks the current top in the slot of the rank
// consumed just before it (free by then, and a compile-time address); folding
// the top into the level below reads that level back.  `parked` holds the slots
// of the parked levels, as scalars chosen by the (wave-uniform) depth: LDS can
// be addressed at run time, registers cannot, and a stack of accumulators in
// registers costs the compiler more in copies between its branches than the
// sums themselves (per rank 150 to 200 moves and selects around 32 additions).
// Rank i is consumed once its own loads have arrived: the loads were the wave's
// last N * U vector memory operations.  The first code always starts an
// accumulator (stack_program sees to that).
template <typename T, int N, int U>
__device__ __forceinline__ void run_stack(unsigned lane_addr, const uint32_t (&codes)[4], U4 (&top)[U]) {
    constexpr int kSlot = U * kLanes * 16;  // bytes
    int depth = 0;                          // accumulators below the top one
    unsigned parked[kStreamStackLevels - 1] = {};
    wait_vector_memory<(N - 1) * U>();
    lds_read<U, 0>(lane_addr, top);
#define BLINK_STACK_STEP(I)                                                                 \
    if constexpr (I < N) {                                                                  \
        const unsigned code = (codes[I / 4] >> ((I & 3) * 8)) & 0xffu;                      \
        if constexpr (I > 0) {                                                              \
            wait_vector_memory<(N - 1 - I) * U>();                                          \
            if (code & 1u) {                                                                \
                lds_write<U, (I - 1) * kSlot>(lane_addr, top);                              \
                _Pragma("unroll") for (int d = 0; d < kStreamStackLevels - 1; ++d)          \
                    if (d == depth) parked[d] = (I - 1) * kSlot;                            \
                ++depth;                                                                    \
                lds_read<U, I * kSlot>(lane_addr, top);                                     \
            } else {                                                                        \
                U4 x[U];                                                                    \
                lds_read<U, I * kSlot>(lane_addr, x);                                       \
                _Pragma("unroll") for (int u = 0; u < U; ++u) top[u] = column_sum<T>(top[u], x[u]); \
            }                                                                               \
        }                                                                                   \
        for (unsigned f = code >> 1; f; --f) { /* the level below += the top level */       \
            --depth;                                                                        \
            unsigned from = parked[0];                                                      \
            _Pragma("unroll") for (int d = 1; d < kStreamStackLevels - 1; ++d)              \
                if (d == depth) from = parked[d];                                           \
            U4 below[U];                                                                    \
            lds_read<U, 0>(lane_addr + from, below);                                        \
            _Pragma("unroll") for (int u = 0; u < U; ++u) top[u] = column_sum<T>(below[u], top[u]); \
        }                                                                                   \
    }
    BLINK_STACK_STEP(0) BLINK_STACK_STEP(1) BLINK_STACK_STEP(2) BLINK_STACK_STEP(3)
    BLINK_STACK_STEP(4) BLINK_STACK_STEP(5) BLINK_STACK_STEP(6) BLINK_STACK_STEP(7)
    BLINK_STACK_STEP(8) BLINK_STACK_STEP(9) BLINK_STACK_STEP(10) BLINK_STACK_STEP(11)
    BLINK_STACK_STEP(12) BLINK_STACK_STEP(13) BLINK_STACK_STEP(14) BLINK_STACK_STEP(15)
#undef BLINK_STACK_STEP
}

// The 16-byte columns of one tile of a stage that reads N ranks: `bytes` bytes
// at element cur.first.  Draws and resolves the wave's next ticket while the
// tile's first loads are in flight, and returns it.
template <typename T, int N, int LD, int ST>
__device__ __forceinline__ Tile stream_tile(U4* __restrict__ slots, RankTable ranks,
                                            const Tile& cur, unsigned bytes, int lane, Resolver& res) {
    constexpr int U = N <= 4 ? 16 : (N <= 8 ? 8 : 4);  // N * U <= kColumnsDirect
    constexpr unsigned kSubBytes = kLanes * U * 16;
    const unsigned long long byte_off = cur.first * 4ull;
    const int n_store = static_cast<int>(cur.n_store);
    const unsigned lane_addr = static_cast<unsigned>(reinterpret_cast<size_t>((LdsPtr)slots)) + lane * 16u;
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
        // The empty statement in end_draw pins the answer's first use to this
        // point of the program: without it the compiler reads it, and waits for
        // it, before issuing the loads.
        if (b == 0) next = res.resolve(res.tickets.end_draw(raw), lane);
        // phase 2: the stage's stack program; rank i is awaited just before its turn
        U4 acc[U];
        run_stack<T, N, U>(lane_addr, cur.seq_codes, acc);
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
    res.n_inst = static_cast<unsigned>(p->n_items / p->tiles_per_chunk);
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
// need for blink_stream to run it: every stack program fits (N / 2 at most).
inline int stream_stack_limit(int) { return kStreamStackLevels; }

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
