// The device side: one persistent gfx950 kernel that consumes the stage list of
// all trees concurrently (paper sections 3.3, 4.1, 4.2.1, 4.2.2), and its launcher.
//
// A workgroup is ONE 64-lane wavefront: nothing in the kernel needs a
// workgroup barrier, and a wave that waits for a dependency holds up nobody
// else.  Work unit: (stage instance, tile).  Waves draw units from one ticket
// counter in the schedule's execution order, so every unit a wave might have
// to wait for has already been drawn by a wave that is running: waiting can
// never deadlock, whatever the grid size.
//
// A tile is kSub sub-tiles; a sub-tile of a stage is processed in three phases
// by the 64 lanes, each owning U 128-bit columns:
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
// on a schedule waits for e * tiles.  A consumer polls with agent-scope atomic
// loads, then acquires; a producer releases at agent scope and increments.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstddef>
#include <cstdio>
#include <vector>

#include "schedule.hpp"
#include "state.hpp"

namespace blink {

constexpr int kLanes = 64;   // one wavefront per workgroup
constexpr int kSub = 4;      // sub-tiles per ticket
// 128-bit columns a lane may hold in registers at once (ranks read x unroll):
// keeps the load phase inside the register file.
constexpr int kMaxColumns = 16;

struct KParams {
    void* buf[BLINK_MAX_RANKS];
    const StageTmpl* tmpl;
    const StageInst* inst;
    unsigned long long* done;
    unsigned long long* ticket;
    unsigned long long ticket_base;
    unsigned long long n_items;
    unsigned long long epoch;
    unsigned tiles_per_chunk;
};

// Address spaces: rank buffers are plain global memory; the kernel arguments
// and the schedule tables are never written by the kernel, so they are read
// through the constant address space, which lets wave-uniform reads use the
// scalar unit.
#define BLINK_GLOBAL __attribute__((address_space(1)))
#define BLINK_CONST __attribute__((address_space(4)))
using ConstParams = const BLINK_CONST KParams*;
using ConstTmpl = const BLINK_CONST StageTmpl*;
using ConstInst = const BLINK_CONST StageInst*;

typedef float F4 __attribute__((ext_vector_type(4)));     // one 128-bit access of fp32
typedef unsigned U4 __attribute__((ext_vector_type(4)));  // int32 payloads add as unsigned: wrap-around, no UB
template <typename V>
__device__ __forceinline__ V vadd(V a, V b) {
    return a + b;
}

// Byte `field_offset + i` of a stage template, fetched as part of a 32-bit word
// so that the scalar unit can do it.
__device__ __forceinline__ unsigned tmpl_byte(ConstTmpl st, unsigned byte_index) {
    const BLINK_CONST uint32_t* w = reinterpret_cast<const BLINK_CONST uint32_t*>(st);
    return (w[byte_index >> 2] >> ((byte_index & 3u) * 8u)) & 0xffu;
}
#define BLINK_TMPL(st, field, i) tmpl_byte(st, static_cast<unsigned>(offsetof(StageTmpl, field)) + (i))

template <typename V>
__device__ __forceinline__ BLINK_GLOBAL V* rank_ptr(ConstParams p, unsigned rank, unsigned long long byte_off) {
    return reinterpret_cast<BLINK_GLOBAL V*>(reinterpret_cast<unsigned long long>(p->buf[rank]) + byte_off);
}

// Phase 1, full tile, NL ranks: issue every load, then park the values in LDS.
template <typename V, int NL, int U>
__device__ __forceinline__ void load_slots_full(V* __restrict__ slots, ConstParams p, ConstTmpl st,
                                                unsigned long long byte_off, int tid) {
    V r[NL][U];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const BLINK_GLOBAL V* src = rank_ptr<V>(p, BLINK_TMPL(st, load_rank, i), byte_off);
#pragma unroll
        for (int u = 0; u < U; ++u) r[i][u] = src[u * kLanes + tid];
    }
#pragma unroll
    for (int i = 0; i < NL; ++i)
#pragma unroll
        for (int u = 0; u < U; ++u) slots[(i * U + u) * kLanes + tid] = r[i][u];
}

// Phases 1-3 for `nvec` elements of type V starting at byte_off.  FULL: the
// tile has all kLanes*U elements (the common case, no per-lane guards).
template <typename V, int U, bool FULL>
__device__ __forceinline__ void run_tile(V* __restrict__ slots, ConstParams p, ConstTmpl st,
                                         unsigned long long byte_off, unsigned nvec, int tid) {
    const int n_load = BLINK_TMPL(st, n_load, 0);
    if constexpr (FULL) {
        switch (n_load) {
#define BLINK_CASE(N)                                                              \
    case N:                                                                        \
        if constexpr (N * U <= kMaxColumns)                                        \
            load_slots_full<V, N, U>(slots, p, st, byte_off, tid);                 \
        break;
            BLINK_CASE(1) BLINK_CASE(2) BLINK_CASE(3) BLINK_CASE(4) BLINK_CASE(5) BLINK_CASE(6)
            BLINK_CASE(7) BLINK_CASE(8) BLINK_CASE(9) BLINK_CASE(10) BLINK_CASE(11) BLINK_CASE(12)
            BLINK_CASE(13) BLINK_CASE(14) BLINK_CASE(15) BLINK_CASE(16)
#undef BLINK_CASE
            default: break;
        }
    } else {
        for (int i = 0; i < n_load; ++i) {
            const BLINK_GLOBAL V* src = rank_ptr<V>(p, BLINK_TMPL(st, load_rank, i), byte_off);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const unsigned idx = u * kLanes + tid;
                if (idx < nvec) slots[(i * U + u) * kLanes + tid] = src[idx];
            }
        }
    }
    V acc[U];
    const int n_op = BLINK_TMPL(st, n_op, 0);
    for (int o = 0; o < n_op; ++o) {
        const unsigned code = BLINK_TMPL(st, op, o);
        V* sl = slots + (code & 63u) * (U * kLanes) + tid;
        const unsigned kind = code >> 6;
        if (kind == OP_LD) {
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] = sl[u * kLanes];
        } else if (kind == OP_ADD) {
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] = vadd(acc[u], sl[u * kLanes]);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) sl[u * kLanes] = acc[u];
        }
    }
    const int n_store = BLINK_TMPL(st, n_store, 0);
    for (int j = 0; j < n_store; ++j) {
        BLINK_GLOBAL V* dst = rank_ptr<V>(p, BLINK_TMPL(st, store_rank, j), byte_off);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned idx = u * kLanes + tid;
            if (FULL || idx < nvec) dst[idx] = acc[u];
        }
    }
}

// T: element type (float, or unsigned for wrap-around int32); V4: its 128-bit vector.
// The by-value argument is only there to size the kernel-argument segment; it is
// read through the constant address space (see ConstParams).
template <typename T, typename V4, int U>
__global__ __launch_bounds__(kLanes) void blink_consume(const KParams) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int lane = threadIdx.x;
    constexpr unsigned kSubTile = kLanes * 4 * U;   // elements per sub-tile
    constexpr unsigned kTile = kSubTile * kSub;     // elements per ticket
    ConstParams p = (ConstParams)__builtin_amdgcn_kernarg_segment_ptr();
    unsigned long long* const ticket = p->ticket;
    unsigned long long* const done = p->done;
    ConstTmpl const tmpl = reinterpret_cast<ConstTmpl>(reinterpret_cast<unsigned long long>(p->tmpl));
    ConstInst const inst = reinterpret_cast<ConstInst>(reinterpret_cast<unsigned long long>(p->inst));
    const unsigned long long n_items = p->n_items, ticket_base = p->ticket_base, epoch = p->epoch;
    const unsigned tiles_per_chunk = p->tiles_per_chunk;
    V4* const slots = reinterpret_cast<V4*>(lds_raw);

    // The loop has exactly one lane-dependent region, at its head, and one back
    // edge: the compiler must never get the chance to let some lanes run ahead
    // of lane 0 around the loop (readfirstlane needs lane 0 present).  Hence the
    // completion signal of a tile is posted together with the next ticket draw.
    long long pending = -1;  // instance whose finished tile still has to be counted
    for (;;) {
        unsigned long long raw = 0;
        if (lane == 0) {
            if (pending >= 0)
                __hip_atomic_fetch_add(done + pending, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            raw = __hip_atomic_fetch_add(ticket, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - ticket_base;
        }
        pending = -1;
        const unsigned lo = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(raw));
        const unsigned hi = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(raw >> 32));
        const unsigned long long t = (static_cast<unsigned long long>(hi) << 32) | lo;
        if (t >= n_items) break;
        const unsigned ii = static_cast<unsigned>(t / tiles_per_chunk);
        const unsigned tile = static_cast<unsigned>(t % tiles_per_chunk);
        ConstInst in = inst + ii;
        const unsigned len = in->len;
        const unsigned long long tile_off = static_cast<unsigned long long>(tile) * kTile;
        if (tile_off < len) {  // a short last chunk has fewer tiles than tickets
            const unsigned tlen = min(kTile, static_cast<unsigned>(len - tile_off));
            ConstTmpl st = tmpl + in->tmpl;

            const int n_dep = in->n_dep;
            if (n_dep) {
                if (lane < n_dep) {
                    const unsigned long long want = epoch * ((len + kTile - 1) / kTile);
                    const unsigned long long* f = done + in->dep[lane];
                    while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < want)
                        __builtin_amdgcn_s_sleep(2);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            }

            const unsigned long long e0 = in->off + tile_off;  // first element of the tile
            if ((e0 & 3ull) == 0) {
                const unsigned nvec = tlen >> 2;
                unsigned v = 0;
                for (; v + kLanes * U <= nvec; v += kLanes * U)
                    run_tile<V4, U, true>(slots, p, st, (e0 + 4ull * v) * 4ull, kLanes * U, lane);
                if (v < nvec) run_tile<V4, U, false>(slots, p, st, (e0 + 4ull * v) * 4ull, nvec - v, lane);
                const unsigned rem = tlen & 3u;  // only where the payload itself ends off a 16-byte boundary
                if (rem)
                    run_tile<T, 1, false>(reinterpret_cast<T*>(lds_raw), p, st, (e0 + (nvec << 2)) * 4ull, rem, lane);
            } else {
                // chunk size not a multiple of 4 elements: element-wise, slow but correct
                for (unsigned done_e = 0; done_e < tlen; done_e += kLanes)
                    run_tile<T, 1, false>(reinterpret_cast<T*>(lds_raw), p, st, (e0 + done_e) * 4ull,
                                          min(static_cast<unsigned>(kLanes), tlen - done_e), lane);
            }

            if (BLINK_TMPL(st, signals, 0)) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                pending = ii;
            }
        }
    }
}

// ---- host side ------------------------------------------------------------------------
namespace {

#define BLINK_HIP(call)                                                                   \
    do {                                                                                  \
        hipError_t err__ = (call);                                                        \
        if (err__ != hipSuccess) {                                                        \
            std::fprintf(stderr, "blink: %s failed: %s\n", #call, hipGetErrorString(err__)); \
            return err__ == hipErrorOutOfMemory ? BLINK_ENOMEM : BLINK_EHIP;              \
        }                                                                                 \
    } while (0)

using KernelFn = void (*)(const KParams);

KernelFn pick_kernel(blink_dtype_t dtype, int unroll) {
    if (dtype == BLINK_FP32) {
        if (unroll == 1) return blink_consume<float, F4, 1>;
        if (unroll == 2) return blink_consume<float, F4, 2>;
        return blink_consume<float, F4, 4>;
    }
    if (unroll == 1) return blink_consume<unsigned, U4, 1>;
    if (unroll == 2) return blink_consume<unsigned, U4, 2>;
    return blink_consume<unsigned, U4, 4>;
}

blink_status_t upload(blink_schedule* h) {
    int dev = -1;
    BLINK_HIP(hipGetDevice(&dev));
    if (h->device == dev) return BLINK_OK;
    if (h->device >= 0) return BLINK_EMISMATCH;  // tables live on another device
    const Schedule& s = h->s;
    BLINK_HIP(hipMalloc(&h->d_tmpl, s.tmpl.size() * sizeof(StageTmpl)));
    BLINK_HIP(hipMalloc(&h->d_inst, s.inst.size() * sizeof(StageInst)));
    BLINK_HIP(hipMalloc(&h->d_counters, (s.inst.size() + 1) * sizeof(unsigned long long)));
    BLINK_HIP(hipMemcpy(h->d_tmpl, s.tmpl.data(), s.tmpl.size() * sizeof(StageTmpl), hipMemcpyHostToDevice));
    BLINK_HIP(hipMemcpy(h->d_inst, s.inst.data(), s.inst.size() * sizeof(StageInst), hipMemcpyHostToDevice));
    BLINK_HIP(hipMemset(h->d_counters, 0, (s.inst.size() + 1) * sizeof(unsigned long long)));
    BLINK_HIP(hipDeviceSynchronize());
    hipDeviceProp_t prop;
    BLINK_HIP(hipGetDeviceProperties(&prop, dev));
    h->n_cu = prop.multiProcessorCount;
    h->device = dev;
    return BLINK_OK;
}

}  // namespace

// Forget all progress (used when the tile size changes: counters of earlier
// calls were counted in other units).  Waits for the device first.
blink_status_t reset_progress(blink_schedule* h) {
    h->epoch = 0;
    h->ticket_base = 0;
    for (auto& row : h->occupancy) for (int& x : row) x = 0;
    if (h->device < 0) return BLINK_OK;
    BLINK_HIP(hipDeviceSynchronize());
    BLINK_HIP(hipMemset(h->d_counters, 0, (h->s.inst.size() + 1) * sizeof(unsigned long long)));
    BLINK_HIP(hipDeviceSynchronize());
    return BLINK_OK;
}

void release_device_state(blink_schedule* h) {
    if (h->device < 0) return;
    (void)hipFree(h->d_tmpl);
    (void)hipFree(h->d_inst);
    (void)hipFree(h->d_counters);
    h->device = -1;
}

blink_status_t execute(blink_schedule* h, void* const* bufs, int k, size_t n, blink_dtype_t dtype,
                       blink_op_t op, void* stream) {
    if (!h || !bufs) return BLINK_EINVAL;
    if (dtype != BLINK_FP32 && dtype != BLINK_INT32) return BLINK_EINVAL;
    const Schedule& s = h->s;
    if (k != s.k || n != s.n || op != s.op) return BLINK_EMISMATCH;
    for (int i = 0; i < k; ++i) {
        if (!bufs[i] || (reinterpret_cast<uintptr_t>(bufs[i]) & 15u)) return BLINK_EINVAL;
        for (int j = 0; j < i; ++j) {
            const char* a = static_cast<const char*>(bufs[i]);
            const char* b = static_cast<const char*>(bufs[j]);
            if (a < b + n * 4 && b < a + n * 4 && n) return BLINK_EINVAL;
        }
    }
    if (n == 0 || s.inst.empty()) return BLINK_OK;
    if (blink_status_t st = upload(h)) return st;

    int unroll = h->unroll;
    if (unroll == 0) unroll = s.max_slots <= 4 ? 4 : (s.max_slots <= 8 ? 2 : 1);
    const unsigned tile = kLanes * 4 * unroll * kSub;
    uint32_t longest = 0;
    for (const StageInst& in : s.inst) longest = std::max(longest, in.len);
    const unsigned tiles_per_chunk = (longest + tile - 1) / tile;
    const unsigned long long n_items = static_cast<unsigned long long>(s.inst.size()) * tiles_per_chunk;
    if (static_cast<int>(s.max_slots) * unroll > kMaxColumns) return BLINK_EINVAL;
    const size_t lds = static_cast<size_t>(s.max_slots) * unroll * kLanes * 16;

    KernelFn fn = pick_kernel(dtype, unroll);
    int& cached = h->occupancy[dtype == BLINK_FP32][unroll == 1 ? 0 : (unroll == 2 ? 1 : 2)];
    if (cached == 0) {
        BLINK_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&cached, fn, kLanes, lds));
        if (cached < 1) {
            cached = 0;
            return BLINK_EHIP;
        }
    }
    int per_cu = cached;
    if (h->wg_per_cu > 0) per_cu = std::min(per_cu, h->wg_per_cu);
    const unsigned long long grid =
        std::min<unsigned long long>(static_cast<unsigned long long>(per_cu) * h->n_cu, n_items);

    KParams p{};
    for (int i = 0; i < k; ++i) p.buf[i] = bufs[i];
    p.tmpl = static_cast<const StageTmpl*>(h->d_tmpl);
    p.inst = static_cast<const StageInst*>(h->d_inst);
    p.done = static_cast<unsigned long long*>(h->d_counters) + 1;
    p.ticket = static_cast<unsigned long long*>(h->d_counters);
    p.ticket_base = h->ticket_base;
    p.n_items = n_items;
    p.epoch = ++h->epoch;
    p.tiles_per_chunk = tiles_per_chunk;
    hipLaunchKernelGGL(fn, dim3(static_cast<unsigned>(grid)), dim3(kLanes), lds,
                       static_cast<hipStream_t>(stream), p);
    BLINK_HIP(hipGetLastError());
    h->ticket_base += n_items + grid;  // every workgroup draws exactly one ticket past the end
    h->last_grid = static_cast<unsigned>(grid);
    h->last_unroll = unroll;
    return BLINK_OK;
}

}  // namespace blink
