// The launcher of the persistent kernel (see kernel.hpp): device-side tables and
// counters of a schedule, the choice of tile size, grid and kernel flavour, the launch.
#include "kernel.hpp"

namespace blink {

constexpr uint64_t kMemorySideCacheBytes = 256ull << 20;

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

KernelFn pick_kernel(blink_dtype_t dtype, int flavour, bool many_waves) {
    if (dtype == BLINK_FP32) return many_waves ? kernel_f32_many(flavour) : kernel_f32_stream(flavour);
    return many_waves ? kernel_i32_many(flavour) : kernel_i32_stream(flavour);
}

// kMaxQueues ticket counters, then one counter per stage instance, all kCounterStride words apart
size_t counter_bytes(const Schedule& s) {
    return (s.inst.size() + kMaxQueues) * static_cast<size_t>(kCounterStride) * sizeof(unsigned long long);
}

blink_status_t upload(blink_schedule* h) {
    int dev = -1;
    BLINK_HIP(hipGetDevice(&dev));
    if (h->device == dev) return BLINK_OK;
    if (h->device >= 0) return BLINK_EMISMATCH;  // tables live on another device
    const Schedule& s = h->s;
    BLINK_HIP(hipMalloc(&h->d_tmpl, s.tmpl.size() * sizeof(StageTmpl)));
    BLINK_HIP(hipMalloc(&h->d_inst, s.inst.size() * sizeof(StageInst)));
    BLINK_HIP(hipMalloc(&h->d_counters, counter_bytes(s)));
    BLINK_HIP(hipMemcpy(h->d_tmpl, s.tmpl.data(), s.tmpl.size() * sizeof(StageTmpl), hipMemcpyHostToDevice));
    BLINK_HIP(hipMemcpy(h->d_inst, s.inst.data(), s.inst.size() * sizeof(StageInst), hipMemcpyHostToDevice));
    BLINK_HIP(hipMemset(h->d_counters, 0, counter_bytes(s)));
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
    for (uint64_t& b : h->ticket_base) b = 0;
    h->tile_elems = 0;
    h->tile_final = false;
    if (h->device < 0) return BLINK_OK;
    BLINK_HIP(hipDeviceSynchronize());
    BLINK_HIP(hipMemset(h->d_counters, 0, counter_bytes(h->s)));
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
                       blink_op_t op, blink_redop_t redop, void* stream) {
    if (!h || !bufs) return BLINK_EINVAL;
    if (dtype != BLINK_FP32 && dtype != BLINK_INT32) return BLINK_EINVAL;
    if (redop != BLINK_SUM && redop != BLINK_PROD && redop != BLINK_MIN && redop != BLINK_MAX) return BLINK_EINVAL;
    const Schedule& s = h->s;
    if (k != s.k || n != s.n || op != s.op) return BLINK_EMISMATCH;
    if (n == 0) return BLINK_OK;  // nothing to move: the buffer pointers are not looked at
    for (int i = 0; i < k; ++i) {
        if (!bufs[i] || (reinterpret_cast<uintptr_t>(bufs[i]) & 15u)) return BLINK_EINVAL;
        for (int j = 0; j < i; ++j) {
            const char* a = static_cast<const char*>(bufs[i]);
            const char* b = static_cast<const char*>(bufs[j]);
            if (a < b + n * 4 && b < a + n * 4) return BLINK_EINVAL;
        }
    }
    if (s.inst.empty()) return BLINK_OK;
    if (blink_status_t st = upload(h)) return st;

    // Tile size, fixed at the first call (the progress counters count tiles):
    // large enough that a ticket moves about kTicketBytes.  A payload too small
    // to give a streaming grid a few dozen such tickets per CU is latency-bound
    // instead ("wide"): then all the waves that fit are used and the tile
    // shrinks until about every other wave has one.
    uint64_t work = 0;  // elements x stages
    if (!h->tile_final)
        for (const StageInst& in : s.inst) work += in.len;
    if (h->tile_elems == 0) {
        const uint64_t bytes_per_elem = std::max<uint64_t>(1, s.traffic_bytes / std::max<uint64_t>(1, work));
        // the power of two nearest (in ratio) to ticket bytes / bytes_per_elem
        const uint64_t ticket_bytes = s.has_deps ? kTicketBytesHandOver : kTicketBytes;
        unsigned tile = kMinTile;
        while (tile < kMaxTile && 2ull * tile * tile * bytes_per_elem * bytes_per_elem < ticket_bytes * ticket_bytes)
            tile *= 2;
        h->wide = work / tile < 24ull * h->n_cu;
        h->tile_elems = tile;
    }
    const uint64_t write_bytes = s.traffic_bytes - s.read_bytes;
    const bool read_heavy = s.read_bytes >= 2 * write_bytes, write_heavy = write_bytes >= 2 * s.read_bytes;
    // Rank buffers that together fit the memory-side cache (256 MiB) are written
    // without the streaming hint: whoever reads the result next (here: the next
    // call) finds it there (8 x 16 MiB: 62 -> 45 us per call; no change from
    // 8 x 64 MiB on, and a loss at 8 x 256 MiB).  That is the read-heavy policy.
    const bool fits_cache = static_cast<uint64_t>(k) * n * 4 <= kMemorySideCacheBytes;
    const int flavour = s.has_deps   ? kHandOver
                        : write_heavy ? kWriteHeavy
                        : (read_heavy || fits_cache) ? kReadHeavy
                                                     : kBalanced;
    KernelFn fn = pick_kernel(dtype, flavour, h->wide);
    int& cached = h->occupancy[dtype == BLINK_FP32];
    if (cached == 0) {
        BLINK_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&cached, fn, kLanes, 0));
        if (cached < 1) {
            cached = 0;
            return BLINK_EHIP;
        }
    }
    if (!h->tile_final) {
        unsigned tile = h->tile_elems;
        if (h->wide)
            while (tile > kMinTile && work / tile < static_cast<uint64_t>(cached) * h->n_cu / 2) tile /= 2;
        h->tile_elems = h->tile_override ? h->tile_override : tile;
        h->tile_final = true;
    }
    // A few waves per CU, each with 32 KiB of loads in flight, saturate HBM;
    // more waves only add ticket and polling traffic.  Measured best: 2, and 3
    // where reads dominate (Reduce: 8 ranks read, 1 written, 0.485 -> 0.412 ms),
    // where stages wait for one another, or where a stage reads more than 8
    // ranks (only 2 columns per rank fit then; 12 ranks: 5.14 -> 5.43 TB/s).
    int per_cu = std::min(cached, read_heavy || s.has_deps || s.max_slots > 8 ? 3 : 2);
    if (h->wg_per_cu > 0) per_cu = std::min(cached, h->wg_per_cu);
    if (h->wide && h->wg_per_cu == 0) per_cu = cached;
    const unsigned long long max_grid = static_cast<unsigned long long>(per_cu) * h->n_cu;
    const unsigned tile = h->tile_elems;
    unsigned tile_shift = 0;
    while ((1u << tile_shift) < tile) ++tile_shift;
    uint64_t tiles_per_chunk = 1;
    for (const StageInst& in : s.inst)
        tiles_per_chunk = std::max<uint64_t>(tiles_per_chunk, ((in.off + in.len + tile - 1) >> tile_shift) - (in.off >> tile_shift));
    const unsigned long long n_items = static_cast<unsigned long long>(s.inst.size()) * tiles_per_chunk;
    const unsigned long long grid = std::min<unsigned long long>(max_grid, n_items);

    KParams p{};
    for (int i = 0; i < k; ++i) p.buf[i] = bufs[i];
    p.tmpl = static_cast<const StageTmpl*>(h->d_tmpl);
    p.inst = static_cast<const StageInst*>(h->d_inst);
    p.done = static_cast<unsigned long long*>(h->d_counters) + kMaxQueues * kCounterStride;
    p.ticket = static_cast<unsigned long long*>(h->d_counters);
    const unsigned n_queues =
        static_cast<unsigned>(std::min<unsigned long long>(s.has_deps ? kQueuesHandOver : 1, grid));
    p.n_queues = n_queues;
    for (unsigned q = 0; q < n_queues; ++q) p.ticket_base[q] = h->ticket_base[q];
    p.n_items = n_items;
    // A dependency-free schedule with at most four tickets per wave is dealt out
    // statically, without the counter (see the kernel).  Larger ones draw every
    // ticket: waves then advance as one compact front through memory, which
    // DRAM likes better (measured: 0.71 ms against 0.79 ms on the 256 MiB case).
    // With dependencies every ticket must come from the counter: only then is
    // a ticket's holder known to be running.
    const unsigned long long static_items = (!s.has_deps && n_items / grid <= 4) ? n_items : 0;
    p.static_items = static_items;
    p.epoch = ++h->epoch;
    p.tiles_per_chunk = static_cast<unsigned>(tiles_per_chunk);
    p.tile_shift = tile_shift;
    p.redop = static_cast<unsigned>(redop);
    // Without dependencies the order of tiles is free: interleave the trees tile by tile.
    p.group = s.has_deps ? 1u : std::min(64u, std::max(1u, s.n_flows));
    // Waiting waves look at their dependency every ~0.2 us in small schedules,
    // where a hand-over is most of the time (16 one-hop trees, 256 elements,
    // per-edge: 47 -> 36 us), and back off to ~0.8 us in large ones.
    p.max_naps = h->wide ? 1 : 4;
    hipLaunchKernelGGL(fn, dim3(static_cast<unsigned>(grid)), dim3(kLanes), 0,
                       static_cast<hipStream_t>(stream), p);
    BLINK_HIP(hipGetLastError());
    if (static_items < n_items) {
        // queue q holds the drawn tickets q, q + n_queues, ...; every wave
        // draws exactly one ticket past the end of every queue
        const unsigned long long drawn = n_items - static_items;
        for (unsigned q = 0; q < n_queues; ++q)
            h->ticket_base[q] += (drawn + n_queues - 1 - q) / n_queues + grid;
    }
    h->last_grid = static_cast<unsigned>(grid);
    return BLINK_OK;
}

}  // namespace blink
