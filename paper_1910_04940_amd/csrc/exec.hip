// The launcher of the persistent kernel (see kernel.hpp): the device block of a
// schedule (status record, progress counters, tables), the launch plan (tile
// size, kernel flavour), the launch and its bookkeeping.
#include "stream.hpp"

#include <atomic>
#include <mutex>

namespace blink {

constexpr uint64_t kMemorySideCacheBytes = 256ull << 20;

// ---- a device block that needs no allocation ------------------------------------------
// For callers that may not allocate (a stream under HIP graph capture, a tight
// serving loop, a harness that forbids it): a block of fixed size in the
// library's own device image.  Every GPU the library runs on holds its own copy
// of the array, at its own address, until the process ends; host code reaches
// it only through the address hipGetSymbolAddress returns with that GPU current
// (the array's name in host code is a host-side stand-in, not a device address).
// All calls of blink_allreduce_noalloc on one GPU share that GPU's block.
constexpr size_t kStaticBlockBytes = 4u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticBlockBytes];

namespace {
constexpr int kMaxDevices = 64;
struct StaticBlock {
    char* ptr = nullptr;   // device address of `scratch` on this GPU
    uint64_t owner = 0;    // id of the schedule whose tables the block holds (0 = none)
};
StaticBlock g_static[kMaxDevices];
std::mutex g_static_mutex;
std::atomic<uint64_t> g_next_id{1};

// Zeroes `words` 64-bit words (a fill kernel rather than hipMemsetAsync, which
// must not be recorded into a captured graph).
__global__ __launch_bounds__(256) void blink_clear(unsigned long long* p, unsigned long long words) {
    for (unsigned long long i = blockIdx.x * 256ull + threadIdx.x; i < words; i += gridDim.x * 256ull) p[i] = 0;
}
}  // namespace

uint64_t next_schedule_id() { return g_next_id.fetch_add(1); }

// ---- host side ------------------------------------------------------------------------
namespace {

void drop_trial_events(blink_schedule* h);  // below, with the choice among the ways to serve a schedule

#define BLINK_HIP(call)                                                                   \
    do {                                                                                  \
        hipError_t err__ = (call);                                                        \
        if (err__ != hipSuccess) {                                                        \
            std::fprintf(stderr, "blink: %s failed: %s\n", #call, hipGetErrorString(err__)); \
            return err__ == hipErrorOutOfMemory ? BLINK_ENOMEM : BLINK_EHIP;              \
        }                                                                                 \
    } while (0)

KernelFn pick_kernel(blink_dtype_t dtype, int flavour, bool many_waves, bool direct) {
    if (dtype == BLINK_FP32) return many_waves ? kernel_f32_many(flavour) : kernel_f32_stream(flavour, direct);
    return many_waves ? kernel_i32_many(flavour) : kernel_i32_stream(flavour, direct);
}

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

BlockLayout layout_of(const Schedule& s) {
    constexpr size_t kLine = static_cast<size_t>(kCounterStride) * sizeof(unsigned long long);
    BlockLayout l;
    l.ticket = static_cast<size_t>(kStatusWords) * sizeof(unsigned long long);
    l.done = l.ticket + kMaxQueues * kLine;
    l.counters_end = l.done + s.inst.size() * kLine;
    l.tmpl = round_up(l.counters_end, 256);
    l.inst = round_up(l.tmpl + s.tmpl.size() * sizeof(StageTmpl), 256);
    l.bytes = round_up(l.inst + s.inst.size() * sizeof(StageInst), 256);
    return l;
}

// Fill a block that lives at `block` on the current device: zero the status
// record and the counters, copy the tables.  Synchronous.
blink_status_t fill_block(const Schedule& s, const BlockLayout& l, char* block) {
    BLINK_HIP(hipMemset(block, 0, l.counters_end));
    BLINK_HIP(hipMemcpy(block + l.tmpl, s.tmpl.data(), s.tmpl.size() * sizeof(StageTmpl), hipMemcpyHostToDevice));
    BLINK_HIP(hipMemcpy(block + l.inst, s.inst.data(), s.inst.size() * sizeof(StageInst), hipMemcpyHostToDevice));
    BLINK_HIP(hipDeviceSynchronize());
    return BLINK_OK;
}

// The schedule's own block: one allocation, made at the first call on a device.
// Nothing is left behind when a step fails.
blink_status_t upload(blink_schedule* h) {
    int dev = -1;
    BLINK_HIP(hipGetDevice(&dev));
    if (h->device == dev) return BLINK_OK;
    if (h->device >= 0) return BLINK_EMISMATCH;  // the block lives on another device
    const BlockLayout l = layout_of(h->s);
    void* block = nullptr;
    BLINK_HIP(hipMalloc(&block, l.bytes));
    const blink_status_t st = fill_block(h->s, l, static_cast<char*>(block));
    if (st != BLINK_OK) {
        (void)hipFree(block);
        return st;
    }
    h->d_block = block;
    h->device = dev;
    h->epoch = 0;
    for (uint64_t& b : h->ticket_base) b = 0;
    return BLINK_OK;
}

// The current device's static block, holding the tables of `h`.  The address is
// looked up once per device.  The tables are copied in when the block last
// held another schedule's (synchronously, after waiting for `stream`, whose
// earlier calls may still be reading the old ones).  Allocates nothing.
blink_status_t claim_static_block(blink_schedule* h, const BlockLayout& l, hipStream_t stream, char** out) {
    int dev = -1;
    BLINK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return BLINK_ELIMIT;
    if (l.bytes > kStaticBlockBytes) {
        std::fprintf(stderr, "blink: the schedule needs a device block of %zu bytes, the static one has %zu\n",
                     l.bytes, kStaticBlockBytes);
        return BLINK_ELIMIT;
    }
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticBlock& sb = g_static[dev];
    if (!sb.ptr) {
        char* ptr = nullptr;
        BLINK_HIP(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
        if (!ptr) return BLINK_EHIP;
        sb.ptr = ptr;
    }
    if (sb.owner != h->id) {
        // waiting and copying are not things a capturing stream can record
        hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream, &capture) != hipSuccess) {
            (void)hipGetLastError();
        } else if (capture != hipStreamCaptureStatusNone) {
            std::fprintf(stderr, "blink: the stream is capturing and the static block holds another schedule's tables; "
                                 "call blink_allreduce_noalloc on this schedule once before the capture\n");
            return BLINK_EINVAL;
        }
        sb.owner = 0;
        BLINK_HIP(hipStreamSynchronize(stream));
        BLINK_HIP(hipMemcpy(sb.ptr + l.tmpl, h->s.tmpl.data(), h->s.tmpl.size() * sizeof(StageTmpl), hipMemcpyHostToDevice));
        BLINK_HIP(hipMemcpy(sb.ptr + l.inst, h->s.inst.data(), h->s.inst.size() * sizeof(StageInst), hipMemcpyHostToDevice));
        sb.owner = h->id;
    }
    h->last_static_device = dev;
    *out = sb.ptr;
    return BLINK_OK;
}

// Tickets of a schedule whose tile grid is moved down by grid_shift elements.
void count_tickets(blink_schedule* h, uint32_t grid_shift) {
    LaunchPlan& pl = h->plan;
    pl.n_items = ticket_count(h->s, ticket_group(h->s), pl.tile_shift, grid_shift, &pl.tiles_per_chunk);
    pl.n_items_turns = ticket_count(h->s, 1, pl.tile_shift, grid_shift, &pl.tiles_per_chunk);
    pl.grid_shift = grid_shift;
}

// Tile size, kernel flavour and ticket count of a schedule on this device.
//
// The tile is large enough that a ticket moves about kTicketBytes.  A payload
// too small to give a streaming grid 16 such tickets per CU is latency-bound
// instead ("wide"): then all the waves that fit are used and the tile shrinks
// (see below).  (Measured on 8 ranks, 4 trees, when the threshold was set, with
// one wave per SIMD: at 11 tickets per CU the wide launch took 52 us and the
// streaming one 72, at 16 they tied at 79, at 18 it was 157 against 130.  With
// two waves per SIMD the wide launch wins by more below the threshold and still
// loses above it: 10 M elements per rank 132 us against 121.)
blink_status_t make_plan(blink_schedule* h, blink_dtype_t dtype) {
    LaunchPlan& pl = h->plan;
    if (pl.made) return BLINK_OK;
    const Schedule& s = h->s;
    if (h->n_cu == 0) {
        int dev = -1, n_cu = 0;
        BLINK_HIP(hipGetDevice(&dev));
        BLINK_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
        if (n_cu < 1) return BLINK_EHIP;
        h->n_cu = n_cu;
    }
    uint64_t work = 0;  // elements x stages
    for (const StageInst& in : s.inst) work += in.len;
    const uint64_t bytes_per_elem = std::max<uint64_t>(1, s.traffic_bytes / std::max<uint64_t>(1, work));
    // the power of two nearest (in ratio) to ticket bytes / bytes_per_elem
    const uint64_t ticket_bytes = s.has_deps ? kTicketBytesHandOver : kTicketBytes;
    unsigned tile = kMinTile;
    while (tile < kMaxTile && 2ull * tile * tile * bytes_per_elem * bytes_per_elem < ticket_bytes * ticket_bytes)
        tile *= 2;
    pl.wide = work / tile < 16ull * h->n_cu;

    const uint64_t write_bytes = s.traffic_bytes - s.read_bytes;
    pl.read_heavy = s.read_bytes >= 2 * write_bytes;
    const bool write_heavy = write_bytes >= 2 * s.read_bytes;
    // Rank buffers that together fit the memory-side cache (256 MiB) are written
    // without the streaming hint: whoever reads the result next (here: the next
    // call) finds it there (8 x 16 MiB: 62 -> 45 us per call).  That is the
    // read-heavy policy.  Larger buffers get it too where calls alternate their
    // direction: a call then starts on the last 256 MiB that the call before it
    // wrote (standalone probe, same kernel structure, repeated in place: 3 ranks x
    // 128 MiB 0.75 -> 0.83 of the HBM peak, 8 x 64 MiB 0.72 -> 0.81, 8 x 256 MiB
    // 0.774 -> 0.787; without the alternation the two policies tie).
    const bool fits_cache = static_cast<uint64_t>(s.k) * s.n * 4 <= kMemorySideCacheBytes;
    pl.flavour = s.has_deps   ? kHandOver
                 : write_heavy ? kWriteHeavy
                 : (pl.read_heavy || fits_cache || h->sweep_alternates) ? kReadHeavy
                                                                        : kBalanced;
    if (pl.wide) {
        int& occ = h->occupancy[dtype == BLINK_FP32][0];
        if (occ == 0) {
            BLINK_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, pick_kernel(dtype, pl.flavour, true, false), kLanes, 0));
            if (occ < 1) {
                occ = 0;
                return BLINK_EHIP;
            }
        }
        // Where stages wait for one another only one time slot's worth of the
        // work can run at a time: the tile shrinks until a slot has about 64
        // tiles, not until half the machine has one (waves beyond what a slot
        // can use do nothing but poll: 4 ranks x 64 Ki elements per edge,
        // 42 -> see the measurements).
        if (s.has_deps)
            while (tile > kMinTile && work / s.n_slots / tile < 64) tile /= 2;
        else {
            // Without dependencies the tickets of such a payload are dealt out in
            // rounds over the waves that fit (drawn, so many small ones would queue
            // at the counter; see execute), and the call lasts as long as the wave
            // with most of them: a tile size costs its rounds times the tile plus
            // what a ticket costs besides its elements (about 2.5 us of latencies,
            // the time in which a wave among a thousand moves 15 KB).
            // Measured, 8 ranks x 4 trees on 1,024 waves, 2,048 -> 1,024-element
            // tiles: 2.7 M elements per rank (1.3 -> 2.6 tickets per wave) 43.8 ->
            // 38.4 us, 4.2 M (2.0 -> 4.0) 59.7 -> 52.7 us, but 3.2 M (1.5 -> 3.05)
            // 42.9 -> 43.3 us: the last round counts whole.
            const uint64_t waves = static_cast<uint64_t>(occ) * h->n_cu;
            unsigned best = tile;
            uint64_t best_cost = ~0ull;
            for (unsigned cand = tile; cand >= kMinTile; cand /= 2) {
                unsigned shift = 0;
                while ((1u << shift) < cand) ++shift;
                uint32_t most = 0;
                const uint64_t tickets = ticket_count(s, ticket_group(s), shift, 0, &most);
                if (tickets / std::min(waves, tickets) > 4) break;  // these would be drawn
                const uint64_t rounds = (tickets + waves - 1) / waves;
                const uint64_t cost = rounds * (cand + 15360 / bytes_per_elem);
                if (cost < best_cost) {
                    best = cand;
                    best_cost = cost;
                }
            }
            tile = best;
        }
    }
    // The streaming kernel (stream.hpp) takes schedules without dependencies all
    // of whose stages have a stack program within its limits.
    pl.direct = !pl.wide && !s.has_deps;
    for (const StageTmpl& st : s.tmpl)
        if (st.seq_depth < 1 || st.seq_depth > stream_stack_limit(st.n_load)) pl.direct = false;
    if (h->tile_override) tile = h->tile_override;
    pl.tile_elems = tile;
    pl.tile_shift = 0;
    while ((1u << pl.tile_shift) < tile) ++pl.tile_shift;
    pl.made = true;
    count_tickets(h, 0);
    return BLINK_OK;
}

}  // namespace

// Forget all progress and the status record, and let the next call plan its
// launch afresh (used when the tile size changes: counters of earlier calls were
// counted in other units; and to recover after a wait was abandoned).  Waits for
// the device first.
blink_status_t reset_progress(blink_schedule* h) {
    h->epoch = 0;
    for (uint64_t& b : h->ticket_base) b = 0;
    h->plan = LaunchPlan();
    for (auto& per_dtype : h->occupancy) per_dtype[0] = per_dtype[1] = 0;
    drop_trial_events(h);
    h->picked = 0;
    h->trial_calls = 0;
    if (h->device < 0) return BLINK_OK;
    BLINK_HIP(hipDeviceSynchronize());
    BLINK_HIP(hipMemset(h->d_block, 0, layout_of(h->s).counters_end));
    BLINK_HIP(hipDeviceSynchronize());
    return BLINK_OK;
}

// Wait for the device, then report what the status record of the block says.
blink_status_t read_status(blink_schedule* h, blink_progress_t* out) {
    *out = blink_progress_t{};
    out->stage = out->awaited_stage = -1;
    const void* block = h->d_block;
    if (h->last_static_device >= 0) {  // the latest call ran on a static block: report on that one
        int dev = -1;
        BLINK_HIP(hipGetDevice(&dev));
        std::lock_guard<std::mutex> lock(g_static_mutex);
        if (dev != h->last_static_device || g_static[dev].owner != h->id) return BLINK_OK;  // record gone
        block = g_static[dev].ptr;
    } else if (h->device < 0) {
        return BLINK_OK;  // never ran: nothing can have gone wrong
    }
    unsigned long long rec[kStatusWords] = {};
    BLINK_HIP(hipDeviceSynchronize());
    BLINK_HIP(hipMemcpy(rec, block, sizeof rec, hipMemcpyDeviceToHost));
    out->state = static_cast<int32_t>(rec[kStatusState]);
    if (rec[kStatusState] == 0) return BLINK_OK;
    out->stage = static_cast<int32_t>(rec[kStatusStage]);
    out->awaited_stage = static_cast<int32_t>(rec[kStatusAwaited]);
    out->seen = rec[kStatusSeen];
    out->wanted = rec[kStatusWanted];
    out->call = rec[kStatusCall];
    return BLINK_ESTUCK;
}

// Picking how a schedule is served.  A schedule without dependencies at
// streaming size can run in up to three ways: on blink_consume (1), on
// blink_stream where the operator is the sum and the stages fit it (2), and,
// with several trees, on blink_consume with the trees taking turns chunk by
// chunk instead of tile by tile (3).  Which is fastest depends on where the
// buffers lie in HBM and how far apart the trees' shares are, in ways addresses
// do not reveal: 1 wins on most placements and by far where the shares are a
// power of two apart (8 x 256 MiB: 0.79 of the HBM peak against 0.73 for 3),
// 2 is steadier where rank buffers are badly placed, 3 where the shares are
// (8 x 117 MiB: 0.66 for 1, 0.73 for 3; sixteen gradient buckets of 64 KiB to
// 400 MiB: 0.665 -> 0.69 overall).  So the first calls on such a schedule go
// round the candidates, kTrialSamples times each, each call timed with a pair
// of events on the caller's stream; the next call waits for the last of them
// (the one time a call waits for the device, besides a schedule's first) and
// the candidate with the smallest minimum serves the rest.  All give the same
// bits.
constexpr int kTrialSamples = 4;
constexpr uint64_t kTrialMinBytes = 64ull << 20;  // smaller calls are too short to time against one another

namespace {
void drop_trial_events(blink_schedule* h) {
    for (void*& e : h->trial_event) {
        if (e) (void)hipEventDestroy(static_cast<hipEvent_t>(e));
        e = nullptr;
    }
    h->trial_events_made = false;
}

// How this call is served (1, 2 or 3, see above); *timed: index of the event
// pair to put around it, or -1.  streams: the schedule can run on blink_stream;
// can_stream: this call can (its operator is the sum); can_turns: way 3 exists.
int choose_kernel(blink_schedule* h, bool static_block, bool streams, bool can_stream, bool can_turns, int* timed) {
    *timed = -1;
    auto allowed = [&](int way) { return way == 1 || (way == 2 && can_stream) || (way == 3 && can_turns); };
    if (h->kernel_choice) return allowed(h->kernel_choice) ? h->kernel_choice : 1;
    if (h->picked) return allowed(h->picked) ? h->picked : 1;
    int ways[3], n_ways = 0;
    ways[n_ways++] = 1;
    if (streams) ways[n_ways++] = 2;
    if (can_turns) ways[n_ways++] = 3;
    // no trial: one way only / nothing may be created here / too short / a call
    // with another operator than the schedule's trial is held with
    if (n_ways == 1 || static_block || h->s.traffic_bytes < kTrialMinBytes || (streams && !can_stream)) return 1;
    const int trial_calls = n_ways * kTrialSamples;
    if (h->trial_calls < trial_calls) {
        if (!h->trial_events_made) {
            for (int e = 0; e < 2 * trial_calls; ++e) {
                hipEvent_t ev = nullptr;
                if (hipEventCreate(&ev) != hipSuccess) {
                    (void)hipGetLastError();
                    drop_trial_events(h);
                    h->picked = 1;
                    return 1;
                }
                h->trial_event[e] = ev;
            }
            h->trial_events_made = true;
        }
        *timed = h->trial_calls;
        return ways[h->trial_calls % n_ways];
    }
    // All trial calls are launched: wait for the last of them (once per
    // schedule) and compare the fastest of each candidate's calls but its first
    // (which carries what happens once: the code's first launch, tables not yet
    // in any cache).  Kernels of a tenth of a millisecond differ by a few
    // percent, which is also what the event pair around a single launch
    // scatters by: hence three samples each, not one.
    float best[3] = {1e30f, 1e30f, 1e30f};
    bool ok = hipEventSynchronize(static_cast<hipEvent_t>(h->trial_event[2 * trial_calls - 1])) == hipSuccess;
    for (int c = 0; ok && c < trial_calls; ++c) {
        float ms = 0.f;
        ok = hipEventElapsedTime(&ms, static_cast<hipEvent_t>(h->trial_event[2 * c]),
                                 static_cast<hipEvent_t>(h->trial_event[2 * c + 1])) == hipSuccess;
        if (c >= n_ways) best[c % n_ways] = std::min(best[c % n_ways], ms);
    }
    if (!ok) (void)hipGetLastError();
    // The first way keeps the schedule unless another beats it by more than the
    // 2 % by which such minima scatter from one trial to the next.
    int fastest = 0;
    float bar = best[0] * 0.98f;
    for (int w = 1; ok && w < n_ways; ++w)
        if (best[w] < bar) {
            fastest = w;
            bar = best[w];
        }
    h->picked = ways[fastest];
    drop_trial_events(h);
    return h->picked;
}
}  // namespace

void release_device_state(blink_schedule* h) {
    drop_trial_events(h);
    if (h->device < 0) return;
    (void)hipFree(h->d_block);
    h->d_block = nullptr;
    h->device = -1;
}

blink_status_t execute(blink_schedule* h, void* const* bufs, int k, size_t n, blink_dtype_t dtype,
                       blink_op_t op, blink_redop_t redop, void* stream, bool static_block) {
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
    const BlockLayout l = layout_of(s);
    char* block = nullptr;
    if (static_block) {
        if (blink_status_t st = claim_static_block(h, l, static_cast<hipStream_t>(stream), &block)) return st;
    } else {
        // A launch carries the call's number on its schedule and the place its
        // ticket counters have reached; replayed from a HIP graph it would carry
        // them again and find the counters elsewhere: waves would draw nothing
        // and stages would not wait.  Say so instead of recording such a launch.
        hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(static_cast<hipStream_t>(stream), &capture) != hipSuccess) {
            (void)hipGetLastError();  // not this call's business: the launch will report a bad stream
        } else if (capture != hipStreamCaptureStatusNone) {
            std::fprintf(stderr, "blink: the stream is capturing; only blink_allreduce_noalloc can be recorded into a HIP graph\n");
            return BLINK_EINVAL;
        }
        if (blink_status_t st = upload(h)) return st;
        block = static_cast<char*>(h->d_block);
        h->last_static_device = -1;
    }
    if (blink_status_t st = make_plan(h, dtype)) return st;
    // Rank buffers that all start the same distance past a 1 KiB boundary (views
    // into larger buffers, allocations at 512-byte granularity): the tile grid
    // is moved down by that distance, so that tiles, and with them the 1 KiB
    // accesses of a wave, start on such boundaries in memory.  Only where no
    // stage waits for another: there a tile is nothing but a range of elements;
    // with dependencies finished tiles are counted, per call number, and the
    // count of an instance must not change from call to call.
    uint32_t grid_shift = 0;
    if (!s.has_deps) {
        const uintptr_t past = reinterpret_cast<uintptr_t>(bufs[0]) & 1023u;
        bool common = true;
        for (int i = 1; i < k; ++i) common = common && (reinterpret_cast<uintptr_t>(bufs[i]) & 1023u) == past;
        if (common) grid_shift = static_cast<uint32_t>(past / 4);
    }
    if (grid_shift != h->plan.grid_shift) count_tickets(h, grid_shift);
    const LaunchPlan& pl = h->plan;

    int timed = -1;
    const unsigned full_group = ticket_group(s);
    const int way = choose_kernel(h, static_block, pl.direct, pl.direct && redop == BLINK_SUM,
                                  !pl.wide && !s.has_deps && full_group > 1, &timed);
    const bool direct = way == 2;
    KernelFn fn = pick_kernel(dtype, pl.flavour, pl.wide, direct);
    int& occ = h->occupancy[dtype == BLINK_FP32][direct];
    if (occ == 0) {
        BLINK_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, fn, kLanes, 0));
        if (occ < 1) {
            occ = 0;
            return BLINK_EHIP;
        }
    }
    // Waves per CU.  blink_stream: 2, each with 64 KiB of loads in flight (all
    // that fit).  blink_consume: 2 waves with 32 KiB each; 3 where reads dominate
    // or where a stage reads more than 8 ranks (only 2 columns per rank fit
    // then); 4 where stages wait for one another (some waves always wait; 8 x
    // 256 MiB per node 1.088 -> 1.023 ms, per edge 1.242 -> 1.230); 1 where writes dominate (Broadcast,
    // AllGather: a wave's sub-tile is then one read and seven writes of 16 KiB
    // each, and a second wave per CU only adds to the queue of stores; 8 ranks,
    // Broadcast: 8 x 64 MiB 83 -> 71 us, 8 x 256 MiB 300 -> 271 us; AllGather
    // 81 -> 73 us and 312 -> 302 us).
    const bool write_heavy = pl.flavour == kWriteHeavy;
    int per_cu = std::min(occ, direct ? 2 : write_heavy ? 1 : s.has_deps ? 4 : (pl.read_heavy || s.max_slots > 8 ? 3 : 2));
    if (h->wg_per_cu > 0) per_cu = std::min(occ, h->wg_per_cu);
    if (pl.wide && h->wg_per_cu == 0) per_cu = occ;
    unsigned long long max_grid = static_cast<unsigned long long>(per_cu) * h->n_cu;
    const unsigned long long n_items = way == 3 ? pl.n_items_turns : pl.n_items;
    // with dependencies no more waves than three time slots' worth of tickets can be busy
    if (s.has_deps) max_grid = std::min(max_grid, std::max<unsigned long long>(64, 3 * (n_items / s.n_slots + 1)));
    const unsigned long long grid = std::min<unsigned long long>(max_grid, n_items);

    KParams p{};
    for (int i = 0; i < k; ++i) p.buf[i] = bufs[i];
    p.tmpl = reinterpret_cast<const StageTmpl*>(block + l.tmpl);
    p.inst = reinterpret_cast<const StageInst*>(block + l.inst);
    p.done = reinterpret_cast<unsigned long long*>(block + l.done);
    p.ticket = reinterpret_cast<unsigned long long*>(block + l.ticket);
    p.status = reinterpret_cast<unsigned long long*>(block);
    p.wait_ticks = (h->wait_limit_us ? h->wait_limit_us : kDefaultWaitMicroseconds) * kTicksPerMicrosecond;
    const unsigned n_queues =
        static_cast<unsigned>(std::min<unsigned long long>(s.has_deps ? kQueuesHandOver : 1, grid));
    p.n_queues = n_queues;
    // A static block is shared by every schedule used on the GPU and keeps the
    // last call's contents: each call on it starts from cleared counters, as
    // call number 1.  The schedule's own block counts on from call to call.
    for (unsigned q = 0; q < n_queues; ++q) p.ticket_base[q] = static_block ? 0 : h->ticket_base[q];
    p.n_items = n_items;
    // A dependency-free schedule with at most four tickets per wave is dealt out
    // statically, without the counter (see the kernel).  Larger ones draw their
    // tickets: waves then advance as one compact front through memory, which
    // DRAM likes better (measured: 0.71 ms against 0.79 ms on the 256 MiB case);
    // but every wave's first ticket is its own number: drawn, the first tickets
    // of 512 waves queue at the counter for up to 8 us (4.4 us on average, seen
    // with a clock in every wave), which is 2 % of a 200 us call.  blink_stream
    // knows all or nothing.  With dependencies every ticket must come from the
    // counter: only then is a ticket's holder known to be running.
    const unsigned long long static_items =
        s.has_deps ? 0 : (n_items / grid <= 4 ? n_items : (direct ? 0 : grid));
    p.static_items = static_items;
    p.epoch = static_block ? 1 : h->epoch + 1;
    p.tiles_per_chunk = pl.tiles_per_chunk;
    p.tile_shift = pl.tile_shift;
    p.redop = static_cast<unsigned>(redop);
    p.group = way == 3 ? 1u : full_group;
    p.grid_shift = pl.grid_shift;
    p.n_inst = static_cast<unsigned>(s.inst.size());
    // Calls on a schedule without dependencies sweep the payload in alternating
    // directions (the second, fourth, ... call backwards), unless switched off.
    p.reverse = !s.has_deps && !static_block && h->sweep_alternates && (p.epoch & 1) == 0;
    // Waiting waves look at their dependency every ~0.2 us in small schedules,
    // where a hand-over is most of the time (16 one-hop trees, 256 elements,
    // per-edge: 47 -> 36 us), and back off to ~0.8 us in large ones.
    p.max_naps = pl.wide ? 1 : 4;

    // The launch's own status decides whether the call counts: an error some
    // earlier HIP call of this thread left behind is not this launch's, and a
    // launch that failed must not consume a call number or move the ticket
    // bases (the next call would wait for tiles that nobody ever counted).
    if (static_block) {
        unsigned long long* words = reinterpret_cast<unsigned long long*>(block);
        unsigned long long n_words = l.counters_end / sizeof(unsigned long long);
        void* clear_args[] = {&words, &n_words};
        const unsigned clear_grid = static_cast<unsigned>(std::min<unsigned long long>((n_words + 255) / 256, 1024));
        const hipError_t cleared = hipLaunchKernel(reinterpret_cast<const void*>(blink_clear), dim3(clear_grid), dim3(256),
                                                   clear_args, 0, static_cast<hipStream_t>(stream));
        if (cleared != hipSuccess) {
            std::fprintf(stderr, "blink: kernel launch failed: %s\n", hipGetErrorString(cleared));
            (void)hipGetLastError();
            return BLINK_EHIP;
        }
    }
    void* args[] = {&p};
    if (timed >= 0 && hipEventRecord(static_cast<hipEvent_t>(h->trial_event[2 * timed]),
                                     static_cast<hipStream_t>(stream)) != hipSuccess) {
        (void)hipGetLastError();  // e.g. a capturing stream: give the trial up
        drop_trial_events(h);
        h->picked = 1;
        timed = -1;
    }
    const hipError_t launched = hipLaunchKernel(reinterpret_cast<const void*>(fn), dim3(static_cast<unsigned>(grid)),
                                                dim3(kLanes), args, 0, static_cast<hipStream_t>(stream));
    if (launched != hipSuccess) {
        std::fprintf(stderr, "blink: kernel launch failed: %s\n", hipGetErrorString(launched));
        (void)hipGetLastError();  // the failed launch's error is reported here, not left for later calls
        return BLINK_EHIP;
    }
    if (timed >= 0) {
        if (hipEventRecord(static_cast<hipEvent_t>(h->trial_event[2 * timed + 1]), static_cast<hipStream_t>(stream)) ==
            hipSuccess) {
            h->trial_calls += 1;
        } else {
            (void)hipGetLastError();
            drop_trial_events(h);
            h->picked = 1;
        }
    }
    h->last_grid = static_cast<unsigned>(grid);
    h->last_kernel = way;
    if (static_block) return BLINK_OK;
    h->epoch += 1;
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
