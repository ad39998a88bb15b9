// The schedule handle: host-side schedule, the launch plan derived from it, and
// the device-side block (status record, progress counters, tables) the kernel uses.
#pragma once
#include <cstddef>
#include <cstdint>

#include "schedule.hpp"

namespace blink {

// What a launch needs besides the schedule itself.  It depends only on the
// schedule, the device and the caller's overrides, so it is worked out once, at
// the first call, and kept until an override changes (the progress counters
// count tiles, so the tile size may not change while they hold progress).
struct LaunchPlan {
    bool made = false;
    bool wide = false;             // small payload: use every wave that fits
    int flavour = 0;               // cache policy of the kernel (see kernel.hpp)
    unsigned tile_elems = 0;       // elements per tile
    unsigned tile_shift = 0;       // log2 of it
    uint32_t tiles_per_chunk = 1;  // most tiles any stage instance has
    uint32_t grid_shift = 0;       // elements the tile grid is moved down by (see execute)
    uint64_t n_items = 0;          // tickets per call
    uint64_t n_items_turns = 0;    // the same when the trees take turns chunk by chunk (group 1)
    bool read_heavy = false;
    bool direct = false;           // the schedule CAN run on the streaming kernel (stream.hpp)
};

// Layout of the device block of a schedule, in bytes from its start:
//   status record (kStatusWords 64-bit words), ticket counters, one counter of
//   finished tiles per stage instance (counters kCounterStride words apart),
//   stage templates, stage instances.
struct BlockLayout {
    size_t ticket = 0, done = 0, tmpl = 0, inst = 0, bytes = 0;
    size_t counters_end = 0;  // status record and counters are [0, counters_end)
};

}  // namespace blink

struct blink_schedule {
    blink::Schedule s;
    blink::LaunchPlan plan;
    int device = -1;              // HIP device holding the block; -1 = not uploaded yet
    void* d_block = nullptr;      // see BlockLayout
    uint64_t id = 0;              // unique per handle (names the owner of a device's static block)
    uint64_t epoch = 0;           // calls made so far on d_block; its counters hold epoch * tiles
    uint64_t ticket_base[16] = {};  // value of each ticket counter when the next call starts
    uint64_t wait_limit_us = 0;   // longest wait for another stage; 0 = default
    int n_cu = 0;
    int wg_per_cu = 0;            // launch override (0 = automatic)
    unsigned tile_override = 0;   // elements per tile requested by the caller (0 = automatic)
    int occupancy[2][2] = {};     // waves per CU of the kernel in use, per dtype and per (streaming kernel or not)
    unsigned last_grid = 0;
    int last_kernel = 0;          // how the latest call ran: 1 = blink_consume, 2 = blink_stream, 3 = blink_consume, trees in turns
    int last_static_device = -1;  // device whose static block the latest call used; -1 = it used d_block
    // What serves a schedule that has the choice (see execute): blink_consume (1),
    // blink_stream (2), or blink_consume with the trees taking turns chunk by
    // chunk instead of tile by tile (3).
    int kernel_choice = 0;        // the caller's wish: 0 = pick the fastest, else one of the three
    bool sweep_alternates = true; // calls on a schedule without dependencies walk the tiles in alternating directions
    int picked = 0;               // the pick once made (1, 2 or 3); 0 = not yet
    int trial_calls = 0;          // timed calls launched so far (the candidates take turns)
    void* trial_event[24] = {};   // hipEvent_t pairs around the timed calls
    bool trial_events_made = false;
};

namespace blink {
// static_block: run on the device's file-scope block instead of the schedule's own.
blink_status_t execute(blink_schedule* h, void* const* bufs, int k, size_t n, blink_dtype_t dtype,
                       blink_op_t op, blink_redop_t redop, void* stream, bool static_block = false);
uint64_t next_schedule_id();
blink_status_t reset_progress(blink_schedule* h);
blink_status_t read_status(blink_schedule* h, blink_progress_t* out);
void release_device_state(blink_schedule* h);
}  // namespace blink
