// The schedule handle: host-side schedule plus the device-side tables and
// progress counters the kernel uses.
#pragma once
#include <cstdint>

#include "schedule.hpp"

struct blink_schedule {
    blink::Schedule s;
    int device = -1;              // HIP device holding the tables; -1 = not uploaded yet
    void* d_tmpl = nullptr;       // StageTmpl[]
    void* d_inst = nullptr;       // StageInst[]
    void* d_counters = nullptr;   // u64 ticket counters, then one u64 of finished tiles per instance
    uint64_t epoch = 0;           // calls made so far; counters hold epoch * tiles
    uint64_t ticket_base[16] = {};  // value of each ticket counter when the next call starts
    int n_cu = 0;
    int wg_per_cu = 0;            // launch override (0 = automatic)
    unsigned tile_override = 0;   // elements per tile requested by the caller (0 = automatic)
    unsigned tile_elems = 0;      // elements per tile in use (0 = not chosen yet)
    bool tile_final = false;      // tile_elems has had its small-payload adjustment
    bool wide = false;            // small payload: use every wave that fits
    int occupancy[2] = {0, 0};    // waves per CU, cached per dtype
    unsigned last_grid = 0;
};

namespace blink {
blink_status_t execute(blink_schedule* h, void* const* bufs, int k, size_t n, blink_dtype_t dtype,
                       blink_op_t op, blink_redop_t redop, void* stream);
blink_status_t reset_progress(blink_schedule* h);
void release_device_state(blink_schedule* h);
}  // namespace blink
