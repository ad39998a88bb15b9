// From weighted trees to what the kernel consumes (paper sections 3.3, 4.1,
// 4.2.1, 4.2.2): per-tree shares, chunks, the tree-edge step list, and the
// "stages" (one or several steps carried out in a single pass over a tile).
#pragma once
#include <cstdint>
#include <vector>

#include "trees.hpp"

namespace blink {

constexpr int kMaxOps = 40;    // micro-operations of one stage (<= 2k - 2 for k <= 16, see eval_tree)
constexpr int kMaxDeps = 8;    // stages one stage may wait for

// Micro-operations on the per-thread accumulator `acc` and the per-thread LDS
// slots (slot i initially holds what was loaded from rank load_rank[i]).
enum : uint8_t { OP_LD = 0, OP_ADD = 1, OP_ST = 2 };  // acc = slot; acc += slot; slot = acc
inline uint8_t make_op(uint8_t kind, uint8_t slot) { return static_cast<uint8_t>((kind << 6) | slot); }

// Shape of one stage, shared by all chunks of a tree.  Plain data: copied to the
// device as is; the kernel reads it as 32-bit words and picks bytes out of them.
struct alignas(4) StageTmpl {
    uint8_t n_load, n_op, n_store, n_dep;
    uint8_t signals;                 // some later stage waits for this one
    uint8_t level;                   // length of the longest dependency chain below it
    uint8_t pad[2];
    uint8_t load_rank[BLINK_MAX_RANKS];
    uint8_t store_rank[BLINK_MAX_RANKS];
    uint8_t op[kMaxOps];
    uint8_t dep_local[kMaxDeps];     // host only: index of the awaited stage among the tree's stages
    // The same micro-program as a stack program over the loaded ranks in the
    // order in which `op` consumes them (see stack_program): seq_rank[i] is the
    // i-th rank consumed, seq_code[i] = (folds << 1) | push.  seq_depth: the
    // accumulators it needs; 0 = `op` has no such form.
    uint8_t seq_rank[BLINK_MAX_RANKS];
    uint8_t seq_code[BLINK_MAX_RANKS];
    uint8_t seq_depth;
    uint8_t pad2[3];
};

// One stage applied to one chunk.  Plain data: copied to the device as is.
struct StageInst {
    uint64_t off;                    // first element
    uint32_t len;                    // elements (a chunk is < 2^32 elements)
    uint32_t tmpl;                   // index into the template table
    uint32_t n_dep;
    uint32_t pad;
    int32_t dep[kMaxDeps];           // indices of earlier instances
};
static_assert(sizeof(StageTmpl) % 4 == 0, "StageTmpl is read as 32-bit words");

// Rewrite st.op as a program for a stack of accumulators, which a kernel can
// run on registers alone: the ranks in the order in which they are consumed,
// each either starting a new accumulator on top of the stack (push) or being
// combined into the top one, followed by `folds` times "combine the top
// accumulator into the one below and drop it".  In `op` terms: LD pushes, ADD
// of a loaded slot combines, ST parks the top accumulator (it simply stays where
// it is while a later LD pushes above it) and ADD of a parked slot folds.  The
// association order is that of `op`; as there, only commutativity of the
// operator is used.  Fills seq_rank, seq_code, seq_depth (0 if `op` does not have
// this shape: a slot consumed twice or never, a fold that is not innermost).
void stack_program(StageTmpl& st);

// Where a stage instance belongs: the packed tree, the chunk inside the flow's
// range, and the flow (one tree carrying one contiguous range in one direction;
// the gathers have several flows per tree).
struct InstWhere {
    int tree, chunk, flow;
};

struct Schedule {
    int k = 0;
    int n_trees = 0;
    uint32_t n_flows = 0;                // (tree, range) pairs the stages were built for
    blink_op_t op = BLINK_OP_ALLREDUCE;
    blink_fusion_t fusion = BLINK_FUSE_EDGE;
    uint64_t n = 0, chunk = 0;
    uint64_t batch = 1;                  // chunks per tree that share a time slot of the step list (see instantiate)
    uint64_t n_slots = 1;                // time slots of the stage list (its stages, not the step list's)
    std::vector<uint64_t> bounds;        // T+1 share boundaries
    std::vector<blink_step_t> steps;     // public tree-edge step list, execution order
    std::vector<StageTmpl> tmpl;
    std::vector<StageInst> inst;         // execution (ticket) order; dependencies point backwards
    std::vector<InstWhere> inst_where;   // per instance: what it belongs to
    uint32_t max_slots = 1;              // largest n_load
    uint32_t max_stack = 0;              // most accumulators any stage's stack program needs (255: some stage has none)
    bool has_deps = false;               // some stage waits for another
    uint64_t traffic_bytes = 0;          // bytes read plus written in rank buffers per call
    uint64_t read_bytes = 0;             // the part of it that is read
};

// ---- the order in which the kernels hand out their work (section 4.2.2) ---------------
// A ticket is (stage instance, tile).  Instances come in the schedule's
// execution order (time slot = chunk + level, the trees taking turns inside a
// slot); `group` consecutive instances (the trees' turns at one chunk position)
// have their tiles handed out in turn, tile by tile across the instances, so
// that all trees advance together; group == 1 keeps an instance's tiles
// together.  Host and device use this one function.
#if defined(__HIP__) || defined(__HIPCC__)
#define BLINK_HOST_DEVICE __host__ __device__
#else
#define BLINK_HOST_DEVICE
#endif
BLINK_HOST_DEVICE inline void ticket_to_tile(unsigned long long t, unsigned group, unsigned tiles_per_chunk,
                                             unsigned n_inst, unsigned* instance, unsigned* tile) {
    const unsigned long long per_group = static_cast<unsigned long long>(group) * tiles_per_chunk;
    const unsigned first = static_cast<unsigned>(t / per_group) * group;
    const unsigned members = group < n_inst - first ? group : n_inst - first;
    const unsigned within = static_cast<unsigned>(t - static_cast<unsigned long long>(first) * tiles_per_chunk);
    *instance = first + within % members;
    *tile = within / members;
}

// `group` for a schedule.  Without dependencies the order of tiles is free: the
// trees are interleaved tile by tile, all of them while a stage reads at most 8
// ranks.  With more ranks per stage that makes too many request streams at a
// time (16 ranks x 16 one-hop trees = 256): there the trees take turns chunk by
// chunk (16 x 1 GiB: 5.5 -> 5.9 TB/s; two servers of 8: 5.7 -> 5.9).  With
// dependencies the tickets follow the execution order itself.
inline unsigned ticket_group(const Schedule& s) {
    if (s.has_deps || s.max_slots > 8) return 1u;
    return s.n_flows < 1u ? 1u : (s.n_flows > 64u ? 64u : s.n_flows);
}

// Number of tickets of a schedule for tiles of 2^tile_shift elements on a grid
// moved down by grid_shift elements, handed out in groups of `group` instances
// (see ticket_to_tile); *tiles_per_chunk receives the tile count
// of the instance that has most (every group of instances but the last gets
// that many tickets per member).  The last group gets only as many per member
// as its own largest instance has: with trees of equal weight every tree's
// short last chunk is there, and tickets that stand for nothing still cost
// their holder a trip to the counter (25.6 MB shares in 4 MiB chunks: an
// eighth of the tickets were such, and 8 % of the time).  Schedules with
// dependencies keep the full count: their groups are single instances.
inline uint64_t ticket_count(const Schedule& s, unsigned group, unsigned tile_shift, uint32_t grid_shift,
                             uint32_t* tiles_per_chunk) {
    const uint64_t tile = 1ull << tile_shift;
    auto tiles_of = [&](const StageInst& in) {
        return ((in.off + grid_shift + in.len + tile - 1) >> tile_shift) - ((in.off + grid_shift) >> tile_shift);
    };
    uint64_t most = 1;
    for (const StageInst& in : s.inst) most = most > tiles_of(in) ? most : tiles_of(in);
    *tiles_per_chunk = static_cast<uint32_t>(most);
    const uint64_t n_inst = s.inst.size();
    if (s.has_deps || n_inst == 0) return n_inst * most;
    const uint64_t first = (n_inst - 1) / group * group;  // the last group's first instance
    uint64_t last_most = 1;
    for (uint64_t i = first; i < n_inst; ++i) last_most = last_most > tiles_of(s.inst[i]) ? last_most : tiles_of(s.inst[i]);
    return first * most + (n_inst - first) * last_most;
}

// Exact floor(n * (w_0+..+w_{t-1}) / (w_0+..+w_{T-1})) rounded down to a multiple of
// `align`, made monotone; b_0 = 0, b_T = n.
std::vector<uint64_t> split_by_weight(uint64_t n, const std::vector<double>& w, uint64_t align);

blink_status_t make_schedule(const Trees& trees, blink_op_t op, uint64_t n, uint64_t chunk,
                             blink_fusion_t fusion, Schedule& out);

// One server of a multi-server AllReduce (section 3.5): its packed local trees
// (null for a server with a single rank) and the global ids of its local
// ranks, ascending.
struct ServerTrees {
    const Trees* trees;
    std::vector<int> ranks;
};

blink_status_t make_schedule_servers(const std::vector<ServerTrees>& servers, uint64_t n,
                                     uint64_t chunk, blink_fusion_t fusion, Schedule& out);

}  // namespace blink
