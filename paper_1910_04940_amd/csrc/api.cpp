// extern "C" boundary: argument checks, handle management, no exceptions out.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <memory>
#include <new>

#include "state.hpp"
#include "trees.hpp"

using blink::Schedule;
using blink::Trees;

#define BLINK_GUARD_BEGIN try {
#define BLINK_GUARD_END                 \
    }                                   \
    catch (const std::bad_alloc&) {     \
        return BLINK_ENOMEM;            \
    }                                   \
    catch (...) {                       \
        return BLINK_EINVAL;            \
    }

extern "C" {

blink_status_t blink_pack_trees(int k, int m, const int32_t* src, const int32_t* dst,
                                const double* cap, int root, double eps, double prune_tol,
                                blink_trees_t** out) {
    if (!out) return BLINK_EINVAL;
    *out = nullptr;
    BLINK_GUARD_BEGIN
    std::unique_ptr<blink_trees_t> h(new blink_trees_t());
    const blink_status_t st = blink::pack_trees(k, m, src, dst, cap, root, eps, prune_tol, h->t);
    if (st != BLINK_OK) return st;
    *out = h.release();
    return BLINK_OK;
    BLINK_GUARD_END
}

blink_status_t blink_trees_from_arrays(int k, int T, const int32_t* roots, const int32_t* parent,
                                       const double* weight, blink_trees_t** out) {
    if (!out) return BLINK_EINVAL;
    *out = nullptr;
    if (k < 2 || k > BLINK_MAX_RANKS || T < 1 || !roots || !parent || !weight) return BLINK_EINVAL;
    BLINK_GUARD_BEGIN
    std::unique_ptr<blink_trees_t> h(new blink_trees_t());
    h->t.k = k;
    for (int t = 0; t < T; ++t) {
        blink::ParentVec p;
        p.fill(-2);
        bool ok = roots[t] >= 0 && roots[t] < k && weight[t] > 0.0 && std::isfinite(weight[t]);
        for (int v = 0; ok && v < k; ++v) {
            const int32_t q = parent[static_cast<size_t>(t) * k + v];
            if (q < -1 || q >= k) ok = false;
            p[v] = static_cast<int8_t>(q);
        }
        if (!ok || !blink::is_spanning_tree(k, roots[t], p)) return BLINK_EINVAL;
        h->t.root.push_back(roots[t]);
        h->t.parent.push_back(p);
        h->t.weight.push_back(weight[t]);
    }
    *out = h.release();
    return BLINK_OK;
    BLINK_GUARD_END
}

int blink_trees_count(const blink_trees_t* trees) { return trees ? trees->t.count() : -1; }
int blink_trees_k(const blink_trees_t* trees) { return trees ? trees->t.k : -1; }

double blink_trees_rate(const blink_trees_t* trees) {
    if (!trees) return 0.0;
    double r = 0.0;
    for (double w : trees->t.weight) r += w;
    return r;
}

blink_status_t blink_trees_get(const blink_trees_t* trees, int t, int32_t* root, int32_t* parent,
                               double* weight) {
    if (!trees || t < 0 || t >= trees->t.count()) return BLINK_EINVAL;
    if (root) *root = trees->t.root[t];
    if (parent)
        for (int v = 0; v < trees->t.k; ++v) parent[v] = trees->t.parent[t][v];
    if (weight) *weight = trees->t.weight[t];
    return BLINK_OK;
}

void blink_trees_free(blink_trees_t* trees) { delete trees; }

blink_status_t blink_make_schedule(const blink_trees_t* trees, blink_op_t op, size_t n_elems,
                                   size_t chunk_elems, blink_fusion_t fusion,
                                   blink_schedule_t** out) {
    if (!out) return BLINK_EINVAL;
    *out = nullptr;
    if (!trees) return BLINK_EINVAL;
    BLINK_GUARD_BEGIN
    std::unique_ptr<blink_schedule_t> h(new blink_schedule_t());
    h->id = blink::next_schedule_id();
    const blink_status_t st = blink::make_schedule(trees->t, op, n_elems, chunk_elems, fusion, h->s);
    if (st != BLINK_OK) return st;
    *out = h.release();
    return BLINK_OK;
    BLINK_GUARD_END
}

blink_status_t blink_make_schedule_servers(int n_servers, const blink_trees_t* const* local,
                                           const int32_t* ranks, size_t n_elems,
                                           size_t chunk_elems, blink_fusion_t fusion,
                                           blink_schedule_t** out) {
    if (!out) return BLINK_EINVAL;
    *out = nullptr;
    if (n_servers < 1 || n_servers > BLINK_MAX_RANKS || !local || !ranks) return BLINK_EINVAL;
    BLINK_GUARD_BEGIN
    std::vector<blink::ServerTrees> servers(n_servers);
    size_t at = 0;
    for (int s = 0; s < n_servers; ++s) {
        servers[s].trees = local[s] ? &local[s]->t : nullptr;
        const size_t ks = local[s] ? static_cast<size_t>(local[s]->t.k) : 1;
        if (at + ks > BLINK_MAX_RANKS) return BLINK_EINVAL;
        servers[s].ranks.assign(ranks + at, ranks + at + ks);
        at += ks;
    }
    std::unique_ptr<blink_schedule_t> h(new blink_schedule_t());
    h->id = blink::next_schedule_id();
    const blink_status_t st = blink::make_schedule_servers(servers, n_elems, chunk_elems, fusion, h->s);
    if (st != BLINK_OK) return st;
    *out = h.release();
    return BLINK_OK;
    BLINK_GUARD_END
}

blink_status_t blink_hybrid_split(double d_total, double bw_slow, double bw_fast, double t_switch,
                                  double* d_slow, double* d_fast) {
    if (!d_slow || !d_fast) return BLINK_EINVAL;
    if (!(bw_slow > 0) || !(bw_fast > 0) || !(d_total >= 0) || !(t_switch >= 0)) return BLINK_EINVAL;
    if (!std::isfinite(d_total) || !std::isfinite(bw_slow) || !std::isfinite(bw_fast) ||
        !std::isfinite(t_switch))
        return BLINK_EINVAL;
    // Equal finishing times: d_slow/bw_slow + t_switch = (d_total - d_slow)/bw_fast.
    const double sum = bw_slow + bw_fast;
    double slow = d_total * (bw_slow / sum) - t_switch * (bw_slow / sum) * bw_fast;
    slow = slow < 0 ? 0 : (slow > d_total ? d_total : slow);
    *d_slow = slow;
    *d_fast = d_total - slow;
    return BLINK_OK;
}

size_t blink_schedule_num_steps(const blink_schedule_t* s) { return s ? s->s.steps.size() : 0; }
size_t blink_schedule_num_stages(const blink_schedule_t* s) { return s ? s->s.inst.size() : 0; }
int blink_schedule_num_trees(const blink_schedule_t* s) { return s ? s->s.n_trees : -1; }
uint64_t blink_schedule_batch(const blink_schedule_t* s) { return s ? s->s.batch : 0; }

blink_status_t blink_schedule_get_steps(const blink_schedule_t* s, blink_step_t* out) {
    if (!s || (!out && !s->s.steps.empty())) return BLINK_EINVAL;
    if (!s->s.steps.empty()) std::memcpy(out, s->s.steps.data(), s->s.steps.size() * sizeof(blink_step_t));
    return BLINK_OK;
}

blink_status_t blink_schedule_get_stages(const blink_schedule_t* s, blink_stage_t* out) {
    static_assert(BLINK_STAGE_MAX_OPS == blink::kMaxOps && BLINK_STAGE_MAX_DEPS == blink::kMaxDeps,
                  "the public stage record mirrors the internal one");
    if (!s || (!out && !s->s.inst.empty())) return BLINK_EINVAL;
    for (size_t i = 0; i < s->s.inst.size(); ++i) {
        const blink::StageInst& in = s->s.inst[i];
        const blink::StageTmpl& st = s->s.tmpl[in.tmpl];
        blink_stage_t& o = out[i];
        std::memset(&o, 0, sizeof o);
        o.off = in.off;
        o.len = in.len;
        o.tree = s->s.inst_where[i].tree;
        o.chunk = s->s.inst_where[i].chunk;
        o.flow = s->s.inst_where[i].flow;
        o.n_load = st.n_load;
        o.n_op = st.n_op;
        o.n_store = st.n_store;
        o.n_dep = static_cast<uint8_t>(in.n_dep);
        std::memcpy(o.load_rank, st.load_rank, sizeof o.load_rank);
        std::memcpy(o.store_rank, st.store_rank, sizeof o.store_rank);
        std::memcpy(o.op, st.op, sizeof o.op);
        std::memcpy(o.seq_rank, st.seq_rank, sizeof o.seq_rank);
        std::memcpy(o.seq_code, st.seq_code, sizeof o.seq_code);
        o.seq_depth = st.seq_depth;
        for (int d = 0; d < BLINK_STAGE_MAX_DEPS; ++d) o.deps[d] = d < static_cast<int>(in.n_dep) ? in.dep[d] : -1;
    }
    return BLINK_OK;
}

blink_status_t blink_schedule_get_bounds(const blink_schedule_t* s, uint64_t* out) {
    if (!s || !out) return BLINK_EINVAL;
    for (size_t i = 0; i < s->s.bounds.size(); ++i) out[i] = s->s.bounds[i];
    return BLINK_OK;
}

blink_status_t blink_schedule_get_tickets(const blink_schedule_t* s, uint32_t tile_elems, uint64_t* n_tickets,
                                          int32_t* stage, int32_t* tile) {
    if (!s || !n_tickets || tile_elems < 256 || tile_elems > 65536 || (tile_elems & (tile_elems - 1))) return BLINK_EINVAL;
    const blink::Schedule& sc = s->s;
    unsigned shift = 0;
    while ((1u << shift) < tile_elems) ++shift;
    uint32_t tiles_per_chunk = 1;
    const unsigned group = blink::ticket_group(sc);
    const uint64_t n = blink::ticket_count(sc, group, shift, 0, &tiles_per_chunk);
    *n_tickets = n;
    if (!stage && !tile) return BLINK_OK;
    if (!stage || !tile) return BLINK_EINVAL;
    for (uint64_t t = 0; t < n; ++t) {
        unsigned ii, tt;
        blink::ticket_to_tile(t, group, tiles_per_chunk, static_cast<unsigned>(sc.inst.size()), &ii, &tt);
        const blink::StageInst& in = sc.inst[ii];
        const uint64_t block = (in.off >> shift) + tt;
        const uint64_t lo = std::max<uint64_t>(in.off, block << shift), hi = std::min<uint64_t>(in.off + in.len, (block + 1) << shift);
        stage[t] = static_cast<int32_t>(ii);
        tile[t] = lo < hi ? static_cast<int32_t>(tt) : -1;
    }
    return BLINK_OK;
}

uint64_t blink_schedule_traffic_bytes(const blink_schedule_t* s) { return s ? s->s.traffic_bytes : 0; }

void blink_schedule_free(blink_schedule_t* s) {
    if (!s) return;
    blink::release_device_state(s);
    delete s;
}

blink_status_t blink_allreduce(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                               blink_schedule_t* s, void* stream) {
    BLINK_GUARD_BEGIN
    return blink::execute(s, bufs, k, n_elems, dtype, BLINK_OP_ALLREDUCE, BLINK_SUM, stream);
    BLINK_GUARD_END
}

blink_status_t blink_allreduce_noalloc(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                                       blink_schedule_t* s, void* stream) {
    BLINK_GUARD_BEGIN
    return blink::execute(s, bufs, k, n_elems, dtype, BLINK_OP_ALLREDUCE, BLINK_SUM, stream, true);
    BLINK_GUARD_END
}

blink_status_t blink_broadcast(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                               blink_schedule_t* s, void* stream) {
    BLINK_GUARD_BEGIN
    return blink::execute(s, bufs, k, n_elems, dtype, BLINK_OP_BROADCAST, BLINK_SUM, stream);
    BLINK_GUARD_END
}

blink_status_t blink_allreduce_op(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                                  blink_redop_t redop, blink_schedule_t* s, void* stream) {
    BLINK_GUARD_BEGIN
    return blink::execute(s, bufs, k, n_elems, dtype, BLINK_OP_ALLREDUCE, redop, stream);
    BLINK_GUARD_END
}

blink_status_t blink_reduce(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                            blink_redop_t redop, blink_schedule_t* s, void* stream) {
    BLINK_GUARD_BEGIN
    return blink::execute(s, bufs, k, n_elems, dtype, BLINK_OP_REDUCE, redop, stream);
    BLINK_GUARD_END
}

blink_status_t blink_allgather(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                               blink_schedule_t* s, void* stream) {
    BLINK_GUARD_BEGIN
    return blink::execute(s, bufs, k, n_elems, dtype, BLINK_OP_ALLGATHER, BLINK_SUM, stream);
    BLINK_GUARD_END
}

blink_status_t blink_gather(void* const* bufs, int k, size_t n_elems, blink_dtype_t dtype,
                            blink_schedule_t* s, void* stream) {
    BLINK_GUARD_BEGIN
    return blink::execute(s, bufs, k, n_elems, dtype, BLINK_OP_GATHER, BLINK_SUM, stream);
    BLINK_GUARD_END
}

blink_status_t blink_schedule_set_launch(blink_schedule_t* s, int wg_per_cu, int tile_elems) {
    const bool tile_ok = tile_elems == 0 || (tile_elems >= 256 && tile_elems <= 65536 &&
                                             (tile_elems & (tile_elems - 1)) == 0);
    if (!s || wg_per_cu < 0 || !tile_ok) return BLINK_EINVAL;
    s->wg_per_cu = wg_per_cu;
    if (static_cast<unsigned>(tile_elems) != s->tile_override) {
        s->tile_override = static_cast<unsigned>(tile_elems);
        return blink::reset_progress(s);  // counters were counted in tiles of the old size
    }
    return BLINK_OK;
}

blink_status_t blink_schedule_status(blink_schedule_t* s, blink_progress_t* out) {
    if (!s || !out) return BLINK_EINVAL;
    BLINK_GUARD_BEGIN
    return blink::read_status(s, out);
    BLINK_GUARD_END
}

blink_status_t blink_schedule_reset(blink_schedule_t* s) {
    if (!s) return BLINK_EINVAL;
    BLINK_GUARD_BEGIN
    return blink::reset_progress(s);
    BLINK_GUARD_END
}

blink_status_t blink_schedule_set_wait_limit(blink_schedule_t* s, uint64_t microseconds) {
    if (!s || microseconds > (1ull << 40)) return BLINK_EINVAL;
    s->wait_limit_us = microseconds;
    return BLINK_OK;
}

blink_status_t blink_schedule_test_skip_call(blink_schedule_t* s) {
    if (!s) return BLINK_EINVAL;
    s->epoch += 1;
    return BLINK_OK;
}

blink_status_t blink_schedule_set_kernel(blink_schedule_t* s, int kernel) {
    if (!s || kernel < 0 || kernel > 3) return BLINK_EINVAL;
    s->kernel_choice = kernel;
    return BLINK_OK;
}

int blink_schedule_last_kernel(const blink_schedule_t* s) { return s ? s->last_kernel : 0; }

blink_status_t blink_schedule_set_sweep(blink_schedule_t* s, int alternate) {
    if (!s || (alternate != 0 && alternate != 1)) return BLINK_EINVAL;
    if (s->sweep_alternates != (alternate == 1)) {
        s->sweep_alternates = alternate == 1;
        // the cache policy, hence the kernel instantiation, follows the mode;
        // tile size and counters do not
        s->plan.made = false;
        for (auto& per_dtype : s->occupancy) per_dtype[0] = per_dtype[1] = 0;
    }
    return BLINK_OK;
}

const char* blink_strerror(blink_status_t st) {
    switch (st) {
        case BLINK_OK: return "ok";
        case BLINK_EINVAL: return "invalid argument";
        case BLINK_EDISCONNECTED: return "a vertex is unreachable from the root";
        case BLINK_ENOMEM: return "out of memory";
        case BLINK_EMISMATCH: return "schedule does not match the call";
        case BLINK_EHIP: return "HIP runtime error";
        case BLINK_ESTUCK: return "a stage gave up waiting for another one";
        case BLINK_ELIMIT: return "the schedule does not fit the static device block";
    }
    return "unknown status";
}

}  // extern "C"
