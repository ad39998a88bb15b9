// Host-side scheduler (paper sections 3.3, 4.1, 4.2.1, 4.2.2).  See schedule.hpp.
#include "schedule.hpp"

#include <algorithm>
#include <climits>
#include <cmath>
#include <functional>

namespace blink {
namespace {

// ---- exact comparison of n*P against c*W for sums of doubles ------------------
// Every finite double is mant * 2^e with a 53-bit integer mant; scaled by the
// smallest exponent in play the weights become (long) non-negative integers.
struct Big {
    std::vector<uint64_t> w;  // little endian
};

Big shifted(uint64_t mant, int shift) {
    Big b;
    b.w.assign(static_cast<size_t>(shift / 64) + 2, 0);
    const int word = shift / 64, bit = shift % 64;
    b.w[word] = mant << bit;
    if (bit) b.w[word + 1] = mant >> (64 - bit);
    return b;
}

void add(Big& a, const Big& b) {
    if (a.w.size() < b.w.size() + 1) a.w.resize(b.w.size() + 1, 0);
    unsigned __int128 carry = 0;
    for (size_t i = 0; i < a.w.size(); ++i) {
        unsigned __int128 s = carry + a.w[i] + (i < b.w.size() ? b.w[i] : 0);
        a.w[i] = static_cast<uint64_t>(s);
        carry = s >> 64;
    }
    if (carry) a.w.push_back(static_cast<uint64_t>(carry));
}

Big mul(const Big& a, uint64_t x) {
    Big r;
    r.w.assign(a.w.size() + 1, 0);
    unsigned __int128 carry = 0;
    for (size_t i = 0; i < a.w.size(); ++i) {
        unsigned __int128 p = static_cast<unsigned __int128>(a.w[i]) * x + carry;
        r.w[i] = static_cast<uint64_t>(p);
        carry = p >> 64;
    }
    r.w[a.w.size()] = static_cast<uint64_t>(carry);
    return r;
}

int cmp(const Big& a, const Big& b) {
    const size_t n = std::max(a.w.size(), b.w.size());
    for (size_t i = n; i-- > 0;) {
        const uint64_t x = i < a.w.size() ? a.w[i] : 0, y = i < b.w.size() ? b.w[i] : 0;
        if (x != y) return x < y ? -1 : 1;
    }
    return 0;
}

// ---- stage shapes of one tree -----------------------------------------------------
StageTmpl blank() {
    StageTmpl t{};
    return t;
}

// Children in the order they are folded in: ascending id, except that the
// vertices in the bit set `late` (attached to their parent by a later phase of
// a multi-server protocol, section 3.5) come after all others.
std::vector<std::vector<int>> ordered_children(int k, const ParentVec& parent, uint16_t late) {
    auto ch = children(k, parent);
    if (late)
        for (auto& cs : ch)
            std::stable_partition(cs.begin(), cs.end(), [late](int c) { return !((late >> c) & 1); });
    return ch;
}

// One stage per tree-edge transfer, in the paper's order: reduce phase child ->
// parent with every vertex after its whole subtree, then copy phase parent ->
// child breadth first.
std::vector<StageTmpl> edge_stages(int k, int root, const ParentVec& parent, uint16_t late,
                                   blink_op_t op) {
    const auto ch = ordered_children(k, parent, late);
    std::vector<StageTmpl> out;
    std::vector<int> red(k, -1), cp(k, -1);
    if (op != BLINK_OP_BROADCAST) {
        std::function<void(int)> visit = [&](int v) {
            for (int c : ch[v]) visit(c);
            if (v == root) return;
            const int p = parent[v];
            StageTmpl t = blank();
            t.n_load = 2;
            t.load_rank[0] = static_cast<uint8_t>(p);   // the accumulating side
            t.load_rank[1] = static_cast<uint8_t>(v);
            t.n_op = 2;
            t.op[0] = make_op(OP_LD, 0);
            t.op[1] = make_op(OP_ADD, 1);
            t.n_store = 1;
            t.store_rank[0] = static_cast<uint8_t>(p);
            if (!ch[v].empty()) t.dep_local[t.n_dep++] = static_cast<uint8_t>(red[ch[v].back()]);
            const auto& sib = ch[p];
            const size_t i = std::find(sib.begin(), sib.end(), v) - sib.begin();
            if (i > 0) t.dep_local[t.n_dep++] = static_cast<uint8_t>(red[sib[i - 1]]);
            red[v] = static_cast<int>(out.size());
            out.push_back(t);
        };
        visit(root);
    }
    if (op == BLINK_OP_REDUCE) return out;
    std::vector<int> frontier{root};
    while (!frontier.empty()) {
        std::vector<int> next;
        for (int p : frontier)
            for (int v : ch[p]) {
                StageTmpl t = blank();
                t.n_load = 1;
                t.load_rank[0] = static_cast<uint8_t>(p);
                t.n_op = 1;
                t.op[0] = make_op(OP_LD, 0);
                t.n_store = 1;
                t.store_rank[0] = static_cast<uint8_t>(v);
                if (p != root)
                    t.dep_local[t.n_dep++] = static_cast<uint8_t>(cp[p]);
                else if (op == BLINK_OP_ALLREDUCE)
                    t.dep_local[t.n_dep++] = static_cast<uint8_t>(red[ch[root].back()]);
                cp[v] = static_cast<int>(out.size());
                out.push_back(t);
                next.push_back(v);
            }
        frontier.swap(next);
    }
    return out;
}

// One stage per fan-in (a node folds itself and all its children, in folding
// order) and one per fan-out; the root's fan-in also writes the result to its children.
std::vector<StageTmpl> node_stages(int k, int root, const ParentVec& parent, uint16_t late,
                                   blink_op_t op) {
    const auto ch = ordered_children(k, parent, late);
    std::vector<StageTmpl> out;
    std::vector<int> fin(k, -1), fout(k, -1);
    if (op != BLINK_OP_BROADCAST) {
        std::function<void(int)> visit = [&](int v) {
            for (int c : ch[v]) visit(c);
            if (ch[v].empty()) return;
            StageTmpl t = blank();
            t.load_rank[t.n_load++] = static_cast<uint8_t>(v);
            t.op[t.n_op++] = make_op(OP_LD, 0);
            for (int c : ch[v]) {
                t.op[t.n_op++] = make_op(OP_ADD, t.n_load);
                t.load_rank[t.n_load++] = static_cast<uint8_t>(c);
                if (!ch[c].empty()) t.dep_local[t.n_dep++] = static_cast<uint8_t>(fin[c]);
            }
            t.store_rank[t.n_store++] = static_cast<uint8_t>(v);
            if (v == root && op == BLINK_OP_ALLREDUCE)
                for (int c : ch[v]) t.store_rank[t.n_store++] = static_cast<uint8_t>(c);
            fin[v] = static_cast<int>(out.size());
            out.push_back(t);
        };
        visit(root);
        fout[root] = fin[root];
    }
    if (op == BLINK_OP_REDUCE) return out;
    std::vector<int> frontier{root};
    while (!frontier.empty()) {
        std::vector<int> next;
        for (int p : frontier) {
            if (ch[p].empty()) continue;
            if (!(p == root && op == BLINK_OP_ALLREDUCE)) {
                StageTmpl t = blank();
                t.n_load = 1;
                t.load_rank[0] = static_cast<uint8_t>(p);
                t.n_op = 1;
                t.op[0] = make_op(OP_LD, 0);
                for (int c : ch[p]) t.store_rank[t.n_store++] = static_cast<uint8_t>(c);
                if (p != root) t.dep_local[t.n_dep++] = static_cast<uint8_t>(fout[parent[p]]);
                fout[p] = static_cast<int>(out.size());
                out.push_back(t);
            }
            for (int c : ch[p]) next.push_back(c);
        }
        frontier.swap(next);
    }
    return out;
}

// acc <- S(v) = ((x_v + S(c_1)) + S(c_2)) + ..., children in folding order.  Slot i
// holds x_i.  The first child's sum is formed first and x_v added to it (IEEE
// addition and multiplication commute bit for bit, and min/max are taken under
// a total order, so the bits equal x_v (+) S(c_1)); before a later child
// that has children of its own the running sum is parked in v's slot, which is
// free once x_v has been consumed.
void eval_tree(int v, const std::vector<std::vector<int>>& ch, StageTmpl& t) {
    if (ch[v].empty()) {
        t.op[t.n_op++] = make_op(OP_LD, static_cast<uint8_t>(v));
        return;
    }
    eval_tree(ch[v][0], ch, t);
    t.op[t.n_op++] = make_op(OP_ADD, static_cast<uint8_t>(v));
    for (size_t i = 1; i < ch[v].size(); ++i) {
        const int c = ch[v][i];
        if (ch[c].empty()) {
            t.op[t.n_op++] = make_op(OP_ADD, static_cast<uint8_t>(c));
        } else {
            t.op[t.n_op++] = make_op(OP_ST, static_cast<uint8_t>(v));
            eval_tree(c, ch, t);
            t.op[t.n_op++] = make_op(OP_ADD, static_cast<uint8_t>(v));
        }
    }
}

// The whole tree in one stage: every rank read once and written once.
std::vector<StageTmpl> tree_stage(int k, int root, const ParentVec& parent, uint16_t late,
                                  blink_op_t op) {
    StageTmpl t = blank();
    if (op != BLINK_OP_BROADCAST) {
        for (int v = 0; v < k; ++v) t.load_rank[t.n_load++] = static_cast<uint8_t>(v);
        eval_tree(root, ordered_children(k, parent, late), t);
        if (op == BLINK_OP_REDUCE)
            t.store_rank[t.n_store++] = static_cast<uint8_t>(root);
        else
            for (int v = 0; v < k; ++v) t.store_rank[t.n_store++] = static_cast<uint8_t>(v);
    } else {
        t.n_load = 1;
        t.load_rank[0] = static_cast<uint8_t>(root);
        t.n_op = 1;
        t.op[0] = make_op(OP_LD, 0);
        for (int v = 0; v < k; ++v)
            if (v != root && parent[v] >= 0) t.store_rank[t.n_store++] = static_cast<uint8_t>(v);
    }
    return {t};
}

}  // namespace

void stack_program(StageTmpl& st) {
    st.seq_depth = 0;
    for (int i = 0; i < BLINK_MAX_RANKS; ++i) st.seq_rank[i] = st.seq_code[i] = 0;
    enum : int { kLoaded = -1, kUsed = -2 };   // else: depth at which a partial sum is parked in the slot
    int state[64];
    for (int i = 0; i < 64; ++i) state[i] = i < st.n_load ? kLoaded : kUsed;
    int depth = 0, deepest = 0, n = 0;
    uint8_t rank[BLINK_MAX_RANKS], code[BLINK_MAX_RANKS];
    for (int o = 0; o < st.n_op; ++o) {
        const int kind = st.op[o] >> 6, slot = st.op[o] & 63;
        if (kind == OP_ST) {
            if (depth < 1 || state[slot] != kUsed) return;  // parks only into a slot whose value is spent
            state[slot] = depth;
        } else if (state[slot] == kLoaded) {
            if (n == BLINK_MAX_RANKS) return;
            if (kind == OP_LD) {
                ++depth;
                deepest = std::max(deepest, depth);
            } else if (depth < 1) {
                return;
            }
            rank[n] = st.load_rank[slot];
            code[n] = kind == OP_LD ? 1 : 0;
            ++n;
            state[slot] = kUsed;
        } else {
            // a parked partial sum: must be the accumulator right below the top
            if (kind != OP_ADD || state[slot] != depth - 1 || n == 0 || (code[n - 1] >> 1) == 63) return;
            code[n - 1] = static_cast<uint8_t>(code[n - 1] + 2);
            --depth;
            state[slot] = kUsed;
        }
    }
    if (depth != 1 || n != st.n_load) return;
    for (int i = 0; i < n; ++i) {
        st.seq_rank[i] = rank[i];
        st.seq_code[i] = code[i];
    }
    st.seq_depth = static_cast<uint8_t>(deepest);
}

namespace {

void finish_levels(std::vector<StageTmpl>& st) {
    for (size_t j = 0; j < st.size(); ++j) {
        int lvl = 0;
        for (int d = 0; d < st[j].n_dep; ++d) {
            lvl = std::max(lvl, st[st[j].dep_local[d]].level + 1);
            st[st[j].dep_local[d]].signals = 1;
        }
        st[j].level = static_cast<uint8_t>(lvl);
    }
}

// One tree carrying one contiguous range of the payload in one direction:
// the unit the stage builders and the chunking work on.  AllReduce, Broadcast
// and Reduce have one flow per tree (its share); AllGather and Gather have one
// per tree and piece (the tree's share of that piece, moving away from, or
// towards the root from, the piece's owner).
struct Flow {
    ParentVec parent;   // -1 at the flow's source, -2 for ranks that take no part
    int root;
    uint64_t lo, hi;    // element range
    int tree;           // index of the packed tree it belongs to
    uint16_t late = 0;  // bit set of vertices folded in after their siblings (see ordered_children)
};

struct Built {
    uint64_t batch = 1;            // chunks per flow and time slot
    uint64_t n_slots = 1;          // time slots in use
    std::vector<StageTmpl> tmpl;
    std::vector<StageInst> inst;
    std::vector<InstWhere> where;  // per instance: tree, chunk, flow
};

// Lay the stages of all flows and chunks out in execution order.  A stage of
// level l on chunk c gets time slot c / B + l: chunks advance through the levels
// in batches of B, a fully pipelined execution with B chunks per stage and time
// step; inside a slot the older chunks come first and, chunk by chunk, the
// flows take turns (section 4.2.2: trees sharing the machine alternate chunk by
// chunk instead of one running ahead).  Dependencies always sit in an earlier
// slot.
//
// B.  Tickets are drawn in this order by hundreds of waves at once, so whatever
// a ticket waits for should lie further back than the waves reach, or most of
// them wait: B is chosen so that a slot holds about kSlotTickets tickets (with
// B = 1 and 64 KiB chunks a slot of the 8-rank per-edge program has 112 tickets
// and 768 waves crowd into seven slots' worth of dependencies: 3.1 ms for
// 8 x 256 MiB; with B = 10: see the measurements), but no more chunks than keep
// what one slot hands to the next within reach of the memory-side cache.
constexpr uint64_t kSlotTickets = 2048;
constexpr uint64_t kSlotElems = (64ull << 20) / 4;   // elements in flight between two slots
constexpr uint64_t kTicketElemsGuess = 8192;         // a ticket of a schedule with dependencies

Built instantiate(const std::vector<std::vector<StageTmpl>>& per_flow, const std::vector<Flow>& flows,
                  uint64_t chunk) {
    Built b;
    struct Key {
        uint64_t slot;
        int flow, local;
        uint64_t chunk_idx;
    };
    std::vector<Key> keys;
    std::vector<size_t> tmpl_base(per_flow.size());
    std::vector<uint64_t> n_chunks(per_flow.size());
    uint64_t stages_per_chunk_step = 0, longest = 0;
    for (size_t f = 0; f < per_flow.size(); ++f) {
        stages_per_chunk_step += per_flow[f].size();
        longest = std::max(longest, flows[f].hi - flows[f].lo);
    }
    const uint64_t chunk_len = std::min(chunk, std::max<uint64_t>(longest, 1));
    const uint64_t tickets_per_chunk_step =
        std::max<uint64_t>(1, stages_per_chunk_step) * ((chunk_len + kTicketElemsGuess - 1) / kTicketElemsGuess);
    const uint64_t by_tickets = (kSlotTickets + tickets_per_chunk_step - 1) / tickets_per_chunk_step;
    const uint64_t by_cache = kSlotElems / std::max<uint64_t>(1, stages_per_chunk_step * chunk_len);
    const uint64_t most_chunks = std::max<uint64_t>(1, (longest + chunk - 1) / chunk);
    const uint64_t batch = std::max<uint64_t>(1, std::min({by_tickets, by_cache, most_chunks}));
    b.batch = batch;
    for (size_t f = 0; f < per_flow.size(); ++f) {
        tmpl_base[f] = b.tmpl.size();
        b.tmpl.insert(b.tmpl.end(), per_flow[f].begin(), per_flow[f].end());
        n_chunks[f] = (flows[f].hi - flows[f].lo + chunk - 1) / chunk;
        for (uint64_t c = 0; c < n_chunks[f]; ++c)
            for (size_t j = 0; j < per_flow[f].size(); ++j)
                keys.push_back({c / batch + per_flow[f][j].level, static_cast<int>(f), static_cast<int>(j), c});
    }
    std::stable_sort(keys.begin(), keys.end(), [](const Key& a, const Key& b2) {
        if (a.slot != b2.slot) return a.slot < b2.slot;
        if (a.chunk_idx != b2.chunk_idx) return a.chunk_idx < b2.chunk_idx;  // older chunks first
        if (a.flow != b2.flow) return a.flow < b2.flow;
        return a.local < b2.local;
    });
    b.n_slots = keys.empty() ? 1 : keys.back().slot + 1;
    // position of (flow, chunk, local) in the order
    std::vector<std::vector<int32_t>> pos(per_flow.size());
    for (size_t f = 0; f < per_flow.size(); ++f) pos[f].assign(n_chunks[f] * per_flow[f].size(), -1);
    for (size_t i = 0; i < keys.size(); ++i)
        pos[keys[i].flow][keys[i].chunk_idx * per_flow[keys[i].flow].size() + keys[i].local] =
            static_cast<int32_t>(i);
    b.inst.resize(keys.size());
    b.where.resize(keys.size());
    for (size_t i = 0; i < keys.size(); ++i) {
        const Key& key = keys[i];
        const StageTmpl& st = per_flow[key.flow][key.local];
        const Flow& fl = flows[key.flow];
        StageInst& in = b.inst[i];
        in.off = fl.lo + key.chunk_idx * chunk;
        in.len = static_cast<uint32_t>(std::min<uint64_t>(chunk, fl.hi - in.off));
        in.tmpl = static_cast<uint32_t>(tmpl_base[key.flow] + key.local);
        in.pad = 0;
        in.n_dep = st.n_dep;
        for (int d = 0; d < kMaxDeps; ++d) in.dep[d] = -1;
        for (int d = 0; d < st.n_dep; ++d)
            in.dep[d] = pos[key.flow][key.chunk_idx * per_flow[key.flow].size() + st.dep_local[d]];
        b.where[i] = {fl.tree, static_cast<int>(key.chunk_idx), key.flow};
    }
    return b;
}

// The same undirected tree with every edge directed away from new_root.
ParentVec reroot(int k, const ParentVec& parent, int new_root) {
    ParentVec out;
    out.fill(-2);
    out[new_root] = -1;
    std::vector<int> stack{new_root};
    while (!stack.empty()) {
        const int u = stack.back();
        stack.pop_back();
        for (int v = 0; v < k; ++v) {
            const bool linked = (parent[v] == u) || (parent[u] == v);
            if (linked && out[v] == -2) {
                out[v] = static_cast<int8_t>(u);
                stack.push_back(v);
            }
        }
    }
    return out;
}

// Piece j climbing to the tree's root: j is the source, each ancestor receives
// from the rank below it; nobody else takes part.  With `direct` the piece goes
// to the root in one hop (what a fully fused pass does).
ParentVec climb(const ParentVec& parent, int root, int j, bool direct) {
    ParentVec out;
    out.fill(-2);
    out[j] = -1;
    if (direct) {
        if (root != j) out[root] = static_cast<int8_t>(j);
        return out;
    }
    for (int v = j; parent[v] >= 0; v = parent[v]) out[parent[v]] = static_cast<int8_t>(v);
    return out;
}

// Stages, instances, the public step list and the totals of a schedule whose
// flows are known.  `fused_flows`: what a fully fused pass works on when that
// differs from the tree-edge flows (empty = the same).
void finish(const std::vector<Flow>& flows, std::vector<Flow> fused_flows, blink_op_t build_as,
            Schedule& out) {
    const int k = out.k;
    const uint64_t chunk = out.chunk;
    const blink_fusion_t fusion = out.fusion;
    if (fused_flows.empty()) fused_flows = flows;
    out.n_flows = static_cast<uint32_t>(fusion == BLINK_FUSE_TREE ? fused_flows.size() : flows.size());

    std::vector<std::vector<StageTmpl>> edge(flows.size()), fused;
    for (size_t f = 0; f < flows.size(); ++f) {
        edge[f] = edge_stages(k, flows[f].root, flows[f].parent, flows[f].late, build_as);
        finish_levels(edge[f]);
    }
    const std::vector<Flow>& ff = fusion == BLINK_FUSE_TREE ? fused_flows : flows;
    if (fusion != BLINK_FUSE_EDGE) {
        fused.resize(ff.size());
        for (size_t f = 0; f < ff.size(); ++f) {
            fused[f] = fusion == BLINK_FUSE_NODE ? node_stages(k, ff[f].root, ff[f].parent, ff[f].late, build_as)
                                                 : tree_stage(k, ff[f].root, ff[f].parent, ff[f].late, build_as);
            finish_levels(fused[f]);
        }
    }
    Built e = instantiate(edge, flows, chunk);
    out.steps.resize(e.inst.size());
    for (size_t i = 0; i < e.inst.size(); ++i) {
        const StageInst& in = e.inst[i];
        const StageTmpl& st = e.tmpl[in.tmpl];
        blink_step_t& s = out.steps[i];
        s.kind = st.n_load == 2 ? BLINK_STEP_REDUCE : BLINK_STEP_COPY;
        s.tree = e.where[i].tree;
        s.chunk = e.where[i].chunk;
        s.src = st.n_load == 2 ? st.load_rank[1] : st.load_rank[0];
        s.dst = st.store_rank[0];
        s.n_deps = in.n_dep;
        s.deps[0] = in.n_dep > 0 ? in.dep[0] : -1;
        s.deps[1] = in.n_dep > 1 ? in.dep[1] : -1;
        s.off = in.off;
        s.len = in.len;
    }
    out.batch = e.batch;
    out.n_slots = e.n_slots;
    if (fusion == BLINK_FUSE_EDGE) {
        out.tmpl = std::move(e.tmpl);
        out.inst = std::move(e.inst);
        out.inst_where = std::move(e.where);
    } else {
        Built f = instantiate(fused, ff, chunk);
        out.n_slots = f.n_slots;
        out.tmpl = std::move(f.tmpl);
        out.inst = std::move(f.inst);
        out.inst_where = std::move(f.where);
    }
    out.max_slots = 1;
    out.traffic_bytes = 0;
    out.read_bytes = 0;
    out.has_deps = false;
    out.max_stack = 0;
    for (StageTmpl& st : out.tmpl) {
        stack_program(st);
        out.max_slots = std::max<uint32_t>(out.max_slots, st.n_load);
        out.has_deps = out.has_deps || st.n_dep > 0;
        out.max_stack = std::max<uint32_t>(out.max_stack, st.seq_depth ? st.seq_depth : 255u);
    }
    for (const StageInst& in : out.inst) {
        const StageTmpl& st = out.tmpl[in.tmpl];
        out.traffic_bytes += static_cast<uint64_t>(in.len) * 4u * (st.n_load + st.n_store);
        out.read_bytes += static_cast<uint64_t>(in.len) * 4u * st.n_load;
    }
}

}  // namespace

std::vector<uint64_t> split_by_weight(uint64_t n, const std::vector<double>& w, uint64_t align) {
    const size_t T = w.size();
    std::vector<uint64_t> mant(T);
    std::vector<int> expo(T);
    int emin = INT_MAX;
    for (size_t t = 0; t < T; ++t) {
        int e;
        const double f = std::frexp(w[t], &e);  // w = f * 2^e, f in [0.5, 1)
        mant[t] = static_cast<uint64_t>(std::ldexp(f, 53));
        expo[t] = e - 53;
        emin = std::min(emin, expo[t]);
    }
    Big total;
    total.w.assign(1, 0);
    long double total_ld = 0.0L;
    for (size_t t = 0; t < T; ++t) {
        add(total, shifted(mant[t], expo[t] - emin));
        total_ld += w[t];
    }
    std::vector<uint64_t> bounds{0};
    Big prefix;
    prefix.w.assign(1, 0);
    long double prefix_ld = 0.0L;
    for (size_t t = 0; t + 1 < T; ++t) {
        add(prefix, shifted(mant[t], expo[t] - emin));
        prefix_ld += w[t];
        long double guess = std::floor(static_cast<long double>(n) * (prefix_ld / total_ld));
        uint64_t c = guess <= 0 ? 0 : (guess >= static_cast<long double>(n) ? n : static_cast<uint64_t>(guess));
        const Big rhs = mul(prefix, n);
        while (c > 0 && cmp(mul(total, c), rhs) > 0) --c;
        while (c < n && cmp(mul(total, c + 1), rhs) <= 0) ++c;
        c -= c % align;
        bounds.push_back(std::max(c, bounds.back()));
    }
    bounds.push_back(n);
    return bounds;
}

blink_status_t make_schedule(const Trees& trees, blink_op_t op, uint64_t n, uint64_t chunk,
                             blink_fusion_t fusion, Schedule& out) {
    const int T = trees.count(), k = trees.k;
    if (T < 1 || k < 2 || k > BLINK_MAX_RANKS || chunk == 0) return BLINK_EINVAL;
    if (chunk > 0xFFFFFFFCull) {  // a chunk is addressed with 32 bits
        if (n > 0xFFFFFFFCull) return BLINK_EINVAL;
        chunk = 0xFFFFFFFCull;    // no payload this small has a longer chunk
    }
    const bool gathers = op == BLINK_OP_ALLGATHER || op == BLINK_OP_GATHER;
    if (op != BLINK_OP_ALLREDUCE && op != BLINK_OP_BROADCAST && op != BLINK_OP_REDUCE && !gathers)
        return BLINK_EINVAL;
    if (fusion != BLINK_FUSE_EDGE && fusion != BLINK_FUSE_NODE && fusion != BLINK_FUSE_TREE)
        return BLINK_EINVAL;
    if (op == BLINK_OP_BROADCAST)
        for (int t = 1; t < T; ++t)
            if (trees.root[t] != trees.root[0]) return BLINK_EMISMATCH;
    if (gathers && n % static_cast<uint64_t>(k) != 0) return BLINK_EINVAL;
    out.k = k;
    out.n_trees = T;
    out.op = op;
    out.fusion = fusion;
    out.n = n;
    out.chunk = chunk;
    // Gathers split every rank's piece (n/k elements) among the trees; the other
    // collectives split the whole payload.
    const uint64_t piece = gathers ? n / k : n;
    out.bounds = split_by_weight(piece, trees.weight, 4);

    // Flows, and the collective each one is built as.  A piece spreading from its
    // owner (AllGather) or climbing to the root (Gather) is a broadcast along a
    // re-directed tree.
    std::vector<Flow> flows, fused_flows;
    const blink_op_t build_as = gathers ? BLINK_OP_BROADCAST : op;
    for (int t = 0; t < T; ++t) {
        if (!gathers) {
            flows.push_back({trees.parent[t], trees.root[t], out.bounds[t], out.bounds[t + 1], t});
            continue;
        }
        for (int j = 0; j < k; ++j) {
            const uint64_t lo = static_cast<uint64_t>(j) * piece + out.bounds[t];
            const uint64_t hi = static_cast<uint64_t>(j) * piece + out.bounds[t + 1];
            if (op == BLINK_OP_ALLGATHER) {
                flows.push_back({reroot(k, trees.parent[t], j), j, lo, hi, t});
            } else if (j != trees.root[t]) {  // the root's own piece is already in place
                flows.push_back({climb(trees.parent[t], trees.root[t], j, false), j, lo, hi, t});
                fused_flows.push_back({climb(trees.parent[t], trees.root[t], j, true), j, lo, hi, t});
            }
        }
    }
    finish(flows, fused_flows, build_as, out);
    return BLINK_OK;
}

// Section 3.5.  The three phases of one (partition, piece) amount to an
// AllReduce along one global tree: the piece's owner (a server-local root) with
// its local tree below it and the other servers' local trees hanging off it
// through their roots, those roots folded in after the owner's local children.
blink_status_t make_schedule_servers(const std::vector<ServerTrees>& servers, uint64_t n,
                                     uint64_t chunk, blink_fusion_t fusion, Schedule& out) {
    const size_t S = servers.size();
    if (S < 1 || chunk == 0) return BLINK_EINVAL;
    if (fusion != BLINK_FUSE_EDGE && fusion != BLINK_FUSE_NODE && fusion != BLINK_FUSE_TREE)
        return BLINK_EINVAL;
    if (chunk > 0xFFFFFFFCull) {
        if (n > 0xFFFFFFFCull) return BLINK_EINVAL;
        chunk = 0xFFFFFFFCull;
    }
    size_t k = 0;
    for (const ServerTrees& sv : servers) k += sv.ranks.size();
    if (k < 2 || k > BLINK_MAX_RANKS) return BLINK_EINVAL;
    std::vector<bool> seen(k, false);
    for (const ServerTrees& sv : servers) {
        const size_t ks = sv.ranks.size();
        if (ks < 1 || (sv.trees ? static_cast<size_t>(sv.trees->k) != ks || sv.trees->count() < 1 : ks != 1))
            return BLINK_EINVAL;
        for (size_t i = 0; i < ks; ++i) {
            const int g = sv.ranks[i];
            if (g < 0 || static_cast<size_t>(g) >= k || seen[g]) return BLINK_EINVAL;
            if (i > 0 && g <= sv.ranks[i - 1]) return BLINK_EINVAL;  // local order = global order
            seen[g] = true;
        }
    }
    out.k = static_cast<int>(k);
    out.op = BLINK_OP_ALLREDUCE;
    out.fusion = fusion;
    out.n = n;
    out.chunk = chunk;

    // partitions: the common refinement of the servers' weighted splits
    std::vector<std::vector<uint64_t>> split(S);
    std::vector<uint64_t> cuts;
    for (size_t s = 0; s < S; ++s) {
        split[s] = servers[s].trees ? split_by_weight(n, servers[s].trees->weight, 4)
                                    : std::vector<uint64_t>{0, n};
        cuts.insert(cuts.end(), split[s].begin(), split[s].end());
    }
    std::sort(cuts.begin(), cuts.end());
    cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());

    std::vector<Flow> flows;
    const std::vector<double> equal(S, 1.0);
    for (size_t c = 0; c + 1 < cuts.size(); ++c) {
        const uint64_t lo = cuts[c], hi = cuts[c + 1];
        ParentVec parent;
        parent.fill(-2);
        std::vector<int> root_ids;
        for (size_t s = 0; s < S; ++s) {
            const ServerTrees& sv = servers[s];
            if (!sv.trees) {
                parent[sv.ranks[0]] = -1;
                root_ids.push_back(sv.ranks[0]);
                continue;
            }
            size_t t = 0;  // the tree whose non-empty share holds lo
            for (size_t i = 0; i + 1 < split[s].size(); ++i)
                if (split[s][i] <= lo && split[s][i] < split[s][i + 1]) t = i;
            for (size_t v = 0; v < sv.ranks.size(); ++v) {
                const int p = sv.trees->parent[t][v];
                parent[sv.ranks[v]] = static_cast<int8_t>(p >= 0 ? sv.ranks[p] : -1);
            }
            root_ids.push_back(sv.ranks[sv.trees->root[t]]);
        }
        std::sort(root_ids.begin(), root_ids.end());
        uint16_t all_roots = 0;
        for (int r : root_ids) all_roots = static_cast<uint16_t>(all_roots | (1u << r));
        const std::vector<uint64_t> piece = split_by_weight(hi - lo, equal, 4);
        for (size_t i = 0; i < S; ++i) {
            if (piece[i] == piece[i + 1]) continue;
            const int owner = root_ids[i];
            Flow f;
            f.parent = parent;
            for (int r : root_ids) f.parent[r] = static_cast<int8_t>(r == owner ? -1 : owner);
            f.root = owner;
            f.lo = lo + piece[i];
            f.hi = lo + piece[i + 1];
            f.tree = static_cast<int>(flows.size());
            f.late = static_cast<uint16_t>(all_roots & ~(1u << owner));
            flows.push_back(f);
        }
    }
    out.n_trees = static_cast<int>(flows.size());
    out.bounds.clear();
    for (const Flow& f : flows) out.bounds.push_back(f.lo);
    out.bounds.push_back(n);
    finish(flows, {}, BLINK_OP_ALLREDUCE, out);
    return BLINK_OK;
}

}  // namespace blink
