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

// One stage per tree-edge transfer, in the paper's order: reduce phase child ->
// parent with every vertex after its whole subtree, then copy phase parent ->
// child breadth first.
std::vector<StageTmpl> edge_stages(int k, int root, const ParentVec& parent, blink_op_t op) {
    const auto ch = children(k, parent);
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

// One stage per fan-in (a node folds itself and all its children, ascending)
// and one per fan-out; the root's fan-in also writes the result to its children.
std::vector<StageTmpl> node_stages(int k, int root, const ParentVec& parent, blink_op_t op) {
    const auto ch = children(k, parent);
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

// acc <- S(v) = ((x_v + S(c_1)) + S(c_2)) + ..., children ascending.  Slot i
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
std::vector<StageTmpl> tree_stage(int k, int root, const ParentVec& parent, blink_op_t op) {
    StageTmpl t = blank();
    if (op != BLINK_OP_BROADCAST) {
        for (int v = 0; v < k; ++v) t.load_rank[t.n_load++] = static_cast<uint8_t>(v);
        eval_tree(root, children(k, parent), t);
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
            if (v != root) t.store_rank[t.n_store++] = static_cast<uint8_t>(v);
    }
    return {t};
}

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

struct Built {
    std::vector<StageTmpl> tmpl;
    std::vector<StageInst> inst;
    std::vector<std::pair<int, int>> where;  // per instance: (tree, chunk)
};

// Lay the stages of all trees and chunks out in execution order.  A stage of
// level l on chunk c gets time slot c + l, the slot in which a fully pipelined
// execution would run it; inside a slot the trees take turns (section 4.2.2:
// trees sharing the machine alternate chunk by chunk instead of one running
// ahead).  Dependencies always sit in an earlier slot.
Built instantiate(const std::vector<std::vector<StageTmpl>>& per_tree,
                  const std::vector<uint64_t>& bounds, uint64_t chunk) {
    Built b;
    struct Key {
        uint64_t slot;
        int tree, local;
        uint64_t chunk_idx;
    };
    std::vector<Key> keys;
    std::vector<size_t> tmpl_base(per_tree.size());
    for (size_t t = 0; t < per_tree.size(); ++t) {
        tmpl_base[t] = b.tmpl.size();
        b.tmpl.insert(b.tmpl.end(), per_tree[t].begin(), per_tree[t].end());
        const uint64_t share = bounds[t + 1] - bounds[t];
        const uint64_t n_chunks = (share + chunk - 1) / chunk;
        for (uint64_t c = 0; c < n_chunks; ++c)
            for (size_t j = 0; j < per_tree[t].size(); ++j)
                keys.push_back({c + per_tree[t][j].level, static_cast<int>(t), static_cast<int>(j), c});
    }
    std::stable_sort(keys.begin(), keys.end(), [](const Key& a, const Key& b2) {
        if (a.slot != b2.slot) return a.slot < b2.slot;
        if (a.chunk_idx != b2.chunk_idx) return a.chunk_idx < b2.chunk_idx;  // older chunks first
        if (a.tree != b2.tree) return a.tree < b2.tree;
        return a.local < b2.local;
    });
    // position of (tree, chunk, local) in the order
    std::vector<std::vector<int32_t>> pos(per_tree.size());
    for (size_t t = 0; t < per_tree.size(); ++t) {
        const uint64_t share = bounds[t + 1] - bounds[t];
        pos[t].assign(((share + chunk - 1) / chunk) * per_tree[t].size(), -1);
    }
    for (size_t i = 0; i < keys.size(); ++i)
        pos[keys[i].tree][keys[i].chunk_idx * per_tree[keys[i].tree].size() + keys[i].local] =
            static_cast<int32_t>(i);
    b.inst.resize(keys.size());
    b.where.resize(keys.size());
    for (size_t i = 0; i < keys.size(); ++i) {
        const Key& key = keys[i];
        const StageTmpl& st = per_tree[key.tree][key.local];
        StageInst& in = b.inst[i];
        in.off = bounds[key.tree] + key.chunk_idx * chunk;
        in.len = static_cast<uint32_t>(std::min<uint64_t>(chunk, bounds[key.tree + 1] - in.off));
        in.tmpl = static_cast<uint32_t>(tmpl_base[key.tree] + key.local);
        in.pad = 0;
        in.n_dep = st.n_dep;
        for (int d = 0; d < kMaxDeps; ++d) in.dep[d] = -1;
        for (int d = 0; d < st.n_dep; ++d)
            in.dep[d] = pos[key.tree][key.chunk_idx * per_tree[key.tree].size() + st.dep_local[d]];
        b.where[i] = {key.tree, static_cast<int>(key.chunk_idx)};
    }
    return b;
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
    if (chunk > 0xFFFFFFFFull) chunk = 0xFFFFFFFFull - 3;  // a chunk is addressed with 32 bits
    if (op != BLINK_OP_ALLREDUCE && op != BLINK_OP_BROADCAST && op != BLINK_OP_REDUCE) return BLINK_EINVAL;
    if (fusion != BLINK_FUSE_EDGE && fusion != BLINK_FUSE_NODE && fusion != BLINK_FUSE_TREE)
        return BLINK_EINVAL;
    if (op == BLINK_OP_BROADCAST)
        for (int t = 1; t < T; ++t)
            if (trees.root[t] != trees.root[0]) return BLINK_EMISMATCH;
    out.k = k;
    out.n_trees = T;
    out.op = op;
    out.fusion = fusion;
    out.n = n;
    out.chunk = chunk;
    out.bounds = split_by_weight(n, trees.weight, 4);

    std::vector<std::vector<StageTmpl>> edge(T), fused(T);
    for (int t = 0; t < T; ++t) {
        edge[t] = edge_stages(k, trees.root[t], trees.parent[t], op);
        finish_levels(edge[t]);
        if (fusion == BLINK_FUSE_NODE) fused[t] = node_stages(k, trees.root[t], trees.parent[t], op);
        if (fusion == BLINK_FUSE_TREE) fused[t] = tree_stage(k, trees.root[t], trees.parent[t], op);
        finish_levels(fused[t]);
    }
    Built e = instantiate(edge, out.bounds, chunk);
    out.steps.resize(e.inst.size());
    for (size_t i = 0; i < e.inst.size(); ++i) {
        const StageInst& in = e.inst[i];
        const StageTmpl& st = e.tmpl[in.tmpl];
        blink_step_t& s = out.steps[i];
        s.kind = st.n_load == 2 ? BLINK_STEP_REDUCE : BLINK_STEP_COPY;
        s.tree = e.where[i].first;
        s.chunk = e.where[i].second;
        s.src = st.n_load == 2 ? st.load_rank[1] : st.load_rank[0];
        s.dst = st.store_rank[0];
        s.n_deps = in.n_dep;
        s.deps[0] = in.n_dep > 0 ? in.dep[0] : -1;
        s.deps[1] = in.n_dep > 1 ? in.dep[1] : -1;
        s.off = in.off;
        s.len = in.len;
    }
    if (fusion == BLINK_FUSE_EDGE) {
        out.tmpl = std::move(e.tmpl);
        out.inst = std::move(e.inst);
    } else {
        Built f = instantiate(fused, out.bounds, chunk);
        out.tmpl = std::move(f.tmpl);
        out.inst = std::move(f.inst);
    }
    out.max_slots = 1;
    out.traffic_bytes = 0;
    out.has_deps = false;
    for (const StageTmpl& st : out.tmpl) {
        out.max_slots = std::max<uint32_t>(out.max_slots, st.n_load);
        out.has_deps = out.has_deps || st.n_dep > 0;
    }
    for (const StageInst& in : out.inst) {
        const StageTmpl& st = out.tmpl[in.tmpl];
        out.traffic_bytes += static_cast<uint64_t>(in.len) * 4u * (st.n_load + st.n_store);
    }
    return BLINK_OK;
}

}  // namespace blink
