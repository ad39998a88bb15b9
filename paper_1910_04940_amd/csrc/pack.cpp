// Tree packing on the host (paper sections 3.1, 3.2, 3.2.1, 3.5).
//
// Section 3.2 describes the multiplicative-weight-update packing in prose and
// leaves its constants open.  This file uses the Garg-Koenemann form of that
// family: arc lengths start at delta/c_e, each round takes the minimum-length
// arborescence, gives it the bottleneck capacity gamma as additional weight and
// stretches its arcs by (1 + eps*gamma/c_e); rounds stop when sum c_e*l_e >= 1
// and the weights are divided by the worst arc congestion.  One addition over
// the plain loop: a tree is re-used for further rounds while its length stays
// within (1+eps) of the length it had when it was found to be minimal (lengths
// only grow, so that value is a lower bound on the current minimum); this
// keeps the (1 - O(eps)) guarantee and saves most arborescence computations.
//
// Section 3.2.1 (fewer trees): weights restricted to unit*{0,1,2,..} over the
// MWU trees, total weight maximised by depth-first branch and bound; unit = 1
// first (the paper's 0/1 program, a multiplicity standing for repeated trees),
// halved until the rate is within prune_tol of the MWU rate (only grids that
// the capacities themselves lie on are tried).  If no grid down to 1/8 gets
// there within the node budget (capacities that are not multiples of a common
// unit), the weights are re-optimised as a linear program over the
// MWU trees, max sum w subject to the arc capacities: a vertex of that
// polytope has at most as many positive weights as there are arcs, and its
// rate is at least MWU's.  The lightest trees are then dropped one at a time,
// the program re-solved over the rest, while the rate stays within prune_tol
// of the MWU rate (the paper's "relax until within the threshold").
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <map>
#include <queue>

#include "trees.hpp"

namespace blink {

bool is_spanning_tree(int k, int root, const ParentVec& parent) {
    if (root < 0 || root >= k || parent[root] != -1) return false;
    for (int v = 0; v < k; ++v) {
        if (v == root) continue;
        if (parent[v] < 0 || parent[v] >= k || parent[v] == v) return false;
    }
    for (int v = 0; v < k; ++v) {
        int x = v, hops = 0;
        while (x != root) {
            x = parent[x];
            if (++hops > k) return false;
        }
    }
    return true;
}

std::vector<std::vector<int>> children(int k, const ParentVec& parent) {
    std::vector<std::vector<int>> ch(k);
    for (int v = 0; v < k; ++v)
        if (parent[v] >= 0) ch[parent[v]].push_back(v);
    return ch;
}

namespace {

struct Arc {
    int u, v;
    double cap;
};

struct Graph {
    int k = 0;
    std::vector<Arc> arcs;            // parallel arcs merged
    int index[BLINK_MAX_RANKS][BLINK_MAX_RANKS];  // arc id of u->v or -1
};

// Minimum-total-length spanning arborescence diverging from root (Chu-Liu /
// Edmonds by repeated cycle contraction).  Each contraction level rewrites an
// arc entering a cycle as a new "record" that remembers which record it stands
// for and which chosen in-arc it would displace; unwinding the records from the
// last to the first yields the arcs of the original graph.  in_arc[v] receives
// the arc id entering v.  Returns false if some vertex is unreachable.  Ties go
// to the arc that comes first.
bool min_arborescence(const Graph& g, int root, const std::vector<double>& len,
                      std::vector<int>& in_arc) {
    struct E {
        int u, v;
        double w;
        int rec;
    };
    const int m = static_cast<int>(g.arcs.size());
    std::vector<E> es;
    es.reserve(m);
    for (int i = 0; i < m; ++i)
        if (g.arcs[i].v != root) es.push_back({g.arcs[i].u, g.arcs[i].v, len[i], i});
    std::vector<int> uses(m, 0), stands_for, displaces;
    int n = g.k, r = root;
    std::vector<double> best;
    std::vector<int> pre, rec_in, comp, mark;
    for (;;) {
        best.assign(n, std::numeric_limits<double>::infinity());
        pre.assign(n, -1);
        rec_in.assign(n, -1);
        for (const E& e : es)
            if (e.w < best[e.v]) {
                best[e.v] = e.w;
                pre[e.v] = e.u;
                rec_in[e.v] = e.rec;
            }
        for (int v = 0; v < n; ++v)
            if (v != r && rec_in[v] < 0) return false;
        for (int v = 0; v < n; ++v)
            if (v != r) ++uses[rec_in[v]];
        int comps = 0;
        comp.assign(n, -1);
        mark.assign(n, -1);
        for (int s = 0; s < n; ++s) {
            int x = s;
            while (x != r && comp[x] == -1 && mark[x] != s) {
                mark[x] = s;
                x = pre[x];
            }
            if (x != r && comp[x] == -1) {  // walked into our own trail: a cycle through x
                for (int y = pre[x]; y != x; y = pre[y]) comp[y] = comps;
                comp[x] = comps++;
            }
        }
        if (comps == 0) break;
        for (int v = 0; v < n; ++v)
            if (comp[v] == -1) comp[v] = comps++;
        std::vector<E> next;
        next.reserve(es.size());
        for (const E& e : es) {
            const int u2 = comp[e.u], v2 = comp[e.v];
            if (u2 == v2) continue;
            const int rec = static_cast<int>(uses.size());
            uses.push_back(0);
            stands_for.push_back(e.rec);
            displaces.push_back(rec_in[e.v]);
            next.push_back({u2, v2, e.w - best[e.v], rec});
        }
        es.swap(next);
        r = comp[r];
        n = comps;
        // arcs into the (possibly renamed) root are never useful
        es.erase(std::remove_if(es.begin(), es.end(), [r](const E& e) { return e.v == r; }), es.end());
    }
    for (int rec = static_cast<int>(uses.size()) - 1; rec >= m; --rec) {
        if (uses[rec] == 0) continue;
        uses[stands_for[rec - m]] += uses[rec];
        uses[displaces[rec - m]] -= uses[rec];
    }
    in_arc.assign(g.k, -1);
    for (int i = 0; i < m; ++i)
        if (uses[i] > 0) in_arc[g.arcs[i].v] = i;
    return true;
}

struct Candidate {
    ParentVec parent;
    std::vector<int> arcs;
    double weight;
};

ParentVec parents_of(const Graph& g, const std::vector<int>& in_arc, int root) {
    ParentVec p;
    p.fill(-2);
    for (int v = 0; v < g.k; ++v) p[v] = (v == root) ? -1 : static_cast<int8_t>(g.arcs[in_arc[v]].u);
    return p;
}

// Upper estimate of the rounds MWU needs (section 3.2: O(m ln m / eps^2)): every
// round multiplies the length of some arc by at least 1 + eps on its way from
// delta / c to at most (1 + eps) / c.
double mwu_round_estimate(int m, double eps) {
    return m * std::log((1.0 + eps) * m) / (eps * std::log1p(eps));
}
constexpr double kMaxMwuRounds = 5e7;  // about a minute of host time on 240 arcs

// MWU fractional packing; returns distinct trees with feasible weights.
//
// The common start value of the arc lengths, delta = (1 + eps) * ((1 + eps) m)^(-1/eps),
// underflows a double for small eps.  Where it does, `len` holds l_e / delta
// instead of l_e and the loop ends when log(sum c_e len_e) reaches -log(delta);
// whenever such relative lengths grow large they are scaled down together (a
// common factor changes no minimum arborescence) and `log_scale` keeps count.
std::vector<Candidate> mwu(const Graph& g, int root, double eps) {
    const int m = static_cast<int>(g.arcs.size());
    double log_goal = std::log((1.0 + eps) * m) / eps - std::log1p(eps);  // -log(delta)
    double start = 1.0, log_scale = 0.0;
    if (log_goal < 690.0) {  // delta is an ordinary double: work with the lengths themselves
        start = (1.0 + eps) * std::pow((1.0 + eps) * m, -1.0 / eps);
        log_goal = 0.0;
    }
    std::vector<double> len(m);
    double potential = 0.0;  // sum c_e * len_e
    for (int i = 0; i < m; ++i) {
        len[i] = start / g.arcs[i].cap;
        potential += start;
    }
    auto unfinished = [&]() { return std::log(potential) + log_scale < log_goal; };
    auto rescale = [&]() {
        if (potential < 0x1p400) return;
        for (double& l : len) l *= 0x1p-400;
        potential *= 0x1p-400;
        log_scale += 400.0 * std::log(2.0);
    };
    std::map<ParentVec, size_t> seen;
    std::vector<Candidate> out;
    std::vector<int> in_arc;
    while (unfinished()) {
        rescale();
        min_arborescence(g, root, len, in_arc);
        std::vector<int> arcs;
        double gamma = std::numeric_limits<double>::infinity(), found_len = 0.0;
        for (int v = 0; v < g.k; ++v)
            if (v != root) {
                arcs.push_back(in_arc[v]);
                gamma = std::min(gamma, g.arcs[in_arc[v]].cap);
                found_len += len[in_arc[v]];
            }
        const ParentVec p = parents_of(g, in_arc, root);
        auto it = seen.find(p);
        if (it == seen.end()) {
            it = seen.emplace(p, out.size()).first;
            out.push_back({p, arcs, 0.0});
        }
        Candidate& c = out[it->second];
        double cur_len = found_len;
        do {
            c.weight += gamma;
            cur_len = 0.0;
            for (int a : arcs) {
                const double grown = len[a] * (1.0 + eps * gamma / g.arcs[a].cap);
                potential += g.arcs[a].cap * (grown - len[a]);
                len[a] = grown;
                cur_len += grown;
            }
        } while (unfinished() && potential < 0x1p800 && cur_len <= (1.0 + eps) * found_len);
    }
    std::vector<double> load(m, 0.0);
    for (const Candidate& c : out)
        for (int a : c.arcs) load[a] += c.weight;
    double congestion = 0.0;
    for (int i = 0; i < m; ++i) congestion = std::max(congestion, load[i] / g.arcs[i].cap);
    for (Candidate& c : out) c.weight /= congestion;
    return out;
}

// max sum x_i over integers x_i >= 0 with sum_i x_i*unit*[a in T_i] <= c_a.
struct GridSearch {
    const Graph& g;
    int root;
    const std::vector<Candidate>& cands;
    double unit;
    long budget;
    std::vector<double> resid;
    std::vector<int> cur, best_x;
    long best = 0, cap_total = 0, nodes = 0;

    GridSearch(const Graph& g_, int root_, const std::vector<Candidate>& c, double unit_, long budget_)
        : g(g_), root(root_), cands(c), unit(unit_), budget(budget_) {
        for (const Arc& a : g.arcs) resid.push_back(a.cap);
        cur.assign(c.size(), 0);
        best_x = cur;
        cap_total = room();
    }
    // no packing exceeds the residual capacity entering any vertex
    long room() const {
        double least = std::numeric_limits<double>::infinity();
        for (int v = 0; v < g.k; ++v) {
            if (v == root) continue;
            double s = 0.0;
            for (int u = 0; u < g.k; ++u)
                if (g.index[u][v] >= 0) s += resid[g.index[u][v]];
            least = std::min(least, s);
        }
        return static_cast<long>(std::floor(least / unit + 1e-9));
    }
    bool descend(size_t i, long count) {
        ++nodes;
        if (count > best) {
            best = count;
            best_x = cur;
            if (best >= cap_total) return true;
        }
        if (i == cands.size() || nodes > budget || count + room() <= best) return false;
        double least = std::numeric_limits<double>::infinity();
        for (int a : cands[i].arcs) least = std::min(least, resid[a]);
        const long most = static_cast<long>(std::floor(least / unit + 1e-9));
        for (long mult = most; mult >= 0; --mult) {
            for (int a : cands[i].arcs) resid[a] -= mult * unit;
            cur[i] = static_cast<int>(mult);
            const bool done = descend(i + 1, count + mult);
            for (int a : cands[i].arcs) resid[a] += mult * unit;
            cur[i] = 0;
            if (done) return true;
        }
        return false;
    }
};

// max sum_j x_j  subject to  sum_j [arc i in tree j] x_j <= cap_i,  x >= 0, by
// the simplex method on a dense tableau (slack basis to start from: the origin
// is feasible).  cols[j] lists the arcs of column j.  Returns a vertex solution
// (hence at most cap.size() positive entries); false if the iteration limit
// was hit.  Dantzig's rule, switching to Bland's after a run of degenerate
// pivots so that it cannot cycle.
bool solve_packing_lp(const std::vector<double>& cap, const std::vector<const std::vector<int>*>& cols,
                      std::vector<double>& x) {
    const int m = static_cast<int>(cap.size()), n = static_cast<int>(cols.size());
    const int width = n + m + 1;  // tree columns, slack columns, right-hand side
    std::vector<double> t(static_cast<size_t>(m + 1) * width, 0.0);
    auto at = [&](int r, int c) -> double& { return t[static_cast<size_t>(r) * width + c]; };
    for (int j = 0; j < n; ++j) {
        for (int a : *cols[j]) at(a, j) = 1.0;
        at(m, j) = -1.0;  // objective row holds the negated reduced costs
    }
    for (int i = 0; i < m; ++i) {
        at(i, n + i) = 1.0;
        at(i, width - 1) = cap[i];
    }
    std::vector<int> basis(m);
    for (int i = 0; i < m; ++i) basis[i] = n + i;
    const double tol = 1e-11;
    int degenerate_run = 0;
    const long limit = 200L * (m + 10);
    for (long it = 0; it < limit; ++it) {
        int enter = -1;
        if (degenerate_run < 2 * m) {
            double most = -1e-9;
            for (int j = 0; j < n + m; ++j)
                if (at(m, j) < most) {
                    most = at(m, j);
                    enter = j;
                }
        } else {
            for (int j = 0; j < n + m && enter < 0; ++j)
                if (at(m, j) < -1e-9) enter = j;
        }
        if (enter < 0) {  // optimal
            x.assign(n, 0.0);
            for (int i = 0; i < m; ++i)
                if (basis[i] < n) x[basis[i]] = std::max(0.0, at(i, width - 1));
            return true;
        }
        int leave = -1;
        double best_ratio = std::numeric_limits<double>::infinity();
        for (int i = 0; i < m; ++i) {
            const double a = at(i, enter);
            if (a <= tol) continue;
            const double ratio = at(i, width - 1) / a;
            if (ratio < best_ratio - 1e-12 || (ratio < best_ratio + 1e-12 && leave >= 0 && basis[i] < basis[leave])) {
                best_ratio = ratio;
                leave = i;
            }
        }
        if (leave < 0) return false;  // unbounded: cannot happen, every tree uses an arc
        degenerate_run = best_ratio <= 1e-12 ? degenerate_run + 1 : 0;
        const double pivot = at(leave, enter);
        for (int c = 0; c < width; ++c) at(leave, c) /= pivot;
        for (int r = 0; r <= m; ++r) {
            if (r == leave) continue;
            const double f = at(r, enter);
            if (f == 0.0) continue;
            for (int c = 0; c < width; ++c) at(r, c) -= f * at(leave, c);
        }
        basis[leave] = enter;
    }
    return false;
}

// The linear-program fallback of section 3.2.1 (see the file header): weights
// for `cands`, at most one positive weight per arc, rate >= target if possible.
bool prune_by_lp(const Graph& g, const std::vector<Candidate>& cands, double target, std::vector<double>& w) {
    std::vector<double> cap;
    for (const Arc& a : g.arcs) cap.push_back(a.cap);
    std::vector<int> support(cands.size());
    for (size_t i = 0; i < cands.size(); ++i) support[i] = static_cast<int>(i);
    auto solve = [&](const std::vector<int>& idx, std::vector<double>& x) {
        std::vector<const std::vector<int>*> cols;
        for (int i : idx) cols.push_back(&cands[i].arcs);
        return solve_packing_lp(cap, cols, x);
    };
    std::vector<double> x;
    if (!solve(support, x)) return false;
    auto shrink = [&](std::vector<int>& idx, std::vector<double>& val) {  // keep the positive entries
        std::vector<int> i2;
        std::vector<double> v2;
        for (size_t j = 0; j < idx.size(); ++j)
            if (val[j] > 1e-9) {
                i2.push_back(idx[j]);
                v2.push_back(val[j]);
            }
        idx.swap(i2);
        val.swap(v2);
    };
    shrink(support, x);
    // drop light trees while the re-optimised rate stays above the target
    for (bool dropped = true; dropped && support.size() > 1;) {
        dropped = false;
        std::vector<size_t> order(support.size());
        for (size_t j = 0; j < order.size(); ++j) order[j] = j;
        std::sort(order.begin(), order.end(), [&](size_t a, size_t b) { return x[a] < x[b]; });
        for (size_t victim : order) {
            std::vector<int> rest;
            for (size_t j = 0; j < support.size(); ++j)
                if (j != victim) rest.push_back(support[j]);
            std::vector<double> y;
            if (!solve(rest, y)) continue;
            double rate = 0.0;
            for (double v : y) rate += v;
            if (rate >= target - 1e-9) {
                support.swap(rest);
                x.swap(y);
                shrink(support, x);
                dropped = true;
                break;
            }
        }
    }
    w.assign(cands.size(), 0.0);
    double rate = 0.0;
    for (size_t j = 0; j < support.size(); ++j) {
        w[support[j]] = x[j];
        rate += x[j];
    }
    return rate >= target - 1e-9;
}

void emit(const std::vector<Candidate>& cands, const std::vector<double>& w, int k, int root, Trees& out) {
    out.k = k;
    for (size_t i = 0; i < cands.size(); ++i) {
        if (!(w[i] > 0.0)) continue;
        out.root.push_back(root);
        out.parent.push_back(cands[i].parent);
        out.weight.push_back(w[i]);
    }
}

}  // namespace

blink_status_t pack_trees(int k, int m, const int32_t* src, const int32_t* dst, const double* cap,
                          int root, double eps, double prune_tol, Trees& out) {
    if (k < 2 || k > BLINK_MAX_RANKS || m < 1 || !src || !dst || !cap) return BLINK_EINVAL;
    if (root != BLINK_ROOT_ANY && (root < 0 || root >= k)) return BLINK_EINVAL;
    if (!(eps > 0.0 && eps <= 0.5) || !(prune_tol >= 0.0 && prune_tol < 1.0)) return BLINK_EINVAL;
    Graph g;
    g.k = k;
    for (auto& row : g.index) std::fill(std::begin(row), std::end(row), -1);
    for (int i = 0; i < m; ++i) {
        const int u = src[i], v = dst[i];
        if (u < 0 || u >= k || v < 0 || v >= k || u == v) return BLINK_EINVAL;
        if (!(cap[i] > 0.0) || !std::isfinite(cap[i])) return BLINK_EINVAL;
        if (g.index[u][v] < 0) {
            g.index[u][v] = static_cast<int>(g.arcs.size());
            g.arcs.push_back({u, v, cap[i]});
        } else {
            g.arcs[g.index[u][v]].cap += cap[i];
        }
    }

    if (root == BLINK_ROOT_ANY) {
        for (int u = 0; u < k; ++u)
            for (int v = 0; v < k; ++v)
                if (u != v && g.index[u][v] < 0) return BLINK_EINVAL;
        out.k = k;
        for (int r = 0; r < k; ++r) {
            ParentVec p;
            p.fill(-2);
            for (int v = 0; v < k; ++v) p[v] = (v == r) ? -1 : static_cast<int8_t>(r);
            out.root.push_back(r);
            out.parent.push_back(p);
            out.weight.push_back(1.0 / k);
        }
        return BLINK_OK;
    }

    // every vertex must be reachable from the root
    {
        std::vector<char> seen(k, 0);
        std::queue<int> q;
        q.push(root);
        seen[root] = 1;
        while (!q.empty()) {
            const int u = q.front();
            q.pop();
            for (int v = 0; v < k; ++v)
                if (g.index[u][v] >= 0 && !seen[v]) {
                    seen[v] = 1;
                    q.push(v);
                }
        }
        for (int v = 0; v < k; ++v)
            if (!seen[v]) return BLINK_EDISCONNECTED;
    }

    // an accuracy that would need more rounds than anybody waits for is refused at once
    if (mwu_round_estimate(static_cast<int>(g.arcs.size()), eps) > kMaxMwuRounds) return BLINK_EINVAL;
    std::vector<Candidate> cands = mwu(g, root, eps);
    std::sort(cands.begin(), cands.end(),
              [](const Candidate& a, const Candidate& b) { return a.weight > b.weight; });
    double mwu_rate = 0.0;
    for (const Candidate& c : cands) mwu_rate += c.weight;
    const double target = (1.0 - prune_tol) * mwu_rate;

    for (double unit = 1.0; unit >= 0.125; unit *= 0.5) {
        // a grid can only reach the optimum if the capacities lie on it
        bool on_grid = true;
        for (const Arc& a : g.arcs) on_grid = on_grid && std::fabs(a.cap / unit - std::round(a.cap / unit)) < 1e-9;
        if (!on_grid) continue;
        GridSearch gs(g, root, cands, unit, 2000000);
        gs.descend(0, 0);
        if (gs.best * unit >= target - 1e-9) {
            std::vector<double> w(cands.size());
            for (size_t i = 0; i < cands.size(); ++i) w[i] = gs.best_x[i] * unit;
            emit(cands, w, k, root, out);
            return BLINK_OK;
        }
    }
    {
        std::vector<double> w;
        if (prune_by_lp(g, cands, target, w)) {
            // guard against rounding: scale down if an arc came out a hair over capacity
            std::vector<double> load(g.arcs.size(), 0.0);
            for (size_t i = 0; i < cands.size(); ++i)
                for (int a : cands[i].arcs) load[a] += w[i];
            double congestion = 1.0;
            for (size_t a = 0; a < load.size(); ++a) congestion = std::max(congestion, load[a] / g.arcs[a].cap);
            for (double& v : w) v /= congestion;
            emit(cands, w, k, root, out);
            return BLINK_OK;
        }
    }
    // last resort: keep the heaviest MWU trees up to the tolerated loss
    std::vector<double> w(cands.size(), 0.0);
    double kept = 0.0;
    for (size_t i = 0; i < cands.size() && kept < target; ++i) {
        w[i] = cands[i].weight;
        kept += w[i];
    }
    emit(cands, w, k, root, out);
    return BLINK_OK;
}

}  // namespace blink
