// Exact solver of the ETS cost model (ETS paper Sec. 4.2, Eq. 4; as an ILP: App. B, Eq. 7).
//
// Without the coverage term the problem decomposes over the tree: a leaf is worth
// a_i = W_i / sum W - c with c = lambda_b / |V_A|, an inner node costs c as soon as a leaf
// beneath it is kept, so best(v) = max(0, sum_children best(child) - c) from the leaves
// up, and "at least one leaf" is met by the best single chain when everything else loses.
// The coverage term pays d = lambda_d / |C_A| once per cluster with a kept leaf: with
// z_k <= sum_{i in C_k} x_i relaxed by multipliers 0 <= u_k <= d the problem decomposes
// again (a leaf of cluster k is worth a_i + u_k, the cluster d - u_k by itself), and the
// best multipliers, found by subgradient steps, give the bound of the linear relaxation.
// Branch and bound on top: every relaxed solution is a candidate; when bound and
// candidate differ, the cluster with the largest share of the gap is decided: either none
// of its leaves is kept, or its first kept leaf (in leaf order) is leaf i -- one branch per
// i, with i forced and the cluster's earlier leaves excluded.
#include "selector.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <new>

namespace ets {

void rebase_weights(int32_t n, const double* rewards, int32_t budget, double temperature,
                    int32_t* weights) {
    std::vector<int32_t> order(n);
    for (int32_t i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return rewards[a] > rewards[b]; });
    std::vector<double> e(n), tail((size_t)n + 1, 0.0);
    for (int32_t p = 0; p < n; ++p) e[p] = std::exp(rewards[order[p]] / temperature);
    for (int32_t p = n - 1; p >= 0; --p) tail[p] = tail[p + 1] + e[p];
    int64_t left = budget;
    for (int32_t i = 0; i < n; ++i) weights[i] = 0;
    for (int32_t p = 0; p < n && left > 0; ++p) {
        const int64_t w = std::min<int64_t>(left, (int64_t)std::ceil((double)left * (e[p] / tail[p])));
        weights[order[p]] = (int32_t)w;
        left -= w;
    }
}

namespace {

constexpr double kEps = 1e-12;
constexpr double kNegInf = -std::numeric_limits<double>::infinity();

enum : int8_t { FREE = 0, EXCLUDED = 1, FORCED = 2 };

struct Solver {
    // live tree, nodes renumbered 0..M-1 in the caller's order (parents first)
    int32_t M = 0, L = 0, K = 0;
    std::vector<int32_t> par;        // [M] parent or -1
    std::vector<int32_t> leaf_of;    // [M] leaf index or -1
    std::vector<int32_t> node_of;    // [L]
    std::vector<double> a;           // [L] W_i / sum W - c
    std::vector<int32_t> clu;        // [L] cluster id 0..K-1 (K = 0: none)
    std::vector<std::vector<int32_t>> members;  // leaves of every cluster, ascending
    double c = 0.0, d = 0.0;
    int64_t node_limit = 0, visited = 0;
    bool hit_limit = false;
    // branch state
    std::vector<int8_t> leaf_state;  // [L]
    std::vector<int8_t> clu_done;    // [K] decided: its bonus is in `paid` or it is excluded
    std::vector<double> u;           // [K] multipliers of the undecided clusters
    // incumbent
    double best = kNegInf;
    std::vector<uint8_t> best_keep;
    // scratch
    std::vector<double> f, g;        // [M] best value of the subtree: anything / at least one leaf
    std::vector<double> sum_f, max_g;  // [M] over the children
    std::vector<int32_t> arg_g;      // [M] child with the best g
    std::vector<uint8_t> forced_below;  // [M] a forced leaf lies at or beneath the node
    std::vector<uint8_t> keep;       // [L]

    double leaf_value(int32_t i) const {
        if (leaf_state[i] == EXCLUDED) return kNegInf;
        return a[i] + ((K > 0 && !clu_done[clu[i]]) ? u[clu[i]] : 0.0);
    }

    // Bound of the current branch state and its selection (keep[]).
    double relax() {
        for (int32_t v = 0; v < M; ++v) {
            sum_f[v] = 0.0;
            max_g[v] = kNegInf;
            arg_g[v] = -1;
            forced_below[v] = 0;
        }
        for (int32_t v = M - 1; v >= 0; --v) {
            if (leaf_of[v] >= 0) {
                const int32_t i = leaf_of[v];
                g[v] = leaf_value(i);
                forced_below[v] = leaf_state[i] == FORCED;
            } else {
                // at least one leaf beneath: every child that gains, else the best one
                g[v] = (sum_f[v] > 0.0 || forced_below[v]) ? sum_f[v] - c : max_g[v] - c;
            }
            f[v] = forced_below[v] ? g[v] : std::max(0.0, g[v]);
            const int32_t p = par[v];
            if (p >= 0) {
                sum_f[p] += f[v];
                if (g[v] > max_g[p]) {
                    max_g[p] = g[v];
                    arg_g[p] = v;
                }
                forced_below[p] |= forced_below[v];
            }
        }
        double total = 0.0, best_root = kNegInf;
        int32_t arg_root = -1;
        bool any = false;
        for (int32_t v = 0; v < M; ++v)
            if (par[v] < 0) {
                total += f[v];
                any |= f[v] > 0.0 || forced_below[v];
                if (g[v] > best_root) {
                    best_root = g[v];
                    arg_root = v;
                }
            }
        std::fill(keep.begin(), keep.end(), 0);
        // walk down: `must` = the subtree has to keep at least one leaf
        std::vector<std::pair<int32_t, bool>> stack;
        if (!any) {
            if (arg_root < 0 || best_root == kNegInf) return kNegInf;  // nothing may be kept
            total = best_root;
            stack.push_back({arg_root, true});
        } else {
            for (int32_t v = 0; v < M; ++v)
                if (par[v] < 0 && (f[v] > 0.0 || forced_below[v])) stack.push_back({v, true});
        }
        // children lists are implicit (parents first): collect once
        if (child_begin.empty()) build_children();
        while (!stack.empty()) {
            const int32_t v = stack.back().first;
            stack.pop_back();
            if (leaf_of[v] >= 0) {
                keep[leaf_of[v]] = 1;
                continue;
            }
            if (sum_f[v] > 0.0 || forced_below[v]) {
                for (int32_t e = child_begin[v]; e < child_begin[v + 1]; ++e) {
                    const int32_t ch = children[e];
                    if (f[ch] > 0.0 || forced_below[ch]) stack.push_back({ch, true});
                }
            } else {
                stack.push_back({arg_g[v], true});
            }
        }
        return total;
    }

    std::vector<int32_t> child_begin, children;
    void build_children() {
        child_begin.assign((size_t)M + 1, 0);
        for (int32_t v = 0; v < M; ++v)
            if (par[v] >= 0) child_begin[par[v] + 1] += 1;
        for (int32_t v = 0; v < M; ++v) child_begin[v + 1] += child_begin[v];
        children.assign(child_begin[M], 0);
        std::vector<int32_t> cur(child_begin.begin(), child_begin.end() - 1);
        for (int32_t v = 0; v < M; ++v)
            if (par[v] >= 0) children[cur[par[v]]++] = v;
    }

    // True objective of keep[] (sums a over kept leaves, c per kept inner node, d per cluster).
    double evaluate(const std::vector<uint8_t>& kp) const {
        std::vector<uint8_t> on(M, 0), cov(std::max(K, 1), 0);
        double val = 0.0;
        bool any = false;
        for (int32_t i = 0; i < L; ++i) {
            if (!kp[i]) continue;
            any = true;
            val += a[i];
            if (K > 0 && !cov[clu[i]]) {
                cov[clu[i]] = 1;
                val += d;
            }
            for (int32_t v = par[node_of[i]]; v >= 0 && !on[v]; v = par[v]) {
                on[v] = 1;
                val -= c;
            }
        }
        return any ? val : kNegInf;
    }

    void branch(double paid) {
        if (hit_limit) return;
        if (++visited > node_limit) {
            hit_limit = true;
            return;
        }
        // subgradient steps on the multipliers of the undecided clusters
        std::vector<int32_t> cnt(std::max(K, 1), 0);
        std::vector<double> u_best = u;
        double bound_best = std::numeric_limits<double>::infinity();
        int32_t pick = -1;
        const int iters = K > 0 ? 60 : 1;
        double theta = 1.0;
        for (int it = 0; it < iters; ++it) {
            const double inner = relax();
            if (inner == kNegInf) return;  // nothing may be kept any more
            double bound = inner + paid;
            for (int32_t k = 0; k < K; ++k)
                if (!clu_done[k]) bound += d - u[k];
            const double val = evaluate(keep);
            if (val > best + kEps) {
                best = val;
                best_keep = keep;
            }
            if (bound < bound_best) {
                bound_best = bound;
                u_best = u;
            } else {
                theta *= 0.8;
            }
            if (bound_best <= best + kEps) return;  // pruned (or solved: the candidate attains it)
            if (K == 0) return;
            // gap of this multiplier vector, cluster by cluster
            std::fill(cnt.begin(), cnt.end(), 0);
            for (int32_t i = 0; i < L; ++i)
                if (keep[i] && !clu_done[clu[i]]) cnt[clu[i]] += 1;
            double norm = 0.0, gap_max = 0.0;
            pick = -1;
            for (int32_t k = 0; k < K; ++k) {
                if (clu_done[k]) continue;
                const double gap = cnt[k] == 0 ? d - u[k] : u[k] * (cnt[k] - 1);
                if (gap > gap_max) {
                    gap_max = gap;
                    pick = k;
                }
                const double sg = cnt[k] - 1.0;
                // a step against a bound of the multiplier does nothing
                if ((sg < 0.0 && u[k] < d) || (sg > 0.0 && u[k] > 0.0)) norm += sg * sg;
            }
            if (pick < 0 || gap_max <= kEps) return;  // bound attained by its own selection
            if (norm == 0.0) break;
            const double step = theta * std::max(bound - best, 1e-9) / norm;
            for (int32_t k = 0; k < K; ++k)
                if (!clu_done[k]) u[k] = std::min(d, std::max(0.0, u[k] - step * (cnt[k] - 1.0)));
        }
        // branch from the best multipliers
        u = u_best;
        relax();
        std::fill(cnt.begin(), cnt.end(), 0);
        for (int32_t i = 0; i < L; ++i)
            if (keep[i] && !clu_done[clu[i]]) cnt[clu[i]] += 1;
        double gap_max = -1.0;
        pick = -1;
        for (int32_t k = 0; k < K; ++k) {
            if (clu_done[k]) continue;
            const double gap = cnt[k] == 0 ? d - u[k] : u[k] * (cnt[k] - 1);
            if (gap > gap_max) {
                gap_max = gap;
                pick = k;
            }
        }
        if (pick < 0) return;
        const std::vector<double> u_node = u;
        const std::vector<int32_t>& mem = members[pick];
        clu_done[pick] = 1;
        // leaves kept by the relaxed solution first: good candidates early
        std::vector<size_t> order;
        for (size_t t = 0; t < mem.size(); ++t)
            if (keep[mem[t]]) order.push_back(t);
        const size_t n_kept_first = order.size();
        for (size_t t = 0; t < mem.size(); ++t)
            if (std::find(order.begin(), order.begin() + (std::ptrdiff_t)n_kept_first, t) ==
                order.begin() + (std::ptrdiff_t)n_kept_first)
                order.push_back(t);
        // the cluster's first kept leaf is mem[t]: the earlier ones are excluded
        for (size_t t : order) {
            if (hit_limit) break;
            for (size_t w = 0; w < t; ++w) leaf_state[mem[w]] = EXCLUDED;
            leaf_state[mem[t]] = FORCED;
            u = u_node;
            branch(paid + d);
            for (size_t w = 0; w <= t; ++w) leaf_state[mem[w]] = FREE;
        }
        // none of its leaves is kept
        if (!hit_limit) {
            for (size_t t = 0; t < mem.size(); ++t) leaf_state[mem[t]] = EXCLUDED;
            u = u_node;
            branch(paid);
            for (size_t t = 0; t < mem.size(); ++t) leaf_state[mem[t]] = FREE;
        }
        clu_done[pick] = 0;
        u = u_node;
    }
};

}  // namespace

ets_status select_leaves(const ets_tree& t, const int32_t* weights, const int32_t* cluster,
                         double lambda_b, double lambda_d, int64_t node_limit, SelectResult& out) {
    if (t.n_nodes < 0 || t.n_leaves <= 0 || !t.parent || !t.leaf_node || !weights)
        return ETS_ERR_INVALID_ARG;
    if (!(lambda_b >= 0.0) || !(lambda_d >= 0.0)) return ETS_ERR_INVALID_ARG;
    const int32_t N = t.n_nodes, L = t.n_leaves;
    for (int32_t i = 0; i < N; ++i)
        if (t.parent[i] < -1 || t.parent[i] >= i) return ETS_ERR_BAD_TREE;
    try {
        std::vector<int32_t> leaf_of(N, -1);
        double wsum = 0.0;
        for (int32_t l = 0; l < L; ++l) {
            const int32_t v = t.leaf_node[l];
            if (v < 0 || v >= N || leaf_of[v] >= 0) return ETS_ERR_BAD_LEAF;
            if (weights[l] < 0) return ETS_ERR_INVALID_ARG;
            leaf_of[v] = l;
            wsum += weights[l];
        }
        if (!(wsum > 0.0)) return ETS_ERR_INVALID_ARG;
        std::vector<uint8_t> live(N, 0);
        for (int32_t l = 0; l < L; ++l)
            for (int32_t v = t.leaf_node[l]; v >= 0 && !live[v]; v = t.parent[v]) live[v] = 1;
        // no leaf beneath another leaf
        for (int32_t l = 0; l < L; ++l)
            for (int32_t v = t.parent[t.leaf_node[l]]; v >= 0; v = t.parent[v])
                if (leaf_of[v] >= 0) return ETS_ERR_BAD_LEAF;
        Solver s;
        std::vector<int32_t> new_id(N, -1);
        for (int32_t v = 0; v < N; ++v)
            if (live[v]) new_id[v] = s.M++;
        s.L = L;
        s.par.assign(s.M, -1);
        s.leaf_of.assign(s.M, -1);
        s.node_of.assign(L, 0);
        for (int32_t v = 0; v < N; ++v) {
            if (!live[v]) continue;
            s.par[new_id[v]] = t.parent[v] >= 0 ? new_id[t.parent[v]] : -1;
            s.leaf_of[new_id[v]] = leaf_of[v];
            if (leaf_of[v] >= 0) s.node_of[leaf_of[v]] = new_id[v];
        }
        s.c = lambda_b / (double)s.M;
        s.a.resize(L);
        for (int32_t l = 0; l < L; ++l) s.a[l] = (double)weights[l] / wsum - s.c;
        if (cluster && lambda_d > 0.0) {
            // dense cluster ids in order of first appearance
            std::vector<int32_t> ids;
            s.clu.resize(L);
            for (int32_t l = 0; l < L; ++l) {
                auto it = std::find(ids.begin(), ids.end(), cluster[l]);
                if (it == ids.end()) {
                    ids.push_back(cluster[l]);
                    it = ids.end() - 1;
                }
                s.clu[l] = (int32_t)(it - ids.begin());
            }
            s.K = (int32_t)ids.size();
            s.members.assign(s.K, {});
            for (int32_t l = 0; l < L; ++l) s.members[s.clu[l]].push_back(l);
            s.d = lambda_d / (double)s.K;
        }
        s.leaf_state.assign(L, FREE);
        s.clu_done.assign(std::max(s.K, 1), 0);
        s.u.assign(std::max(s.K, 1), s.d);
        s.f.resize(s.M);
        s.g.resize(s.M);
        s.sum_f.resize(s.M);
        s.max_g.resize(s.M);
        s.arg_g.resize(s.M);
        s.forced_below.resize(s.M);
        s.keep.assign(L, 0);
        s.node_limit = node_limit > 0 ? node_limit : (int64_t)1 << 22;
        s.branch(0.0);
        if (s.best == kNegInf) return ETS_ERR_INVALID_ARG;
        out.keep = s.best_keep;
        out.objective = s.best;
        out.bb_nodes = s.visited;
        out.optimal = !s.hit_limit;
        out.live_nodes = s.M;
        out.clusters = s.K;
        std::vector<uint8_t> on(s.M, 0), cov(std::max(s.K, 1), 0);
        out.kept_nodes = 0;
        out.kept_clusters = 0;
        for (int32_t l = 0; l < L; ++l) {
            if (!out.keep[l]) continue;
            if (s.K > 0 && !cov[s.clu[l]]) {
                cov[s.clu[l]] = 1;
                out.kept_clusters += 1;
            }
            for (int32_t v = s.node_of[l]; v >= 0 && !on[v]; v = s.par[v]) {
                on[v] = 1;
                out.kept_nodes += 1;
            }
        }
        return ETS_OK;
    } catch (const std::bad_alloc&) {
        return ETS_ERR_NOMEM;
    }
}

}  // namespace ets
