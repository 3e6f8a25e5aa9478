// Planner of step-prefill attention: per distinct leaf node one run list (ancestors'
// rows merged where they are contiguous in the pool and cut into pieces of at most 32,
// then the node's own rows in pieces of 32 counted from its first row), per leaf query
// blocks of 128 / G query tokens.  Leaf queries are taken in depth-first order of their
// nodes, so that workgroups that run at the same time walk the same ancestors.
#include "prefill_plan.h"

#include <algorithm>
#include <limits>
#include <new>

namespace ets {
namespace {

ets_status check(const ets_tree& t) {
    if (t.n_nodes < 0 || t.n_leaves < 0) return ETS_ERR_INVALID_ARG;
    if (t.n_nodes > 0 && (!t.parent || !t.tok_offset || !t.n_tokens)) return ETS_ERR_INVALID_ARG;
    if (t.n_leaves > 0 && !t.leaf_node) return ETS_ERR_INVALID_ARG;
    for (int32_t i = 0; i < t.n_nodes; ++i) {
        if (t.parent[i] < -1 || t.parent[i] >= i) return ETS_ERR_BAD_TREE;
        if (t.n_tokens[i] < 0 || t.tok_offset[i] < 0) return ETS_ERR_BAD_TREE;
        if (t.tok_offset[i] > std::numeric_limits<int64_t>::max() - t.n_tokens[i])
            return ETS_ERR_BAD_TREE;
    }
    for (int32_t l = 0; l < t.n_leaves; ++l)
        if (t.leaf_node[l] < 0 || t.leaf_node[l] >= t.n_nodes) return ETS_ERR_BAD_LEAF;
    return ETS_OK;
}

ets_status build(const ets_shape& shape, const ets_tree& tree, PrefillPlan& p,
                 int64_t kv_elem_bytes) {
    const int32_t N = tree.n_nodes, L = tree.n_leaves;
    const int32_t G = shape.n_q_heads / shape.n_kv_heads;
    const int32_t tq = kPrefillRowsPerItem / G;  // query tokens per item
    p.parent.assign(tree.parent, tree.parent + N);
    p.tok_offset.assign(tree.tok_offset, tree.tok_offset + N);
    p.n_tokens.assign(tree.n_tokens, tree.n_tokens + N);
    p.leaf_node.assign(tree.leaf_node, tree.leaf_node + L);
    p.runs.clear();
    p.items.clear();
    p.q_ptr.assign((size_t)L + 1, 0);
    p.item_begin.assign((size_t)L, 0);
    for (int32_t l = 0; l < L; ++l) p.q_ptr[l + 1] = p.q_ptr[l] + p.n_tokens[p.leaf_node[l]];

    // depth-first position of every node: children (larger ids) in id order
    std::vector<int32_t> first_child(N, -1), next_sibling(N, -1), last_child(N, -1), roots;
    for (int32_t i = 0; i < N; ++i) {
        const int32_t par = p.parent[i];
        if (par < 0) {
            roots.push_back(i);
        } else if (first_child[par] < 0) {
            first_child[par] = last_child[par] = i;
        } else {
            next_sibling[last_child[par]] = i;
            last_child[par] = i;
        }
    }
    std::vector<int32_t> dfs_pos(N, 0), stack;
    int32_t pos = 0;
    for (auto r = roots.rbegin(); r != roots.rend(); ++r) stack.push_back(*r);
    while (!stack.empty()) {
        const int32_t n = stack.back();
        stack.pop_back();
        dfs_pos[n] = pos++;
        // push the siblings' chain in reverse so that the smallest id is visited first
        const size_t mark = stack.size();
        for (int32_t c = first_child[n]; c >= 0; c = next_sibling[c]) stack.push_back(c);
        std::reverse(stack.begin() + (std::ptrdiff_t)mark, stack.end());
    }
    std::vector<int32_t> order(L);
    for (int32_t l = 0; l < L; ++l) order[l] = l;
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
        return dfs_pos[p.leaf_node[x]] < dfs_pos[p.leaf_node[y]];
    });

    ets_prefill_stats& st = p.stats;
    st = ets_prefill_stats{};
    st.n_leaves = L;
    st.n_q_rows = p.q_ptr[L];
    st.rows_per_item = kPrefillRowsPerItem;
    std::vector<char> live(N, 0);

    std::vector<int32_t> chain;
    std::vector<int32_t> run_begin_of(N, -1), anc_runs_of(N, 0);  // per distinct leaf node
    std::vector<int64_t> anc_tokens_of(N, 0);
    std::vector<std::vector<PrefillItem>> per_leaf((size_t)L);
    for (int32_t oi = 0; oi < L; ++oi) {
        const int32_t l = order[oi];
        const int32_t v = p.leaf_node[l];
        const int32_t len = p.n_tokens[v];
        if (run_begin_of[v] < 0 && len > 0) {
            chain.clear();
            for (int32_t x = v; x >= 0; x = p.parent[x]) chain.push_back(x);
            std::reverse(chain.begin(), chain.end());
            run_begin_of[v] = (int32_t)p.runs.size();
            // ancestors: contiguous rows merge, then pieces of 32
            int64_t cur_tok = 0, cur_n = 0, anc_tokens = 0;
            auto flush = [&]() {
                for (int64_t off = 0; off < cur_n; off += 32)
                    p.runs.push_back(Run{cur_tok + off, (int32_t)std::min<int64_t>(32, cur_n - off),
                                         kAncestorRun});
                cur_n = 0;
            };
            for (size_t c = 0; c + 1 < chain.size(); ++c) {
                const int32_t n = chain[c];
                live[n] = 1;
                if (p.n_tokens[n] <= 0) continue;
                anc_tokens += p.n_tokens[n];
                if (cur_n > 0 && cur_tok + cur_n == p.tok_offset[n]) {
                    cur_n += p.n_tokens[n];
                } else {
                    flush();
                    cur_tok = p.tok_offset[n];
                    cur_n = p.n_tokens[n];
                }
            }
            flush();
            live[v] = 1;
            anc_runs_of[v] = (int32_t)p.runs.size() - run_begin_of[v];
            anc_tokens_of[v] = anc_tokens;
            for (int32_t off = 0; off < len; off += 32)
                p.runs.push_back(Run{p.tok_offset[v] + off, std::min(32, len - off), off});
            if (p.runs.size() > (size_t)std::numeric_limits<int32_t>::max() - 64)
                return ETS_ERR_UNSUPPORTED;
        }
        for (int32_t t0 = 0; t0 < len; t0 += tq) {
            PrefillItem it{};
            it.n_tok = std::min(tq, len - t0);
            it.tok0 = t0;
            it.run_begin = run_begin_of[v];
            it.run_end = run_begin_of[v] + anc_runs_of[v] + (t0 + it.n_tok - 1) / 32 + 1;
            it.q_row0 = p.q_ptr[l] + t0;
            it.leaf = l;
            per_leaf[l].push_back(it);
            // what the block's queries see: ancestors in full, own rows causally
            const int64_t a = t0, b = t0 + it.n_tok;  // own rows visible: a + 1 .. b
            st.visible_pairs += it.n_tok * anc_tokens_of[v] + (b * (b + 1) - a * (a + 1)) / 2;
            for (int32_t r = it.run_begin; r < it.run_end; ++r) st.streamed_tokens += p.runs[r].n;
        }
    }
    // items in the depth-first leaf order; item_begin indexes them per leaf query
    std::vector<int32_t> n_items_of(L, 0);
    for (int32_t oi = 0; oi < L; ++oi) {
        const int32_t l = order[oi];
        n_items_of[l] = (int32_t)per_leaf[l].size();
        for (const PrefillItem& it : per_leaf[l]) p.items.push_back(it);
    }
    {
        // position of leaf query l's first item in p.items
        int32_t cursor = 0;
        std::vector<int32_t> first(L, 0);
        for (int32_t oi = 0; oi < L; ++oi) {
            first[order[oi]] = cursor;
            cursor += n_items_of[order[oi]];
        }
        for (int32_t l = 0; l < L; ++l) p.item_begin[l] = first[l];
    }
    st.n_items = (int64_t)p.items.size();
    st.n_runs = (int64_t)p.runs.size();
    for (int32_t i = 0; i < N; ++i) {
        if (!live[i]) continue;
        st.unique_tokens += p.n_tokens[i];
        if (p.n_tokens[i] > 0)
            st.min_pool_tokens = std::max(st.min_pool_tokens, p.tok_offset[i] + p.n_tokens[i]);
    }
    const int64_t tok_bytes = 2 * (int64_t)shape.n_kv_heads * shape.head_dim * kv_elem_bytes;
    st.unique_kv_bytes = st.unique_tokens * tok_bytes;
    st.streamed_kv_bytes = st.streamed_tokens * tok_bytes;
    // two contractions of head_dim per (query row, visible key row), 2 flops per multiply-add
    st.flops = 4 * (int64_t)shape.head_dim * shape.n_q_heads * st.visible_pairs;
    p.valid = true;
    return ETS_OK;
}

}  // namespace

ets_status build_prefill_plan(const ets_shape& shape, const ets_tree& tree, PrefillPlan& plan,
                              int64_t kv_elem_bytes) {
    plan.valid = false;
    const ets_status s = check(tree);
    if (s != ETS_OK) return s;
    try {
        return build(shape, tree, plan, kv_elem_bytes);
    } catch (const std::bad_alloc&) {
        plan.valid = false;
        return ETS_ERR_NOMEM;
    }
}

bool prefill_cover(const PrefillPlan& p, int32_t leaf, int32_t tok, std::vector<int64_t>& rows) {
    rows.clear();
    // the items of a leaf query are consecutive, in token order
    for (size_t i = (size_t)p.item_begin[leaf]; i < p.items.size() && p.items[i].leaf == leaf; ++i) {
        const PrefillItem& it = p.items[i];
        if (tok < it.tok0 || tok >= it.tok0 + it.n_tok) continue;
        for (int32_t r = it.run_begin; r < it.run_end; ++r) {
            const Run& run = p.runs[r];
            for (int32_t t = 0; t < run.n; ++t)
                if ((int64_t)run.pad + t <= tok) rows.push_back(run.tok + t);
        }
        return true;
    }
    return false;
}

bool check_prefill_plan(const PrefillPlan& p, const ets_shape& shape, PlanCheck& out) {
    out = PlanCheck{};
    const int G = shape.n_q_heads / shape.n_kv_heads;
    const int64_t n_runs = (int64_t)p.runs.size();
    auto bad = [&](bool cond) {
        if (cond) out.violations += 1;
    };
    for (const PrefillItem& it : p.items) {
        out.items += 1;
        bad(it.run_begin < 0 || it.run_end < it.run_begin || it.run_end > n_runs);
        bad(it.n_tok < 1 || it.n_tok * G > kPrefillRowsPerItem);
        bad(it.leaf < 0 || it.leaf >= p.stats.n_leaves);
        // query tokens past n_tok are clamped to the block's last one by the kernel
        bad(it.q_row0 < 0 || it.q_row0 + it.n_tok > p.stats.n_q_rows);
        for (int64_t r = it.run_begin; r < it.run_end && r < n_runs; ++r) {
            const Run& run = p.runs[(size_t)r];
            bad(run.n < 0 || run.n > 32 || run.tok < 0);
            if (run.n > 0) {
                bad(run.tok + run.n > p.stats.min_pool_tokens);
                out.max_pool_row = std::max(out.max_pool_row, run.tok + run.n - 1);
            }
        }
    }
    return out.violations == 0;
}

}  // namespace ets
