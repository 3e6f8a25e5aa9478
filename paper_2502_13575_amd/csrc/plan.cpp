// Host planner: validates the tree, counts leaf queries per node, compacts
// chains of nodes with identical leaf sets into segments, cuts segments into
// work items for the two attention kernels and numbers the partial results.
//
// Tree semantics after the ETS paper, Sec. 4.1 and App. B: a non-leaf node is
// needed iff some retained leaf is among its descendants, and all trajectories
// through a node share that node's KV.
#include "plan.h"

#include <algorithm>
#include <limits>
#include <new>

namespace ets {
namespace {

// Whether the planner, left to decide, merges inside the attention launch.
bool fuse_by_default(const ets_stats&) { return false; }

struct Seg {
    int32_t parent_seg = -1;
    int64_t cnt = 0;             // leaf queries at or beneath the segment
    std::vector<int32_t> nodes;  // chain, root side first
    int64_t tokens = 0;
    int32_t ent_begin = 0;       // range in Plan::ent_order
    int32_t own_filled = 0;
    int32_t child_cursor = 0;
    int32_t prefix = 0;          // partial slots used by the segments above
    int32_t n_chunks = 0;
    bool cascade = false;
    bool wide = false;           // read by the wide kernel (many query rows)
};

struct Chunk {
    int32_t run_begin, run_end, tokens;
};

constexpr int64_t kMaxPiecesPerChunk = kTreeAttnMaxSteps;  // step list the kernel keeps in LDS

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t m) { return ceil_div(a, m) * m; }

// Appends the (merged) pool runs of a node list to `out`.  A node that holds leaf
// queries grows by a token per decode step: the run that ends such a node is marked
// (pad = 1) and nothing is merged behind it.  Returns false if a growing node has no
// rows yet (there is no run to mark).
bool collect_runs(const Plan& p, const std::vector<int32_t>& nodes, const std::vector<int64_t>& own,
                  std::vector<Run>& out) {
    bool ok = true;
    bool closed = true;  // the previous run must not be extended
    for (int32_t n : nodes) {
        const int32_t len = p.n_tokens[n];
        const bool grows = own[n] > 0;
        if (len <= 0) {
            if (grows) ok = false;
            continue;
        }
        const int64_t tok = p.tok_offset[n];
        if (!closed && !out.empty() && out.back().tok + out.back().n == tok &&
            (int64_t)out.back().n + len <= std::numeric_limits<int32_t>::max()) {
            out.back().n += len;
        } else {
            out.push_back(Run{tok, len, 0});
        }
        out.back().pad = grows ? 1 : 0;
        closed = grows;
    }
    return ok;
}

// Cuts `src` (total `tokens` rows) into chunks of at most `cap` rows, sized
// evenly in multiples of 32 rows, appending the chunks' runs to plan.runs.  With
// piece > 0 no emitted run is longer than `piece` rows (the matrix-core kernel
// walks its run list in steps of at most 32 rows).  Behind the last piece of a marked
// run (a growing node's tail) an empty spare run is emitted and an AdvEntry recorded;
// returns false if a chunk's step list had no room for a spare.
bool cut_runs(Plan& p, const std::vector<Run>& src, int64_t tokens, int64_t cap, int64_t piece,
              std::vector<Chunk>& chunks) {
    chunks.clear();
    if (tokens <= 0) return true;
    bool ok = true;
    cap = std::max<int64_t>(cap, 32);
    int64_t n_chunks = ceil_div(tokens, cap);
    int64_t per = std::min(cap, round_up(ceil_div(tokens, n_chunks), 32));
    size_t ri = 0;
    int64_t used = 0;  // rows of src[ri] already handed out
    int64_t left = tokens;
    while (left > 0) {
        int64_t want = std::min(per, left);
        Chunk c{(int32_t)p.runs.size(), 0, 0};
        int64_t pieces = 0;
        while (want > 0 && (piece <= 0 || pieces < kMaxPiecesPerChunk)) {
            const int64_t avail = src[ri].n - used;
            int64_t take = std::min(avail, want);
            if (piece > 0) take = std::min(take, piece);
            p.runs.push_back(Run{src[ri].tok + used, (int32_t)take, 0});
            used += take;
            want -= take;
            c.tokens += (int32_t)take;
            ++pieces;
            if (used == src[ri].n) {
                if (src[ri].pad) {
                    if (piece > 0 && pieces >= kMaxPiecesPerChunk) {
                        ok = false;
                    } else {
                        const int32_t r_last = (int32_t)p.runs.size() - 1;
                        const int64_t end0 = src[ri].tok + src[ri].n;
                        p.adv.push_back(AdvEntry{r_last, r_last + 1, end0, 1, 0});
                        p.runs.push_back(Run{end0, 0, 0});
                        ++pieces;
                    }
                }
                ++ri;
                used = 0;
            }
        }
        c.run_end = (int32_t)p.runs.size();
        left -= c.tokens;
        chunks.push_back(c);
    }
    return ok;
}

// Fills the slot's copies of its item's steps from the step lists.  Returns whether one of
// them is a run that an advance may extend.
bool fill_unit_steps(const Plan& p, UnitSlot& u, int wave, const std::vector<char>* grows) {
    bool may_grow = false;
    Run* dst[2] = {&u.first, &u.second};
    for (int j = 0; j < 2; ++j) {
        const int k = unit_step_index(u.item, wave, j);
        const int64_t r = (int64_t)u.item.run_begin + k;
        if (k < 0 || r >= u.item.run_end) {
            *dst[j] = Run{0, 0, 0};
            continue;
        }
        *dst[j] = p.runs[(size_t)r];
        if (grows) may_grow = may_grow || (*grows)[(size_t)r];
    }
    return may_grow;
}

// The table the matrix-core kernel starts from (see UnitSlot), and the slots whose copies
// of steps an advance has to refresh.
void build_units(Plan& p) {
    const size_t n_units = p.wg_map.size();
    p.units.assign(4 * n_units, UnitSlot{});  // zero: n_ent = 0, nothing to do
    p.adv_slots.clear();
    std::vector<char> grows(p.runs.size(), 0);
    for (const AdvEntry& e : p.adv) grows[(size_t)e.r_last] = grows[(size_t)e.r_spare] = 1;
    const int64_t n_items = (int64_t)p.cascade_items.size();
    for (size_t y = 0; y < n_units; ++y) {
        const int32_t code = p.wg_map[y];
        for (int w = 0; w < 4; ++w) {
            const int64_t idx = code >= 0 ? code : p.n_single + 4 * (-(int64_t)code - 1) + w;
            if (idx >= n_items) continue;
            UnitSlot& u = p.units[4 * y + (size_t)w];
            u.item = p.cascade_items[(size_t)idx];
            u.item.wave_item = code < 0 ? 1 : 0;
            if (fill_unit_steps(p, u, w, &grows)) p.adv_slots.push_back((int32_t)(4 * y + (size_t)w));
        }
    }
}

// After an advance: the unit table's copies follow the step lists.
void refresh_units(Plan& p) {
    for (int32_t slot : p.adv_slots) fill_unit_steps(p, p.units[(size_t)slot], slot & 3, nullptr);
}

ets_status validate(const ets_tree& t) {
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

ets_status build(const ets_shape& shape, const PlanOptions& opt, const ets_tree& tree, int mode,
                 Plan& p) {
    const int32_t N = tree.n_nodes, L = tree.n_leaves;
    const int32_t G = shape.n_q_heads / shape.n_kv_heads;
    const int64_t esz = opt.kv_elem_bytes > 0 ? opt.kv_elem_bytes : shape.dtype == ETS_F32 ? 4 : 2;

    p.mode = mode;
    p.parent.assign(tree.parent, tree.parent + N);
    p.tok_offset.assign(tree.tok_offset, tree.tok_offset + N);
    p.n_tokens.assign(tree.n_tokens, tree.n_tokens + N);
    p.leaf_node.assign(tree.leaf_node, tree.leaf_node + L);

    // leaf queries at or beneath every node (children have larger ids)
    std::vector<int64_t> own(N, 0);
    for (int32_t l = 0; l < L; ++l) own[p.leaf_node[l]] += 1;
    p.leaf_count = own;
    for (int32_t i = N - 1; i >= 0; --i)
        if (p.parent[i] >= 0) p.leaf_count[p.parent[i]] += p.leaf_count[i];

    ets_stats& st = p.stats;
    st = ets_stats{};
    st.n_nodes = N;
    st.n_leaves = L;
    for (int32_t i = 0; i < N; ++i) {
        if (p.leaf_count[i] == 0) continue;
        st.live_nodes += 1;
        st.unique_tokens += p.n_tokens[i];
        st.flat_tokens += p.leaf_count[i] * (int64_t)p.n_tokens[i];
        if (p.n_tokens[i] > 0)
            st.min_pool_tokens = std::max(st.min_pool_tokens, p.tok_offset[i] + p.n_tokens[i]);
    }
    const int64_t tok_bytes = 2 * (int64_t)shape.n_kv_heads * shape.head_dim * esz;
    st.unique_kv_bytes = st.unique_tokens * tok_bytes;
    st.flat_kv_bytes = st.flat_tokens * tok_bytes;

    // chain compaction: a live node joins its parent's segment when both have
    // the same leaf set, i.e. the same count
    std::vector<Seg> segs;
    std::vector<int32_t> seg_of(N, -1);
    for (int32_t i = 0; i < N; ++i) {
        if (p.leaf_count[i] == 0) continue;
        const int32_t par = p.parent[i];
        if (par >= 0 && p.leaf_count[par] == p.leaf_count[i]) {
            seg_of[i] = seg_of[par];
        } else {
            Seg s;
            s.parent_seg = par >= 0 ? seg_of[par] : -1;
            s.cnt = p.leaf_count[i];
            seg_of[i] = (int32_t)segs.size();
            segs.push_back(std::move(s));
        }
        Seg& s = segs[seg_of[i]];
        s.nodes.push_back(i);
        s.tokens += p.n_tokens[i];
    }
    st.n_segments = (int64_t)segs.size();

    p.runs.clear();
    p.stream_items.clear();
    p.cascade_items.clear();
    p.wide_items.clear();
    p.ent_order.assign(L, 0);
    p.part_base.assign((size_t)L + 1, 0);
    p.max_cascade_ent = 0;
    p.adv.clear();
    p.adv_in_place = true;
    p.advances = 0;

    std::vector<Run> tmp_runs;
    std::vector<Chunk> chunks;
    std::vector<int32_t> stream_tokens;   // per stream item, for ordering
    std::vector<int64_t> cascade_cost;    // per cascade item, for ordering

    // leaf queries in depth-first segment order: the queries beneath a segment
    // form one contiguous range of ent_order
    {
        std::vector<int64_t> seg_own(segs.size(), 0);
        for (int32_t l = 0; l < L; ++l) seg_own[seg_of[p.leaf_node[l]]] += 1;
        int64_t root_cursor = 0;
        for (size_t s = 0; s < segs.size(); ++s) {
            Seg& sg = segs[s];
            if (sg.parent_seg < 0) {
                sg.ent_begin = (int32_t)root_cursor;
                root_cursor += sg.cnt;
            } else {
                Seg& ps = segs[sg.parent_seg];
                sg.ent_begin = ps.child_cursor;
                ps.child_cursor += (int32_t)sg.cnt;
            }
            sg.child_cursor = sg.ent_begin + (int32_t)seg_own[s];
        }
        for (int32_t l = 0; l < L; ++l) {
            Seg& sg = segs[seg_of[p.leaf_node[l]]];
            p.ent_order[sg.ent_begin + sg.own_filled++] = l;
        }
    }

    // Which kernel reads which segment.  The matrix-core kernel reads a shared
    // segment once for all `cnt` leaf queries beneath it but costs one partial
    // result per query and query head (written, then read by the merge); otherwise
    // every query reads the segment itself as part of its own item.  A segment is
    // shared when the KV bytes this saves exceed the partial bytes it adds.
    const bool use_mfma = opt.mfma != 0 && shape.dtype == ETS_BF16;  // head_dim 64 or 128
    const bool cascade_ok = mode == ETS_PLAN_TREE && use_mfma && opt.cascade_min_leaves > 0;
    if (mode == ETS_PLAN_TREE && opt.require_sharing && !cascade_ok) return ETS_ERR_UNSUPPORTED;
    st.shares_nodes = cascade_ok ? 1 : 0;
    const int64_t piece = use_mfma ? 32 : 0;
    p.piece = (int32_t)piece;
    auto grow_end_of = [&](int32_t node) { return p.tok_offset[node] + p.n_tokens[node]; };
    const int64_t partial_bytes = 2 * (int64_t)shape.n_q_heads * (shape.head_dim + 2) * 4;
    const int64_t ent_per_item = std::max<int64_t>(1, opt.cascade_rows / G);
    // cost model in nanoseconds: a resident workgroup needs about t_tile per tile of 64
    // tokens whether it waits on memory (few rows) or computes (many rows), and t_item to
    // start and to store its partial results; 768 workgroups are resident (three per
    // compute unit).  Measured: 2.1-2.7 us per tile, 6.5-8.5 us per item; the sum predicts the
    // attention launch of the configurations within 5 %.
    const int64_t t_tile = 2500, t_mem = t_tile, t_item = 7000, kTile = 64, kResident = 768;
    auto tile_cost = [&](int64_t) { return t_tile; };
    // wide kernel: one workgroup per compute unit, about t_wide per 64-token tile of 256 rows.
    // Off unless asked for: with the launch order merged, items of 64 rows measure 5-6 %
    // faster on every shape, also with 8 query heads per kv head.  It does not merge, so
    // a plan that uses it keeps the merge launch.
    const int64_t wide_rows = opt.wide_rows >= 0 && shape.head_dim == 128 ? opt.wide_rows : 0;
    const int64_t ent_per_wide = std::max<int64_t>(1, kWideRowsPerItem / G);
    const int64_t t_wide = 1500;
    int64_t own_total = 0, work_ns = 0, wide_work_ns = 0;
    int64_t items_est = L;  // one item per leaf query for what it reads itself, plus:
    for (Seg& sg : segs) {
        sg.cascade = cascade_ok && sg.cnt >= 2 && sg.cnt >= opt.cascade_min_leaves &&
                     sg.tokens > 0 &&
                     (sg.cnt - 1) * sg.tokens * tok_bytes > sg.cnt * partial_bytes;
        // A segment with many query rows is work for the matrix cores, not for the memory
        // system: items of 64 rows would stream it rows / 64 times through the compute
        // units.  The wide kernel takes 256 rows per item.
        sg.wide = sg.cascade && wide_rows > 0 && sg.cnt * G > wide_rows;
        if (sg.wide) {
            st.cascade_tokens += sg.tokens;
            st.wide_tokens += sg.tokens;
            wide_work_ns += ceil_div(sg.tokens, kTile) * ceil_div(sg.cnt, ent_per_wide) * t_wide *
                            shape.n_kv_heads;
        } else if (sg.cascade) {
            st.cascade_tokens += sg.tokens;
            for (int64_t e0 = 0; e0 < sg.cnt; e0 += ent_per_item) {
                work_ns += ceil_div(sg.tokens, kTile) *
                           tile_cost(std::min(ent_per_item, sg.cnt - e0) * G) * shape.n_kv_heads;
                items_est += 1;
            }
        } else {
            st.stream_tokens += sg.tokens * sg.cnt;
            own_total += sg.tokens * sg.cnt;
            work_ns += ceil_div(sg.tokens, kTile) * t_mem * sg.cnt * shape.n_kv_heads;
        }
    }
    // time the whole call is expected to take: the larger of the HBM time of the
    // unique bytes (at ~5.5 TB/s) and the modelled work spread over the resident
    // workgroups; no single item should take more than half of it: finer items balance no
    // better (the launch order starts the long ones first) and every further chunk of a
    // shared segment costs one more partial result for each leaf query beneath it
    // (measured on the configurations: the optimum lies at 45-55 % of the call time)
    // (1-byte pools are budgeted like 2-byte ones: their launch is bound by the number
    // of loads, not by their bytes, and finer items would only add partial results)
    const int64_t hbm_ns = st.unique_kv_bytes * (esz < 2 ? 2 : 1) / 5500;
    // (plus the start and the end of the items on the critical path, which is what a small
    // call mostly consists of)
    const int64_t call_ns =
        std::max(hbm_ns, (work_ns + items_est * t_item * shape.n_kv_heads) / kResident) +
        2 * t_item;
    const int64_t item_budget_ns = std::max<int64_t>(call_ns / 2, 4 * t_mem);

    // wide items: no longer than a quarter of the time their launch is expected to take on
    // 256 compute units, and not so short that start-up dominates
    const int64_t wide_budget_ns = std::max<int64_t>(wide_work_ns / 256 / 4, 16 * t_wide);

    int64_t scap = opt.stream_chunk;
    if (scap <= 0) {
        if (use_mfma) {
            scap = item_budget_ns / t_mem * kTile;
        } else {
            scap = round_up(ceil_div(own_total * shape.n_kv_heads, 2048), 32);
            scap = std::min<int64_t>(std::max<int64_t>(scap, 64), 2048);
        }
    }

    // shared segments: chunk counts first (they fix the slot numbering)
    std::vector<std::vector<Chunk>> seg_chunks(segs.size());
    for (size_t s = 0; s < segs.size(); ++s) {
        Seg& sg = segs[s];
        sg.prefix =
            sg.parent_seg < 0 ? 0 : segs[sg.parent_seg].prefix + segs[sg.parent_seg].n_chunks;
        sg.n_chunks = 0;
        if (!sg.cascade) continue;
        int64_t ccap = opt.cascade_chunk;
        if (ccap <= 0 && sg.wide)
            ccap = wide_budget_ns / t_wide * kTile;
        else if (ccap <= 0)
            ccap = item_budget_ns / tile_cost(std::min(ent_per_item, sg.cnt) * G) * kTile;
        tmp_runs.clear();
        if (!collect_runs(p, sg.nodes, own, tmp_runs)) p.adv_in_place = false;
        if (!cut_runs(p, tmp_runs, sg.tokens, ccap, piece, seg_chunks[s]))
            p.adv_in_place = false;
        sg.n_chunks = (int32_t)seg_chunks[s].size();
    }

    // per leaf query: the segments of its chain that no shared item reads are read
    // by the query itself, as one run list cut into items
    std::vector<int32_t> ent_pos(L, 0);
    for (int32_t i = 0; i < L; ++i) ent_pos[p.ent_order[i]] = i;
    {
        std::vector<int32_t> own_nodes, seg_chain;
        int64_t slot = 0;
        for (int32_t l = 0; l < L; ++l) {
            const int32_t s_leaf = seg_of[p.leaf_node[l]];
            p.part_base[l] = (int32_t)slot;
            const int32_t shared_slots = segs[s_leaf].prefix + segs[s_leaf].n_chunks;
            slot += shared_slots;
            seg_chain.clear();
            for (int32_t s = s_leaf; s >= 0; s = segs[s].parent_seg)
                if (!segs[s].cascade) seg_chain.push_back(s);
            own_nodes.clear();
            for (size_t i = seg_chain.size(); i-- > 0;)
                own_nodes.insert(own_nodes.end(), segs[seg_chain[i]].nodes.begin(),
                                 segs[seg_chain[i]].nodes.end());
            tmp_runs.clear();
            if (!collect_runs(p, own_nodes, own, tmp_runs)) p.adv_in_place = false;
            int64_t tokens = 0;
            for (const Run& r : tmp_runs) tokens += r.n;
            if (!cut_runs(p, tmp_runs, tokens, scap, piece, chunks)) p.adv_in_place = false;
            int32_t c_idx = 0;
            for (const Chunk& c : chunks) {
                if (slot >= std::numeric_limits<int32_t>::max()) return ETS_ERR_UNSUPPORTED;
                if (use_mfma) {
                    p.cascade_items.push_back(CascadeItem{c.run_begin, c.run_end, ent_pos[l], 1,
                                                          shared_slots + c_idx, c.tokens, 1, 0});
                    cascade_cost.push_back(ceil_div(c.tokens, kTile) * t_mem);
                    p.max_cascade_ent = std::max(p.max_cascade_ent, 1);
                } else {
                    p.stream_items.push_back(
                        StreamItem{l, c.run_begin, c.run_end, (int32_t)slot});
                    stream_tokens.push_back(c.tokens);
                }
                ++c_idx;
                ++slot;
            }
            if (slot >= std::numeric_limits<int32_t>::max()) return ETS_ERR_UNSUPPORTED;
        }
        p.part_base[L] = (int32_t)slot;
    }

    std::vector<int64_t> wide_cost;
    for (size_t s = 0; s < segs.size(); ++s) {
        const Seg& sg = segs[s];
        for (int32_t c = 0; c < sg.n_chunks; ++c) {
            const Chunk& ch = seg_chunks[s][c];
            if (sg.wide) {
                for (int64_t e0 = 0; e0 < sg.cnt; e0 += ent_per_wide) {
                    const int32_t ne = (int32_t)std::min<int64_t>(ent_per_wide, sg.cnt - e0);
                    p.wide_items.push_back(CascadeItem{ch.run_begin, ch.run_end,
                                                       sg.ent_begin + (int32_t)e0, ne, sg.prefix + c,
                                                       ch.tokens, sg.cnt <= ent_per_wide ? 1 : 0, 0});
                    wide_cost.push_back(ceil_div(ch.tokens, kTile) * ceil_div((int64_t)ne * G, 32));
                }
                continue;
            }
            for (int64_t e0 = 0; e0 < sg.cnt; e0 += ent_per_item) {
                const int32_t ne = (int32_t)std::min<int64_t>(ent_per_item, sg.cnt - e0);
                p.cascade_items.push_back(CascadeItem{ch.run_begin, ch.run_end,
                                                      sg.ent_begin + (int32_t)e0, ne,
                                                      sg.prefix + c, ch.tokens,
                                                      sg.cnt <= ent_per_item ? 1 : 0, 0});
                cascade_cost.push_back(ceil_div(ch.tokens, kTile) * tile_cost((int64_t)ne * G));
                p.max_cascade_ent = std::max(p.max_cascade_ent, ne);
            }
        }
    }

    // longest items first, so that the tail of each launch is made of short ones
    {
        std::vector<int32_t> idx(p.stream_items.size());
        for (size_t i = 0; i < idx.size(); ++i) idx[i] = (int32_t)i;
        std::stable_sort(idx.begin(), idx.end(), [&](int32_t a, int32_t b) {
            return stream_tokens[a] > stream_tokens[b];
        });
        std::vector<StreamItem> sorted(idx.size());
        for (size_t i = 0; i < idx.size(); ++i) sorted[i] = p.stream_items[idx[i]];
        p.stream_items.swap(sorted);
    }
    {
        std::vector<int32_t> idx(p.wide_items.size());
        for (size_t i = 0; i < idx.size(); ++i) idx[i] = (int32_t)i;
        std::stable_sort(idx.begin(), idx.end(),
                         [&](int32_t a, int32_t b) { return wide_cost[a] > wide_cost[b]; });
        std::vector<CascadeItem> sorted(idx.size());
        for (size_t i = 0; i < idx.size(); ++i) sorted[i] = p.wide_items[idx[i]];
        p.wide_items.swap(sorted);
    }
    {
        std::vector<int32_t> idx(p.cascade_items.size());
        for (size_t i = 0; i < idx.size(); ++i) idx[i] = (int32_t)i;
        std::stable_sort(idx.begin(), idx.end(), [&](int32_t a, int32_t b) {
            return cascade_cost[a] > cascade_cost[b];
        });
        // Small items with at most 16 query rows follow the others (both groups longest
        // first): one wave walks such an item alone, four of them share a workgroup,
        // which divides the number of short workgroups the device has to start by four.
        std::vector<CascadeItem> sorted;
        sorted.reserve(idx.size());
        // A lone wave needs about 2.5 us per 16-token unit; such an item should not
        // last longer than a quarter of the time the whole call is expected to take.
        const int64_t wave_cap = std::min<int64_t>(opt.wave_items, hbm_ns / 4 / 2500 * 16);
        auto small = [&](const CascadeItem& it) {
            return (int64_t)it.n_ent * G <= 16 && it.n_tokens <= wave_cap;
        };
        for (size_t i = 0; i < idx.size(); ++i)
            if (!small(p.cascade_items[idx[i]])) sorted.push_back(p.cascade_items[idx[i]]);
        p.n_single = (int32_t)sorted.size();
        for (size_t i = 0; i < idx.size(); ++i)
            if (small(p.cascade_items[idx[i]])) sorted.push_back(p.cascade_items[idx[i]]);
        p.cascade_items.swap(sorted);
        // Launch order.  Items with many query rows keep a workgroup slot busy for a long
        // time per byte they bring in from memory; items with few rows (a leaf's private
        // rows, segments shared by a handful of leaves) stream at the memory system's pace.
        // The device hands workgroups out in index order, so the two kinds are merged into
        // one sequence in which each advances at the same fraction of its total tokens:
        // memory traffic and arithmetic are then spread evenly over the launch instead of
        // following each other.  Within a kind the order stays longest first.
        const int64_t n_w = ((int64_t)p.cascade_items.size() - p.n_single + 3) / 4;
        std::vector<std::pair<int64_t, int32_t>> heavy, light;  // (tokens, code)
        for (int32_t i = 0; i < p.n_single; ++i) {
            const CascadeItem& it = p.cascade_items[(size_t)i];
            ((int64_t)it.n_ent * G > 16 ? heavy : light).push_back({it.n_tokens, i});
        }
        for (int64_t g = 0; g < n_w; ++g) {
            int64_t tok = 0;
            for (int64_t k = 4 * g; k < std::min<int64_t>(4 * g + 4, (int64_t)p.cascade_items.size() - p.n_single); ++k)
                tok += p.cascade_items[(size_t)(p.n_single + k)].n_tokens;
            light.push_back({tok, (int32_t)(-g - 1)});
        }
        p.wg_map.clear();
        p.wg_map.reserve(heavy.size() + light.size());
        if (!opt.interleave) {
            for (int32_t i = 0; i < p.n_single; ++i) p.wg_map.push_back(i);
            for (int64_t g = 0; g < n_w; ++g) p.wg_map.push_back((int32_t)(-g - 1));
        } else {
            auto by_tokens = [](const std::pair<int64_t, int32_t>& a,
                                const std::pair<int64_t, int32_t>& b) { return a.first > b.first; };
            std::stable_sort(heavy.begin(), heavy.end(), by_tokens);
            std::stable_sort(light.begin(), light.end(), by_tokens);
            int64_t tot_h = 0, tot_l = 0, done_h = 0, done_l = 0;
            for (const auto& x : heavy) tot_h += std::max<int64_t>(x.first, 1);
            for (const auto& x : light) tot_l += std::max<int64_t>(x.first, 1);
            size_t ih = 0, il = 0;
            while (ih < heavy.size() || il < light.size()) {
                // the kind that lags behind in its own total goes next (fractions compared
                // without division: done_h / tot_h <= done_l / tot_l)
                const bool take_heavy =
                    il >= light.size() ||
                    (ih < heavy.size() && (__int128)done_h * tot_l <= (__int128)done_l * tot_h);
                if (take_heavy) {
                    p.wg_map.push_back(heavy[ih].second);
                    done_h += std::max<int64_t>(heavy[ih++].first, 1);
                } else {
                    p.wg_map.push_back(light[il].second);
                    done_l += std::max<int64_t>(light[il++].first, 1);
                }
            }
        }
    }

    if (p.runs.size() >= (size_t)std::numeric_limits<int32_t>::max() ||
        p.wg_map.size() >= (size_t)std::numeric_limits<int32_t>::max() / 16)
        return ETS_ERR_UNSUPPORTED;
    build_units(p);
    {
        std::vector<int32_t> first(N, -1);
        p.adv_node.clear();
        p.adv_src.clear();
        p.adv_last_row.clear();
        for (int32_t l = 0; l < L; ++l) {
            const int32_t n = p.leaf_node[l];
            if (first[n] >= 0) continue;
            first[n] = l;
            p.adv_node.push_back(n);
            p.adv_src.push_back(l);
            p.adv_last_row.push_back(p.n_tokens[n] > 0 ? grow_end_of(n) - 1 : kNoRow);
        }
        p.adv_room = piece > 0 ? 32 : std::numeric_limits<int32_t>::max();
    }
    p.ent_base.resize((size_t)L);
    for (int32_t i = 0; i < L; ++i) p.ent_base[i] = p.part_base[p.ent_order[i]];
    st.n_partials = p.part_base[L];
    // the kernels number partial rows, (leaf, head) pairs and workgroups with 32-bit integers
    const int64_t i32_max = std::numeric_limits<int32_t>::max();
    if (st.n_partials * shape.n_q_heads >= i32_max || (int64_t)L * shape.n_q_heads >= i32_max ||
        (int64_t)p.stream_items.size() * shape.n_kv_heads >= i32_max)
        return ETS_ERR_UNSUPPORTED;
    st.n_stream_items = (int64_t)p.stream_items.size();
    st.n_cascade_items = (int64_t)p.cascade_items.size();
    st.n_wide_items = (int64_t)p.wide_items.size();
    st.workspace_bytes = st.n_partials * shape.n_q_heads * ((int64_t)shape.head_dim + 2) * 4;
    // The matrix-core kernel can run the merge itself when it writes every partial and every
    // leaf query has at least one (the wave that stores a leaf's last partial merges them).
    // (the merging kernel addresses the workspace with 32-bit byte offsets)
    bool can_fuse = use_mfma && L > 0 && p.stream_items.empty() && p.wide_items.empty() &&
                    !p.cascade_items.empty() &&
                    st.n_partials * shape.n_q_heads * shape.head_dim * 4 < (int64_t(1) << 31);
    for (int32_t l = 0; can_fuse && l < L; ++l) can_fuse = p.part_base[l + 1] > p.part_base[l];
    p.fused = can_fuse && (opt.fuse_merge == 1 || (opt.fuse_merge < 0 && fuse_by_default(st)));
    st.merge_fused = p.fused ? 1 : 0;
    p.valid = true;
    return ETS_OK;
}

}  // namespace

void advance_tree(Plan& plan) {
    ets_stats& st = plan.stats;
    const int64_t tok_bytes = st.unique_tokens > 0 ? st.unique_kv_bytes / st.unique_tokens : 0;
    for (int32_t n : plan.adv_node) {
        plan.n_tokens[n] += 1;
        st.unique_tokens += 1;
        st.flat_tokens += plan.leaf_count[n];
        st.min_pool_tokens =
            std::max(st.min_pool_tokens, plan.tok_offset[n] + (int64_t)plan.n_tokens[n]);
    }
    if (tok_bytes > 0) {
        st.unique_kv_bytes = st.unique_tokens * tok_bytes;
        st.flat_kv_bytes = st.flat_tokens * tok_bytes;
    }
}

bool advance_in_place(Plan& plan) {
    if (!plan.valid || !plan.adv_in_place || plan.adv_room <= 0) return false;
    for (const AdvEntry& e : plan.adv) {
        Run& last = plan.runs[e.r_last];
        if (e.mergeable && (plan.piece == 0 || last.n < plan.piece)) {
            last.n += 1;
        } else {
            Run& spare = plan.runs[e.r_spare];
            if (spare.n == 0) spare.tok = e.end0 + plan.advances;
            spare.n += 1;
        }
    }
    refresh_units(plan);
    plan.advances += 1;
    plan.adv_room -= 1;
    advance_tree(plan);
    return true;
}

void chain_of(const Plan& plan, int32_t leaf, std::vector<int32_t>& out) {
    const size_t first = out.size();
    for (int32_t x = plan.leaf_node[leaf]; x >= 0; x = plan.parent[x]) out.push_back(x);
    std::reverse(out.begin() + (std::ptrdiff_t)first, out.end());
}

ets_status build_plan(const ets_shape& shape, const PlanOptions& opt, const ets_tree& tree,
                      int mode, Plan& plan) {
    plan.valid = false;
    if (mode != ETS_PLAN_TREE && mode != ETS_PLAN_FLAT) return ETS_ERR_INVALID_ARG;
    ets_status s = validate(tree);
    if (s != ETS_OK) return s;
    try {
        return build(shape, opt, tree, mode, plan);
    } catch (const std::bad_alloc&) {
        plan.valid = false;
        return ETS_ERR_NOMEM;
    }
}

bool check_plan(const Plan& p, const ets_shape& shape, PlanCheck& out) {
    out = PlanCheck{};
    const int64_t L = (int64_t)p.leaf_node.size();
    const int G = shape.n_q_heads / shape.n_kv_heads;
    const int per_block = std::max(1, 16 / G);  // entries whose rows make up a 16-row block
    const int64_t n_runs = (int64_t)p.runs.size();
    out.entry_table_entries = (int64_t)p.ent_order.size() + kEntryPadding;
    auto bad = [&](bool cond) {
        if (cond) out.violations += 1;
    };
    auto entry_leaf = [&](int64_t idx) -> int64_t {  // padding entries hold zero
        return idx < (int64_t)p.ent_order.size() ? p.ent_order[(size_t)idx] : 0;
    };
    bad(p.ent_base.size() != p.ent_order.size());
    // every partial slot has exactly one writer: the merge reads all of a leaf's slots, and the
    // merge inside the attention launch starts when as many have arrived as the leaf has slots
    std::vector<char> written((size_t)std::max<int64_t>(p.stats.n_partials, 0), 0);
    auto writes = [&](int64_t slot) {
        if (slot < 0 || slot >= (int64_t)written.size() || written[(size_t)slot]++) out.violations += 1;
    };
    for (size_t i = 0; i < p.cascade_items.size(); ++i) {
        const CascadeItem& it = p.cascade_items[i];
        const bool wave_item = (int64_t)i >= p.n_single;
        out.items += 1;
        // the step list
        bad(it.run_begin < 0 || it.run_end < it.run_begin || it.run_end > n_runs);
        if (!wave_item) bad(it.run_end - it.run_begin > kTreeAttnMaxSteps);
        for (int64_t r = it.run_begin; r < it.run_end && r < n_runs; ++r) {
            const Run& run = p.runs[(size_t)r];
            bad(run.n < 0 || run.n > 32 || run.tok < 0);
            if (run.n > 0) {
                bad(run.tok + run.n > p.stats.min_pool_tokens);
                out.max_pool_row = std::max(out.max_pool_row, run.tok + run.n - 1);
            }
        }
        // the entries: every wave loads 16 consecutive entries from its block's first one
        const int64_t R = (int64_t)it.n_ent * G;
        bad(it.n_ent < 1 || R > kTreeAttnRowsPerItem || it.ent_begin < 0 ||
            (int64_t)it.ent_begin + it.n_ent > L);
        if (wave_item) bad(R > 16);
        const bool rowpar = R > 16;
        const int n_blocks = (int)((R + 15) / 16);
        for (int w = 0; w < 4; ++w) {
            const int blk = rowpar && w < n_blocks ? w : 0;
            const int64_t first = (int64_t)it.ent_begin + (16 * blk) / G;
            const int64_t last_loaded = first + 15;
            out.max_entry_index = std::max(out.max_entry_index, last_loaded);
            out.max_entry_overreach = std::max(
                out.max_entry_overreach, last_loaded - ((int64_t)it.ent_begin + it.n_ent - 1));
            bad(last_loaded >= out.entry_table_entries);
            // the entries whose query rows the wave fetches (rows past R included)
            for (int k = 0; k < per_block; ++k) {
                const int64_t leaf = entry_leaf(first + k);
                bad(leaf < 0 || leaf >= std::max<int64_t>(L, 1));
            }
            if (wave_item) break;  // one wave walks the item
        }
        // the partial rows it writes
        for (int32_t e = 0; e < it.n_ent && (int64_t)it.ent_begin + e < L; ++e) {
            const int32_t leaf = p.ent_order[(size_t)(it.ent_begin + e)];
            const int64_t slot = (int64_t)p.part_base[(size_t)leaf] + it.slot_off;
            bad(it.slot_off < 0 || slot >= p.part_base[(size_t)leaf + 1]);
            writes(slot);
            out.max_partial_row =
                std::max(out.max_partial_row, slot * shape.n_q_heads + shape.n_q_heads - 1);
        }
    }
    // wide items: a lane looks up the entry of its own query row, clamped to the item's last
    for (const CascadeItem& it : p.wide_items) {
        out.items += 1;
        bad(it.run_begin < 0 || it.run_end < it.run_begin || it.run_end > n_runs);
        bad(it.n_ent < 1 || (int64_t)it.n_ent * G > kWideRowsPerItem || it.ent_begin < 0 ||
            (int64_t)it.ent_begin + it.n_ent > L);
        out.max_entry_index = std::max(out.max_entry_index, (int64_t)it.ent_begin + it.n_ent - 1);
        for (int64_t r = it.run_begin; r < it.run_end && r < n_runs; ++r) {
            const Run& run = p.runs[(size_t)r];
            bad(run.n < 0 || run.n > 32 || run.tok < 0);
            if (run.n > 0) {
                bad(run.tok + run.n > p.stats.min_pool_tokens);
                out.max_pool_row = std::max(out.max_pool_row, run.tok + run.n - 1);
            }
        }
        for (int32_t e = 0; e < it.n_ent && (int64_t)it.ent_begin + e < L; ++e) {
            const int32_t leaf = p.ent_order[(size_t)(it.ent_begin + e)];
            const int64_t slot = (int64_t)p.part_base[(size_t)leaf] + it.slot_off;
            bad(it.slot_off < 0 || slot >= p.part_base[(size_t)leaf + 1]);
            writes(slot);
            out.max_partial_row =
                std::max(out.max_partial_row, slot * shape.n_q_heads + shape.n_q_heads - 1);
        }
    }
    for (const StreamItem& it : p.stream_items) {
        out.items += 1;
        bad(it.run_begin < 0 || it.run_end < it.run_begin || it.run_end > n_runs);
        bad(it.entry < 0 || it.entry >= L);
        if (it.entry >= 0 && it.entry < L)
            bad(it.slot < p.part_base[(size_t)it.entry] || it.slot >= p.part_base[(size_t)it.entry + 1]);
        writes(it.slot);
        out.max_partial_row = std::max(
            out.max_partial_row, (int64_t)it.slot * shape.n_q_heads + shape.n_q_heads - 1);
        for (int64_t r = it.run_begin; r < it.run_end && r < n_runs; ++r) {
            const Run& run = p.runs[(size_t)r];
            bad(run.n < 0 || run.tok < 0);
            if (run.n > 0) {
                bad(run.tok + run.n > p.stats.min_pool_tokens);
                out.max_pool_row = std::max(out.max_pool_row, run.tok + run.n - 1);
            }
        }
    }
    // the unit table says what the launch order and the step lists say
    bad(p.units.size() != 4 * p.wg_map.size());
    for (size_t y = 0; y < p.wg_map.size() && 4 * y + 3 < p.units.size(); ++y) {
        const int32_t code = p.wg_map[y];
        for (int w = 0; w < 4; ++w) {
            const UnitSlot& u = p.units[4 * y + (size_t)w];
            const int64_t idx = code >= 0 ? code : p.n_single + 4 * (-(int64_t)code - 1) + w;
            if (idx < 0 || idx >= (int64_t)p.cascade_items.size()) {
                bad(u.item.n_ent != 0);
                continue;
            }
            const CascadeItem& it = p.cascade_items[(size_t)idx];
            bad(u.item.run_begin != it.run_begin || u.item.run_end != it.run_end ||
                u.item.ent_begin != it.ent_begin || u.item.n_ent != it.n_ent ||
                u.item.slot_off != it.slot_off || u.item.sole_reader != it.sole_reader ||
                u.item.wave_item != (code < 0 ? 1 : 0));
            const Run* held[2] = {&u.first, &u.second};
            for (int j = 0; j < 2; ++j) {
                const int k = unit_step_index(u.item, w, j);
                const int64_t r = (int64_t)it.run_begin + k;
                if (k >= 0 && r < it.run_end && r < n_runs)
                    bad(held[j]->tok != p.runs[(size_t)r].tok || held[j]->n != p.runs[(size_t)r].n);
                else
                    bad(held[j]->n != 0);
            }
        }
    }
    // the launch order names every item that takes a workgroup and every group of small
    // items exactly once
    {
        const int64_t n_w = ((int64_t)p.cascade_items.size() - p.n_single + 3) / 4;
        bad((int64_t)p.wg_map.size() != p.n_single + n_w);
        std::vector<char> seen_single((size_t)p.n_single, 0), seen_group((size_t)n_w, 0);
        for (int32_t code : p.wg_map) {
            if (code >= 0) {
                if (code >= p.n_single || seen_single[(size_t)code]++) out.violations += 1;
            } else {
                const int64_t g = -(int64_t)code - 1;
                if (g >= n_w || seen_group[(size_t)g]++) out.violations += 1;
            }
        }
    }
    bad(out.max_partial_row >= p.stats.n_partials * shape.n_q_heads);
    for (char w : written) bad(w != 1);
    if (p.fused) {
        // only the matrix-core kernel's own items count arrivals, and a leaf query without a
        // partial would never be merged
        bad(!p.stream_items.empty() || !p.wide_items.empty());
        for (int64_t l = 0; l < L; ++l) bad(p.part_base[(size_t)l + 1] <= p.part_base[(size_t)l]);
    }
    return out.violations == 0;
}

bool leaf_cover(const Plan& plan, int32_t leaf, std::vector<int64_t>& rows,
                int32_t& n_partials) {
    const int32_t base = plan.part_base[leaf];
    n_partials = plan.part_base[leaf + 1] - base;
    // run range of every slot of this leaf, taken from the work items themselves
    std::vector<std::pair<int32_t, int32_t>> by_slot((size_t)n_partials, {-1, -1});
    bool ok = true;
    auto put = [&](int32_t slot, int32_t rb, int32_t re) {
        const int32_t k = slot - base;
        if (k < 0 || k >= n_partials || by_slot[k].first >= 0) {
            ok = false;
            return;
        }
        by_slot[k] = {rb, re};
    };
    for (const StreamItem& it : plan.stream_items)
        if (it.entry == leaf) put(it.slot, it.run_begin, it.run_end);
    for (const std::vector<CascadeItem>* items : {&plan.cascade_items, &plan.wide_items})
        for (const CascadeItem& it : *items)
            for (int32_t i = 0; i < it.n_ent; ++i)
                if (plan.ent_order[it.ent_begin + i] == leaf)
                    put(base + it.slot_off, it.run_begin, it.run_end);
    rows.clear();
    for (const auto& rr : by_slot) {
        if (rr.first < 0) {
            ok = false;
            continue;
        }
        for (int32_t r = rr.first; r < rr.second; ++r)
            for (int32_t t = 0; t < plan.runs[r].n; ++t) rows.push_back(plan.runs[r].tok + t);
    }
    return ok;
}

}  // namespace ets
