// Host planner of step-prefill attention (scoring a new step with the reward model,
// ETS paper Abstract, Sec. 1 and Sec. 5.1): every token of a leaf query's node is a
// query that sees the node's strict ancestors in full and the node itself causally.
// Integer work only.
#pragma once

#include <cstdint>
#include <vector>

#include "etsattn.h"
#include "plan.h"

namespace ets {

// Run::pad of a prefill run holds `kpos`, the index inside the querying node of the
// run's first row; rows of ancestors carry kAncestorRun and are seen by every query.
// Query token i sees row t of a run iff t < n and kpos + t <= i.
constexpr int32_t kAncestorRun = -(1 << 30);
constexpr int32_t kPrefillRowsPerItem = 256;  // query rows (tokens x heads per kv head)

// Work item of the prefill kernel: query tokens [tok0, tok0 + n_tok) of one leaf
// query's node against runs [run_begin, run_end): the ancestors' rows, then the node's
// own rows in pieces of 32 up to the piece that holds token tok0 + n_tok - 1.  32 bytes.
struct PrefillItem {
    int32_t run_begin;
    int32_t run_end;
    int64_t q_row0;  // query row of token tok0
    int32_t n_tok;   // 1 .. kPrefillRowsPerItem / G
    int32_t tok0;
    int32_t leaf;    // leaf query index
    int32_t pad;
};

struct PrefillPlan {
    bool valid = false;
    std::vector<int32_t> parent, n_tokens, leaf_node;
    std::vector<int64_t> tok_offset;
    std::vector<int64_t> q_ptr;        // [L + 1] first query row of every leaf query
    std::vector<Run> runs;
    std::vector<PrefillItem> items;    // leaf queries in depth-first order of their nodes
    std::vector<int32_t> item_begin;   // [L] first item of leaf query l (its blocks follow)
    ets_prefill_stats stats{};
};

// Builds `plan`; ETS_OK, ETS_ERR_BAD_TREE, ETS_ERR_BAD_LEAF, ETS_ERR_INVALID_ARG,
// ETS_ERR_UNSUPPORTED (more than 2^31 - 1 runs or query rows per node) or ETS_ERR_NOMEM.
// kv_elem_bytes: bytes per pool element for the byte statistics (2 = bf16, 1 = E4M3 codes)
ets_status build_prefill_plan(const ets_shape& shape, const ets_tree& tree, PrefillPlan& plan,
                              int64_t kv_elem_bytes = 2);

// Pool rows that query token `tok` of leaf query `leaf` sees according to the work
// items (their run lists and the visibility rule above), in the order they are read.
// Returns false if no item holds that token.
bool prefill_cover(const PrefillPlan& plan, int32_t leaf, int32_t tok, std::vector<int64_t>& rows);

// Replays what the prefill kernel reads and writes from its tables (run lists against the
// pool, query and output rows against n_q_rows); true when everything is in bounds.
// Only items, max_pool_row and violations of `out` are filled.
bool check_prefill_plan(const PrefillPlan& plan, const ets_shape& shape, PlanCheck& out);

}  // namespace ets
