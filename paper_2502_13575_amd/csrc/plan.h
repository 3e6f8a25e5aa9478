// Host-side planner of libetsattn: integer work on the search tree.
//
// Follows the tree semantics of the ETS paper (Sec. 4.1, App. B): nodes are
// reasoning steps, a trajectory is a root->leaf chain, a non-leaf node is kept
// iff a retained leaf lies beneath it, and ancestors' KV is shared by every
// trajectory through them.
#pragma once

#include <cstdint>
#include <vector>

#include "etsattn.h"

namespace ets {

// A run of consecutive pool rows.  16 bytes, read by the kernels.
struct Run {
    int64_t tok;  // first pool row
    int32_t n;    // rows
    int32_t pad;
};

// Work item of the per-leaf streaming kernel: one leaf query reads `runs`
// for each kv head and writes partial `slot`.
struct StreamItem {
    int32_t entry;      // leaf query index
    int32_t run_begin;  // [run_begin, run_end) in Plan::runs
    int32_t run_end;
    int32_t slot;       // partial index (already includes part_base[entry])
};

// Work item of the matrix-core kernel: the leaf queries
// ent_order[ent_begin .. ent_begin + n_ent) all attend to `runs` (each run at
// most 32 rows); the partial of entry e goes to slot part_base[e] + slot_off.
struct CascadeItem {
    int32_t run_begin;
    int32_t run_end;
    int32_t ent_begin;
    int32_t n_ent;
    int32_t slot_off;
    int32_t n_tokens;
    int32_t sole_reader;  // 1: no other item reads these rows
    int32_t wave_item;    // 1: a small item walked by one wavefront (set in the unit table)
};

// What a wavefront of the matrix-core kernel starts from, in launch order: wave w of
// workgroup y reads units[4 y + w]: its work item (n_ent = 0: nothing to do) and the step
// it fetches first (n = 0: none), so that the first tile can be requested after a single
// table read.  Item of a workgroup: four copies, `first` = step w / 2 of the item (the wave
// fetches half w % 2 of it), `second` unused.  Small item of a wave: `first` = its step 0,
// `second` = its step 1.  64 bytes.
struct UnitSlot {
    CascadeItem item;
    Run first;
    Run second;
};

// Step j of the slot's item as the unit table holds it: 0 = first, 1 = second (-1: none).
// Used by the host planner and by the kernel that refreshes the table after an advance.
#if defined(__HIPCC__)
__host__ __device__
#endif
inline int unit_step_index(const CascadeItem& item, int wave, int j) {
    return item.wave_item ? j : (j == 0 ? wave >> 1 : -1);
}

// Where a growing node's next token goes (decode-step advance): one record per copy of
// the node's tail in Plan::runs.  The token joins run `r_last` if that run ends at the
// node's end and has room, else the spare run `r_spare` that follows it.  24 bytes, read
// by the advance kernel.
struct AdvEntry {
    int32_t r_last;
    int32_t r_spare;
    int64_t end0;       // first free pool row of the node when the plan was built
    int32_t mergeable;  // 1: run r_last ends at end0
    int32_t pad;
};

// Geometry of the matrix-core kernel that the planner and the launch code rely on.
constexpr int kTreeAttnRowsPerItem = 64;  // query rows one work item serves at most
constexpr int kTreeAttnMaxSteps = 256;    // steps per work item that takes a workgroup
constexpr int kWideRowsPerItem = 256;     // query rows per work item of the wide kernel (8 waves x 32)
// Both per-entry tables (ent_order, ent_base) end in this many zero entries on the device:
// a wave fetches the entries of its 16 query rows with one 16-entry scalar load, which may
// run up to 15 entries past the item's last entry (see check_plan).
constexpr int kEntryPadding = 64;

// adv_last_row of a node that has no row yet; stays negative under any number of advances
constexpr int64_t kNoRow = -(int64_t(1) << 62);

struct PlanOptions {
    int64_t kv_elem_bytes = 0;       // bytes per pool element; 0 = by the shape's dtype
    int64_t stream_chunk = 0;        // 0 = auto
    int64_t cascade_chunk = 0;       // 0 = auto
    int64_t cascade_rows = 64;       // query rows per shared work item (16, 32 or 64)
    int64_t wave_items = 512;        // an item of <= 16 rows and at most this many tokens is
                                     // walked by one wave, four such items to a workgroup (0 = off)
    int64_t mfma = 1;                // 0 = never use the matrix-core kernel
    int64_t cascade_min_leaves = 2;  // 0 = never use the shared-node kernel
    int64_t wide_rows = -1;          // a shared segment with more query rows than this goes to the
                                     // wide kernel, 256 rows per item (0 or -1 = never)
    int64_t interleave = 1;          // 1 = workgroups of small items are spread among the others
    int64_t require_sharing = 0;     // 1 = a tree-mode plan that cannot share nodes is refused
    int64_t fuse_merge = -1;         // merge inside the attention launch: 1 = whenever the plan allows
                                     // it, 0 = never, -1 = the planner decides
};

struct Plan {
    bool valid = false;
    int mode = ETS_PLAN_TREE;
    // copies of the caller's tree
    std::vector<int32_t> parent, n_tokens, leaf_node;
    std::vector<int64_t> tok_offset;
    // derived
    std::vector<int64_t> leaf_count;  // [N]
    std::vector<Run> runs;
    std::vector<StreamItem> stream_items;
    std::vector<CascadeItem> cascade_items;
    std::vector<CascadeItem> wide_items;  // up to kWideRowsPerItem query rows each, any number of runs
    std::vector<int32_t> ent_order;   // leaf queries in depth-first segment order
    std::vector<int32_t> part_base;   // [L + 1] first partial slot of every leaf query
    std::vector<int32_t> ent_base;    // [L] part_base of ent_order[i], for the kernel's scalar loads
    int32_t max_cascade_ent = 0;      // largest n_ent over the cascade items
    int32_t n_single = 0;             // cascade_items[0, n_single): one workgroup each; the rest:
                                      // small items, four to a workgroup (one wave each)
    std::vector<int32_t> wg_map;      // launch order of the matrix-core kernel: workgroup i takes
                                      // item wg_map[i] when that is >= 0, else the four small
                                      // items of group -wg_map[i] - 1 (n_single + 4 g ..)
    std::vector<UnitSlot> units;      // [4 * wg_map.size()] what the kernel reads: see UnitSlot
    std::vector<int32_t> adv_slots;   // slots of `units` whose copies of the first steps hold a
                                      // run that an advance may extend (refreshed after it)
    // decode-step advance: every distinct node of leaf_node grows by one token
    std::vector<AdvEntry> adv;        // tails to extend
    std::vector<int32_t> adv_node;    // distinct leaf nodes, in order of first appearance
    std::vector<int32_t> adv_src;     // first leaf query of that node (supplies the new token)
    std::vector<int64_t> adv_last_row;  // newest pool row of that node at plan time (kNoRow: none);
                                        // after a advances in place it is this + a
    bool adv_in_place = false;        // every tail has a record (else advancing re-plans)
    int32_t adv_room = 0;             // advances the spare runs still hold
    int32_t advances = 0;             // advances applied in place since the plan was built
    int32_t piece = 0;                // longest run the kernels accept (0 = any)
    bool fused = false;               // the matrix-core kernel merges (no merge launch): every
                                      // partial comes from it and every leaf query has one
    ets_stats stats{};
};

// Grows every distinct leaf node by one token in place.  Returns false (and changes
// nothing) when the plan has no room left: the caller then re-plans.
bool advance_in_place(Plan& plan);
// The same bookkeeping on the plan's copy of the tree only (lengths and statistics).
void advance_tree(Plan& plan);

// Builds `plan` from `tree`.  Returns ETS_OK, ETS_ERR_BAD_TREE, ETS_ERR_BAD_LEAF,
// ETS_ERR_INVALID_ARG or ETS_ERR_NOMEM; on error plan.valid is false.
ets_status build_plan(const ets_shape& shape, const PlanOptions& opt, const ets_tree& tree,
                      int mode, Plan& plan);

// Root->leaf chain of leaf query `leaf` (node ids), appended to `out`.
void chain_of(const Plan& plan, int32_t leaf, std::vector<int32_t>& out);

// What the kernels will touch, replayed on the host from the tables they read: the
// highest index into the per-entry tables any wave loads, the leaf queries whose q rows it
// fetches, the partial rows it writes, the pool rows its steps name.
struct PlanCheck {
    int64_t items = 0;
    int64_t entry_table_entries = 0;  // entries of each table on the device, padding included
    int64_t max_entry_index = -1;     // highest entry index loaded
    int64_t max_entry_overreach = 0;  // entries loaded past an item's own last entry, at most
    int64_t max_pool_row = -1;        // highest pool row named by a step
    int64_t max_partial_row = -1;     // highest (slot, head) row written
    int64_t violations = 0;
};
// Returns true when every access stays inside its table / the pool / the workspace.
bool check_plan(const Plan& plan, const ets_shape& shape, PlanCheck& out);

// Rows read for `leaf` according to the work items, ordered by partial slot.
// Returns false if a slot of the leaf is produced twice or never.
bool leaf_cover(const Plan& plan, int32_t leaf, std::vector<int64_t>& rows, int32_t& n_partials);

}  // namespace ets
