// Decode-step advance on the device: between two tokens of one search step the tree's
// topology is fixed (ETS paper, Sec. 4.1) and only the nodes that hold leaf queries grow.
//   advance_runs_kernel  extends, in the step lists the attention kernels read, the tail
//                        of every copy of every growing node by one row
//                        (refresh_units_kernel then updates the start table's copies);
//   kv_append_kernel     writes the new token's K and V row of every growing node into
//                        the pools.
#pragma once

#include "device_utils.hpp"
#include "plan.h"

namespace ets {

// One thread per AdvEntry.  `advances` = advances already applied since the plan was built.
__global__ void advance_runs_kernel(Run* __restrict__ runs, const AdvEntry* __restrict__ adv,
                                    int n_adv, int piece, int advances) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_adv) return;
    const AdvEntry e = adv[i];
    Run* last = runs + e.r_last;
    if (e.mergeable && (piece == 0 || last->n < piece)) {
        last->n += 1;
    } else {
        Run* spare = runs + e.r_spare;
        if (spare->n == 0) spare->tok = e.end0 + advances;
        spare->n += 1;
    }
}

// Launched behind advance_runs_kernel, one thread per listed slot: the attention kernel's
// start table holds copies of every item's first two steps, which follow the step lists.
__global__ void refresh_units_kernel(UnitSlot* __restrict__ units, const int32_t* __restrict__ slots,
                                     int n_slots, const Run* __restrict__ runs) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_slots) return;
    const int slot = slots[i];
    UnitSlot* u = units + slot;
    const CascadeItem item = u->item;
    for (int j = 0; j < 2; ++j) {
        const int k = unit_step_index(item, slot & 3, j);
        if (k < 0 || item.run_begin + k >= item.run_end) continue;
        const Run r = runs[item.run_begin + k];
        if (j == 0) u->first = r;
        else u->second = r;
    }
}

// One workgroup per growing node: for every kv head, head_bytes = head_dim * element
// size (a multiple of 16) of K and of V go from row src[node] of k_new / v_new
// ([leaf][kv head][head_dim]) to the node's newest row, last_row[node] + advances, of that
// head's plane of the pool ([kv head][pool row][head_dim]).  A node that has no row yet
// (negative entry) is skipped.
__global__ __launch_bounds__(256) void kv_append_kernel(char* __restrict__ k_pool,
                                                        char* __restrict__ v_pool,
                                                        const char* __restrict__ k_new,
                                                        const char* __restrict__ v_new,
                                                        const int32_t* __restrict__ src,
                                                        const int64_t* __restrict__ last_row,
                                                        int advances, int n_kv_heads,
                                                        int head_bytes, int64_t pool_tokens) {
    const int node = blockIdx.x;
    const int64_t row = last_row[node] + advances;
    if (row < 0) return;
    const int64_t from = (int64_t)src[node] * n_kv_heads * head_bytes;
    const int per_head = head_bytes / 16;
    const int pieces = n_kv_heads * per_head;
    for (int i = threadIdx.x; i < 2 * pieces; i += blockDim.x) {
        const bool is_v = i >= pieces;
        const int piece = is_v ? i - pieces : i;
        const int h = piece / per_head;
        const int64_t dst = (h * pool_tokens + row) * head_bytes + (piece - h * per_head) * 16;
        const uint4 val =
            *reinterpret_cast<const uint4*>((is_v ? v_new : k_new) + from + piece * 16);
        *reinterpret_cast<uint4*>((is_v ? v_pool : k_pool) + dst) = val;
    }
}

}  // namespace ets
