// The ETS selection step on the host (ETS paper Sec. 4.1-4.2, App. B): REBASE weights
// (Eq. 1 / Eq. 3) and the set of leaves that maximises the cost model
//   sum_{i in S} W_i / sum_i W_i  -  lambda_b |V_S| / |V_A|  +  lambda_d |C_S| / |C_A|
// (Eq. 2 without and Eq. 4 with the coverage term; as ILPs Eq. 6 and Eq. 7 of App. B), solved exactly: a tree recursion gives the optimum for the
// budget term, the coverage term is handled by branch and bound over the clusters.
#pragma once

#include <cstdint>
#include <vector>

#include "etsattn.h"

namespace ets {

// Eq. 1: visits the trajectories from the highest reward to the lowest (equal rewards in
// input order); trajectory i receives ceil(N_i e_i / sum_{k in A_i} e_k) of the N_i
// continuations still to hand out, e = exp(R / T).
void rebase_weights(int32_t n, const double* rewards, int32_t budget, double temperature,
                    int32_t* weights);

struct SelectResult {
    std::vector<uint8_t> keep;  // [L]
    double objective = 0.0;
    int64_t kept_nodes = 0, live_nodes = 0;   // |V_S|, |V_A|
    int64_t kept_clusters = 0, clusters = 0;  // |C_S|, |C_A|
    int64_t bb_nodes = 0;                     // branch-and-bound nodes visited
    bool optimal = true;                      // false: node limit hit, best found returned
};

// Leaves must be distinct and none may lie beneath another (ETS_ERR_BAD_LEAF otherwise);
// weights >= 0 with a positive sum; cluster may be null (no coverage term).
ets_status select_leaves(const ets_tree& tree, const int32_t* weights, const int32_t* cluster,
                         double lambda_b, double lambda_d, int64_t node_limit, SelectResult& out);

}  // namespace ets
