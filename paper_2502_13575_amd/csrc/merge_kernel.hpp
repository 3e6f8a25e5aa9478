// Log-sum-exp merge of the partial results along every leaf's chain.
//
// One wavefront per (leaf query, query head).  With partials (o_i, m_i, l_i),
// m in log2 units:  m* = max m_i,  w_i = 2^(m_i - m*),  l* = sum l_i w_i,
// out = sum o_i w_i / l*,  lse = (m* + log2 l*) ln 2.  The partials of a leaf
// are consecutive slots and are combined in slot order, so the result does not
// depend on scheduling.  A leaf without partials (empty chain) gets out = 0,
// lse = -inf.
#pragma once

#include "device_utils.hpp"

namespace ets {

template <int D>
__global__ __launch_bounds__(256) void merge_kernel(const int32_t* __restrict__ part_base,
                                                    int n_leaves, int n_q_heads,
                                                    const float* __restrict__ ws_o,
                                                    const float2* __restrict__ ws_ml,
                                                    float* __restrict__ out,
                                                    float* __restrict__ lse) {
    constexpr int EPL = D / 64;  // floats per lane
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int64_t pair = (int64_t)blockIdx.x * 4 + wave;  // (leaf, head) index
    if (pair >= (int64_t)n_leaves * n_q_heads) return;
    const int leaf = (int)(pair / n_q_heads), j = (int)(pair % n_q_heads);
    const int p0 = part_base[leaf], p1 = part_base[leaf + 1];

    float ms = -INFINITY;
    for (int p = p0; p < p1; ++p) ms = fmaxf(ms, ws_ml[(int64_t)p * n_q_heads + j].x);

    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;
    float ls = 0.f;
    for (int p = p0; p < p1; ++p) {
        const int64_t row = (int64_t)p * n_q_heads + j;
        const float2 ml = ws_ml[row];
        const float w = fast_exp2(ml.x - ms);
        ls = fmaf(ml.y, w, ls);
        const float* src = ws_o + row * D + lane * EPL;
        if constexpr (EPL == 2) {
            const float2 v = *reinterpret_cast<const float2*>(src);
            acc[0] = fmaf(v.x, w, acc[0]);
            acc[1] = fmaf(v.y, w, acc[1]);
        } else {
            acc[0] = fmaf(src[0], w, acc[0]);
        }
    }
    const bool empty = p1 == p0;
    const float inv = empty ? 0.f : 1.f / ls;
    float* dst = out + pair * D + lane * EPL;
#pragma unroll
    for (int i = 0; i < EPL; ++i) dst[i] = acc[i] * inv;
    if (lane == 0)
        lse[pair] = empty ? -INFINITY : (ms + __builtin_amdgcn_logf(ls)) * 0.6931471805599453f;
}

}  // namespace ets
