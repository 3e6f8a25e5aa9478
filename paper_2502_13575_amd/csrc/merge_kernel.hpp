// Log-sum-exp merge of the partial results along every leaf's chain.
//
// One wavefront per (leaf query, query head).  With partials (o_i, m_i, l_i),
// m in log2 units:  m* = max m_i,  w_i = 2^(m_i - m*),  l* = sum l_i w_i,
// out = sum o_i w_i / l*,  lse = (m* + log2 l*) ln 2.  The partials of a leaf
// are consecutive slots and are combined in slot order, so the result does not
// depend on scheduling.  A leaf without partials (empty chain) gets out = 0,
// lse = -inf.  out may be written as fp32 or rounded to bf16 (nearest even), and is
// multiplied first by the factor of its kv head (the scale of a quantised V pool; 1
// otherwise); `group` = query heads per kv head.
#pragma once

#include "device_utils.hpp"

namespace ets {

// float -> bfloat16 bits, round to nearest even (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
    const uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

template <int D, typename OutT>
__global__ __launch_bounds__(256) void merge_kernel(const int32_t* __restrict__ part_base,
                                                    int n_leaves, int n_q_heads,
                                                    const float* __restrict__ ws_o,
                                                    const float2* __restrict__ ws_ml,
                                                    OutT* __restrict__ out,
                                                    float* __restrict__ lse, HeadScales v_scales,
                                                    int group) {
    constexpr int EPL = D / 64;  // floats per lane
    struct alignas(4 * EPL) RowPiece {
        float f[EPL];
    };
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int64_t pair = (int64_t)blockIdx.x * 4 + wave;  // (leaf, head) index
    if (pair >= (int64_t)n_leaves * n_q_heads) return;
    const int leaf = (int)(pair / n_q_heads), j = (int)(pair % n_q_heads);
    const int p0 = part_base[leaf], p1 = part_base[leaf + 1];

    // Lanes first take one partial each (its m and l), so that the maximum and the
    // weights of up to 64 partials cost one round trip; the weighted rows are then
    // accumulated four at a time with the weight read from the owning lane.
    float ms = -INFINITY;
    for (int c0 = p0; c0 < p1; c0 += 64) {
        const int p = c0 + lane;
        float mv = p < p1 ? ws_ml[(int64_t)p * n_q_heads + j].x : -INFINITY;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mv = fmaxf(mv, __shfl_xor(mv, off, 64));
        ms = fmaxf(ms, mv);
    }

    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;
    float ls = 0.f;
    for (int c0 = p0; c0 < p1; c0 += 64) {
        const int p = c0 + lane;
        float wv = 0.f, lw = 0.f;
        if (p < p1) {
            const float2 ml = ws_ml[(int64_t)p * n_q_heads + j];
            wv = fast_exp2(ml.x - ms);
            lw = ml.y * wv;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) lw += __shfl_xor(lw, off, 64);
        ls += lw;
        const int cn = min(64, p1 - c0);
        const float* base = ws_o + ((int64_t)c0 * n_q_heads + j) * D + lane * EPL;
        const int64_t stride = (int64_t)n_q_heads * D;
        int k = 0;
        for (; k + 4 <= cn; k += 4) {
            RowPiece v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[u] = *reinterpret_cast<const RowPiece*>(base + (k + u) * stride);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float w = __builtin_bit_cast(
                    float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv), k + u));
#pragma unroll
                for (int i = 0; i < EPL; ++i) acc[i] = fmaf(v[u].f[i], w, acc[i]);
            }
        }
        for (; k < cn; ++k) {
            const float w =
                __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv), k));
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] = fmaf(base[k * stride + i], w, acc[i]);
        }
    }
    const bool empty = p1 == p0;
    const float out_scale = v_scales.s[j / group];
    const float inv = empty ? 0.f : 1.f / ls;
    if constexpr (sizeof(OutT) == 4) {
        float* dst = reinterpret_cast<float*>(out) + pair * D + lane * EPL;
#pragma unroll
        for (int i = 0; i < EPL; ++i) dst[i] = acc[i] * inv * out_scale;
    } else {
        uint16_t* dst = reinterpret_cast<uint16_t*>(out) + pair * D + lane * EPL;
#pragma unroll
        for (int i = 0; i < EPL; ++i) dst[i] = f32_to_bf16_rne(acc[i] * inv * out_scale);
    }
    if (lane == 0)
        lse[pair] = empty ? -INFINITY : (ms + __builtin_amdgcn_logf(ls)) * 0.6931471805599453f;
}

}  // namespace ets
