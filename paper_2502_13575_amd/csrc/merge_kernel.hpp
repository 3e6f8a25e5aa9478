// Log-sum-exp merge of the partial results along every leaf's chain.
//
// One wavefront per (leaf query, kv head): it merges the G query heads of that kv
// head together, whose rows of a partial slot are adjacent in the workspace (G * D
// floats in one piece).  With partials (o_i, m_i, l_i), m in log2 units:
// m* = max m_i,  w_i = 2^(m_i - m*),  l* = sum l_i w_i,  out = sum o_i w_i / l*,
// lse = (m* + log2 l*) ln 2.  The partials of a leaf are consecutive slots and are
// combined in slot order, so the result does not depend on scheduling or on which
// kernel runs the merge.  A leaf without partials (empty chain) gets out = 0,
// lse = -inf.  out is written as fp32 or rounded to bf16 (nearest even), and is
// multiplied first by the factor of its kv head (the scale of a quantised V pool; 1
// otherwise).
#pragma once

#include "device_utils.hpp"

namespace ets {

// float -> bfloat16 bits, round to nearest even (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
    const uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// Maximum / sum over the lanes that share `lane % G` (strides G, 2 G, .., 32).
template <int G>
__device__ __forceinline__ float strided_max(float x) {
#pragma unroll
    for (int off = 32; off >= G; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
    return x;
}
template <int G>
__device__ __forceinline__ float strided_sum(float x) {
#pragma unroll
    for (int off = 32; off >= G; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// Cache policy bit of a buffer access at device scope: the access is coherent with the
// same kind of access from compute units behind another L2 (a store is written through,
// a load does not take a line that may be stale).
constexpr int kDeviceScope = 16;

// The whole wave merges partial slots [p0, p1) of leaf query `leaf` for the G query
// heads of kv head h.  Two lane layouts: for the (m, l) pairs lane = slot-in-round * G +
// head, 64 / G slots per round; for the rows lane = piece of the G * D adjacent floats
// (EPL each), i.e. head = lane / (64 / G).
// COHERENT: the partials were stored by other workgroups of this very launch, with
// device-scope stores that had completed before their writer counted itself in; they are
// read with device-scope loads (byte offsets into the workspace are below 2^32 then).
template <int D, int G, bool COHERENT = false>
__device__ __forceinline__ void merge_leaf_heads(int lane, int64_t leaf, int h, int p0, int p1,
                                                 int n_q_heads, const float* ws_o,
                                                 const float2* ws_ml, int64_t n_ws_rows, void* out,
                                                 bool out_bf16, float* lse, float out_scale) {
    constexpr int EPL = D * G / 64;  // floats per lane of a slot's G rows
    constexpr int LPH = 64 / G;      // lanes per head in the row layout; slots per round
    constexpr int VEC = EPL >= 4 ? 4 : EPL;
    struct alignas(4 * VEC) Piece {
        float f[VEC];
    };
    // workspace as buffer resources (uniform), used by the device-scope loads only
    const __amdgpu_buffer_rsrc_t rs_o = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(ws_o), 0, COHERENT ? (int)(uint32_t)(n_ws_rows * D * 4) : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_ml = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float2*>(ws_ml), 0, COHERENT ? (int)(uint32_t)(n_ws_rows * 8) : 0, 0x00020000);
    auto load_ml = [&](int64_t row) {
        if constexpr (COHERENT) {
            const auto r = __builtin_amdgcn_raw_buffer_load_b64(rs_ml, (uint32_t)row * 8u, 0, kDeviceScope);
            return __builtin_bit_cast(float2, r);
        } else {
            return ws_ml[row];
        }
    };
    auto load_piece = [&](int64_t float_off) {
        if constexpr (COHERENT) {
            const uint32_t off = (uint32_t)float_off * 4u;
            if constexpr (VEC == 4)
                return __builtin_bit_cast(Piece, __builtin_amdgcn_raw_buffer_load_b128(rs_o, off, 0, kDeviceScope));
            else if constexpr (VEC == 2)
                return __builtin_bit_cast(Piece, __builtin_amdgcn_raw_buffer_load_b64(rs_o, off, 0, kDeviceScope));
            else
                return __builtin_bit_cast(Piece, __builtin_amdgcn_raw_buffer_load_b32(rs_o, off, 0, kDeviceScope));
        } else {
            return *reinterpret_cast<const Piece*>(ws_o + float_off);
        }
    };
    const int g_ml = lane % G, k_ml = lane / G;
    const int j0 = h * G;
    const int64_t stride = (int64_t)n_q_heads * D;  // floats between slots

    // Loads are issued as early as their addresses are known, and a batch of rows at a time:
    // the first round's (m, l) pairs and the first batch of rows go out together, before
    // anything is reduced (a leaf rarely has more partials than one round holds), so that a
    // typical leaf costs two or three memory round trips.
    // rows in flight per lane and batch (inside the attention kernel registers are scarce)
    constexpr int UNROLL = COHERENT && EPL >= 8 ? 2 : 4;
    const int g_row = lane / LPH;
    auto load_rows = [&](Piece (&v)[UNROLL][EPL / VEC], int64_t base, int k, int cn) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (k + u < cn) {  // uniform
#pragma unroll
                for (int c = 0; c < EPL / VEC; ++c)
                    v[u][c] = load_piece(base + (k + u) * stride + c * VEC);
            }
        }
    };
    const int cn0 = min(LPH, p1 - p0);
    const int64_t base0 = ((int64_t)p0 * n_q_heads + j0) * D + lane * EPL;  // in floats
    float2 ml0 = make_float2(-INFINITY, 0.f);
    if (p0 + k_ml < p1) ml0 = load_ml((int64_t)(p0 + k_ml) * n_q_heads + j0 + g_ml);
    Piece v0[UNROLL][EPL / VEC];
    load_rows(v0, base0, 0, cn0);

    float ms = strided_max<G>(ml0.x);  // per head lane % G
    for (int c0 = p0 + LPH; c0 < p1; c0 += LPH) {
        const int p = c0 + k_ml;
        const float mv = p < p1 ? load_ml((int64_t)p * n_q_heads + j0 + g_ml).x : -INFINITY;
        ms = fmaxf(ms, strided_max<G>(mv));
    }

    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;
    float ls = 0.f;  // per head lane % G
    for (int c0 = p0; c0 < p1; c0 += LPH) {
        const int p = c0 + k_ml;
        float wv = 0.f, lw = 0.f;
        if (p < p1) {
            const float2 ml = c0 == p0 ? ml0 : load_ml((int64_t)p * n_q_heads + j0 + g_ml);
            wv = fast_exp2(ml.x - ms);
            lw = ml.y * wv;
        }
        ls += strided_sum<G>(lw);
        const int cn = min(LPH, p1 - c0);
        const int64_t base = ((int64_t)c0 * n_q_heads + j0) * D + lane * EPL;  // in floats
        auto accumulate = [&](int k, const Piece (&v)[EPL / VEC]) {
            const float w = __shfl(wv, k * G + g_row, 64);
#pragma unroll
            for (int c = 0; c < EPL / VEC; ++c)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[c * VEC + i] = fmaf(v[c].f[i], w, acc[c * VEC + i]);
        };
        int k = 0;
        if (c0 == p0) {  // the batch that is already here
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (u < cn) accumulate(u, v0[u]);
            k = UNROLL;
        }
        for (; k < cn; k += UNROLL) {
            Piece v[UNROLL][EPL / VEC];
            load_rows(v, base, k, cn);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (k + u < cn) accumulate(k + u, v[u]);
        }
    }
    const bool empty = p1 == p0;
    // the sums live in lanes by lane % G; lane g (< G) holds head g's
    const float ls_row = __shfl(ls, g_row, 64);
    const float inv = empty ? 0.f : 1.f / ls_row;
    const int64_t o_off = (leaf * n_q_heads + j0) * D + lane * EPL;
    if (!out_bf16) {
        float* dst = static_cast<float*>(out) + o_off;
#pragma unroll
        for (int c = 0; c < EPL / VEC; ++c) {
            Piece r;
#pragma unroll
            for (int i = 0; i < VEC; ++i) r.f[i] = acc[c * VEC + i] * inv * out_scale;
            *reinterpret_cast<Piece*>(dst + c * VEC) = r;
        }
    } else {
        uint16_t* dst = static_cast<uint16_t*>(out) + o_off;
        if constexpr (EPL == 1) {
            dst[0] = f32_to_bf16_rne(acc[0] * inv * out_scale);
        } else {
            constexpr int WPV = EPL >= 8 ? 4 : EPL / 2;  // 32-bit words per store
            struct alignas(4 * WPV) Words {
                uint32_t u[WPV];
            };
#pragma unroll
            for (int c = 0; c < EPL / 2 / WPV; ++c) {
                Words r;
#pragma unroll
                for (int i = 0; i < WPV; ++i) {
                    const int e = 2 * (c * WPV + i);
                    r.u[i] = (uint32_t)f32_to_bf16_rne(acc[e] * inv * out_scale) |
                             ((uint32_t)f32_to_bf16_rne(acc[e + 1] * inv * out_scale) << 16);
                }
                *reinterpret_cast<Words*>(dst + 2 * c * WPV) = r;
            }
        }
    }
    if (lane < G)
        lse[leaf * n_q_heads + j0 + lane] =
            empty ? -INFINITY : (ms + __builtin_amdgcn_logf(ls)) * 0.6931471805599453f;
}

template <int D, int G>
__global__ __launch_bounds__(256) void merge_kernel(const int32_t* __restrict__ part_base,
                                                    int n_leaves, int n_kv_heads,
                                                    const float* __restrict__ ws_o,
                                                    const float2* __restrict__ ws_ml,
                                                    void* __restrict__ out, int out_bf16,
                                                    float* __restrict__ lse, HeadScales v_scales) {
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int64_t pair = (int64_t)blockIdx.x * 4 + wave;  // (leaf, kv head) index
    if (pair >= (int64_t)n_leaves * n_kv_heads) return;
    const int leaf = (int)(pair / n_kv_heads), h = (int)(pair % n_kv_heads);
    merge_leaf_heads<D, G>(lane, leaf, h, part_base[leaf], part_base[leaf + 1], n_kv_heads * G, ws_o,
                           ws_ml, 0, out, out_bf16 != 0, lse, v_scales.s[h]);
}

}  // namespace ets
