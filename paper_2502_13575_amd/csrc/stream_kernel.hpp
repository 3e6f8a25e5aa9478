// Per-leaf streaming attention: one wavefront = one (work item, kv head).
//
// A work item names one leaf query and a list of pool runs (its private
// suffix of the tree, or in the flat baseline its whole root->leaf chain).
// The wave streams the runs' K and V rows from HBM with 16-byte loads that
// cover whole head rows contiguously (D * sizeof(T) bytes per token and head),
// keeps the G query heads of the kv head in registers, and carries a running
// (max, sum, weighted V) per query head: the online form of the softmax whose
// result is defined by out = sum_t exp(s_t - lse) V_t.  It writes one
// unnormalised partial (o, m, l) per query head; the merge kernel combines the
// partials along the leaf's chain.  m is kept in log2 units (scores are
// pre-multiplied by log2 e) so that exp2 can be used throughout.
#pragma once

#include "device_utils.hpp"
#include "plan.h"

namespace ets {

template <typename T, int D, int G, int U>
__global__ __launch_bounds__(64) void stream_attn_kernel(
    const T* __restrict__ k_pool, const T* __restrict__ v_pool, int64_t pool_tokens,
    const T* __restrict__ q, const Run* __restrict__ runs, const StreamItem* __restrict__ items,
    int n_kv_heads,
    float scale_log2e, float* __restrict__ ws_o, float2* __restrict__ ws_ml) {
    constexpr int EPL = Vec16<T>::N;  // elements per lane per load
    constexpr int LPT = D / EPL;      // lanes per token row
    constexpr int TPS = 64 / LPT;     // tokens per wave-wide load
    static_assert(LPT >= 2 && LPT <= 64 && TPS >= 1, "unsupported row size");

    const int h = blockIdx.x % n_kv_heads;
    const StreamItem item = items[blockIdx.x / n_kv_heads];
    const int lane = threadIdx.x;
    const int a = lane % LPT;  // which 16-byte piece of the row
    const int b = lane / LPT;  // which token of the step
    const int n_q_heads = n_kv_heads * G;
    constexpr int64_t row_stride = D;  // pools are [kv head][pool row][D]

    float qf[G][EPL];
    {
        const T* qp = q + ((int64_t)item.entry * n_q_heads + (int64_t)h * G) * D + a * EPL;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            Vec16<T> v;
            v.load(qp + g * D);
            v.unpack(qf[g]);
#pragma unroll
            for (int i = 0; i < EPL; ++i) qf[g][i] *= scale_log2e;
        }
    }

    float m[G], l[G], o[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) o[g][i] = 0.f;
    }

    for (int r = item.run_begin; r < item.run_end; ++r) {
        const Run run = runs[r];
        const int64_t base = ((int64_t)h * pool_tokens + run.tok) * (int64_t)D + a * EPL;
        const T* kb = k_pool + base;
        const T* vb = v_pool + base;
        for (int t0 = 0; t0 < run.n; t0 += TPS * U) {
            Vec16<T> kraw[U], vraw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int tok = min(t0 + u * TPS + b, run.n - 1);  // clamp: stays inside the run
                kraw[u].load(kb + tok * row_stride);
                vraw[u].load(vb + tok * row_stride);
            }
            float s[U][G];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float kf[EPL];
                kraw[u].unpack(kf);
                const bool valid = t0 + u * TPS + b < run.n;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float acc = 0.f;
#pragma unroll
                    for (int i = 0; i < EPL; ++i) acc = fmaf(qf[g][i], kf[i], acc);
                    acc = group_sum<LPT>(acc);
                    s[u][g] = valid ? acc : -INFINITY;
                }
            }
            float alpha[G], mu[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mn = m[g];
#pragma unroll
                for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[u][g]);
                mu[g] = (mn == -INFINITY) ? 0.f : mn;
                alpha[g] = fast_exp2(m[g] - mu[g]);
                m[g] = mn;
                l[g] *= alpha[g];
#pragma unroll
                for (int i = 0; i < EPL; ++i) o[g][i] *= alpha[g];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float vf[EPL];
                vraw[u].unpack(vf);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float p = fast_exp2(s[u][g] - mu[g]);
                    l[g] += p;
#pragma unroll
                    for (int i = 0; i < EPL; ++i) o[g][i] = fmaf(p, vf[i], o[g][i]);
                }
            }
        }
    }

    // fold the TPS token lanes of the wave together
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float mt = m[g];
#pragma unroll
        for (int off = LPT; off < 64; off <<= 1) mt = fmaxf(mt, __shfl_xor(mt, off, 64));
        const float mu = (mt == -INFINITY) ? 0.f : mt;
        const float f = fast_exp2(m[g] - mu);
        float lt = l[g] * f;
#pragma unroll
        for (int off = LPT; off < 64; off <<= 1) lt += __shfl_xor(lt, off, 64);
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            float x = o[g][i] * f;
#pragma unroll
            for (int off = LPT; off < 64; off <<= 1) x += __shfl_xor(x, off, 64);
            o[g][i] = x;
        }
        if (b == 0) {
            const int64_t row = (int64_t)item.slot * n_q_heads + h * G + g;
            float4* dst = reinterpret_cast<float4*>(ws_o + row * D + a * EPL);
#pragma unroll
            for (int i = 0; i < EPL / 4; ++i)
                dst[i] = make_float4(o[g][4 * i], o[g][4 * i + 1], o[g][4 * i + 2],
                                     o[g][4 * i + 3]);
            if (a == 0) ws_ml[row] = make_float2(mt, lt);
        }
    }
}

}  // namespace ets
