// Shared-node ("cascade") attention on the matrix cores: one wavefront = one
// (work item, kv head).  A work item names a run list of pool rows (a chunk of
// a tree segment) and the leaf queries beneath the segment; the wave reads the
// chunk's K and V once and applies them to all R = n_ent * G query rows
// (G query heads per leaf share the kv head), R <= 16 * NB.
//
// bf16, head_dim 128, v_mfma_f32_16x16x32_bf16.  Per step of 32 tokens:
//   S^T = K Q^T   tokens on M, query rows on N: A = K rows (8 consecutive d per
//                 lane), B = Q rows (same 8 d), 4 MFMAs per 16-token tile.
//   softmax       each lane holds one query row (column of S^T) x 8 tokens;
//                 running max / sum per row, two cross-lane exchanges per step.
//   O^T += V^T P^T  the C layout of S^T is already the B layout of P^T when
//                 the 8 contraction slots of lane group kg are mapped to tokens
//                 {4kg..4kg+3} of tile 0 and of tile 1; the A operand V^T is
//                 built to the same slot order by an 8x8 transpose in
//                 registers of eight coalesced 16-byte row pieces.
// K goes through a wave-private LDS tile (coalesced 256-byte row loads in,
// MFMA A-layout out, rows padded to 272 bytes against bank conflicts).
// The result is the unnormalised partial (o, m, l) per query row, m in log2
// units, merged later along each leaf's chain.
#pragma once

#include "device_utils.hpp"
#include "plan.h"

namespace ets {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }
__device__ __forceinline__ u32x4_t load16(const void* p) {
    return *reinterpret_cast<const u32x4_t*>(p);
}

template <int NB>
__global__ __launch_bounds__(64) void cascade_attn_kernel(
    const bf16_t* __restrict__ k_pool, const bf16_t* __restrict__ v_pool,
    const bf16_t* __restrict__ q, const Run* __restrict__ runs,
    const CascadeItem* __restrict__ items, const int32_t* __restrict__ ent_order,
    const int32_t* __restrict__ part_base, int n_kv_heads, int g_shift, float scale_log2e,
    float* __restrict__ ws_o, float2* __restrict__ ws_ml) {
    constexpr int D = 128;
    constexpr int KROW = 17;  // uint4 per padded K row in LDS (272 bytes)
    __shared__ u32x4_t ks[32 * KROW];

    const int lane = threadIdx.x;
    const int a = lane & 15;   // 16-byte piece of a row when loading; MFMA row/column index
    const int b = lane >> 4;   // token sub-index when loading; MFMA contraction group kg
    const int h = blockIdx.x % n_kv_heads;
    const CascadeItem it = items[blockIdx.x / n_kv_heads];
    const int G = 1 << g_shift;
    const int n_q_heads = n_kv_heads << g_shift;
    const int R = it.n_ent << g_shift;
    const int64_t row_stride = (int64_t)n_kv_heads * D;  // elements between tokens

    // Q rows as B operands: lane (column a = query row, group b) holds
    // q[row][32 kk + 8 b .. + 8) for kk = 0..3.
    bf16x8_t qf[NB][4];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        const int r = 16 * blk + a;
        const int rr = r < R ? r : 0;  // padding rows read a valid row; never written
        const int ent = ent_order[it.ent_begin + (rr >> g_shift)];
        const int head = h * G + (rr & (G - 1));
        const bf16_t* qp = q + ((int64_t)ent * n_q_heads + head) * D;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[blk][kk] = as_bf16x8(load16(qp + 32 * kk + 8 * b));
    }

    f32x4_t oacc[NB][8];
    float m[NB], lsum[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        m[blk] = -INFINITY;
        lsum[blk] = 0.f;
#pragma unroll
        for (int x = 0; x < 8; ++x) oacc[blk][x] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    // step cursor over (run, 32-token window)
    int r_cur = it.run_begin, t_cur = 0;
    Run run = runs[r_cur];

    u32x4_t kraw[8], vraw[8];
    auto issue_loads = [&](const Run& rn, int t0) {
        const int last = rn.n - 1;
        const int64_t base = (rn.tok * n_kv_heads + h) * (int64_t)D + a * 8;
        const bf16_t* kb = k_pool + base;
        const bf16_t* vb = v_pool + base;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // K: token 4 i + b, a whole 256-byte row per 16 lanes
            const int tk = min(t0 + 4 * i + b, last);
            kraw[i] = load16(kb + tk * row_stride);
            // V: contraction slot i of group b = token 16 (i / 4) + 4 b + i % 4
            const int tv = min(t0 + 16 * (i >> 2) + 4 * b + (i & 3), last);
            vraw[i] = load16(vb + tv * row_stride);
        }
    };
    issue_loads(run, 0);

    while (true) {
        const int n_valid = min(32, run.n - t_cur);

        // K tile -> LDS (row-major, padded); V tile -> A fragments by transposing in registers
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; ++i) ks[(4 * i + b) * KROW + a] = kraw[i];
        bf16x8_t vf[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
            u32x4_t t;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                t[w] = __builtin_amdgcn_perm(vraw[2 * w + 1][x >> 1], vraw[2 * w][x >> 1], sel);
            vf[x] = as_bf16x8(t);
        }

        // advance the cursor and start the next step's loads
        int t_next = t_cur + 32, r_next = r_cur;
        bool more = true;
        Run run_next = run;
        if (t_next >= run.n) {
            t_next = 0;
            r_next = r_cur + 1;
            more = r_next < it.run_end;
            if (more) run_next = runs[r_next];
        }
        if (more) issue_loads(run_next, t_next);

        __syncthreads();
        bf16x8_t kf[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                kf[t][kk] = as_bf16x8(ks[(16 * t + a) * KROW + 4 * kk + b]);

#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            if (16 * blk >= R) break;
            f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][kk], qf[blk][kk], s0, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][kk], qf[blk][kk], s1, 0, 0, 0);
            }
            // lane holds row a of the block, tokens 4 b + i (tile 0) and 16 + 4 b + i (tile 1)
            float s[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
            if (n_valid < 32) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (16 * (j >> 2) + 4 * b + (j & 3) >= n_valid) s[j] = -INFINITY;
            }
            float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])),
                             fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m[blk], mx);
            if (__any(m_new > m[blk])) {
                const float alpha = fast_exp2((m[blk] - m_new) * scale_log2e);
                lsum[blk] *= alpha;
#pragma unroll
                for (int x = 0; x < 8; ++x) oacc[blk][x] *= alpha;
                m[blk] = m_new;
            }
            const float mc = m_new * scale_log2e;
            float p[8];
            float psum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                p[j] = fast_exp2(fmaf(s[j], scale_log2e, -mc));
                psum += p[j];
            }
            lsum[blk] += psum;
            bf16x8_t pf;
#pragma unroll
            for (int j = 0; j < 8; ++j) pf[j] = (__bf16)p[j];
#pragma unroll
            for (int x = 0; x < 8; ++x)
                oacc[blk][x] =
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[x], pf, oacc[blk][x], 0, 0, 0);
        }

        if (!more) break;
        run = run_next;
        r_cur = r_next;
        t_cur = t_next;
    }

    // partial results: row a of every block; lane group b holds d = 32 b + 8 i + x
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        const int r = 16 * blk + a;
        float l = lsum[blk];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (r < R) {
            const int ent = ent_order[it.ent_begin + (r >> g_shift)];
            const int64_t row =
                ((int64_t)part_base[ent] + it.slot_off) * n_q_heads + h * G + (r & (G - 1));
            float* dst = ws_o + row * D + 32 * b;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float4 lo4 = make_float4(oacc[blk][0][i], oacc[blk][1][i], oacc[blk][2][i],
                                         oacc[blk][3][i]);
                float4 hi4 = make_float4(oacc[blk][4][i], oacc[blk][5][i], oacc[blk][6][i],
                                         oacc[blk][7][i]);
                *reinterpret_cast<float4*>(dst + 8 * i) = lo4;
                *reinterpret_cast<float4*>(dst + 8 * i + 4) = hi4;
            }
            if (b == 0) ws_ml[row] = make_float2(m[blk] * scale_log2e, l);
        }
    }
}

}  // namespace ets
