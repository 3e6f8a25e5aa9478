// Tree attention on the matrix cores: one workgroup of four wavefronts = one
// (work item, kv head).
//
// A work item names a list of steps (pieces of at most 32 consecutive pool
// rows: a chunk of a tree segment, or a leaf's private suffix) and the leaf
// queries that attend to them.  The workgroup reads the item's K and V from
// HBM exactly once, 128 tokens (four steps) at a time, stages them in LDS and
// applies them to all R = n_ent * G query rows (the G query heads of a leaf
// share the kv head):
//   R  > 32  "row parallel":   every wave walks all steps, wave w owns query
//            rows [32 w, 32 w + 32); the staged tile is reused by the four waves.
//   R <= 32  "token parallel": every wave owns all rows, wave w walks step w of
//            each tile; the four running results are folded through LDS at the
//            end, so the item still yields one partial per query row.
//
// bf16, head_dim 128, v_mfma_f32_16x16x32_bf16.  Per step of 32 tokens and per
// block of 16 query rows:
//   S^T = K Q^T    tokens on M, query rows on N: A = K rows (8 consecutive d per
//                  lane, read from the LDS tile), B = Q rows (registers).
//   softmax        each lane holds one query row x 8 tokens; weights are taken
//                  against a per-row reference score that is raised only when a
//                  score exceeds it by more than 2^8 in weight, so the common
//                  step needs no cross-lane traffic.
//   O^T += V^T P^T with P = P_hi + P_lo (two bf16 terms, ~16 significant bits).
//                  The C layout of S^T is already the B layout of P^T when the
//                  8 contraction slots of lane group kg are mapped to tokens
//                  {4kg..4kg+3} of both 16-token tiles; V^T is brought to that
//                  slot order by an 8x8 transpose in registers of eight
//                  coalesced 16-byte row pieces before it is staged in LDS.
// Loads of the next tile are in flight while the current one is computed.
// The result per query row is the unnormalised partial (o, m, l), m in log2
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

constexpr int kTreeAttnRowsPerItem = 128;  // 4 waves x 2 blocks x 16 rows

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void tree_attn_kernel(
    const bf16_t* __restrict__ k_pool, const bf16_t* __restrict__ v_pool,
    const bf16_t* __restrict__ q, const Run* __restrict__ steps,
    const CascadeItem* __restrict__ items, const int32_t* __restrict__ ent_order,
    const int32_t* __restrict__ part_base, int n_kv_heads, int g_shift, float scale_log2e,
    float* __restrict__ ws_o, float2* __restrict__ ws_ml) {
    constexpr int D = 128;
    constexpr int NB = 2;     // blocks of 16 query rows per wave
    constexpr int KROW = 17;  // 16-byte units per padded K row in LDS (272 bytes)
    constexpr int KS_UNITS = 128 * KROW;
    constexpr int VS_UNITS = 4 * 8 * 64;
    // K tile, then V^T fragments; reused for the fold of the token-parallel mode
    __shared__ u32x4_t smem[KS_UNITS + VS_UNITS];
    __shared__ float sm_m[4][NB][16];
    __shared__ float sm_l[4][NB][16];
    __shared__ int sm_n[4];  // tokens in each of the staged tile's four steps (0 = none)
    u32x4_t* ks = smem;
    u32x4_t* vs = smem + KS_UNITS;

    // wave index, made known-uniform so that per-wave descriptors come through scalar loads
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int a = lane & 15;  // 16-byte piece of a row when loading; MFMA row/column index
    const int b = lane >> 4;  // token sub-index when loading; MFMA contraction group kg
    const int h = blockIdx.x % n_kv_heads;
    const CascadeItem it = items[blockIdx.x / n_kv_heads];
    const int G = 1 << g_shift;
    const int n_q_heads = n_kv_heads << g_shift;
    const int R = it.n_ent << g_shift;
    const bool rowpar = R > 16 * NB;
    const int row0 = rowpar ? w * 16 * NB : 0;  // first query row of this wave
    const int nbv = min(NB, max(0, (R - row0 + 15) >> 4));  // row blocks this wave owns
    const int n_steps = it.run_end - it.run_begin;
    const int n_tiles = (n_steps + 3) >> 2;
    const Run* my_steps = steps + it.run_begin;
    const int64_t row_stride = (int64_t)n_kv_heads * D;  // elements between tokens
    const float raise_margin = 8.0f / scale_log2e;       // raw-score distance of 2^8 in weight

    // Q rows as B operands: lane (column a = query row, group b) holds
    // q[row][32 kk + 8 b .. + 8) for kk = 0..3.
    bf16x8_t qf[NB][4];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        const int r = row0 + 16 * blk + a;
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

    // wave w fetches step 4 tile + w of every tile; the step descriptor is read one
    // tile ahead of the loads that use it
    u32x4_t kraw[8], vraw[8];
    auto read_desc = [&](int tile) {
        const int sidx = 4 * tile + w;
        return sidx < n_steps ? my_steps[sidx] : Run{0, 0, 0};
    };
    auto issue_loads = [&](const Run& sd) {
        if (sd.n > 0) {
            const int last = sd.n - 1;
            const int64_t base = (sd.tok * n_kv_heads + h) * (int64_t)D + a * 8;
            const bf16_t* kb = k_pool + base;
            const bf16_t* vb = v_pool + base;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                // K: token 4 i + b, a whole 256-byte row per 16 lanes
                kraw[i] = load16(kb + min(4 * i + b, last) * row_stride);
                // V: contraction slot i of group b = token 16 (i / 4) + 4 b + i % 4
                vraw[i] = load16(vb + min(16 * (i >> 2) + 4 * b + (i & 3), last) * row_stride);
            }
        }
    };
    auto stage = [&](const Run& sd) {
        if (lane == 0) sm_n[w] = sd.n;
        if (sd.n > 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) ks[(32 * w + 4 * i + b) * KROW + a] = kraw[i];
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
                u32x4_t t;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    t[j] = __builtin_amdgcn_perm(vraw[2 * j + 1][x >> 1], vraw[2 * j][x >> 1], sel);
                vs[(w * 8 + x) * 64 + lane] = t;
            }
        }
    };

    Run sd_loaded = read_desc(0);  // descriptor of the loads in flight
    issue_loads(sd_loaded);
    Run sd_next = read_desc(1);
    stage(sd_loaded);
    // Everything issued so far (Q rows, first tile) has to have landed on every path
    // before the loop: a load still counted as outstanding here would make each
    // iteration wait for the next tile's loads as well.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    for (int tile = 0; tile < n_tiles; ++tile) {
        sd_loaded = sd_next;         // tile + 1 (a descriptor past the end has n = 0)
        issue_loads(sd_loaded);
        sd_next = read_desc(tile + 2);

        const int st_lo = rowpar ? 0 : w;
        const int st_hi = rowpar ? 4 : w + 1;
#pragma unroll 1
        for (int st = st_lo; st < st_hi; ++st) {
            const int n_valid = __builtin_amdgcn_readfirstlane(sm_n[st]);
            if (n_valid == 0 || nbv == 0) break;

            // scores S^T = K Q^T of every row block; K fragments come from the LDS
            // tile one at a time and serve all blocks
            f32x4_t sacc[2][NB];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int blk = 0; blk < NB; ++blk) sacc[t][blk] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const bf16x8_t kf =
                        as_bf16x8(ks[(32 * st + 16 * t + a) * KROW + 4 * kk + b]);
#pragma unroll
                    for (int blk = 0; blk < NB; ++blk)
                        if (blk < nbv)
                            sacc[t][blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                kf, qf[blk][kk], sacc[t][blk], 0, 0, 0);
                }
            }
            // lane holds row a of each block, tokens 4 b + i (tile 0), 16 + 4 b + i (tile 1)
            float s[NB][8];
#pragma unroll
            for (int blk = 0; blk < NB; ++blk)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    s[blk][j] = sacc[0][blk][j];
                    s[blk][4 + j] = sacc[1][blk][j];
                }
            bool need = false;
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) {
                if (n_valid < 32) {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (16 * (j >> 2) + 4 * b + (j & 3) >= n_valid) s[blk][j] = -INFINITY;
                }
                const float mx =
                    fmaxf(fmaxf(fmaxf(s[blk][0], s[blk][1]), fmaxf(s[blk][2], s[blk][3])),
                          fmaxf(fmaxf(s[blk][4], s[blk][5]), fmaxf(s[blk][6], s[blk][7])));
                need |= (blk < nbv) && (mx > m[blk] + raise_margin);
            }
            if (__any(need)) {
                // raise the reference of every row to its running maximum
#pragma unroll
                for (int blk = 0; blk < NB; ++blk) {
                    if (blk < nbv) {
                        float mx =
                            fmaxf(fmaxf(fmaxf(s[blk][0], s[blk][1]), fmaxf(s[blk][2], s[blk][3])),
                                  fmaxf(fmaxf(s[blk][4], s[blk][5]), fmaxf(s[blk][6], s[blk][7])));
                        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                        const float m_new = fmaxf(m[blk], mx);
                        const float alpha = fast_exp2((m[blk] - m_new) * scale_log2e);
                        lsum[blk] *= alpha;
#pragma unroll
                        for (int x = 0; x < 8; ++x) oacc[blk][x] *= alpha;
                        m[blk] = m_new;
                    }
                }
            }
            // A bf16 weight carries 8 significant bits, too few for the output tolerance
            // when a handful of tokens dominate; the weight is therefore split into a
            // bf16 head and a bf16 remainder (together ~16 bits) and both enter P V.
            bf16x8_t pf[NB], pl[NB];
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) {
                if (blk < nbv) {
                    const float mc = m[blk] * scale_log2e;
                    float psum = 0.f;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float p = fast_exp2(fmaf(s[blk][j], scale_log2e, -mc));
                        psum += p;
                        const __bf16 hi = (__bf16)p;
                        pf[blk][j] = hi;
                        pl[blk][j] = (__bf16)(p - (float)hi);
                    }
                    lsum[blk] += psum;
                }
            }
            // O^T += V^T (P_hi + P_lo)^T
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const bf16x8_t vf = as_bf16x8(vs[(st * 8 + x) * 64 + lane]);
#pragma unroll
                for (int blk = 0; blk < NB; ++blk)
                    if (blk < nbv) {
                        oacc[blk][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[blk],
                                                                               oacc[blk][x], 0, 0, 0);
                        oacc[blk][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pl[blk],
                                                                               oacc[blk][x], 0, 0, 0);
                    }
            }
        }

        __syncthreads();  // every wave is done reading the staged tile
        stage(sd_loaded);
        __syncthreads();
    }

    if (rowpar) {
        // each wave owns its rows: lane group b holds d = 32 b + 8 i + x of row a
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            const int r = row0 + 16 * blk + a;
            float l = lsum[blk];
            l += __shfl_xor(l, 16, 64);
            l += __shfl_xor(l, 32, 64);
            if (blk < nbv && r < R) {
                const int ent = ent_order[it.ent_begin + (r >> g_shift)];
                const int64_t row =
                    ((int64_t)part_base[ent] + it.slot_off) * n_q_heads + h * G + (r & (G - 1));
                float* dst = ws_o + row * D + 32 * b;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    *reinterpret_cast<float4*>(dst + 8 * i) =
                        make_float4(oacc[blk][0][i], oacc[blk][1][i], oacc[blk][2][i],
                                    oacc[blk][3][i]);
                    *reinterpret_cast<float4*>(dst + 8 * i + 4) =
                        make_float4(oacc[blk][4][i], oacc[blk][5][i], oacc[blk][6][i],
                                    oacc[blk][7][i]);
                }
                if (b == 0) ws_ml[row] = make_float2(m[blk] * scale_log2e, l);
            }
        }
        return;
    }

    // token parallel: fold the four waves' running results (same rows, disjoint tokens)
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        float l = lsum[blk];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (b == 0) {
            sm_m[w][blk][a] = m[blk];
            sm_l[w][blk][a] = l;
        }
    }
    __syncthreads();
    float m_all[NB], l_all[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        float ms = sm_m[0][blk][a];
#pragma unroll
        for (int ww = 1; ww < 4; ++ww) ms = fmaxf(ms, sm_m[ww][blk][a]);
        const float mu = (ms == -INFINITY) ? 0.f : ms;
        float ls = 0.f;
#pragma unroll
        for (int ww = 0; ww < 4; ++ww)
            ls += sm_l[ww][blk][a] * fast_exp2((sm_m[ww][blk][a] - mu) * scale_log2e);
        const float f = fast_exp2((m[blk] - mu) * scale_log2e);
        f32x4_t* dst = reinterpret_cast<f32x4_t*>(smem) + ((w * NB + blk) * 8) * 64 + lane;
#pragma unroll
        for (int x = 0; x < 8; ++x) dst[x * 64] = oacc[blk][x] * f;
        m_all[blk] = ms;
        l_all[blk] = ls;
    }
    __syncthreads();
    {
        // wave w sums block w / 2, columns x in [4 (w % 2), + 4): 16 contiguous bytes per i
        const int blk = w >> 1, xh = w & 1;
        const int r = 16 * blk + a;
        f32x4_t acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) {
            const f32x4_t* src =
                reinterpret_cast<const f32x4_t*>(smem) + ((ww * NB + blk) * 8 + 4 * xh) * 64 + lane;
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] += src[j * 64];
        }
        if (r < R) {
            const int ent = ent_order[it.ent_begin + (r >> g_shift)];
            const int64_t row =
                ((int64_t)part_base[ent] + it.slot_off) * n_q_heads + h * G + (r & (G - 1));
            float* dst = ws_o + row * D + 32 * b + 4 * xh;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *reinterpret_cast<float4*>(dst + 8 * i) =
                    make_float4(acc[0][i], acc[1][i], acc[2][i], acc[3][i]);
            if (b == 0 && xh == 0) {
                const float ms = blk == 0 ? m_all[0] : m_all[1];
                const float ls = blk == 0 ? l_all[0] : l_all[1];
                ws_ml[row] = make_float2(ms * scale_log2e, ls);
            }
        }
    }
}

}  // namespace ets
