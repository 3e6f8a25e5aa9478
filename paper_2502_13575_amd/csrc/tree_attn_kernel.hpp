// Tree attention on the matrix cores: one workgroup of four wavefronts = one
// (work item, kv head).
//
// A work item names a list of steps (pieces of at most 32 consecutive pool
// rows: a chunk of a tree segment, or a leaf's private suffix) and the leaf
// queries that attend to them.  The workgroup reads the item's K and V from
// HBM exactly once, 128 tokens (four steps) at a time, stages them in LDS and
// applies them to all R = n_ent * G query rows (the G query heads of a leaf
// share the kv head):
//   R  > 32  "row parallel":   every wave walks all steps, wave w owns the 16-row
//            blocks w and w + 4; the staged tile is reused by the four waves.
//   R <= 32  "token parallel": every wave owns all rows, wave w walks step w of
//            each tile; the four running results are folded through LDS at the
//            end, so the item still yields one partial per query row.
//
// bf16 pools, head_dim 128.  Per step of 32 tokens and per block of 16 query rows:
//   S^T = K Q^T    v_mfma_f32_16x16x32_bf16, tokens on M, query rows on N:
//                  A = K rows (8 consecutive d per lane, read from the LDS tile),
//                  B = Q rows (registers).
//   softmax        each lane holds one query row x 8 tokens; weights are taken
//                  against a per-row reference score that is raised only when a
//                  score exceeds it by more than 2^8 in weight, so the common
//                  step needs no cross-lane traffic.
//   O^T += V^T P^T v_mfma_f32_16x16x32_f16.  A bf16 weight has 8 significant
//                  bits, too few for the output tolerance when a handful of
//                  tokens dominate; fp16 has 11, and a bf16 value converts to
//                  fp16 without rounding (magnitudes above 65504 saturate,
//                  below 2^-24 flush), so V is converted once while it is staged
//                  and P is rounded to fp16.  The C layout of S^T is already the
//                  B layout of P^T when the 8 contraction slots of lane group kg
//                  are mapped to tokens {4kg..4kg+3} of both 16-token tiles; V^T
//                  is brought to that slot order by an 8x8 transpose in registers
//                  of eight coalesced 16-byte row pieces before it is staged.
// Loads of the next tile are in flight while the current one is computed.
// The result per query row is the unnormalised partial (o, m, l), m in log2
// units, merged later along each leaf's chain.
#pragma once

#include "device_utils.hpp"
#include "plan.h"

namespace ets {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }
__device__ __forceinline__ f16x8_t as_f16x8(u32x4_t v) { return __builtin_bit_cast(f16x8_t, v); }
__device__ __forceinline__ u32x4_t load16(const void* p) {
    return *reinterpret_cast<const u32x4_t*>(p);
}
// Two bf16 packed in a dword -> the same two values as packed fp16.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t v) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16_lo(v), bf16_hi(v)));
}

constexpr int kTreeAttnRowsPerItem = 128;  // 4 waves x 2 blocks x 16 rows
constexpr int kTreeAttnMaxSteps = 512;     // steps per work item (planner's cap)

// One step: 32 staged tokens against NBV blocks of 16 query rows of one wave.
// Straight-line code (NBV is a compile-time constant) so that LDS reads, matrix
// and vector instructions can be interleaved by the scheduler.
template <int NBV>
__device__ __forceinline__ void attn_step(const u32x4_t* __restrict__ ks_lane,
                                          const u32x4_t* __restrict__ vs_lane, int b, int n_valid,
                                          const bf16x8_t (&qf)[2][4], f32x4_t (&oacc)[2][8],
                                          float (&m)[2], float (&lsum)[2], float scale_log2e,
                                          float raise_margin) {
    constexpr int KROW = 17;
    // scores S^T = K Q^T; a K fragment serves every row block
    bf16x8_t kf[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kf[t][kk] = as_bf16x8(ks_lane[16 * t * KROW + 4 * kk]);
    f32x4_t sacc[2][NBV];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int blk = 0; blk < NBV; ++blk) sacc[t][blk] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int blk = 0; blk < NBV; ++blk)
                sacc[t][blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][kk], qf[blk][kk],
                                                                       sacc[t][blk], 0, 0, 0);
    // lane holds row a of each block, tokens 4 b + i (tile 0) and 16 + 4 b + i (tile 1)
    float s[NBV][8];
    bool need = false;
#pragma unroll
    for (int blk = 0; blk < NBV; ++blk) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            s[blk][j] = sacc[0][blk][j];
            s[blk][4 + j] = sacc[1][blk][j];
        }
        if (n_valid < 32) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (16 * (j >> 2) + 4 * b + (j & 3) >= n_valid) s[blk][j] = -INFINITY;
        }
        const float mx = fmaxf(fmaxf(fmaxf(s[blk][0], s[blk][1]), fmaxf(s[blk][2], s[blk][3])),
                               fmaxf(fmaxf(s[blk][4], s[blk][5]), fmaxf(s[blk][6], s[blk][7])));
        need |= mx > m[blk] + raise_margin;
    }
    if (__any(need)) {
        // raise the reference of every row to its running maximum
#pragma unroll
        for (int blk = 0; blk < NBV; ++blk) {
            float mx = fmaxf(fmaxf(fmaxf(s[blk][0], s[blk][1]), fmaxf(s[blk][2], s[blk][3])),
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
    f16x8_t pf[NBV];
#pragma unroll
    for (int blk = 0; blk < NBV; ++blk) {
        const float mc = m[blk] * scale_log2e;
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float p = fast_exp2(fmaf(s[blk][j], scale_log2e, -mc));
            psum += p;
            pf[blk][j] = (_Float16)p;
        }
        lsum[blk] += psum;
    }
    // O^T += V^T P^T
#pragma unroll
    for (int x = 0; x < 8; ++x) {
        const f16x8_t vf = as_f16x8(vs_lane[x * 64]);
#pragma unroll
        for (int blk = 0; blk < NBV; ++blk)
            oacc[blk][x] =
                __builtin_amdgcn_mfma_f32_16x16x32_f16(vf, pf[blk], oacc[blk][x], 0, 0, 0);
    }
}

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
    __shared__ u32x4_t sm_desc[kTreeAttnMaxSteps];  // the item's step list
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
    // Row blocks of 16 query rows: token-parallel waves all own blocks 0 and 1;
    // row-parallel wave w owns blocks w and w + 4, so that up to 64 rows every wave
    // has one block and the work is spread evenly.
    const int n_blocks = (R + 15) >> 4;
    const int blk_stride = rowpar ? 4 : 1;
    const int blk0 = rowpar ? w : 0;
    const int nbv = (blk0 < n_blocks) + (blk0 + blk_stride < n_blocks);  // blocks this wave owns
    const int n_steps = it.run_end - it.run_begin;
    const int n_tiles = (n_steps + 3) >> 2;
    const Run* my_steps = steps + it.run_begin;
    const float raise_margin = 8.0f / scale_log2e;  // raw-score distance of 2^8 in weight

    // wave w fetches step 4 tile + w of every tile
    u32x4_t kraw[8], vraw[8];
    const uint32_t stride_b = (uint32_t)n_kv_heads * D * 2;             // bytes between tokens
    const uint32_t k_lane_off = (uint32_t)b * stride_b + a * 16;        // K: token 4 i + b
    const uint32_t v_lane_off = (uint32_t)(4 * b) * stride_b + a * 16;  // V: token 16 (i/4) + 4 b + i%4
    auto issue_loads = [&](const Run& sd) {
        if (sd.n > 0) {
            const int64_t base = (sd.tok * n_kv_heads + h) * (int64_t)D * 2;
            const char* kb = reinterpret_cast<const char*>(k_pool) + base;  // uniform
            const char* vb = reinterpret_cast<const char*>(v_pool) + base;
            if (sd.n == 32) {
                // full step: uniform base + per-lane offset that never changes
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    kraw[i] = load16(kb + (uint32_t)(4 * i) * stride_b + k_lane_off);
                    vraw[i] = load16(vb + (uint32_t)(16 * (i >> 2) + (i & 3)) * stride_b + v_lane_off);
                }
            } else {
                // ragged tail of a run: rows past the end re-read the last row (masked later)
                const int last = sd.n - 1;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t tk = (uint32_t)min(4 * i + b, last);
                    const uint32_t tv = (uint32_t)min(16 * (i >> 2) + 4 * b + (i & 3), last);
                    kraw[i] = load16(kb + tk * stride_b + a * 16);
                    vraw[i] = load16(vb + tv * stride_b + a * 16);
                }
            }
        }
    };

    // The first tile's loads start as soon as this wave's first step is known (read
    // straight from the step list); everything else the prologue needs overlaps them.
    Run sd_loaded = w < n_steps ? my_steps[w] : Run{0, 0, 0};  // descriptor of the loads in flight
    issue_loads(sd_loaded);

    // the item's step descriptors go to LDS once; nothing but K, V is fetched afterwards
    for (int i = threadIdx.x; i < n_steps; i += 256)
        sm_desc[i] = load16(reinterpret_cast<const char*>(my_steps + i));

    // Q rows as B operands: lane (column a = query row, group b) holds
    // q[row][32 kk + 8 b .. + 8) for kk = 0..3.  The workspace row of the lane's
    // partial result is looked up here as well, off the critical path.
    bf16x8_t qf[NB][4];
    int64_t out_row[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        const int r = 16 * (blk0 + blk * blk_stride) + a;
        const int rr = r < R ? r : 0;  // padding rows read a valid row; never written
        const int ent = ent_order[it.ent_begin + (rr >> g_shift)];
        const int head = h * G + (rr & (G - 1));
        const bf16_t* qp = q + ((int64_t)ent * n_q_heads + head) * D;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[blk][kk] = as_bf16x8(load16(qp + 32 * kk + 8 * b));
        out_row[blk] = ((int64_t)part_base[ent] + it.slot_off) * n_q_heads + head;
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

    auto read_desc = [&](int sidx) {
        Run sd{0, 0, 0};
        if (sidx < n_steps) {
            const u32x4_t d = sm_desc[sidx];  // same address in every lane
            const uint32_t lo = __builtin_amdgcn_readfirstlane(d[0]);
            const uint32_t hi = __builtin_amdgcn_readfirstlane(d[1]);
            sd.tok = (int64_t)(((uint64_t)hi << 32) | lo);
            sd.n = __builtin_amdgcn_readfirstlane(d[2]);
        }
        return sd;
    };
    auto stage = [&](const Run& sd) {
        if (sd.n > 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) ks[(32 * w + 4 * i + b) * KROW + a] = kraw[i];
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
                u32x4_t t;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    t[j] = bf16x2_to_f16x2(
                        __builtin_amdgcn_perm(vraw[2 * j + 1][x >> 1], vraw[2 * j][x >> 1], sel));
                vs[(w * 8 + x) * 64 + lane] = t;
            }
        }
    };

    // Row-parallel waves share the staged tile: workgroup barriers.  Token-parallel
    // waves stage and read only their own quarter of it, and the LDS executes one
    // wave's accesses in order, so a compiler-level fence is enough there.
    auto tile_sync = [&]() {
        if (rowpar) {
            __syncthreads();
        } else {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    };

    stage(sd_loaded);
    // Everything issued so far (Q rows, first tile) has to have landed on every path
    // before the loop: a load still counted as outstanding here would make each
    // iteration wait for the next tile's loads as well.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();  // step list and first tile are in LDS

    for (int tile = 0; tile < n_tiles; ++tile) {
        sd_loaded = read_desc(4 * (tile + 1) + w);  // a step past the end has n = 0
        issue_loads(sd_loaded);

        const int st_lo = rowpar ? 0 : w;
        const int st_hi = rowpar ? 4 : w + 1;
#pragma unroll 1
        for (int st = st_lo; st < st_hi; ++st) {
            const int sidx = 4 * tile + st;
            if (sidx >= n_steps || nbv == 0) break;
            const int n_valid = __builtin_amdgcn_readfirstlane(sm_desc[sidx][2]);
            const u32x4_t* ks_lane = ks + (32 * st + a) * KROW + b;
            const u32x4_t* vs_lane = vs + st * 8 * 64 + lane;
            if (nbv == 2)
                attn_step<2>(ks_lane, vs_lane, b, n_valid, qf, oacc, m, lsum, scale_log2e,
                             raise_margin);
            else
                attn_step<1>(ks_lane, vs_lane, b, n_valid, qf, oacc, m, lsum, scale_log2e,
                             raise_margin);
        }

        tile_sync();  // the staged tile has been read by everyone who shares it
        stage(sd_loaded);
        tile_sync();
    }

    if (rowpar) {
        // each wave owns its rows: lane group b holds d = 32 b + 8 i + x of row a
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            const int r = 16 * (blk0 + blk * blk_stride) + a;
            float l = lsum[blk];
            l += __shfl_xor(l, 16, 64);
            l += __shfl_xor(l, 32, 64);
            if (blk < nbv && r < R) {
                float* dst = ws_o + out_row[blk] * D + 32 * b;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    *reinterpret_cast<float4*>(dst + 8 * i) =
                        make_float4(oacc[blk][0][i], oacc[blk][1][i], oacc[blk][2][i],
                                    oacc[blk][3][i]);
                    *reinterpret_cast<float4*>(dst + 8 * i + 4) =
                        make_float4(oacc[blk][4][i], oacc[blk][5][i], oacc[blk][6][i],
                                    oacc[blk][7][i]);
                }
                if (b == 0) ws_ml[out_row[blk]] = make_float2(m[blk] * scale_log2e, l);
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
    __syncthreads();  // also: every wave has left the main loop, the tile buffer is free
    float m_all[NB], l_all[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        m_all[blk] = 0.f;
        l_all[blk] = 0.f;
        if (blk < n_blocks) {
            float ms = sm_m[0][blk][a];
#pragma unroll
            for (int ww = 1; ww < 4; ++ww) ms = fmaxf(ms, sm_m[ww][blk][a]);
            float ls = 0.f;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww)
                ls += sm_l[ww][blk][a] * fast_exp2((sm_m[ww][blk][a] - ms) * scale_log2e);
            const float f = fast_exp2((m[blk] - ms) * scale_log2e);
            f32x4_t* dst = reinterpret_cast<f32x4_t*>(smem) + ((w * NB + blk) * 8) * 64 + lane;
#pragma unroll
            for (int x = 0; x < 8; ++x) dst[x * 64] = oacc[blk][x] * f;
            m_all[blk] = ms;
            l_all[blk] = ls;
        }
    }
    __syncthreads();
    {
        // wave w sums block w / 2, columns x in [4 (w % 2), + 4): 16 contiguous bytes per i
        const int blk = w >> 1, xh = w & 1;
        const int r = 16 * blk + a;
        if (blk < n_blocks && r < R) {
            f32x4_t acc[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                const f32x4_t* src = reinterpret_cast<const f32x4_t*>(smem) +
                                     ((ww * NB + blk) * 8 + 4 * xh) * 64 + lane;
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] += src[j * 64];
            }
            const int64_t row = blk == 0 ? out_row[0] : out_row[1];
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
