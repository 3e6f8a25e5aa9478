// Tree attention on the matrix cores: one workgroup of four wavefronts = one
// (work item, kv head).
//
// A work item names a list of steps (pieces of at most 32 consecutive pool
// rows: a chunk of a tree segment, or a leaf's private suffix) and the leaf
// queries that attend to them.  The workgroup reads the item's K and V from
// HBM exactly once, 64 tokens (two steps) at a time, stages them in LDS and
// applies them to all R = n_ent * G <= 64 query rows (the G query heads of a
// leaf share the kv head).  Each wave fetches and stages half a step (16
// tokens) and owns at most one block of 16 query rows, which keeps the kernel
// at 168 registers per lane and 38 KB of LDS: three workgroups (12 waves) per
// compute unit, so that one workgroup's memory latency overlaps the others'
// arithmetic.
//   R  > 16  "row parallel":   wave w owns row block w and walks both steps of
//            every tile; the staged tile is reused by the waves.
//   R <= 16  "token parallel": waves 0 and 2 each walk one of the tile's two
//            steps for the single row block; their two running results are
//            folded through LDS at the end, so the item still yields one
//            partial per query row.
//
// bf16 pools, head_dim 128.  Per step of 32 tokens and block of 16 query rows:
//   S^T = K Q^T    v_mfma_f32_16x16x32_bf16, tokens on M, query rows on N:
//                  A = K rows (8 consecutive d per lane, read from the LDS tile),
//                  B = Q rows (registers).
//   softmax        each lane holds one query row x 8 tokens; weights are taken
//                  against a per-row reference score that is raised only when a
//                  score exceeds it by more than 2^8 in weight, so the common
//                  step needs no cross-lane traffic.
//   O^T += V^T P^T A bf16 weight has 8 significant bits, too few for the output
//                  tolerance when a handful of tokens dominate.  Row-parallel
//                  items convert V to fp16 once while it is staged (a bf16 value
//                  converts without rounding; magnitudes above 65504 saturate,
//                  below 2^-24 flush) and round P to fp16 (11 bits):
//                  v_mfma_f32_16x16x32_f16.  Token-parallel items, where that
//                  conversion would not be shared by several row blocks, keep V
//                  in bf16 and enter P as a bf16 head plus a bf16 remainder.
//                  The C layout of S^T is already the B layout of P^T when the
//                  8 contraction slots of lane group kg are mapped to tokens
//                  {4kg..4kg+3} of both 16-token halves; V^T is brought to that
//                  slot order by a transpose in registers of coalesced 16-byte
//                  row pieces before it is staged.
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
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }
__device__ __forceinline__ f16x8_t as_f16x8(u32x4_t v) { return __builtin_bit_cast(f16x8_t, v); }
__device__ __forceinline__ u32x4_t load16(const void* p) {
    return *reinterpret_cast<const u32x4_t*>(p);
}
// Two bf16 packed in a dword -> the same two values as packed fp16.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t v) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16_lo(v), bf16_hi(v)));
}

constexpr int kTreeAttnRowsPerItem = 64;  // 4 waves x 16 rows
constexpr int kTreeAttnMaxSteps = 256;    // steps per work item (planner's cap)
constexpr int kTreeAttnKRow = 17;         // 16-byte units per padded K row in LDS (272 bytes)

// One step: 32 staged tokens against one block of 16 query rows.  F16V tells
// how V was staged (fp16, or bf16 with split weights).
template <bool F16V>
__device__ __forceinline__ void attn_step(const u32x4_t* __restrict__ ks_lane,
                                          const u32x4_t* __restrict__ vs_lane, int b, int n_valid,
                                          const bf16x8_t (&qf)[4], f32x4_t (&oacc)[8], float& m,
                                          float& lsum, float scale_log2e, float raise_margin) {
    constexpr int KROW = kTreeAttnKRow;
    // scores S^T = K Q^T
    f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ks_lane[4 * kk]), qf[kk], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ks_lane[16 * KROW + 4 * kk]), qf[kk],
                                                     s1, 0, 0, 0);
    }
    // lane holds row a of the block, tokens 4 b + i (first half) and 16 + 4 b + i (second half)
    float s[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
    if (n_valid < 32) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (16 * (j >> 2) + 4 * b + (j & 3) >= n_valid) s[j] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])),
                     fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
    if (__any(mx > m + raise_margin)) {
        // raise the reference of every row to its running maximum
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2((m - m_new) * scale_log2e);
        lsum *= alpha;
#pragma unroll
        for (int x = 0; x < 8; ++x) oacc[x] *= alpha;
        m = m_new;
    }
    const float mc = m * scale_log2e;
    float psum = 0.f;
    if constexpr (F16V) {
        f16x8_t pf;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float p = fast_exp2(fmaf(s[j], scale_log2e, -mc));
            psum += p;
            pf[j] = (_Float16)p;
        }
#pragma unroll
        for (int x = 0; x < 8; ++x)
            oacc[x] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(vs_lane[x * 64]), pf, oacc[x],
                                                             0, 0, 0);
    } else {
        bf16x8_t ph, pl;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float p = fast_exp2(fmaf(s[j], scale_log2e, -mc));
            psum += p;
            const __bf16 hi = (__bf16)p;
            ph[j] = hi;
            pl[j] = (__bf16)(p - (float)hi);
        }
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const bf16x8_t vf = as_bf16x8(vs_lane[x * 64]);
            oacc[x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, ph, oacc[x], 0, 0, 0);
            oacc[x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pl, oacc[x], 0, 0, 0);
        }
    }
    lsum += psum;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void tree_attn_kernel(
    const bf16_t* __restrict__ k_pool, const bf16_t* __restrict__ v_pool,
    const bf16_t* __restrict__ q, const Run* __restrict__ steps,
    const CascadeItem* __restrict__ items, const int32_t* __restrict__ ent_order,
    const int32_t* __restrict__ part_base, int n_kv_heads, int g_shift, float scale_log2e,
    float* __restrict__ ws_o, float2* __restrict__ ws_ml) {
    constexpr int D = 128;
    constexpr int KROW = kTreeAttnKRow;
    constexpr int KS_UNITS = 64 * KROW;    // K tile: 64 padded rows
    constexpr int VS_UNITS = 2 * 8 * 64;   // V^T fragments: [step][x][lane]
    // K tile, then V^T fragments; the K part is reused for the token-parallel fold
    __shared__ u32x4_t smem[KS_UNITS + VS_UNITS];
    __shared__ float sm_m[2][16];
    __shared__ float sm_l[2][16];
    __shared__ u32x4_t sm_desc[kTreeAttnMaxSteps];  // the item's step list
    u32x4_t* ks = smem;
    u32x4_t* vs = smem + KS_UNITS;

    // wave index, made known-uniform so that per-wave descriptors come through scalar loads
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sw = w >> 1;  // which step of a tile this wave fetches
    const int hw = w & 1;   // which 16-token half of that step
    const int lane = threadIdx.x & 63;
    const int a = lane & 15;  // 16-byte piece of a row when loading; MFMA row/column index
    const int b = lane >> 4;  // token sub-index when loading; MFMA contraction group kg
    const int h = blockIdx.x % n_kv_heads;
    const CascadeItem it = items[blockIdx.x / n_kv_heads];
    const int G = 1 << g_shift;
    const int n_q_heads = n_kv_heads << g_shift;
    const int R = it.n_ent << g_shift;
    const bool rowpar = R > 16;
    const int n_blocks = (R + 15) >> 4;
    // the row block this wave computes: block w when row parallel, block 0 otherwise
    const int blk = rowpar ? w : 0;
    const bool computes = rowpar ? (w < n_blocks) : (hw == 0);
    const int n_steps = it.run_end - it.run_begin;
    const int n_tiles = (n_steps + 1) >> 1;
    const Run* my_steps = steps + it.run_begin;
    const float raise_margin = 8.0f / scale_log2e;  // raw-score distance of 2^8 in weight

    // wave w fetches half hw of step 2 tile + sw of every tile
    u32x4_t kraw[4], vraw[4];
    const uint32_t stride_b = (uint32_t)n_kv_heads * D * 2;  // bytes between tokens
    // K: token 16 hw + 4 i + b;  V: contraction slot 4 hw + j of group b = token 16 hw + 4 b + j
    const uint32_t k_lane_off = (uint32_t)(16 * hw + b) * stride_b + a * 16;
    const uint32_t v_lane_off = (uint32_t)(16 * hw + 4 * b) * stride_b + a * 16;
    auto issue_loads = [&](const Run& sd) {
        if (sd.n > 0) {
            const int64_t base = (sd.tok * n_kv_heads + h) * (int64_t)D * 2;
            const char* kb = reinterpret_cast<const char*>(k_pool) + base;  // uniform
            const char* vb = reinterpret_cast<const char*>(v_pool) + base;
            if (sd.n == 32) {
                // full step: uniform base + per-lane offset that never changes
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    kraw[i] = load16(kb + (uint32_t)(4 * i) * stride_b + k_lane_off);
                    vraw[i] = load16(vb + (uint32_t)i * stride_b + v_lane_off);
                }
            } else {
                // ragged tail of a run: rows past the end re-read the last row (masked later)
                const int last = sd.n - 1;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t tk = (uint32_t)min(16 * hw + 4 * i + b, last);
                    const uint32_t tv = (uint32_t)min(16 * hw + 4 * b + i, last);
                    kraw[i] = load16(kb + tk * stride_b + a * 16);
                    vraw[i] = load16(vb + tv * stride_b + a * 16);
                }
            }
        }
    };

    // The first tile's loads start as soon as this wave's first step is known (read
    // straight from the step list); everything else the prologue needs overlaps them.
    Run sd_loaded = sw < n_steps ? my_steps[sw] : Run{0, 0, 0};  // descriptor of the loads in flight
    issue_loads(sd_loaded);

    // the item's step descriptors go to LDS once; nothing but K, V is fetched afterwards
    if ((int)threadIdx.x < n_steps)
        sm_desc[threadIdx.x] = load16(reinterpret_cast<const char*>(my_steps + threadIdx.x));

    // Q rows as B operands: lane (column a = query row, group b) holds
    // q[row][32 kk + 8 b .. + 8) for kk = 0..3.  The workspace row of the lane's
    // partial result is looked up here as well, off the critical path.
    bf16x8_t qf[4];
    int32_t out_row;
    const int r_lane = 16 * blk + a;
    {
        const int rr = r_lane < R ? r_lane : 0;  // padding rows read a valid row; never written
        const int ent = ent_order[it.ent_begin + (rr >> g_shift)];
        const int head = h * G + (rr & (G - 1));
        const bf16_t* qp = q + ((int64_t)ent * n_q_heads + head) * D;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[kk] = as_bf16x8(load16(qp + 32 * kk + 8 * b));
        out_row = (part_base[ent] + it.slot_off) * n_q_heads + head;
    }

    f32x4_t oacc[8];
    float m = -INFINITY, lsum = 0.f;
#pragma unroll
    for (int x = 0; x < 8; ++x) oacc[x] = f32x4_t{0.f, 0.f, 0.f, 0.f};

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
            for (int i = 0; i < 4; ++i) ks[(32 * sw + 16 * hw + 4 * i + b) * KROW + a] = kraw[i];
            // this half's four contraction slots of every V^T fragment: 8 of its 16 bytes
            u32x2_t* vs2 = reinterpret_cast<u32x2_t*>(vs);
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
                u32x2_t t;
                t[0] = __builtin_amdgcn_perm(vraw[1][x >> 1], vraw[0][x >> 1], sel);
                t[1] = __builtin_amdgcn_perm(vraw[3][x >> 1], vraw[2][x >> 1], sel);
                if (rowpar) {
                    // shared by several row blocks: convert once to fp16 for the P V product
                    t[0] = bf16x2_to_f16x2(t[0]);
                    t[1] = bf16x2_to_f16x2(t[1]);
                }
                vs2[((sw * 8 + x) * 64 + lane) * 2 + hw] = t;
            }
        }
    };

    stage(sd_loaded);
    // Everything issued so far (Q rows, first tile) has to have landed on every path
    // before the loop: a load still counted as outstanding here would make each
    // iteration wait for the next tile's loads as well.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();  // step list and first tile are in LDS

    for (int tile = 0; tile < n_tiles; ++tile) {
        sd_loaded = read_desc(2 * (tile + 1) + sw);  // a step past the end has n = 0
        issue_loads(sd_loaded);

        if (computes) {
            const int st_lo = rowpar ? 0 : sw;
            const int st_hi = rowpar ? 2 : sw + 1;
#pragma unroll 1
            for (int st = st_lo; st < st_hi; ++st) {
                const int sidx = 2 * tile + st;
                if (sidx >= n_steps) break;
                const int n_valid = __builtin_amdgcn_readfirstlane(sm_desc[sidx][2]);
                const u32x4_t* ks_lane = ks + (32 * st + a) * KROW + b;
                const u32x4_t* vs_lane = vs + st * 8 * 64 + lane;
                if (rowpar)
                    attn_step<true>(ks_lane, vs_lane, b, n_valid, qf, oacc, m, lsum, scale_log2e,
                                    raise_margin);
                else
                    attn_step<false>(ks_lane, vs_lane, b, n_valid, qf, oacc, m, lsum, scale_log2e,
                                     raise_margin);
            }
        }

        __syncthreads();  // the staged tile has been read by everyone who shares it
        stage(sd_loaded);
        __syncthreads();
    }

    float l = lsum;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    float scale_o = 1.f;
    if (!rowpar) {
        // token parallel: waves 0 and 2 hold the same rows over disjoint tokens; wave 2
        // hands its result to wave 0 through LDS (the tile buffer is free now)
        if (hw == 0 && b == 0) {
            sm_m[sw][a] = m;
            sm_l[sw][a] = l;
        }
        __syncthreads();
        const float ms = fmaxf(sm_m[0][a], sm_m[1][a]);
        const float f0 = fast_exp2((sm_m[0][a] - ms) * scale_log2e);
        const float f1 = fast_exp2((sm_m[1][a] - ms) * scale_log2e);
        f32x4_t* fold = reinterpret_cast<f32x4_t*>(smem) + lane;
        if (w == 2) {
#pragma unroll
            for (int x = 0; x < 8; ++x) fold[x * 64] = oacc[x] * f1;
        }
        __syncthreads();
        if (w != 0) return;
        l = sm_l[0][a] * f0 + sm_l[1][a] * f1;
        m = ms;
        scale_o = f0;
#pragma unroll
        for (int x = 0; x < 8; ++x) oacc[x] = oacc[x] * f0 + fold[x * 64];
    } else if (!computes) {
        return;
    }

    // partial result of row a of the wave's block: lane group b holds d = 32 b + 8 i + x
    if (r_lane < R) {
        float* dst = ws_o + (int64_t)out_row * D + 32 * b;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *reinterpret_cast<float4*>(dst + 8 * i) =
                make_float4(oacc[0][i], oacc[1][i], oacc[2][i], oacc[3][i]);
            *reinterpret_cast<float4*>(dst + 8 * i + 4) =
                make_float4(oacc[4][i], oacc[5][i], oacc[6][i], oacc[7][i]);
        }
        if (b == 0) ws_ml[out_row] = make_float2(m * scale_log2e, l);
    }
    (void)scale_o;
}

}  // namespace ets
