// Step-prefill attention on the matrix cores: one workgroup of four wavefronts = one
// block of query tokens of a leaf query's node, one kv head.
//
// Scoring a new step with the reward model is a prefill of that step's tokens over the
// tree of cached steps: query token i of the node sees every row of the node's strict
// ancestors and rows 0..i of the node itself.  A workgroup takes 128 query rows
// (128 / G consecutive tokens x the G query heads of the kv head), walks the ancestors'
// rows and then the node's own rows up to its last token, 64 rows (two runs of at most
// 32) at a time through LDS, and keeps the running softmax of its rows in registers:
// there are no partial results and no merge, the normalised output leaves at the end.
// With 128 rows against every K/V row read, the walk is bound by the matrix cores, not
// by HBM; blocks of the same node and of sibling nodes run next to each other and find
// their shared ancestors in L2.
//
// Wave w owns NB = 2 blocks of 16 rows.  Per run of 32 rows and block:
//   S^T = K Q^T     v_mfma_f32_16x16x32_bf16, K rows from the LDS tile (read once for
//                   both blocks), Q in registers;
//   mask            lane (a, b) holds query row a against rows 4 b + i and 16 + 4 b + i
//                   of the run: row t counts iff t < n and kpos + t <= i_row, kpos being
//                   the run's position inside the node (ancestors: always).  Runs that
//                   need no mask take a path without the compares; scores are consumed
//                   in the basic block of their matrix instructions on both paths;
//   softmax         against a per-row reference that is raised only when a score exceeds
//                   it by 2^8 in weight;
//   O^T += V^T P^T  v_mfma_f32_16x16x32_f16 with V converted to fp16 while it is staged
//                   and P rounded to fp16, as in the decode kernel's row-parallel path.
// K and V are fetched as there: each wave loads half a run (16 rows, 16 bytes per lane
// and load) with range-checked buffer loads, the next tile's loads in flight while the
// current tile is computed.  The run list can be long (a path of thousands of rows), so
// its descriptors travel through a ring of 256 entries in LDS that is refilled 128 at a
// time, 64 tiles ahead of their use.
#pragma once

#include "device_utils.hpp"
#include "prefill_plan.h"
#include "tree_attn_kernel.hpp"

namespace ets {

constexpr int kPrefillBlocksPerWave = 2;  // prefill_step is written for two

// Softmax pieces of one block of 16 query rows against one run of 32 rows.  Lane (a, b)
// holds query row a against rows 4 b + i (s0) and 16 + 4 b + i (s1) of the run.
// Masks the rows the query does not see (lim = rows of the run it sees, may be <= 0) and
// returns the lane's largest score.
__device__ __forceinline__ float prefill_mask_max(f32x4_t& s0, f32x4_t& s1, int b, int lim) {
    const int rem = lim - 4 * b;  // row 4 b + i counts iff i < rem, row 16 + 4 b + i iff 16 + i < rem
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s0[i] = i < rem ? s0[i] : -INFINITY;
        s1[i] = 16 + i < rem ? s1[i] : -INFINITY;
    }
    return fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                 fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
}

// Raises the block's reference score when a score exceeds it by more than the margin.
__device__ __forceinline__ void prefill_raise(float mx, float& m, float& lsum, f32x4_t (&oacc)[8],
                                              float scale_log2e, float raise_margin) {
    if (__any(mx > m + raise_margin)) {
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2((m - m_new) * scale_log2e);
        lsum *= alpha;
#pragma unroll
        for (int x = 0; x < 8; ++x) oacc[x] *= alpha;
        m = m_new;
    }
}

// Weights of the masked scores against the reference, rounded to fp16 for the P V product.
__device__ __forceinline__ f16x8_t prefill_weights(const f32x4_t& s0, const f32x4_t& s1, float m,
                                                   float& lsum, float scale_log2e) {
    const float mc = m * scale_log2e;
    f16x8_t pf;
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float p0 = fast_exp2(fmaf(s0[i], scale_log2e, -mc));
        const float p1 = fast_exp2(fmaf(s1[i], scale_log2e, -mc));
        psum += p0 + p1;
        pf[i] = (_Float16)p0;
        pf[4 + i] = (_Float16)p1;
    }
    lsum += psum;
    return pf;
}

// n groups of one matrix instruction followed by `valu` vector-ALU instructions: the
// order in which the surrounding basic block is to be issued, so that a block's softmax
// arithmetic runs while the matrix pipe works on the other block.
template <int N, int VALU>
__device__ __forceinline__ void interleave_mfma_valu() {
#pragma unroll
    for (int i = 0; i < N; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x002, VALU, 0);  // VALU
    }
}

// One run of 32 staged rows against the wave's two blocks of 16 query rows.  The two
// blocks are independent, so their phases are staggered: while the matrix pipe computes
// the scores of block 1 the vector ALU turns block 0's scores into weights, and while it
// applies block 0's weights to V the vector ALU does the same for block 1.  K and V
// fragments are read from LDS once per block (LDS bandwidth is not what limits here).
__device__ __forceinline__ void prefill_step(const u32x4_t* __restrict__ ks_lane,
                                             const u32x4_t* __restrict__ vs_lane, int b,
                                             const int (&lim)[2], const bf16x8_t (&qf)[2][4],
                                             f32x4_t (&oacc)[2][8], float (&m)[2], float (&lsum)[2],
                                             float scale_log2e, float raise_margin) {
    constexpr int KROW = kTreeAttnKRow;
    f32x4_t s0a = {0.f, 0.f, 0.f, 0.f}, s1a = s0a, s0b = s0a, s1b = s0a;
    // scores of block 0
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        s0a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ks_lane[4 * kk]), qf[0][kk], s0a, 0, 0, 0);
        s1a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ks_lane[16 * KROW + 4 * kk]), qf[0][kk],
                                                      s1a, 0, 0, 0);
    }
    const float mxa = prefill_mask_max(s0a, s1a, b, lim[0]);
    prefill_raise(mxa, m[0], lsum[0], oacc[0], scale_log2e, raise_margin);
    // scores of block 1 || weights of block 0
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        s0b = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ks_lane[4 * kk]), qf[1][kk], s0b, 0, 0, 0);
        s1b = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ks_lane[16 * KROW + 4 * kk]), qf[1][kk],
                                                      s1b, 0, 0, 0);
    }
    const f16x8_t pfa = prefill_weights(s0a, s1a, m[0], lsum[0], scale_log2e);
    interleave_mfma_valu<8, 4>();
    const float mxb = prefill_mask_max(s0b, s1b, b, lim[1]);
    prefill_raise(mxb, m[1], lsum[1], oacc[1], scale_log2e, raise_margin);
    // P V of block 0 || weights of block 1
#pragma unroll
    for (int x = 0; x < 8; ++x)
        oacc[0][x] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(vs_lane[x * 64]), pfa, oacc[0][x], 0, 0, 0);
    const f16x8_t pfb = prefill_weights(s0b, s1b, m[1], lsum[1], scale_log2e);
    interleave_mfma_valu<8, 4>();
    // P V of block 1
#pragma unroll
    for (int x = 0; x < 8; ++x)
        oacc[1][x] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(vs_lane[x * 64]), pfb, oacc[1][x], 0, 0, 0);
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void prefill_attn_kernel(
    const bf16_t* __restrict__ k_pool, const bf16_t* __restrict__ v_pool, int64_t pool_tokens,
    const bf16_t* __restrict__ q, const Run* __restrict__ runs,
    const PrefillItem* __restrict__ items, int item_base, int g_shift, float scale_log2e,
    float* __restrict__ out, float* __restrict__ lse) {
    constexpr int D = 128;
    constexpr int NB = kPrefillBlocksPerWave;
    constexpr int KROW = kTreeAttnKRow;
    constexpr int KS_UNITS = 64 * KROW;
    constexpr int VS_UNITS = 2 * 8 * 64;
    constexpr int RING = 256;
    __shared__ u32x4_t smem[KS_UNITS + VS_UNITS];
    __shared__ u32x4_t sm_desc[RING];
    u32x4_t* ks = smem;
    u32x4_t* vs = smem + KS_UNITS;

    const int n_kv_heads = (int)gridDim.x;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sw = w >> 1;  // which run of a tile this wave fetches
    const int hw = w & 1;   // which 16-row half of that run
    const int lane = threadIdx.x & 63;
    const int a = lane & 15;
    const int b = lane >> 4;
    const int h = blockIdx.x;
    const PrefillItem it = items[item_base + (int)blockIdx.y];
    const int G = 1 << g_shift;
    const int n_q_heads = n_kv_heads << g_shift;
    const int n_runs = it.run_end - it.run_begin;
    const int n_tiles = (n_runs + 1) >> 1;
    const Run* my_runs = runs + it.run_begin;
    const float raise_margin = 8.0f / scale_log2e;

    u32x4_t kraw[4], vraw[4];
    constexpr uint32_t stride_b = D * 2;
    const int64_t plane = (int64_t)h * pool_tokens;
    const uint32_t k_lane_off = (uint32_t)(16 * hw + b) * stride_b + a * 16;
    const uint32_t v_lane_off = (uint32_t)(16 * hw + 4 * b) * stride_b + a * 16;
    // a run's rows through a descriptor that covers exactly the run: rows past the end of
    // a short run read as zero (and are masked)
    auto issue_loads = [&](const Run& sd) {
        if (sd.n > 0) {
            const int64_t base = (plane + sd.tok) * (int64_t)D * 2;
            char* kb = const_cast<char*>(reinterpret_cast<const char*>(k_pool)) + base;
            char* vb = const_cast<char*>(reinterpret_cast<const char*>(v_pool)) + base;
            const int bytes = sd.n * (int)stride_b;
            const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc(kb, 0, bytes, 0x00020000);
            const __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc(vb, 0, bytes, 0x00020000);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                kraw[i] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                          kr, k_lane_off + (uint32_t)(4 * i) * stride_b, 0, 0));
                vraw[i] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                          vr, v_lane_off + (uint32_t)i * stride_b, 0, 0));
            }
        }
    };
    auto stage = [&](const Run& sd) {
        if (sd.n > 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) ks[(32 * sw + 16 * hw + 4 * i + b) * KROW + a] = kraw[i];
            u32x2_t* vs2 = reinterpret_cast<u32x2_t*>(vs);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u32x2_t te, to;
                te[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(
                                                         bf16_lo(vraw[0][j]), bf16_lo(vraw[1][j])));
                te[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(
                                                         bf16_lo(vraw[2][j]), bf16_lo(vraw[3][j])));
                to[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(
                                                         bf16_hi(vraw[0][j]), bf16_hi(vraw[1][j])));
                to[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(
                                                         bf16_hi(vraw[2][j]), bf16_hi(vraw[3][j])));
                vs2[((sw * 8 + 2 * j) * 64 + lane) * 2 + hw] = te;
                vs2[((sw * 8 + 2 * j + 1) * 64 + lane) * 2 + hw] = to;
            }
        }
    };
    // descriptor of run idx from the ring (same address in every lane)
    auto read_desc = [&](int idx) {
        Run sd{0, 0, 0};
        if (idx < n_runs) {
            const u32x4_t d = sm_desc[idx & (RING - 1)];
            const uint32_t lo = __builtin_amdgcn_readfirstlane(d[0]);
            const uint32_t hi = __builtin_amdgcn_readfirstlane(d[1]);
            sd.tok = (int64_t)(((uint64_t)hi << 32) | lo);
            sd.n = __builtin_amdgcn_readfirstlane(d[2]);
            sd.pad = __builtin_amdgcn_readfirstlane(d[3]);
        }
        return sd;
    };

    // prologue: first tile, the first 256 descriptors, the query rows
    Run sd_loaded = sw < n_runs ? my_runs[sw] : Run{0, 0, 0};
    issue_loads(sd_loaded);
    u32x4_t desc_raw = {0u, 0u, 0u, 0u};
    if ((int)threadIdx.x < n_runs)
        desc_raw = load16(reinterpret_cast<const char*>(my_runs + threadIdx.x));

    // block nb of wave w holds rows 16 (NB w + nb) .. + 15 of the item; row r is token
    // r >> g_shift of the block, query head r & (G - 1) of the kv head's group
    bf16x8_t qf[NB][4];
    int i_row[NB];  // the lane's query token, as an index into its node
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int r = 16 * (NB * w + nb) + a;
        const int tq = min(r >> g_shift, it.n_tok - 1);  // rows past the block repeat its last token
        i_row[nb] = it.tok0 + tq;
        const bf16_t* qp = q + ((it.q_row0 + tq) * n_q_heads + h * G + (r & (G - 1))) * D;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[nb][kk] = as_bf16x8(load16(qp + 32 * kk + 8 * b));
    }
    // smallest and largest query token of the wave's rows (uniform)
    const int i_lo = it.tok0 + min((16 * NB * w) >> g_shift, it.n_tok - 1);
    const int i_hi = it.tok0 + min((16 * NB * w + 16 * NB - 1) >> g_shift, it.n_tok - 1);

    sm_desc[threadIdx.x] = desc_raw;
    f32x4_t oacc[NB][8];
    float m[NB], lsum[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        m[nb] = -INFINITY;
        lsum[nb] = 0.f;
#pragma unroll
        for (int x = 0; x < 8; ++x) oacc[nb][x] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    stage(sd_loaded);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();  // descriptors and the first tile are in LDS

    for (int tile = 0; tile < n_tiles; ++tile) {
        sd_loaded = read_desc(2 * (tile + 1) + sw);
        issue_loads(sd_loaded);
        // ring refill: when run 128 k starts (k >= 1), runs [128 (k + 1), 128 (k + 2)) take
        // the slots of the 128 runs that were finished before it; they are used from 64
        // tiles later on
        const bool refill = tile > 0 && (tile & 63) == 0;
        const int refill_idx = 2 * tile + 128 + (int)threadIdx.x;
        if (refill && threadIdx.x < 128 && refill_idx < n_runs)
            desc_raw = load16(reinterpret_cast<const char*>(my_runs + refill_idx));

#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const int sidx = 2 * tile + st;
            if (sidx >= n_runs) break;
            const u32x4_t d = sm_desc[sidx & (RING - 1)];
            const int n_valid = __builtin_amdgcn_readfirstlane(d[2]);
            const int kpos = __builtin_amdgcn_readfirstlane(d[3]);
            const u32x4_t* ks_lane = ks + (32 * st + a) * KROW + b;
            const u32x4_t* vs_lane = vs + st * 8 * 64 + lane;
            // one code path for every run (the accumulators stay in place): the mask is
            // always applied, a run that needs none has lim = 32
            int lim[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) lim[nb] = min(n_valid, i_row[nb] - kpos + 1);
            prefill_step(ks_lane, vs_lane, b, lim, qf, oacc, m, lsum, scale_log2e, raise_margin);
        }

        __syncthreads();  // the staged tile has been read by every wave
        stage(sd_loaded);
        if (refill && threadIdx.x < 128 && refill_idx < n_runs)
            sm_desc[refill_idx & (RING - 1)] = desc_raw;
        __syncthreads();
    }

    // normalised rows out: lane (a, b) holds row a, d = 32 b + 8 i + x; through the wave's
    // own LDS region (the tile is no longer read) so that whole 512-byte rows are stored
    constexpr int OROW = 132;
    float* ob = reinterpret_cast<float*>(smem) + w * (16 * OROW);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        float l = lsum[nb];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const float inv = 1.0f / l;
        const int r0 = 16 * (NB * w + nb);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float* p = ob + a * OROW + 32 * b + 8 * i;
            *reinterpret_cast<float4*>(p) = make_float4(oacc[nb][0][i] * inv, oacc[nb][1][i] * inv,
                                                        oacc[nb][2][i] * inv, oacc[nb][3][i] * inv);
            *reinterpret_cast<float4*>(p + 4) = make_float4(oacc[nb][4][i] * inv, oacc[nb][5][i] * inv,
                                                            oacc[nb][6][i] * inv, oacc[nb][7][i] * inv);
        }
        {
            const int r = r0 + a;
            const int tq = r >> g_shift;
            if (b == 0 && tq < it.n_tok)
                lse[(it.q_row0 + tq) * n_q_heads + h * G + (r & (G - 1))] =
                    (m[nb] * scale_log2e + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int col = (lane & 31) * 4;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int r = r0 + 2 * k + (lane >> 5);
            const int tq = r >> g_shift;
            const float4 v = *reinterpret_cast<const float4*>(ob + (r - r0) * OROW + col);
            if (tq < it.n_tok)
                *reinterpret_cast<float4*>(
                    out + ((it.q_row0 + tq) * n_q_heads + h * G + (r & (G - 1))) * D + col) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace ets
