// Step-prefill attention on the matrix cores: one workgroup of eight wavefronts = one
// block of query tokens of a leaf query's node, one kv head.
//
// Scoring a new step with the reward model is a prefill of that step's tokens over the
// tree of cached steps: query token i of the node sees every row of the node's strict
// ancestors and rows 0..i of the node itself.  A workgroup takes 256 query rows
// (256 / G consecutive tokens x the G query heads of the kv head), walks the ancestors'
// rows and then the node's own rows up to its last token, 64 rows (two runs of at most
// 32) at a time through LDS, and keeps the running softmax of its rows in registers:
// there are no partial results and no merge, the normalised output leaves at the end.
// Every K/V row a workgroup reads (512 bytes per kv head) meets 256 query rows, 256 flop
// per byte: with 128 rows the walk was bound by the 5.8 TB/s at which L2 and the memory
// side cache feed the compute units, not by the matrix cores.  Blocks of the same node
// and of sibling nodes run next to each other and find their shared ancestors in L2.
//
// Wave w owns 32 query rows.  The 32x32x16 matrix instructions are used: on this chip
// they take as long as the 16x16x32 ones and do twice the work.  Lane l = (n, g), n =
// l % 32, g = l / 32.  Per run of 32 rows:
//   S^T = K Q^T     8 x v_mfma_f32_32x32x16_bf16: run rows on M, query rows on N.  A = K
//                   rows from the LDS tile (lane (n, g): row n, d = 16 kk + 8 g .. + 7),
//                   B = Q in registers.  Lane (n, g) receives query row n against run
//                   rows 8 c + 4 g + r (c, r = 0..3);
//   mask            run row t counts iff t < n_run and kpos + t <= i_row, kpos being the
//                   run's position inside the node (ancestors: always).  One code path:
//                   a run that needs no mask sees lim = 32;
//   softmax         against a per-row reference that is raised only when a score exceeds
//                   it by 2^8 in weight (then one cross-lane exchange);
//   O^T += V^T P^T  8 x v_mfma_f32_32x32x16_f16: d on M (4 blocks of 32), query rows on
//                   N, run rows on the contraction (2 halves of 16).  P rounded to fp16
//                   sits in the B layout as it is when contraction slot 8 g + 4 c' + r
//                   of half t stands for run row 16 t + 8 c' + 4 g + r; V, converted to
//                   fp16 while it is staged, is written to LDS as A fragments in that
//                   slot order.
// The work on a run is software pipelined inside the wave, because matrix and vector
// instructions only overlap when they alternate in program order:
//   [ scores(u + 1) || weights(u) ]  [ apply(u) || mask, maximum(u + 1) ]  raise(u + 1)
// (half t of the weights takes the scores of c = 2 t and 2 t + 1)
// and the pipeline runs on across tiles: the first run of the next tile is read from
// the next LDS buffer.  Three tile buffers rotate, so that the next tile can be staged
// while the previous one may still be read by a slower wave: one barrier per tile (new
// contents visible), and the staging sits in the same basic block as the matrix work.
// K and V are fetched with range-checked buffer loads, three tiles ahead of their use
// (two register sets alternate; one tile ahead left the waves waiting for memory):
// waves 0..3 each fetch and stage half a run (16 rows, 16 bytes per lane and load) of K,
// waves 4..7 of V.  The run list can be long (a
// path of thousands of rows), so its descriptors travel through a ring of 256 entries in
// LDS that is refilled 128 at a time, 64 tiles ahead of their use.
//
// The same kernel serves decode attention for tree segments that MANY leaf queries share
// (template parameter DECODE): there the 256 query rows of a work item are up to 256 / G
// leaf queries x the G query heads of the kv head, every row sees every row of the item's
// runs, and instead of a normalised output the workgroup leaves the unnormalised partial
// (o, m, l) of each query row in the decode workspace, where the log-sum-exp merge picks
// it up.  A root prompt shared by 512 leaves is 2048 query rows per kv head: that is this
// kernel's shape of problem (bound by the matrix cores), not the streaming kernel's.
#pragma once

#include "device_utils.hpp"
#include "prefill_plan.h"
#include "tree_attn_kernel.hpp"

namespace ets {

typedef float f32x16_t __attribute__((ext_vector_type(16)));

// Scores of the wave's 32 query rows against one staged run: S^T = K Q^T.
// ks_lane: the run's K rows in LDS at row n, 16-byte unit g.
__device__ __forceinline__ void prefill_scores(const u32x4_t* __restrict__ ks_lane,
                                               const bf16x8_t (&qf)[8], f32x16_t& s) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ks_lane[2 * kk]), qf[kk], s, 0, 0, 0);
}

// Masks the run rows the lane's query does not see (lim = rows of the run it sees, may
// be <= 0) and returns the lane's largest score.  Score i stands for run row
// 8 (i / 4) + 4 g + i % 4.
__device__ __forceinline__ float prefill_mask_max(f32x16_t& s, int g, int lim) {
    const int rem = lim - 4 * g;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = (8 * (i >> 2) + (i & 3)) < rem ? s[i] : -INFINITY;
    float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
#pragma unroll
    for (int c = 1; c < 4; ++c)
        mx = fmaxf(mx, fmaxf(fmaxf(s[4 * c], s[4 * c + 1]), fmaxf(s[4 * c + 2], s[4 * c + 3])));
    return mx;
}

// Raises the rows' reference score when a score exceeds it by more than the margin.
__device__ __forceinline__ void prefill_raise(float mx, float& m, float& lsum, f32x16_t (&oacc)[4],
                                              float scale_log2e, float raise_margin) {
    if (__any(mx > m + raise_margin)) {
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));  // the row's other half of the run
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2((m - m_new) * scale_log2e);
        lsum *= alpha;
#pragma unroll
        for (int x = 0; x < 4; ++x) oacc[x] *= alpha;
        m = m_new;
    }
}

// Where lane s of a V^T fragment of d block x sits inside the fragment's 64 slots of 16
// bytes.  The staging writes of one instruction go to 8 slots in each of the 4 d blocks;
// the swizzle spreads those 32 slots evenly over the LDS banks (two per bank group, the
// minimum) while 16 consecutive lanes of a fragment read still cover every bank once.
__device__ __forceinline__ int vfrag_slot(int s, int x) {
    const int k = ((s >> 4) & 1) | ((s >> 5) << 1) | (x << 2);
    return (s & 48) | ((s & 15) ^ k);
}

// One pipeline stage: the scores of run u + 1 and the weights of run u, then the
// application of run u's weights and the masking of run u + 1's scores, written in the
// order in which it is to be issued: every matrix instruction is followed by the LDS read
// of a fragment four instructions on and by two scores' worth of vector arithmetic, and a
// scheduling fence keeps the group together.  Matrix and vector instructions of one wave
// overlap only when they alternate like this.
//   ks_next  K rows of run u + 1 in LDS (at row n, 16-byte unit g)
//   vs_run   V^T fragments of run u
//   s_cur    masked scores of run u (in), s_next: masked scores of run u + 1 (out)
// Returns the lane's largest score of run u + 1.
__device__ __forceinline__ float prefill_unit(const u32x4_t* __restrict__ ks_next,
                                              const u32x4_t* __restrict__ vs_run,
                                              const int (&slot_x)[4], const bf16x8_t (&qf)[8],
                                              const f32x16_t& s_cur, f32x16_t& s_next, int g,
                                              int lim_next, float m, float& lsum, f32x16_t (&oacc)[4],
                                              float scale_log2e) {
    constexpr int AHEAD = 4;
    u32x4_t fr[AHEAD];
    f16x8_t pf[2];
    const float mc = m * scale_log2e;
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s_next[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < AHEAD; ++kk) fr[kk] = ks_next[2 * kk];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fr[kk % AHEAD]), qf[kk], s_next, 0, 0, 0);
        if (kk + AHEAD < 8) fr[kk % AHEAD] = ks_next[2 * (kk + AHEAD)];
        const float p0 = fast_exp2(fmaf(s_cur[2 * kk], scale_log2e, -mc));
        const float p1 = fast_exp2(fmaf(s_cur[2 * kk + 1], scale_log2e, -mc));
        psum += p0 + p1;
        pf[kk >> 2][2 * (kk & 3)] = (_Float16)p0;
        pf[kk >> 2][2 * (kk & 3) + 1] = (_Float16)p1;
        __builtin_amdgcn_sched_barrier(0);
    }
    lsum += psum;
    // apply(u): d block x, half t, both halves of a block back to back
#pragma unroll
    for (int j = 0; j < AHEAD; ++j) fr[j] = vs_run[((j & 1) * 4 + (j >> 1)) * 64 + slot_x[j >> 1]];
    __builtin_amdgcn_sched_barrier(0);
    const int rem = lim_next - 4 * g;
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int x = j >> 1, t = j & 1;
        oacc[x] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(fr[j % AHEAD]), pf[t], oacc[x], 0, 0, 0);
        if (j + AHEAD < 8) {
            const int jn = j + AHEAD;
            fr[j % AHEAD] = vs_run[((jn & 1) * 4 + (jn >> 1)) * 64 + slot_x[jn >> 1]];
        }
        // scores 2 j and 2 j + 1 of run u + 1 stand for run rows 8 (i / 4) + 4 g + i % 4
#pragma unroll
        for (int i = 2 * j; i < 2 * j + 2; ++i) {
            s_next[i] = (8 * (i >> 2) + (i & 3)) < rem ? s_next[i] : -INFINITY;
            mx = fmaxf(mx, s_next[i]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    return mx;
}

// FP8: the pools hold E4M3 codes (128-byte rows, 8 bytes per lane and load); the codes are
// widened while the tile is staged (K to bf16, V straight to the fp16 fragments), the kv
// head's K scale enters the score scale and its V scale multiplies the normalised rows.
// DECODE: `items_raw` are CascadeItem (leaf queries ent_order[ent_begin .. + n_ent), at most
// 256 / G of them), `out` is the partial workspace ws_o, `lse` is unused, and ent_order,
// ent_base, ws_ml are the decode plan's tables; otherwise `items_raw` are PrefillItem and
// the last three arguments are unused.
template <bool FP8, bool DECODE>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2))) void prefill_attn_kernel(
    const void* __restrict__ k_pool, const void* __restrict__ v_pool, int64_t pool_tokens,
    const bf16_t* __restrict__ q, const Run* __restrict__ runs,
    const void* __restrict__ items_raw, int item_base, int g_shift, float scale_log2e_base,
    HeadScales k_scales, HeadScales v_scales, float* __restrict__ out, float* __restrict__ lse,
    const int32_t* __restrict__ ent_order, const int32_t* __restrict__ ent_base,
    float2* __restrict__ ws_ml) {
    constexpr int D = 128;
    constexpr int KROW = kTreeAttnKRow;
    constexpr int KS_UNITS = 64 * KROW;    // K tile: 64 rows of 272 bytes
    constexpr int VS_UNITS = 2 * 8 * 64;   // V^T fragments: [run][half][d block][lane]
    constexpr int BUF_UNITS = KS_UNITS + VS_UNITS;
    constexpr int RING = 256;
    __shared__ u32x4_t smem[3 * BUF_UNITS];  // three tile buffers
    __shared__ u32x4_t sm_desc[RING];

    const int n_kv_heads = (int)gridDim.x;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool loads_v = w >= 4;   // waves 0..3 fetch K, waves 4..7 fetch V
    const int sw = (w & 3) >> 1;   // which run of a tile this wave fetches
    const int hw = w & 1;          // which 16-row half of that run
    const int lane = threadIdx.x & 63;
    const int a = lane & 15;  // when loading: 16-byte piece of a row
    const int b = lane >> 4;  // when loading: row group
    const int n = lane & 31;  // in the matrix layouts: query row / run row / d
    const int g = lane >> 5;
    const int h = blockIdx.x;
    const float scale_log2e = FP8 ? scale_log2e_base * k_scales.s[h] : scale_log2e_base;
    // the work item, in the terms both modes share: its runs, and the number of row
    // groups (query tokens, or leaf queries) whose G heads make up its query rows
    int run_begin, run_end, n_grp, tok0 = 0, ent_begin = 0, slot_off = 0;
    int64_t q_row0 = 0;
    if constexpr (DECODE) {
        const CascadeItem it = static_cast<const CascadeItem*>(items_raw)[item_base + (int)blockIdx.y];
        run_begin = it.run_begin;
        run_end = it.run_end;
        n_grp = it.n_ent;
        ent_begin = it.ent_begin;
        slot_off = it.slot_off;
    } else {
        const PrefillItem it = static_cast<const PrefillItem*>(items_raw)[item_base + (int)blockIdx.y];
        run_begin = it.run_begin;
        run_end = it.run_end;
        n_grp = it.n_tok;
        tok0 = it.tok0;
        q_row0 = it.q_row0;
    }
    const int G = 1 << g_shift;
    const int n_q_heads = n_kv_heads << g_shift;
    const int n_runs = run_end - run_begin;
    const int n_tiles = (n_runs + 1) >> 1;
    const Run* my_runs = runs + run_begin;
    const float raise_margin = 8.0f / scale_log2e;

    // the wave's 16 rows of K (rows b + 4 i) or of V (rows 4 b + i) of two tiles in flight:
    // loads are issued three tiles ahead of their use, and a register set is busy from
    // the issue until its tile is staged, so two sets alternate
    using raw_t = std::conditional_t<FP8, u32x2_t, u32x4_t>;
    raw_t raw0[4], raw1[4];
    constexpr uint32_t stride_b = FP8 ? D : D * 2;
    const int64_t plane = (int64_t)h * pool_tokens;
    const void* pool = loads_v ? v_pool : k_pool;
    const uint32_t lane_off =
        (uint32_t)(16 * hw + (loads_v ? 4 * b : b)) * stride_b + a * (FP8 ? 8 : 16);
    const uint32_t load_step = (loads_v ? 1u : 4u) * stride_b;
    // a run's rows through a descriptor that covers exactly the run: rows past the end of
    // a short run read as zero (and are masked); an empty run (past the end of an odd
    // list) is staged as zeros
    auto issue_loads = [&](const Run& sd, raw_t (&raw)[4]) {
        // always four loads (an empty run's descriptor covers nothing: every lane reads
        // zero without a memory access), so that the number of loads in flight is known
        // at every wait
        const int64_t base = (plane + sd.tok) * (int64_t)stride_b;
        char* pb = const_cast<char*>(reinterpret_cast<const char*>(pool)) + base;
        const int bytes = sd.n * (int)stride_b;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(pb, 0, bytes, 0x00020000);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (FP8)
                raw[i] = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_raw_buffer_load_b64(
                                                         rs, lane_off + (uint32_t)i * load_step, 0, 0));
            else
                raw[i] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                         rs, lane_off + (uint32_t)i * load_step, 0, 0));
        }
    };
    // K: row-major rows of 272 bytes.  V: lane (a, b) holds run rows 16 hw + 4 b + i
    // (i = 0..3) at d = 8 a + x (x = 0..7); the four rows at one d are half (b >> 1) of
    // the 16-byte A fragment of lane (d % 32, b & 1) in d block d / 32 of half hw.
    auto stage = [&](int buf, const raw_t (&raw)[4]) {
        u32x4_t* ks = smem + buf * BUF_UNITS;
        u32x2_t* vs2 = reinterpret_cast<u32x2_t*>(ks + KS_UNITS);
        if (!loads_v) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (FP8)
                    ks[(32 * sw + 16 * hw + 4 * i + b) * KROW + a] = e4m3x8_to_bf16x8(raw[i]);
                else
                    ks[(32 * sw + 16 * hw + 4 * i + b) * KROW + a] = raw[i];
            }
        } else {
            const int frag = (sw * 2 + hw) * 4 + (a >> 2);    // [run][half][d block]
            const int dst_lane = 32 * (b & 1) + 8 * (a & 3);  // + x
            // slot of lane dst_lane + x: x only enters the low three bits, which the
            // swizzle XORs with bits that do not depend on x
            u32x2_t* dst = vs2 + (frag * 64 * 2 + (b >> 1));
            const int slot0 = vfrag_slot(dst_lane, a >> 2);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u32x2_t te, to;
                if constexpr (FP8) {
                    // elements 2 j and 2 j + 1 of the four rows as floats (exact), then
                    // fp16 pairs across rows
                    typedef float f32x2_t __attribute__((ext_vector_type(2)));
                    f32x2_t f[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        f[i] = (j & 1) ? __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[i][j >> 1], true)
                                       : __builtin_amdgcn_cvt_pk_f32_fp8((int)raw[i][j >> 1], false);
                    te[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(f[0][0], f[1][0]));
                    te[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(f[2][0], f[3][0]));
                    to[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(f[0][1], f[1][1]));
                    to[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(f[2][1], f[3][1]));
                } else {
                    te[0] = __builtin_bit_cast(
                        uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16_lo(raw[0][j]), bf16_lo(raw[1][j])));
                    te[1] = __builtin_bit_cast(
                        uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16_lo(raw[2][j]), bf16_lo(raw[3][j])));
                    to[0] = __builtin_bit_cast(
                        uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16_hi(raw[0][j]), bf16_hi(raw[1][j])));
                    to[1] = __builtin_bit_cast(
                        uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16_hi(raw[2][j]), bf16_hi(raw[3][j])));
                }
                dst[(slot0 ^ (2 * j)) * 2] = te;      // x = 2 j
                dst[(slot0 ^ (2 * j + 1)) * 2] = to;  // x = 2 j + 1
            }
        }
    };
    // descriptor of run idx from the ring (same address in every lane); past the end: empty
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
    issue_loads(sw < n_runs ? my_runs[sw] : Run{0, 0, 0}, raw0);
    u32x4_t desc_raw = {0u, 0u, 0u, 0u};
    if ((int)threadIdx.x < min(n_runs, RING))
        desc_raw = load16(reinterpret_cast<const char*>(my_runs + threadIdx.x));

    // row r = 32 w + n of the item is token r >> g_shift of the block, query head
    // r & (G - 1) of the kv head's group; rows past the block repeat its last token
    // (decode: row r is leaf query r >> g_shift of the item, in ent_order)
    const int r_lane = 32 * w + n;
    const int tq_lane = min(r_lane >> g_shift, n_grp - 1);
    const int i_row = tok0 + tq_lane;  // the lane's query token, as an index into its node
    // a wave whose 32 rows all lie past the block's last token (the last block of a node
    // is rarely full) only fetches and stages: its SIMD is left to the other wave
    const bool active = ((32 * w) >> g_shift) < n_grp;
    bf16x8_t qf[8];
    int64_t out_row;  // row of the lane's query in `out` (and in lse / ws_ml)
    {
        const int head = h * G + (r_lane & (G - 1));
        int64_t q_row;
        if constexpr (DECODE) {
            q_row = ent_order[ent_begin + tq_lane];
            out_row = (int64_t)(ent_base[ent_begin + tq_lane] + slot_off) * n_q_heads + head;
        } else {
            q_row = q_row0 + tq_lane;
            out_row = q_row * n_q_heads + head;
        }
        const bf16_t* qp = q + (q_row * n_q_heads + head) * D;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = as_bf16x8(load16(qp + 16 * kk + 8 * g));
    }

    if (threadIdx.x < RING) sm_desc[threadIdx.x] = desc_raw;
    f32x16_t oacc[4];  // d block x: lane (n, g) holds d = 32 x + 8 c + 4 g + r at index 4 c + r
    float m = -INFINITY, lsum = 0.f;
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[x][i] = 0.f;
    stage(0, raw0);
    // the loads of the second and third tile are in flight while the first is computed
    // (their descriptors straight from memory: the ring is not visible before the barrier)
    issue_loads(2 + sw < n_runs ? my_runs[2 + sw] : Run{0, 0, 0}, raw0);
    issue_loads(4 + sw < n_runs ? my_runs[4 + sw] : Run{0, 0, 0}, raw1);
    __syncthreads();  // descriptors and the first tile are in LDS

    auto lim_of = [&](const u32x4_t& d) {
        // rows of the run that the lane's query row sees
        const int n_valid = __builtin_amdgcn_readfirstlane(d[2]);
        if constexpr (DECODE) return n_valid;  // the query is newer than every row
        const int kpos = __builtin_amdgcn_readfirstlane(d[3]);
        return min(n_valid, i_row - kpos + 1);
    };
    const u32x4_t empty_desc = {0u, 0u, 0u, 0u};  // n = 0: everything masked
    auto desc_of = [&](int idx) { return idx < n_runs ? sm_desc[idx & (RING - 1)] : empty_desc; };

    int slot_x[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) slot_x[x] = vfrag_slot(lane, x);
    f32x16_t s_a, s_b;  // scores of the runs in flight (even and odd run of a tile)
    if (active) {
        // first run: scores, mask and maximum
        prefill_scores(smem + n * KROW + g, qf, s_a);
        const float mx = prefill_mask_max(s_a, g, lim_of(desc_of(0)));
        prefill_raise(mx, m, lsum, oacc, scale_log2e, raise_margin);
    }

    int cur = 0, nxt = 1;  // tile % 3, (tile + 1) % 3
    // one tile; `raw` holds the rows of tile + 1 and takes those of tile + 3
    auto do_tile = [&](int tile, raw_t (&raw)[4]) {
        const u32x4_t* ks = smem + cur * BUF_UNITS;
        const u32x4_t* vs = ks + KS_UNITS;
        const u32x4_t* ks_next = smem + nxt * BUF_UNITS;
        const u32x4_t d1 = desc_of(2 * tile + 1), d2 = desc_of(2 * tile + 2);
        // ring refill: when run 128 k starts (k >= 1), runs [128 (k + 1), 128 (k + 2)) take
        // the slots of the 128 runs that were finished before it; they are used from 64
        // tiles later on
        const bool refill = tile > 0 && (tile & 63) == 0;
        const int refill_idx = 2 * tile + 128 + (int)threadIdx.x;
        if (refill && threadIdx.x < 128 && refill_idx < n_runs)
            desc_raw = load16(reinterpret_cast<const char*>(my_runs + refill_idx));

        // the buffer of tile - 2 is free: every wave has passed the barrier of tile - 1.
        // Past the end of the list zeros are staged (never read).
        stage(nxt, raw);  // waits for the loads of tile + 1
        issue_loads(read_desc(2 * (tile + 3) + sw), raw);
        if (refill && threadIdx.x < 128 && refill_idx < n_runs)
            sm_desc[refill_idx & (RING - 1)] = desc_raw;

        // [ scores(run 1) || weights(run 0) ]  [ apply(run 0) || mask, maximum(run 1) ]
        if (active) {
            const float mx1 = prefill_unit(ks + (32 + n) * KROW + g, vs, slot_x, qf, s_a, s_b, g,
                                           lim_of(d1), m, lsum, oacc, scale_log2e);
            prefill_raise(mx1, m, lsum, oacc, scale_log2e, raise_margin);
        }

        __syncthreads();  // the next tile is staged
        // [ scores(next tile, run 0) || weights(run 1) ]  [ apply(run 1) || mask, maximum ]
        // (past the last tile the scores are masked away as a whole)
        if (active) {
            const float mx0 = prefill_unit(ks_next + n * KROW + g, vs + 8 * 64, slot_x, qf, s_b, s_a, g,
                                           lim_of(d2), m, lsum, oacc, scale_log2e);
            prefill_raise(mx0, m, lsum, oacc, scale_log2e, raise_margin);
        }
        cur = nxt;
        nxt = nxt == 2 ? 0 : nxt + 1;
    };
    // (no branch inside the loop body: the waits for a register set then leave the other
    // set's loads in flight)
    for (int tile = 0; tile + 1 < n_tiles; tile += 2) {
        do_tile(tile, raw0);
        do_tile(tile + 1, raw1);
    }
    if (n_tiles & 1) do_tile(n_tiles - 1, raw0);
    __syncthreads();  // every wave is done with the tiles: the epilogue reuses the buffers

    // rows out through the wave's own LDS region (16 rows padded to 132 floats, two
    // passes), so that whole 512-byte rows are stored: normalised in step prefill,
    // unnormalised next to (m, l) in decode
    constexpr int OROW = 132;
    float* ob = reinterpret_cast<float*>(smem) + w * (16 * OROW);
    float l = lsum;
    l += __shfl_xor(l, 32, 64);
    float inv = 1.0f;
    if constexpr (!DECODE) {
        inv = 1.0f / l;
        if constexpr (FP8) inv *= v_scales.s[h];
    }
    if (g == 0 && (r_lane >> g_shift) < n_grp) {
        if constexpr (DECODE)
            ws_ml[out_row] = make_float2(m * scale_log2e, l);
        else
            lse[out_row] = (m * scale_log2e + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    }
    const int col = (lane & 31) * 4;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if ((n >> 4) == pass) {
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    *reinterpret_cast<float4*>(ob + (n & 15) * OROW + 32 * x + 8 * c + 4 * g) =
                        make_float4(oacc[x][4 * c] * inv, oacc[x][4 * c + 1] * inv,
                                    oacc[x][4 * c + 2] * inv, oacc[x][4 * c + 3] * inv);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int rr = 2 * k + (lane >> 5);  // row of this pass that the lane stores
            const int r = 32 * w + 16 * pass + rr;
            // lane 16 pass + rr (g = 0) holds the output row of query row r
            const int64_t row_out = __shfl(out_row, 16 * pass + rr, 64);
            const float4 v = *reinterpret_cast<const float4*>(ob + rr * OROW + col);
            if ((r >> g_shift) < n_grp) *reinterpret_cast<float4*>(out + row_out * D + col) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace ets
