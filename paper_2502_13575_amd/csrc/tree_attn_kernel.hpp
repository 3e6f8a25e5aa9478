// Tree attention on the matrix cores: one workgroup of four wavefronts = one
// (work item, kv head).
//
// A work item names a list of steps (pieces of at most 32 consecutive pool
// rows: a chunk of a tree segment, or a leaf's private suffix) and the leaf
// queries that attend to them.  The workgroup reads the item's K and V from
// HBM exactly once, 64 tokens (two steps) at a time, stages them in LDS and
// applies them to all R = n_ent * G <= 64 query rows (the G query heads of a
// leaf share the kv head).  Each wave fetches half a step (16 tokens) and owns
// at most one block of 16 query rows, which keeps the kernel under 170
// registers per lane and at 38 KB of LDS: three workgroups (12 waves) per
// compute unit, so that one workgroup's memory latency overlaps the others'
// arithmetic.
//   R  > 16  "row parallel":   the tile is staged in LDS once and reused by the
//            waves; wave w owns row block w and walks both steps of every tile.
//   R <= 16  "token parallel": nothing is shared, so every wave walks the
//            16-token units it fetched itself through a private LDS region,
//            with no workgroup barrier in the loop; the four running results
//            are folded through LDS at the end, so the item still yields one
//            partial per query row.
//   small items (R <= 16, few tokens): four items per workgroup, each walked by
//            one wave alone, without fold or barrier.
//
// bf16 pools laid out [kv head][pool row][128]: the rows of a step are contiguous
// within a head, 256 bytes each.  Per step of 32 tokens and block of 16 query rows:
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
// Pools of E4M3 codes (template parameter FP8; one scale per pool, applied by the
// caller to the score scale and to the merged output): rows are 128 bytes, a lane
// fetches the same 8 elements with an 8-byte load, and the codes are widened to bf16
// (exactly: 4 significant bits) when the tile is staged; everything after the staging
// is the bf16 path unchanged.
// head_dim 64 (template parameter D; either pool format): rows of 8 pieces of 8 elements, two
// score products and four output fragments per 16 tokens; for the V transposition two
// neighbouring lanes fetch the same piece and take one half of it each.
// Loads of the next tile are in flight while the current one is computed.
// The result per query row is the unnormalised partial (o, m, l), m in log2
// units, merged later along each leaf's chain.
#pragma once

#include <type_traits>

#include "device_utils.hpp"
#include "merge_kernel.hpp"
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
// Eight E4M3 codes (two dwords) -> eight bf16 values, element order kept.  Every E4M3
// value is a bf16 value, so the float -> bf16 conversion (one packed instruction per
// pair) does not round.
__device__ __forceinline__ u32x4_t e4m3x8_to_bf16x8(u32x2_t r) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    u32x4_t o;
#pragma unroll
    for (int dw = 0; dw < 2; ++dw) {
        const f32x2_t lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)r[dw], false);  // bytes 0, 1
        const f32x2_t hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)r[dw], true);   // bytes 2, 3
        o[2 * dw] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2_t));
        o[2 * dw + 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2_t));
    }
    return o;
}
__device__ __forceinline__ u32x4_t widen_raw(u32x4_t r) { return r; }
__device__ __forceinline__ u32x4_t widen_raw(u32x2_t r) { return e4m3x8_to_bf16x8(r); }
template <bool FP8>
__device__ __forceinline__ std::conditional_t<FP8, u32x2_t, u32x4_t> load_row_piece(
    __amdgpu_buffer_rsrc_t rsrc, uint32_t voff, int soff, std::integral_constant<int, 0>) {
    if constexpr (FP8)
        return __builtin_bit_cast(u32x2_t, __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff, soff, 0));
    else
        return __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, 0));
}
template <bool FP8>
__device__ __forceinline__ std::conditional_t<FP8, u32x2_t, u32x4_t> load_row_piece(
    __amdgpu_buffer_rsrc_t rsrc, uint32_t voff, int soff, std::integral_constant<int, 2>) {
    if constexpr (FP8)
        return __builtin_bit_cast(u32x2_t, __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff, soff, 2));
    else
        return __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, 2));
}

static_assert(kTreeAttnRowsPerItem == 64, "4 waves x 16 rows");
constexpr int kTreeAttnKRow = 17;         // 16-byte units per padded K row in LDS (272 bytes)

// Geometry by head_dim D (128 or 64): a K row in LDS is D / 8 16-byte units plus one of
// padding; the score product contracts over D in D / 32 matrix instructions; the output
// has D / 16 blocks of 16 rows of V^T (fragments).
template <int D>
constexpr int k_row_units() {
    return D / 8 + 1;
}
static_assert(k_row_units<128>() == kTreeAttnKRow, "the step-prefill kernel stages K the same way");

// One step of a row-parallel item: 32 staged tokens (V already fp16) against one block
// of 16 query rows.
template <int D>
__device__ __forceinline__ void attn_step(const u32x4_t* __restrict__ ks_lane,
                                          const u32x4_t* __restrict__ vs_lane, int b, int n_valid,
                                          const bf16x8_t (&qf)[D / 32], f32x4_t (&oacc)[D / 16],
                                          float& m, float& lsum, float scale_log2e,
                                          float raise_margin) {
    constexpr int KROW = k_row_units<D>();
    constexpr int NKK = D / 32, NX = D / 16, HX = NX / 2;
    // scores S^T = K Q^T
    f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    // one accumulator after the other: consecutive matrix instructions that accumulate
    // into the same registers issue twice as fast as alternating ones
    for (int kk = 0; kk < NKK; ++kk)
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ks_lane[4 * kk]), qf[kk], s0, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ks_lane[16 * KROW + 4 * kk]), qf[kk],
                                                     s1, 0, 0, 0);
    // The first half of the V^T fragments is requested from LDS before the softmax
    // arithmetic, so that they arrive while it runs; the other half follows behind the first
    // matrix instructions.  (Left to itself the compiler reads each fragment just ahead of
    // its use.)
    u32x4_t vf[HX];
#pragma unroll
    for (int x = 0; x < HX; ++x) vf[x] = vs_lane[x * 64];
    __builtin_amdgcn_sched_barrier(0);
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
        for (int x = 0; x < NX; ++x) oacc[x] *= alpha;
        m = m_new;
    }
    const float mc = m * scale_log2e;
    float psum = 0.f;
    f16x8_t pf;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float p = fast_exp2(fmaf(s[j], scale_log2e, -mc));
        psum += p;
        pf[j] = (_Float16)p;
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int x = 0; x < HX; ++x) {
        oacc[x] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(vf[x]), pf, oacc[x], 0, 0, 0);
        vf[x] = vs_lane[(HX + x) * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int x = 0; x < HX; ++x)
        oacc[HX + x] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(vf[x]), pf, oacc[HX + x], 0, 0, 0);
    lsum += psum;
}

// Token-parallel unit: the 16 tokens one wave fetched itself, against the single
// block of query rows.  K rows and transposed V pieces sit in the wave's own LDS
// region.  The weight enters the P V product as a bf16 head in contraction slots
// 0..3 and its bf16 remainder in slots 4..7, against the same four V rows in both
// slot halves, so one MFMA per fragment applies both.
template <int D>
__device__ __forceinline__ void attn_half_step(const u32x4_t* __restrict__ ks_lane,
                                               const u32x2_t* __restrict__ vs_lane, int b,
                                               int n_valid, const bf16x8_t (&qf)[D / 32],
                                               f32x4_t (&oacc)[D / 16], float& m, float& lsum,
                                               float scale_log2e, float raise_margin) {
    constexpr int NKK = D / 32, NX = D / 16;
    f32x4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ks_lane[4 * kk]), qf[kk], s, 0, 0, 0);
    // lane holds row a, tokens 4 b + i; masking is unconditional so that the scores are
    // consumed in straight-line code after the matrix instructions
    const int rem = n_valid - 4 * b;
#pragma unroll
    for (int i = 0; i < 4; ++i) s[i] = i < rem ? s[i] : -INFINITY;
    float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    if (__any(mx > m + raise_margin)) {
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2((m - m_new) * scale_log2e);
        lsum *= alpha;
#pragma unroll
        for (int x = 0; x < NX; ++x) oacc[x] *= alpha;
        m = m_new;
    }
    const float mc = m * scale_log2e;
    float psum = 0.f;
    bf16x8_t pf;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float p = fast_exp2(fmaf(s[i], scale_log2e, -mc));
        psum += p;
        const __bf16 hi = (__bf16)p;
        pf[i] = hi;
        pf[4 + i] = (__bf16)(p - (float)hi);
    }
#pragma unroll
    for (int x = 0; x < NX; ++x) {
        const u32x2_t t = vs_lane[x * 64];
        const u32x4_t vf = {t[0], t[1], t[0], t[1]};
        oacc[x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vf), pf, oacc[x], 0, 0, 0);
    }
    lsum += psum;
}

// What the merge inside the attention launch needs (instantiations with FUSED only).
struct MergeTail {
    const int32_t* part_base;  // [leaf queries + 1] first partial slot of every leaf query
    int32_t* arrived;          // [leaf queries][kv heads] partial slots stored so far; all
                               // zero whenever no call is in flight
    int64_t n_ws_rows;         // partial rows in the workspace; their bytes stay below 2^32
    void* out;                 // merged output, fp32 or bf16
    float* lse;
    int out_bf16;
    HeadScales v_scales;       // factor of the merged output per kv head
};

template <bool FP8, bool FUSED, int D = 128>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void tree_attn_kernel(
    const void* __restrict__ k_pool, const void* __restrict__ v_pool, int64_t pool_tokens,
    const bf16_t* __restrict__ q, const Run* __restrict__ steps,
    const UnitSlot* __restrict__ units, int unit_base,
    const int32_t* __restrict__ ent_order, const int32_t* __restrict__ ent_base, int g_shift,
    float scale_log2e_base, HeadScales k_scales,
    float* __restrict__ ws_o, float2* __restrict__ ws_ml, MergeTail tail) {
    static_assert(D == 128 || D == 64, "head_dim");
    const int n_kv_heads = (int)gridDim.x;
    constexpr int KROW = k_row_units<D>();
    constexpr int NKK = D / 32;            // matrix instructions of a score product
    constexpr int NX = D / 16;             // V^T fragments (blocks of 16 output elements)
    constexpr int PPR = D / 8;             // 16-byte pieces (8 elements) per row
    constexpr int RPL = 64 / PPR;          // K rows one load instruction of a wave covers
    constexpr int NKL = 16 / RPL;          // K loads per 16 tokens
    constexpr int KS_UNITS = 64 * KROW;    // K tile: 64 padded rows
    constexpr int VS_UNITS = 2 * NX * 64;  // V^T fragments: [step][x][lane]
    // K tile, then V^T fragments; the K part is reused for the token-parallel fold
    __shared__ u32x4_t smem[KS_UNITS + VS_UNITS];
    __shared__ float sm_m[4][16];
    __shared__ float sm_l[4][16];
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
    const int h = blockIdx.x;  // kv head; consecutive workgroups share an item
    // E4M3 pools: the K scale of this kv head is part of the score scale
    const float scale_log2e = FP8 ? scale_log2e_base * k_scales.s[h] : scale_log2e_base;
    // A workgroup takes one item, or four small items, one per wave, which then works alone
    // (no barrier below this point on that path); the planner's launch order says which.
    // One table read (uniform per wave: scalar loads) brings the item and the step this wave
    // fetches first, in launch order.
    const UnitSlot* my_unit = units + 4 * (unit_base + (int)blockIdx.y) + w;
    const CascadeItem it = my_unit->item;
    const Run first_step = my_unit->first;
    const bool wave_item = it.wave_item != 0;
    if (it.n_ent == 0) return;
    const int G = 1 << g_shift;
    const int n_q_heads = n_kv_heads << g_shift;
    const int R = it.n_ent << g_shift;
    const bool rowpar = R > 16;
    const int n_blocks = (R + 15) >> 4;
    // the row block this wave computes: block w when row parallel, block 0 otherwise.  A
    // row-parallel wave past the item's last block computes nothing; it looks up (and
    // fetches the query rows of) block 0 instead of entries that are not the item's.
    const bool computes = w < n_blocks;  // row parallel only; token parallel: every wave
    const int blk = rowpar && computes ? w : 0;
    // a token-parallel wave needs its half of a step only if the step reaches it
    const int load_min = rowpar ? 0 : 16 * hw;
    const int n_steps = it.run_end - it.run_begin;
    const int n_tiles = (n_steps + 1) >> 1;
    const Run* my_steps = steps + it.run_begin;
    const float raise_margin = 8.0f / scale_log2e;  // raw-score distance of 2^8 in weight

    // wave w fetches half hw of step 2 tile + sw of every tile
    std::conditional_t<FP8, u32x2_t, u32x4_t> kraw[NKL], vraw[4];
    constexpr uint32_t stride_b = FP8 ? D : D * 2;  // bytes between the tokens of a head plane
    constexpr uint32_t piece_b = FP8 ? 8 : 16;      // bytes of a lane's 8 elements
    const int64_t plane = (int64_t)h * pool_tokens;  // first row of this kv head
    // K: a load covers RPL consecutive rows, the lane's piece pa of row rb: token
    // 16 hw + RPL i + rb (head_dim 128: pa = a, rb = b).
    // V: contraction slot 4 hw + j of group b = token 16 hw + 4 b + j.  With head_dim 128
    // the lane's piece is a, of which it transposes all 8 elements; with head_dim 64 a row
    // has 8 pieces, lanes 2 p and 2 p + 1 both fetch piece p and transpose one half each
    // (output element 4 a + x of fragment x).
    const int pa = lane & (PPR - 1), rb = lane / PPR;
    const int va = D == 128 ? a : a >> 1;
    const uint32_t k_lane_off = (uint32_t)(16 * hw + rb) * stride_b + pa * piece_b;
    const uint32_t v_lane_off = (uint32_t)(16 * hw + 4 * b) * stride_b + va * piece_b;
    // Buffer loads: a step's rows are addressed through a descriptor that covers exactly
    // the step (base = its first row at this kv head, size = n rows), so a load is a
    // scalar descriptor plus a 32-bit lane offset, and rows past the end of a ragged step
    // read as zero instead of needing clamped addresses (they are masked later).
    auto issue_loads = [&](const Run& sd, auto aux_tag) {
        // cache policy of the loads: 2 = non-temporal, for rows that no other item reads
        if (sd.n > load_min) {
            const int64_t base = (plane + sd.tok) * (int64_t)stride_b;
            char* kb = const_cast<char*>(reinterpret_cast<const char*>(k_pool)) + base;  // uniform
            char* vb = const_cast<char*>(reinterpret_cast<const char*>(v_pool)) + base;
            const int bytes = sd.n * (int)stride_b;
            const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc(kb, 0, bytes, 0x00020000);
            const __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc(vb, 0, bytes, 0x00020000);
            if (sd.n == 32) {
                // full step: every row is in range; the row stepping rides in the scalar offset
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (i < NKL)
                        kraw[i] = load_row_piece<FP8>(kr, k_lane_off, RPL * i * (int)stride_b, aux_tag);
                    vraw[i] = load_row_piece<FP8>(vr, v_lane_off, i * (int)stride_b, aux_tag);
                }
            } else {
                // ragged step: the whole offset is in the range-checked lane offset
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (i < NKL)
                        kraw[i] = load_row_piece<FP8>(kr, k_lane_off + (uint32_t)(RPL * i) * stride_b,
                                                      0, aux_tag);
                    vraw[i] = load_row_piece<FP8>(vr, v_lane_off + (uint32_t)i * stride_b, 0,
                                                  aux_tag);
                }
            }
        }
    };

    // Prologue loads, in the order their results are needed (vector loads return in
    // order): the lane's query index, the first tile, the step list, then the query
    // row, which depends on the first.
    // The leaf queries of the wave's 16 rows and their partial slots come through scalar
    // loads (uniform addresses; a 16-entry load may run up to 15 entries past the item's
    // own, which is what the tables' zero padding is for: those name leaf query 0 or a
    // neighbouring item's leaf queries, whose rows are read and never written): scalar
    // loads do not queue behind the CU's K/V loads, and the query rows can be requested
    // one memory round trip earlier.
    const int r_lane = 16 * blk + a;
    const int e_lane = a >> g_shift;  // entry of the lane's row within the wave's block
    const int32_t* s_ent = ent_order + it.ent_begin + ((16 * blk) >> g_shift);
    const int32_t* s_base = ent_base + it.ent_begin + ((16 * blk) >> g_shift);
    int32_t t_ent[16], t_base[16];  // loaded unconditionally: two wide scalar loads
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        t_ent[k] = s_ent[k];
        t_base[k] = s_base[k];
    }
    int ent = t_ent[0], ent_slot = t_base[0];
#pragma unroll
    for (int k = 1; k < 16; ++k) {
        if (k < (16 >> g_shift)) {
            ent = e_lane == k ? t_ent[k] : ent;
            ent_slot = e_lane == k ? t_base[k] : ent_slot;
        }
    }
    const int rr = r_lane;  // rows past R belong to padding entries: read, never written

    // Partial result of the wave's block.  Lane (a, b) holds row a, d = 32 b + 8 i + x
    // (head_dim 64: d = 16 b + 4 i + x): written from there, every store instruction would
    // touch 64 different cache lines with 16 bytes each.  The block goes through a
    // wave-private LDS region (rows padded by 4 floats) instead, and each store
    // instruction writes whole rows (two of 512 bytes, or four of 256).
    // the workspace as buffer resources, for the device-scope stores of the merging variant
    const __amdgpu_buffer_rsrc_t rs_ws_o = __builtin_amdgcn_make_buffer_rsrc(
        ws_o, 0, FUSED ? (int)(uint32_t)(tail.n_ws_rows * D * 4) : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_ws_ml = __builtin_amdgcn_make_buffer_rsrc(
        ws_ml, 0, FUSED ? (int)(uint32_t)(tail.n_ws_rows * 8) : 0, 0x00020000);
    auto store_partial = [&](const f32x4_t (&oacc)[NX], float m, float l, int32_t out_row) {
        constexpr int OROW = D + 4;
        float* ob = reinterpret_cast<float*>(smem) + w * (16 * OROW);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float* p = ob + a * OROW + (D / 4) * b + (D / 16) * i;
            *reinterpret_cast<float4*>(p) =
                make_float4(oacc[0][i], oacc[1][i], oacc[2][i], oacc[3][i]);
            if constexpr (D == 128)
                *reinterpret_cast<float4*>(p + 4) =
                    make_float4(oacc[4][i], oacc[5][i], oacc[6][i], oacc[7][i]);
        }
        if (b == 0 && r_lane < R) {
            if constexpr (FUSED)
                __builtin_amdgcn_raw_buffer_store_b64(
                    __builtin_bit_cast(u32x2_t, make_float2(m * scale_log2e, l)), rs_ws_ml,
                    (uint32_t)out_row * 8u, 0, kDeviceScope);
            else
                ws_ml[out_row] = make_float2(m * scale_log2e, l);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        constexpr int LPR = D / 4;       // lanes that store a row, 16 bytes each
        constexpr int RPS = 64 / LPR;    // rows per store instruction
        const int col = (lane & (LPR - 1)) * 4;
#pragma unroll
        for (int k = 0; k < 16 / RPS; ++k) {
            const int r = RPS * k + lane / LPR;              // row of the block this lane stores
            const int32_t row_out = __shfl(out_row, r, 64);  // lane r holds row r (a = r, b = 0)
            const float4 v = *reinterpret_cast<const float4*>(ob + r * OROW + col);
            if (16 * blk + r < R) {
                if constexpr (FUSED)
                    __builtin_amdgcn_raw_buffer_store_b128(
                        __builtin_bit_cast(u32x4_t, v), rs_ws_o,
                        ((uint32_t)row_out * D + (uint32_t)col) * 4u, 0, kDeviceScope);
                else
                    *reinterpret_cast<float4*>(ws_o + (int64_t)row_out * D + col) = v;
            }
        }
        if constexpr (FUSED) {
            // Merge in the same launch: every entry (leaf query) whose rows this wave
            // has just stored counts one arrival for (leaf query, kv head); the wave that
            // brings the count to the leaf's number of partial slots merges them.  The
            // partial rows are stored at device scope and have completed (the wait below)
            // before the wave counts itself in, and the merging wave reads them at device
            // scope after its own count has returned, so it sees every slot without any
            // cache being written back or invalidated as a whole.  It then puts the
            // counter back to zero for the next call.  Which wave merges depends on
            // timing; what it computes does not.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
            const bool arriver = b == 0 && (a & (G - 1)) == 0 && r_lane < R;
            int leaf = 0, p0 = 0, np = 0, seen = -2;
            if (arriver) {
                leaf = s_ent[e_lane];  // the lane's entry again (not kept over the loop)
                p0 = tail.part_base[leaf];
                np = tail.part_base[leaf + 1] - p0;
                seen = __hip_atomic_fetch_add(tail.arrived + (int64_t)leaf * n_kv_heads + h, 1,
                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            uint64_t todo = __ballot(arriver && seen + 1 == np);
            if (todo != 0) {
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                const float out_scale = tail.v_scales.s[h];
                while (todo != 0) {
                    const int src = __builtin_ctzll(todo);
                    todo &= todo - 1;
                    const int m_leaf = __shfl(leaf, src, 64);
                    const int m_p0 = __shfl(p0, src, 64);
                    const int m_p1 = m_p0 + __shfl(np, src, 64);
                    switch (g_shift) {
                        case 0:
                            merge_leaf_heads<D, 1, true>(lane, m_leaf, h, m_p0, m_p1, n_q_heads, ws_o,
                                                   ws_ml, tail.n_ws_rows, tail.out, tail.out_bf16 != 0, tail.lse, out_scale);
                            break;
                        case 1:
                            merge_leaf_heads<D, 2, true>(lane, m_leaf, h, m_p0, m_p1, n_q_heads, ws_o,
                                                   ws_ml, tail.n_ws_rows, tail.out, tail.out_bf16 != 0, tail.lse, out_scale);
                            break;
                        case 2:
                            merge_leaf_heads<D, 4, true>(lane, m_leaf, h, m_p0, m_p1, n_q_heads, ws_o,
                                                   ws_ml, tail.n_ws_rows, tail.out, tail.out_bf16 != 0, tail.lse, out_scale);
                            break;
                        default:
                            merge_leaf_heads<D, 8, true>(lane, m_leaf, h, m_p0, m_p1, n_q_heads, ws_o,
                                                   ws_ml, tail.n_ws_rows, tail.out, tail.out_bf16 != 0, tail.lse, out_scale);
                            break;
                    }
                    if (lane == 0) tail.arrived[(int64_t)m_leaf * n_kv_heads + h] = 0;
                }
            }
        }
    };

    // A wave's own 16 tokens into its private LDS region (small and token-parallel items):
    // K rows as they are, V as bf16 transposed pieces (two tokens per dword).
    auto stage_private = [&](u32x4_t* ksw, u32x2_t* vsw) {
#pragma unroll
        for (int i = 0; i < NKL; ++i) ksw[(RPL * i + rb) * KROW + pa] = widen_raw(kraw[i]);
        const u32x4_t vw[4] = {widen_raw(vraw[0]), widen_raw(vraw[1]), widen_raw(vraw[2]),
                               widen_raw(vraw[3])};
        if constexpr (D == 128) {
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
                u32x2_t t;
                t[0] = __builtin_amdgcn_perm(vw[1][x >> 1], vw[0][x >> 1], sel);
                t[1] = __builtin_amdgcn_perm(vw[3][x >> 1], vw[2][x >> 1], sel);
                vsw[x * 64 + lane] = t;
            }
        } else {
            // the lane's half of the piece: elements 4 (a & 1) + x, x = 0..3
            uint32_t hv[4][2];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                hv[i][0] = (a & 1) ? vw[i][2] : vw[i][0];
                hv[i][1] = (a & 1) ? vw[i][3] : vw[i][1];
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
                u32x2_t t;
                t[0] = __builtin_amdgcn_perm(hv[1][x >> 1], hv[0][x >> 1], sel);
                t[1] = __builtin_amdgcn_perm(hv[3][x >> 1], hv[2][x >> 1], sel);
                vsw[x * 64 + lane] = t;
            }
        }
    };

    if (wave_item) {
        // ---- A small item walked by this wave alone: 16-token units in order (unit u =
        // half u & 1 of step u >> 1) through the wave's own LDS region, next unit's loads
        // in flight while the current one is computed; no fold, no workgroup barrier.
        const uint32_t k_off0 = (uint32_t)rb * stride_b + pa * piece_b;       // K row rb (+ RPL i)
        const uint32_t v_off0 = (uint32_t)(4 * b) * stride_b + va * piece_b;  // V row 4 b (+ i)
        u32x4_t* ksw = smem + w * (16 * KROW + NX * 32);
        u32x2_t* vsw = reinterpret_cast<u32x2_t*>(ksw + 16 * KROW);
        auto unit_rows = [&](int u, int64_t& tok) {
            // steps 0 and 1 stand in the unit table; the others: uniform, a scalar load
            const Run sd = u < 2 ? first_step : u < 4 ? my_unit->second : my_steps[u >> 1];
            tok = sd.tok + 16 * (u & 1);
            return min(16, max(0, sd.n - 16 * (u & 1)));
        };
        auto issue_unit = [&](int64_t tok, int n) {
            if (n > 0) {
                const int64_t base = (plane + tok) * (int64_t)stride_b;
                char* kb = const_cast<char*>(reinterpret_cast<const char*>(k_pool)) + base;
                char* vb = const_cast<char*>(reinterpret_cast<const char*>(v_pool)) + base;
                const __amdgpu_buffer_rsrc_t kr =
                    __builtin_amdgcn_make_buffer_rsrc(kb, 0, n * (int)stride_b, 0x00020000);
                const __amdgpu_buffer_rsrc_t vr =
                    __builtin_amdgcn_make_buffer_rsrc(vb, 0, n * (int)stride_b, 0x00020000);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (i < NKL)
                        kraw[i] = load_row_piece<FP8>(kr, k_off0 + (uint32_t)(RPL * i) * stride_b, 0,
                                                      std::integral_constant<int, 2>{});
                    vraw[i] = load_row_piece<FP8>(vr, v_off0 + (uint32_t)i * stride_b, 0,
                                                  std::integral_constant<int, 2>{});
                }
            }
        };
        auto stage_own = [&](int n) {
            if (n > 0) stage_private(ksw, vsw);
        };
        const int n_units = 2 * n_steps;
        int64_t tok = 0;
        int n_cur = n_units > 0 ? unit_rows(0, tok) : 0;
        issue_unit(tok, n_cur);
        const int head = h * G + (rr & (G - 1));
        const bf16_t* qp = q + ((int64_t)ent * n_q_heads + head) * D;
        bf16x8_t qf[NKK];
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) qf[kk] = as_bf16x8(load16(qp + 32 * kk + 8 * b));
        const int32_t out_row = (ent_slot + it.slot_off) * n_q_heads + head;
        f32x4_t oacc[NX];
        float m = -INFINITY, lsum = 0.f;
#pragma unroll
        for (int x = 0; x < NX; ++x) oacc[x] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        stage_own(n_cur);
        __builtin_amdgcn_s_waitcnt(0);  // nothing issued so far may count against the loop's waits
        for (int u = 0; u < n_units; ++u) {
            int64_t tok_next = 0;
            const int n_next = u + 1 < n_units ? unit_rows(u + 1, tok_next) : 0;
            issue_unit(tok_next, n_next);
            if (n_cur > 0)
                attn_half_step<D>(ksw + a * KROW + b, vsw + lane, b, n_cur, qf, oacc, m, lsum,
                                  scale_log2e, raise_margin);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            stage_own(n_next);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            n_cur = n_next;
        }
        float l = lsum;
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        store_partial(oacc, m, l, out_row);
        return;
    }

    // descriptor of the loads in flight: the wave's step of the first tile came with the
    // item (a step the item does not have reads n = 0 there)
    Run sd_loaded = first_step;
    if (rowpar && !it.sole_reader)
        issue_loads(sd_loaded, std::integral_constant<int, 0>{});
    else
        issue_loads(sd_loaded, std::integral_constant<int, 2>{});

    // the item's step descriptors go to LDS once; nothing but K, V is fetched afterwards
    u32x4_t desc_raw = {0u, 0u, 0u, 0u};
    if ((int)threadIdx.x < n_steps)
        desc_raw = load16(reinterpret_cast<const char*>(my_steps + threadIdx.x));

    // Q rows as B operands: lane (column a = query row, group b) holds
    // q[row][32 kk + 8 b .. + 8) for kk = 0..3.  The workspace row of the lane's
    // partial result is looked up here as well, off the critical path.
    bf16x8_t qf[NKK];
    int32_t out_row;
    {
        const int head = h * G + (rr & (G - 1));
        const bf16_t* qp = q + ((int64_t)ent * n_q_heads + head) * D;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) qf[kk] = as_bf16x8(load16(qp + 32 * kk + 8 * b));
        out_row = (ent_slot + it.slot_off) * n_q_heads + head;
    }
    if ((int)threadIdx.x < n_steps) sm_desc[threadIdx.x] = desc_raw;

    f32x4_t oacc[NX];
    float m = -INFINITY, lsum = 0.f;
#pragma unroll
    for (int x = 0; x < NX; ++x) oacc[x] = f32x4_t{0.f, 0.f, 0.f, 0.f};

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
            for (int i = 0; i < NKL; ++i)
                ks[(32 * sw + 16 * hw + RPL * i + rb) * KROW + pa] = widen_raw(kraw[i]);
            const u32x4_t vw[4] = {widen_raw(vraw[0]), widen_raw(vraw[1]), widen_raw(vraw[2]),
                                   widen_raw(vraw[3])};
            // This half's four contraction slots of every V^T fragment (8 of its 16
            // bytes), converted to fp16 for the P V product once for all row blocks:
            // element x of the lane's 16-byte piece (head_dim 64: of the lane's half of
            // it), tokens 4 b .. 4 b + 3.
            u32x2_t* vs2 = reinterpret_cast<u32x2_t*>(vs);
            uint32_t dw[4][NX / 2];  // the dwords (two elements each) this lane transposes
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (D == 128) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) dw[i][j] = vw[i][j];
                } else {
                    dw[i][0] = (a & 1) ? vw[i][2] : vw[i][0];
                    dw[i][1] = (a & 1) ? vw[i][3] : vw[i][1];
                }
            }
#pragma unroll
            for (int j = 0; j < NX / 2; ++j) {
                u32x2_t te, to;
                te[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(
                                                         bf16_lo(dw[0][j]), bf16_lo(dw[1][j])));
                te[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(
                                                         bf16_lo(dw[2][j]), bf16_lo(dw[3][j])));
                to[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(
                                                         bf16_hi(dw[0][j]), bf16_hi(dw[1][j])));
                to[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(
                                                         bf16_hi(dw[2][j]), bf16_hi(dw[3][j])));
                vs2[((sw * NX + 2 * j) * 64 + lane) * 2 + hw] = te;
                vs2[((sw * NX + 2 * j + 1) * 64 + lane) * 2 + hw] = to;
            }
        }
    };

    if (rowpar) {
        stage(sd_loaded);
        // Everything issued so far (Q rows, first tile) has to have landed on every path
        // before the loop: a load still counted as outstanding here would make each
        // iteration wait for the next tile's loads as well.
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();  // step list and first tile are in LDS

        // rows that no other item reads (a segment whose queries fit one item) are
        // fetched non-temporally; rows that further row groups re-read stay in L2
        auto tile_loop = [&](auto aux_tag) {
        for (int tile = 0; tile < n_tiles; ++tile) {
            sd_loaded = read_desc(2 * (tile + 1) + sw);  // a step past the end has n = 0
            issue_loads(sd_loaded, aux_tag);

            if (computes) {
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    const int sidx = 2 * tile + st;
                    if (sidx >= n_steps) break;
                    const int n_valid = __builtin_amdgcn_readfirstlane(sm_desc[sidx][2]);
                    if (n_valid > 0)  // an empty spare step was never staged
                        attn_step<D>(ks + (32 * st + a) * KROW + b, vs + st * NX * 64 + lane, b,
                                     n_valid, qf, oacc, m, lsum, scale_log2e, raise_margin);
                }
            }

            __syncthreads();  // the staged tile has been read by everyone who shares it
            stage(sd_loaded);
            __syncthreads();
        }
        };
        if (it.sole_reader)
            tile_loop(std::integral_constant<int, 2>{});
        else
            tile_loop(std::integral_constant<int, 0>{});
        if (!computes) return;
    } else {
        // Token parallel: every wave walks its own 16-token units (half hw of step
        // 2 tile + sw) through a private LDS region; no workgroup barrier in the loop.
        u32x4_t* ksw = ks + 16 * w * KROW;
        u32x2_t* vsw = reinterpret_cast<u32x2_t*>(vs) + w * (NX * 64);
        auto stage_unit = [&](const Run& sd) {
            if (sd.n > 16 * hw) stage_private(ksw, vsw);
        };
        stage_unit(sd_loaded);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();  // step list is in LDS

        for (int tile = 0; tile < n_tiles; ++tile) {
            const int n_cur = sd_loaded.n - 16 * hw;  // tokens of the staged unit
            sd_loaded = read_desc(2 * (tile + 1) + sw);
            issue_loads(sd_loaded, std::integral_constant<int, 2>{});
            if (n_cur > 0)
                attn_half_step<D>(ksw + a * KROW + b, vsw + lane, b, n_cur, qf, oacc, m, lsum,
                                  scale_log2e, raise_margin);
            // the wave's LDS accesses complete in order; keep the compiler from moving them
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            stage_unit(sd_loaded);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }

    float l = lsum;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (!rowpar) {
        // The four waves hold the same rows over disjoint tokens (a wave that saw no
        // token has m = -inf, l = 0); waves 1..3 hand their results to wave 0 through
        // LDS, so the item still yields one partial per query row.
        if (b == 0) {
            sm_m[w][a] = m;
            sm_l[w][a] = l;
        }
        __syncthreads();  // also: every wave is done with its tile region
        const float ms = fmaxf(fmaxf(sm_m[0][a], sm_m[1][a]), fmaxf(sm_m[2][a], sm_m[3][a]));
        const float f_own = fast_exp2((m - ms) * scale_log2e);
        f32x4_t* fold = reinterpret_cast<f32x4_t*>(smem) + lane;
        if (w != 0) {
#pragma unroll
            for (int x = 0; x < NX; ++x) fold[((w - 1) * NX + x) * 64] = oacc[x] * f_own;
        }
        __syncthreads();
        if (w != 0) return;
        l *= f_own;
#pragma unroll
        for (int k = 1; k < 4; ++k)
            l += sm_l[k][a] * fast_exp2((sm_m[k][a] - ms) * scale_log2e);
        m = ms;
#pragma unroll
        for (int x = 0; x < NX; ++x)
            oacc[x] = oacc[x] * f_own + fold[x * 64] + fold[(NX + x) * 64] + fold[(2 * NX + x) * 64];
    }

    if (rowpar ? !computes : w != 0) return;
    store_partial(oacc, m, l, out_row);
}

}  // namespace ets
