// Small device helpers shared by the kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace ets {

struct bf16_t {
    uint16_t bits;
};

// One factor per kv head, passed to kernels by value (kernel argument memory).
constexpr int kMaxScaledHeads = 64;
struct HeadScales {
    float s[kMaxScaledHeads];
};

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) {
    return __uint_as_float(packed & 0xFFFF0000u);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Data-parallel-primitive lane exchange inside a row of 16 lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// Sum over aligned groups of LANES consecutive lanes (2..64); every lane of a
// group receives the group's sum.
template <int LANES>
__device__ __forceinline__ float group_sum(float x) {
    if constexpr (LANES >= 2) x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
    if constexpr (LANES >= 4) x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
    if constexpr (LANES >= 8) x += dpp_move<0x141>(x);  // row_half_mirror
    if constexpr (LANES >= 16) x += dpp_move<0x140>(x); // row_mirror
    if constexpr (LANES >= 32) x += __shfl_xor(x, 16, 64);
    if constexpr (LANES >= 64) x += __shfl_xor(x, 32, 64);
    return x;
}

// 16 bytes of pool data widened to floats.
template <typename T>
struct Vec16;

template <>
struct Vec16<float> {
    static constexpr int N = 4;
    float4 raw;
    __device__ __forceinline__ void load(const float* p) {
        raw = *reinterpret_cast<const float4*>(p);
    }
    __device__ __forceinline__ void unpack(float (&f)[4]) const {
        f[0] = raw.x; f[1] = raw.y; f[2] = raw.z; f[3] = raw.w;
    }
};

template <>
struct Vec16<bf16_t> {
    static constexpr int N = 8;
    uint4 raw;
    __device__ __forceinline__ void load(const bf16_t* p) {
        raw = *reinterpret_cast<const uint4*>(p);
    }
    __device__ __forceinline__ void unpack(float (&f)[8]) const {
        f[0] = bf16_lo(raw.x); f[1] = bf16_hi(raw.x);
        f[2] = bf16_lo(raw.y); f[3] = bf16_hi(raw.y);
        f[4] = bf16_lo(raw.z); f[5] = bf16_hi(raw.z);
        f[6] = bf16_lo(raw.w); f[7] = bf16_hi(raw.w);
    }
};

}  // namespace ets
