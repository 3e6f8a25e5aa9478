// Benchmark hooks: kernels that do no attention work and exist so that a benchmark can
// put the attention kernels' HBM figures next to what the same device sustains for the
// plainest access pattern.
#pragma once

#include "device_utils.hpp"

namespace ets {

// Plain streaming read: every lane fetches 16 bytes per load, a wavefront 1 KiB of
// consecutive memory, eight loads in flight per lane; the workgroups walk the buffer with
// a grid stride.  The values are folded into one word per workgroup so that the loads
// cannot be dropped.  n16 = number of 16-byte pieces (a multiple of 256 * 8 is read in
// full; a ragged tail is read piece by piece).
typedef uint32_t bench_u32x4_t __attribute__((ext_vector_type(4)));

template <bool NONTEMPORAL>
__global__ __launch_bounds__(256) void read_stream_kernel(const bench_u32x4_t* __restrict__ src,
                                                          int64_t n16,
                                                          uint32_t* __restrict__ sink) {
    constexpr int U = 8;
    bench_u32x4_t acc = {0u, 0u, 0u, 0u};
    const int64_t span = 256 * U;
    const int64_t n_spans = n16 / span;
    for (int64_t s = blockIdx.x; s < n_spans; s += gridDim.x) {
        const bench_u32x4_t* p = src + s * span + threadIdx.x;
        bench_u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            v[u] = NONTEMPORAL ? __builtin_nontemporal_load(p + 256 * u) : p[256 * u];
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    if (blockIdx.x == 0)
        for (int64_t i = n_spans * span + threadIdx.x; i < n16; i += 256) {
            acc ^= src[i];
        }
    uint32_t r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) r ^= __shfl_xor(r, off, 64);
    if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], r);
}

}  // namespace ets
