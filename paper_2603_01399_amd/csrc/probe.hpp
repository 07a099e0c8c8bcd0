// Bandwidth probes: a pure read stream with the same per-wave load ring as the linear
// kernels, and a plain copy of known size for calibrating hardware byte counters.
#pragma once

#include "quasar_device.hpp"

namespace quasar {

template <int NW, int D>
__global__ __launch_bounds__(NW * 64) void read_stream_kernel(const u32x4 *src, long long nsteps,
                                                              unsigned int *sink) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long long G = gridDim.x, b = blockIdx.x;
    // workgroup range, then wave range inside it: every wave streams a contiguous span
    const long long s0 = nsteps * b / G, s1 = nsteps * (b + 1) / G;
    const long long n = s1 - s0;
    const long long lo = s0 + n * w / NW, hi = s0 + n * (w + 1) / NW;
    const long long total = hi - lo;
    const u32x4 *ptr = src + lo * 64 + lane;
    u32x4 ring[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        ring[d] = u32x4{0u, 0u, 0u, 0u};
        if (d < total) ring[d] = __builtin_nontemporal_load(ptr + (long long)d * 64);
    }
    unsigned int sum = 0;
    for (long long j = 0; j < total; j += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (j + d < total) {
                const u32x4 v = ring[d];
                sum += v.x ^ v.y ^ v.z ^ v.w;
                if (j + d + D < total) ring[d] = __builtin_nontemporal_load(ptr + (j + d + D) * 64);
            }
        }
    }
    sum += __shfl_xor(sum, 1, 64);
    sum += __shfl_xor(sum, 2, 64);
    sum += __shfl_xor(sum, 4, 64);
    sum += __shfl_xor(sum, 8, 64);
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    if (lane == 0) atomicAdd(&sink[b & 2047], sum);
}

__global__ __launch_bounds__(256) void copy_stream_kernel(u32x4 *dst, const u32x4 *src, long long n16) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += (long long)gridDim.x * 256)
        dst[i] = src[i];
}

}  // namespace quasar
