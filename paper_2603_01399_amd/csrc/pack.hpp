// Offline weight preparation kernels: quantise + pack, unpack, bf16 pack (gfx950).
//
// Packed order (both dtypes): a "step" is 1024 contiguous bytes read by one wave-wide
// 128-bit load; lane l = 16*g + i of step s of tile t holds, for int8,
//     W[16 t + i][64 s + 16 g + 0..15]        (16 codes)
// and for bf16
//     W[16 t + i][32 s +  8 g + 0..7]         (8 values).
// Steps of a tile are contiguous, tiles follow each other, so a workgroup that owns a
// tile range streams one contiguous address range.
#pragma once

#include "quasar_device.hpp"

namespace quasar {

template <bool SRC_BF16>
__device__ __forceinline__ float load_w(const void *w, long long idx) {
    if constexpr (SRC_BF16)
        return bf16_bits_to_float(reinterpret_cast<const uint16_t *>(w)[idx]);
    else
        return reinterpret_cast<const float *>(w)[idx];
}
// element k of a row, with the offline side of the smoothing transformation applied
// (W diag(s)^-1, one fp32 division) when a smoothing vector is given
template <bool SRC_BF16>
__device__ __forceinline__ float load_w_smoothed(const void *w, long long row_base, int k, const float *smooth) {
    const float v = load_w<SRC_BF16>(w, row_base + k);
    return smooth ? __fdiv_rn(v, smooth[k]) : v;
}

// One workgroup (256 threads) per 16-row tile.
template <bool SRC_BF16>
__global__ __launch_bounds__(256) void quantize_pack_kernel(const void *w, long long ldw, int N, int K,
                                                            const float *smooth, u32x4 *packed, uint16_t *scales) {
    __shared__ float row_scale[kTileRows];
    const int tid = threadIdx.x;
    const int t = blockIdx.x;
    const int S = K / kStepK8;

    // pass 1: row maxima.  16 threads per row.
    {
        const int r = tid >> 4, c = tid & 15;
        const long long base = (long long)(t * kTileRows + r) * ldw;
        float amax = 0.f;
        for (int k = c; k < K; k += 16) amax = fmaxf(amax, fabsf(load_w_smoothed<SRC_BF16>(w, base, k, smooth)));
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        if (c == 0) {
            const float step = __fdiv_rn(amax, 127.0f);
            unsigned int sb = float_to_bf16_bits(step);
            float s = bf16_bits_to_float(sb);
            if (!(s > 0.f)) { sb = 0; s = 0.f; }
            row_scale[r] = s;
            scales[t * kTileRows + r] = (uint16_t)sb;
        }
    }
    __syncthreads();

    // pass 2: each thread produces one 16-byte lane slot of one step at a time
    for (int slot = tid; slot < S * 64; slot += 256) {
        const int s = slot >> 6, l = slot & 63;
        const int g = l >> 4, i = l & 15;
        const float sc = row_scale[i];
        const long long base = (long long)(t * kTileRows + i) * ldw;
        const int k0 = s * kStepK8 + 16 * g;
        unsigned int out[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            unsigned int word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int code = 0;
                if (sc > 0.f) {
                    const float ratio = __fdiv_rn(load_w_smoothed<SRC_BF16>(w, base, k0 + 4 * q + e, smooth), sc);
                    float r = rintf(ratio);                 // round half to even
                    r = fminf(fmaxf(r, -127.f), 127.f);
                    code = (int)r;
                }
                word |= ((unsigned int)code & 0xffu) << (8 * e);
            }
            out[q] = word;
        }
        packed[((long long)t * S + s) * 64 + l] = u32x4{out[0], out[1], out[2], out[3]};
    }
}

__global__ __launch_bounds__(256) void unpack_kernel(const u32x4 *packed, int N, int K, int8_t *q) {
    const int S = K / kStepK8;
    const long long nslots = (long long)(N / kTileRows) * S * 64;
    for (long long slot = (long long)blockIdx.x * 256 + threadIdx.x; slot < nslots;
         slot += (long long)gridDim.x * 256) {
        const int l = (int)(slot & 63);
        const long long ts = slot >> 6;
        const int s = (int)(ts % S);
        const long long t = ts / S;
        const int g = l >> 4, i = l & 15;
        const u32x4 v = packed[slot];
        *reinterpret_cast<u32x4 *>(q + (t * kTileRows + i) * (long long)K + (long long)s * kStepK8 + 16 * g) = v;
    }
}

template <bool SRC_BF16>
__global__ __launch_bounds__(256) void pack_bf16_kernel(const void *w, long long ldw, int N, int K,
                                                        u32x4 *packed) {
    const int S = K / kStepK16;
    const long long nslots = (long long)(N / kTileRows) * S * 64;
    for (long long slot = (long long)blockIdx.x * 256 + threadIdx.x; slot < nslots;
         slot += (long long)gridDim.x * 256) {
        const int l = (int)(slot & 63);
        const long long ts = slot >> 6;
        const int s = (int)(ts % S);
        const long long t = ts / S;
        const int g = l >> 4, i = l & 15;
        const long long base = (t * kTileRows + i) * ldw + (long long)s * kStepK16 + 8 * g;
        unsigned int h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if constexpr (SRC_BF16)
                h[e] = reinterpret_cast<const uint16_t *>(w)[base + e];
            else
                h[e] = float_to_bf16_bits(reinterpret_cast<const float *>(w)[base + e]);
        }
        packed[slot] = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    }
}

// ---- 4-bit group-wise weights -------------------------------------------------------------
// Packed order: step s of tile t is 1056 contiguous bytes: 16 rows x 128 k of codes (lane
// l = 16*g + i holds row i; dword j of the lane holds k = 32 j + 8 g + e, e = 0..7, as
// code + 8 in nibble (e >> 1) + 4 (e & 1)), then the rows' 16 bf16 step sizes of this group.
constexpr int kW4StepK = 128;
constexpr int kW4StepBytes = 1056;

// One workgroup (256 threads) per 16-row tile; 16 threads per row, each owns 8 consecutive k of
// the current group, which is exactly one dword of the packed step.
template <bool SRC_BF16>
__global__ __launch_bounds__(256) void quantize_pack_w4_kernel(const void *w, long long ldw, int N, int K,
                                                               unsigned char *packed) {
    const int tid = threadIdx.x;
    const int t = blockIdx.x;
    const int S = K / kW4StepK;
    const int r = tid >> 4, c = tid & 15;
    const long long base = (long long)(t * kTileRows + r) * ldw;
    for (int s = 0; s < S; ++s) {
        float v[8];
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            v[e] = load_w<SRC_BF16>(w, base + (long long)s * kW4StepK + 8 * c + e);
            amax = fmaxf(amax, fabsf(v[e]));
        }
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        unsigned int sb = float_to_bf16_bits(__fdiv_rn(amax, 7.0f));
        float sc = bf16_bits_to_float(sb);
        if (!(sc > 0.f)) { sb = 0; sc = 0.f; }
        unsigned int word = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int code = 0;
            if (sc > 0.f) {
                float q = rintf(__fdiv_rn(v[e], sc));           // round half to even
                q = fminf(fmaxf(q, -7.f), 7.f);
                code = (int)q;
            }
            word |= (unsigned int)(code + 8) << (4 * ((e >> 1) + 4 * (e & 1)));
        }
        unsigned char *step = packed + ((long long)t * S + s) * kW4StepBytes;
        const int j = c >> 2, g = c & 3;
        reinterpret_cast<unsigned int *>(step)[(16 * g + r) * 4 + j] = word;
        if (c == 0) reinterpret_cast<uint16_t *>(step + 1024)[r] = (uint16_t)sb;
    }
}

// codes -> q[N, K] int8 row-major, step sizes -> scales[N, K / 128] bf16 (for checking)
__global__ __launch_bounds__(256) void unpack_w4_kernel(const unsigned char *packed, int N, int K, int8_t *q,
                                                        uint16_t *scales) {
    const int S = K / kW4StepK;
    const long long nwords = (long long)(N / kTileRows) * S * 256;
    for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < nwords; idx += (long long)gridDim.x * 256) {
        const int wd = (int)(idx & 255);
        const long long ts = idx >> 8;
        const int s = (int)(ts % S);
        const long long t = ts / S;
        const int l = wd >> 2, j = wd & 3;
        const int g = l >> 4, i = l & 15;
        const unsigned char *step = packed + ts * kW4StepBytes;
        const unsigned int word = reinterpret_cast<const unsigned int *>(step)[wd];
        int8_t *dst = q + (t * kTileRows + i) * (long long)K + (long long)s * kW4StepK + 32 * j + 8 * g;
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e] = (int8_t)((int)((word >> (4 * ((e >> 1) + 4 * (e & 1)))) & 15u) - 8);
        if (wd < kTileRows)
            scales[(t * kTileRows + wd) * (long long)S + s] = reinterpret_cast<const uint16_t *>(step + 1024)[wd];
    }
}

}  // namespace quasar
