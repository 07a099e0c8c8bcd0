// W8A8 weight-streaming kernels (gfx950): int8 codes on both sides of the matrix cores.
//
// The activations are smoothed and quantised per token inside the kernel (Sec. 3.3, online
// activation smoothing and quantisation), the packed weight step goes from the load
// straight into one v_mfma_i32_16x16x64_i8 (no per-weight vector-ALU work at all), the
// integer sums are exact, and the epilogue applies (delta_w . delta_x) once per output
// (Eq. 10).
//
// Every floating-point step that decides an integer code or the bits of the result is one
// IEEE fp32 operation, in this order:
//     x~ = float(x) * s[k]            (skipped without a smoothing vector)
//     amax = max_k |x~|,  dx = amax / 127,  inv = 127 / amax
//     code = clamp(rint(x~ * inv), -127, 127)
//     y = bf16( float(acc_i32) * (dx * dw) )
//
// Work decomposition, ring of weight loads and the fixed-order cross-wave sum are those of
// the bf16-activation kernel (stream_gemm.hpp); integer addition makes the sum exact, so the
// result does not depend on the split at all.
#pragma once

#include "stream_gemm.hpp"

namespace quasar {

typedef int i32x4 __attribute__((ext_vector_type(4)));

// eight bf16 activations (one 16-byte piece at column k) -> smoothed fp32 values
__device__ __forceinline__ void smooth_piece(const u32x4 &v, const float *smooth, long long k, float (&xt)[8]) {
    const unsigned int wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        xt[2 * q] = __uint_as_float(wd[q] << 16);
        xt[2 * q + 1] = __uint_as_float(wd[q] & 0xFFFF0000u);
    }
    if (smooth) {
        const f32x4 s0 = *reinterpret_cast<const f32x4 *>(smooth + k);
        const f32x4 s1 = *reinterpret_cast<const f32x4 *>(smooth + k + 4);
        xt[0] = xt[0] * s0.x; xt[1] = xt[1] * s0.y; xt[2] = xt[2] * s0.z; xt[3] = xt[3] * s0.w;
        xt[4] = xt[4] * s1.x; xt[5] = xt[5] * s1.y; xt[6] = xt[6] * s1.z; xt[7] = xt[7] * s1.w;
    }
}

__device__ __forceinline__ float piece_amax(const float (&xt)[8]) {
    float a = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(xt[j]));
    return a;
}

// eight smoothed values -> eight int8 codes packed into two dwords
__device__ __forceinline__ u32x2 quantize_piece(const float (&xt)[8], float inv) {
    unsigned int o[2] = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float r = rintf(xt[j] * inv);                       // round half to even
        r = fminf(fmaxf(r, -127.f), 127.f);
        o[j >> 2] |= ((unsigned int)(int)r & 0xFFu) << (8 * (j & 3));
    }
    return u32x2{o[0], o[1]};
}

__device__ __forceinline__ float step_of(float amax) { return amax > 0.f ? __fdiv_rn(amax, 127.0f) : 0.f; }
__device__ __forceinline__ float inverse_step_of(float amax) { return amax > 0.f ? __fdiv_rn(127.0f, amax) : 0.f; }

// ------------------------------------------------------------------------------------
// Stand-alone activation quantiser: x[M, K] bf16 -> codes[M, K] int8 row-major, dx[M] fp32.
// One workgroup (256 threads) per token.  The fused kernels below run the same three
// device functions; this entry makes the codes observable.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void quantize_activations_kernel(const uint16_t *x, long long ldx, int K,
                                                                   const float *smooth, int8_t *xq, float *dx) {
    __shared__ float red[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    const uint16_t *row = x + (long long)m * ldx;
    float amax = 0.f;
    for (int p8 = tid; p8 < K / 8; p8 += 256) {
        float xt[8];
        smooth_piece(*reinterpret_cast<const u32x4 *>(row + 8ll * p8), smooth, 8ll * p8, xt);
        amax = fmaxf(amax, piece_amax(xt));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    if ((tid & 63) == 0) red[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float inv = inverse_step_of(amax);
    if (tid == 0) dx[m] = step_of(amax);
    for (int p8 = tid; p8 < K / 8; p8 += 256) {
        float xt[8];
        smooth_piece(*reinterpret_cast<const u32x4 *>(row + 8ll * p8), smooth, 8ll * p8, xt);
        *reinterpret_cast<u32x2 *>(xq + (long long)m * K + 8ll * p8) = quantize_piece(xt, inv);
    }
}

// ------------------------------------------------------------------------------------
// Fused W8A8 linear / vocabulary-argmax kernel.
// A operand = one packed weight step (16 rows x 64 k int8), B operand = 64 k x 16 tokens of
// int8 codes from LDS, D = 16 rows x 16 tokens int32.  Lane l = 16*g + i holds weight row i,
// k-group g (A) / token i, k-group g (B) and accumulates rows 4g..4g+3 of token i (D).
// LDS: [codes of the chunk: [k/16][token][16 B]][row scales, then dx[32] and amax[32]]
//      [2 x NW staging tiles][tile sums (C > 1)]
// ------------------------------------------------------------------------------------
template <int MP, int EPI, int NW, int D>
__global__ __launch_bounds__(NW * 64) void stream_w8a8_kernel(const GemmParams p) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int NB = (MP == 32) ? 2 : 1;
    constexpr int LMP = (MP == 8) ? 3 : (MP == 16 ? 4 : 5);
    constexpr int XB = 4;
    constexpr int nthreads = NW * 64;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, mcol = lane & 15;

    const int G = gridDim.x, b = blockIdx.x;
    const int t0 = tile_split(p.T, b, G);
    const int t1 = tile_split(p.T, b + 1, G);
    const int ntiles = t1 - t0;

    unsigned char *xq = lds;                                                          // [SC*4][MP][16]
    uint16_t *sc_lds = reinterpret_cast<uint16_t *>(lds + p.xs_bytes);                 // [tpw*16]
    float *tok_dx = reinterpret_cast<float *>(lds + p.xs_bytes + p.sc_bytes - 256);    // [32]
    unsigned int *tok_amax = reinterpret_cast<unsigned int *>(lds + p.xs_bytes + p.sc_bytes - 128);   // [32]
    i32x4 *stage = reinterpret_cast<i32x4 *>(lds + p.xs_bytes + p.sc_bytes);          // [2][NW][NB][64]
    i32x4 *accs = stage + 2 * NW * NB * 64;                                            // [ntiles][NB][64] (C > 1)

    // requests in the order they are needed back: the first batch of activations (kept in
    // registers for both passes below), then the weight ring
    const int m_own = tid & (MP - 1);          // every thread always sees the same token
    const int npieces_all = (p.K / 8) * MP;
    u32x4 xfirst[XB];
#pragma unroll
    for (int i = 0; i < XB; ++i) {
        const int idx = i * nthreads + tid;
        xfirst[i] = u32x4{0u, 0u, 0u, 0u};
        if (idx < npieces_all && m_own < p.M)
            xfirst[i] = *reinterpret_cast<const u32x4 *>(p.x + m_own * p.ldx + 8ll * (idx >> LMP));
    }
    WaveWalk<NW, D> walk{p, w, lane, t0, ntiles};
    typename WaveWalk<NW, D>::Front ld;
    walk.begin(ld);
    u32x4 ring[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        ring[d] = ring_refill(walk.addr(ld), u32x4{0u, 0u, 0u, 0u});
        walk.advance(ld);
    }

    // ---- per-token step sizes over the whole K
    if (tid < 32) tok_amax[tid] = 0u;
    lds_barrier();
    if (m_own < p.M) {
        float amax = 0.f;
#pragma unroll
        for (int i = 0; i < XB; ++i) {
            const int idx = i * nthreads + tid;
            if (idx < npieces_all) {
                float xt[8];
                smooth_piece(xfirst[i], p.smooth, 8ll * (idx >> LMP), xt);
                amax = fmaxf(amax, piece_amax(xt));
            }
        }
        for (int base = nthreads * XB; base < npieces_all; base += nthreads * XB) {
            u32x4 v[XB];
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                v[i] = u32x4{0u, 0u, 0u, 0u};
                if (idx < npieces_all) v[i] = *reinterpret_cast<const u32x4 *>(p.x + m_own * p.ldx + 8ll * (idx >> LMP));
            }
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                if (idx < npieces_all) {
                    float xt[8];
                    smooth_piece(v[i], p.smooth, 8ll * (idx >> LMP), xt);
                    amax = fmaxf(amax, piece_amax(xt));
                }
            }
        }
        // non-negative floats order like their bit patterns
        __hip_atomic_fetch_max(&tok_amax[m_own], __float_as_uint(amax), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    lds_barrier();
    const float amax_own = __uint_as_float(tok_amax[m_own]);
    const float inv = inverse_step_of(amax_own);
    if (tid < MP) tok_dx[tid] = step_of(amax_own);

    // codes of K chunk c -> LDS in B-operand order; the first batch of chunk 0 is still in registers
    auto x_quant = [&](int c) {
        const int scc = min(p.SC, p.S - c * p.SC);
        const int npieces = scc * 8 * MP;
        for (int base = 0; base < npieces; base += nthreads * XB) {
            u32x4 v[XB];
            const bool held = c == 0 && base == 0;
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                v[i] = xfirst[i];
                if (!held) {
                    v[i] = u32x4{0u, 0u, 0u, 0u};
                    if (idx < npieces && m_own < p.M)
                        v[i] = *reinterpret_cast<const u32x4 *>(p.x + m_own * p.ldx + (long long)c * p.SC * kStepK8 +
                                                                8ll * (idx >> LMP));
                }
            }
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                if (idx < npieces) {
                    const int p8 = idx >> LMP;
                    u32x2 codes = {0u, 0u};
                    if (m_own < p.M) {
                        float xt[8];
                        smooth_piece(v[i], p.smooth, (long long)c * p.SC * kStepK8 + 8ll * p8, xt);
                        codes = quantize_piece(xt, inv);
                    }
                    *reinterpret_cast<u32x2 *>(xq + (((p8 >> 1) * MP + m_own) * 16 + 8 * (p8 & 1))) = codes;
                }
            }
        }
    };
    x_quant(0);
    for (int i = 2 * tid; i < ntiles * kTileRows; i += 2 * nthreads)
        reinterpret_cast<unsigned int *>(sc_lds)[i >> 1] =
            *reinterpret_cast<const unsigned int *>(p.scales + (long long)t0 * kTileRows + i);
    // known-empty load queue: the staging loads are conditional, and without this the compiler
    // would fall back to draining the ring on every round
    __builtin_amdgcn_s_waitcnt(0x0F70);
    lds_barrier();

    i32x4 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = i32x4{0, 0, 0, 0};
    float bestv[NB];
    unsigned int besti[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) { bestv[nb] = -__builtin_inff(); besti[nb] = 0x7FFFFFFFu; }
    int parity = 0;
    const int xm = (MP == 8) ? (mcol & 7) : mcol;

    for (int c = 0; c < p.C; ++c) {
        if (c > 0) {
            x_quant(c);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            lds_barrier();
        }
        typename WaveWalk<NW, D>::Front cs;
        walk.slice(c, cs);
        int tl = 0, si = 0;
        const int rounds = cs.padded / D;
        for (int r = 0; r < rounds; ++r) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const int idx = r * D + d;
                const bool in_range = idx < cs.items;
                const bool valid = in_range && si < cs.spw;
                u32x4 wv = ring[d];
                if (!valid) wv = u32x4{0u, 0u, 0u, 0u};
                const int step_in_chunk = valid ? cs.s_lo + si : 0;
                const i32x4 a = __builtin_bit_cast(i32x4, wv);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const i32x4 bq =
                        *reinterpret_cast<const i32x4 *>(xq + ((step_in_chunk * 4 + g) * MP + xm + 16 * nb) * 16);
                    acc[nb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bq, acc[nb], 0, 0, 0);
                }
                ring[d] = ring_refill(walk.addr(ld), wv);
                walk.advance(ld);
                if (in_range && si == cs.nsl - 1) {
                    // ---- tile end: exact integer sum over the waves through LDS
                    i32x4 *st = stage + (parity * NW) * NB * 64;
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        st[(w * NB + nb) * 64 + lane] = acc[nb];
                        acc[nb] = i32x4{0, 0, 0, 0};
                    }
                    lds_barrier();
                    if (w == (tl % NW)) {
                        i32x4 rsum[NB];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            rsum[nb] = st[nb * 64 + lane];
#pragma unroll
                            for (int ww = 1; ww < NW; ++ww) rsum[nb] += st[(ww * NB + nb) * 64 + lane];
                            if (p.C > 1) {
                                i32x4 *sum = accs + (tl * NB + nb) * 64 + lane;
                                if (c > 0) rsum[nb] += *sum;
                                if (c < p.C - 1) *sum = rsum[nb];
                            }
                        }
                        if (c == p.C - 1) {
                            const int n0 = (t0 + tl) * kTileRows + 4 * g;
                            const u32x2 sb = *reinterpret_cast<const u32x2 *>(sc_lds + tl * kTileRows + 4 * g);
                            const float dw0 = bf16_bits_to_float(sb.x & 0xFFFFu), dw1 = bf16_bits_to_float(sb.x >> 16);
                            const float dw2 = bf16_bits_to_float(sb.y & 0xFFFFu), dw3 = bf16_bits_to_float(sb.y >> 16);
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb) {
                                const int m = mcol + 16 * nb;
                                const float dxm = tok_dx[m];
                                // Eq. 10: fp32(acc) * (dx * dw), each one fp32 operation
                                const float v0 = (float)rsum[nb].x * (dxm * dw0);
                                const float v1 = (float)rsum[nb].y * (dxm * dw1);
                                const float v2 = (float)rsum[nb].z * (dxm * dw2);
                                const float v3 = (float)rsum[nb].w * (dxm * dw3);
                                if constexpr (EPI == EPI_LINEAR) {
                                    if (m < p.M) {
                                        u32x2 o;
                                        o.x = float_to_bf16_bits(v0) | (float_to_bf16_bits(v1) << 16);
                                        o.y = float_to_bf16_bits(v2) | (float_to_bf16_bits(v3) << 16);
                                        *reinterpret_cast<u32x2 *>(p.y + m * p.ldy + n0) = o;
                                    }
                                } else {
                                    // strictly greater keeps the lowest index inside a lane
                                    if (v0 > bestv[nb]) { bestv[nb] = v0; besti[nb] = n0; }
                                    if (v1 > bestv[nb]) { bestv[nb] = v1; besti[nb] = n0 + 1; }
                                    if (v2 > bestv[nb]) { bestv[nb] = v2; besti[nb] = n0 + 2; }
                                    if (v3 > bestv[nb]) { bestv[nb] = v3; besti[nb] = n0 + 3; }
                                }
                            }
                        }
                    }
                    parity ^= 1;
                }
                if (in_range) {
                    ++si;
                    if (si >= cs.nsl) { si = 0; ++tl; }
                }
            }
        }
    }

    if constexpr (EPI == EPI_ARGMAX) {
        unsigned long long *red = reinterpret_cast<unsigned long long *>(stage);   // [NW][MP]
        lds_barrier();   // all tile-end reads of the staging area are done
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            unsigned long long key = argmax_key(bestv[nb], besti[nb]);
            unsigned long long o = shfl_xor_u64(key, 16);
            key = o > key ? o : key;
            o = shfl_xor_u64(key, 32);
            key = o > key ? o : key;
            if (g == 0 && (MP != 8 || mcol < 8)) red[w * MP + mcol + 16 * nb] = key;
        }
        lds_barrier();
        if (tid < MP) {
            unsigned long long key = red[tid];
            for (int ww = 1; ww < NW; ++ww) {
                const unsigned long long o = red[ww * MP + tid];
                key = o > key ? o : key;
            }
            p.partial[(long long)b * MP + tid] = key;
        }
    }
}

}  // namespace quasar
