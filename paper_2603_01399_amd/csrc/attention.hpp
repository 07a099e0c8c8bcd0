// Attention of a verification step: M new positions against a key/value cache (gfx950).
//
// Grouped-query attention with head dimension 128.  The cache is laid out for the matrix-core
// operand order, so that every wave-wide 128-bit load is 1 KB of contiguous memory AND already
// an MFMA operand (no transpose through LDS):
//   keys,   per kv head and block of 32 positions: [sub 2][kstep 4][g4 4][p 16][8 d] bf16, element
//           (position 32 b + 16 sub + p, d = 32 kstep + 8 g4 + e): the A operand of
//           v_mfma_f32_16x16x32_bf16 (16 positions x 32 d) for lane 16 g4 + p;
//   values, per kv head and block of 32 positions: [dt 8][g4 4][dd 16][slot 8] bf16, element
//           (d = 16 dt + dd, position 32 b + o) with o = 4 g4 + slot (slot < 4) or 16 + 4 g4 + slot - 4:
//           the A operand (16 d x 32 positions) for lane 16 g4 + dd, its eight positions being
//           exactly those whose scores the same lane group holds after the score MFMAs.
// Everything is computed transposed: S^T = K Q^T (positions x queries), O^T = V^T P^T (d x queries),
// so that a lane owns ONE query column in every accumulator: the running maximum, the rescaling
// of the output and the probabilities (B operand of the second product) never cross lanes.
//
// Work split: grid (splits, kv heads); the waves of a workgroup take the split's 32-position
// blocks in turn with private online-softmax state, merge through LDS, and the workgroup writes
// one partial (max, sum, output) per split; attention_merge_kernel combines the splits.
#pragma once

#include "quasar_device.hpp"

namespace quasar {

constexpr int kHeadDim = 128;
constexpr int kKvBlock = 32;                 // positions per cache block
constexpr int kKvBlockBytes = 8192;          // 32 positions x 128 d x 2 B

struct AttnParams {
    const uint16_t *q;        // [M, Hq * 128] bf16 (normalised, rotated)
    long long ldq;
    const unsigned char *kcache, *vcache;   // per kv head: nblocks_max blocks of 8 KB
    long long head_stride;    // bytes between kv heads in one cache
    uint16_t *out;            // [M, Hq * 128] bf16
    long long ldo;
    float *part_o;            // [Hkv][nsplit][NQT][8][64] f32x4
    float *part_ml;           // [Hkv][nsplit][NQT][16][2]
    int M, G, Hkv, L_total, nblk, nsplit;
    int row0;                 // first query row (m * G + g) of this launch; rows row0 .. row0 + 16 NQT - 1
    float scale_log2;         // log2(e) / sqrt(128)
};

__device__ __forceinline__ long long k_cache_index(int pos_in_block, int d) {
    const int sub = pos_in_block >> 4, p = pos_in_block & 15;
    return ((((long long)sub * 4 + (d >> 5)) * 4 + ((d & 31) >> 3)) * 16 + p) * 8 + (d & 7);
}
__device__ __forceinline__ long long v_cache_index(int pos_in_block, int d) {
    const int o = pos_in_block & 15;
    const int g4 = o >> 2, slot = (o & 3) + ((pos_in_block >> 4) << 2);
    return ((((long long)(d >> 4)) * 4 + g4) * 16 + (d & 15)) * 8 + slot;
}

// ---------------------------------------------------------------------------------------------
// Per head of the fused q/k/v projection output: RMSNorm over the head, rotary embedding at the
// token's position (queries and keys), then queries to q_out and keys/values into the cache at
// positions L .. L + M - 1.  One wave per (token, head); lane i holds elements i and i + 64, the
// two halves of a rotary pair.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void attn_prepare_kernel(const uint16_t *qkv, long long ld, int M, int Hq, int Hkv,
                                                          int L, const uint16_t *q_gamma, const uint16_t *k_gamma,
                                                          float eps, double log2_theta, uint16_t *q_out, long long ldq,
                                                          unsigned char *kcache, unsigned char *vcache,
                                                          long long head_stride) {
    const int lane = threadIdx.x;
    const int nheads = Hq + 2 * Hkv;
    const int m = blockIdx.x / nheads, h = blockIdx.x % nheads;
    const uint16_t *src = qkv + m * ld + (long long)h * kHeadDim;
    const float x1 = bf16_bits_to_float(src[lane]), x2 = bf16_bits_to_float(src[lane + 64]);
    const int pos = L + m;
    const long long blk = pos / kKvBlock;
    const int pib = pos % kKvBlock;
    if (h >= Hq + Hkv) {                                   // value head: stored as is
        uint16_t *dst = reinterpret_cast<uint16_t *>(vcache + (h - Hq - Hkv) * head_stride + blk * kKvBlockBytes);
        dst[v_cache_index(pib, lane)] = src[lane];
        dst[v_cache_index(pib, lane + 64)] = src[lane + 64];
        return;
    }
    float ss = x1 * x1 + x2 * x2;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
    const float r = __fdiv_rn(1.0f, __fsqrt_rn(__fdiv_rn(ss, (float)kHeadDim) + eps));
    const uint16_t *gamma = h < Hq ? q_gamma : k_gamma;
    const float n1 = bf16_bits_to_float(float_to_bf16_bits(bf16_bits_to_float(float_to_bf16_bits(x1 * r)) *
                                                           bf16_bits_to_float(gamma[lane])));
    const float n2 = bf16_bits_to_float(float_to_bf16_bits(bf16_bits_to_float(float_to_bf16_bits(x2 * r)) *
                                                           bf16_bits_to_float(gamma[lane + 64])));
    // angle = pos * theta^(-2 i / 128) in double: positions reach tens of thousands of radians
    const double angle = (double)pos * exp2(-(2.0 * lane / kHeadDim) * log2_theta);
    const float c = (float)cos(angle), s = (float)sin(angle);
    const uint16_t o1 = (uint16_t)float_to_bf16_bits(n1 * c - n2 * s);
    const uint16_t o2 = (uint16_t)float_to_bf16_bits(n2 * c + n1 * s);
    if (h < Hq) {
        uint16_t *dst = q_out + m * ldq + (long long)h * kHeadDim;
        dst[lane] = o1;
        dst[lane + 64] = o2;
    } else {
        uint16_t *dst = reinterpret_cast<uint16_t *>(kcache + (h - Hq) * head_stride + blk * kKvBlockBytes);
        dst[k_cache_index(pib, lane)] = o1;
        dst[k_cache_index(pib, lane + 64)] = o2;
    }
}

// Plain [L, Hkv, 128] keys or values into the cache layout (filling a cache with a prompt, tests).
__global__ __launch_bounds__(256) void kv_cache_fill_kernel(const uint16_t *src, long long n_elems, int Hkv, int pos0,
                                                            unsigned char *cache, long long head_stride, int is_value) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n_elems; i += (long long)gridDim.x * 256) {
        const int d = (int)(i % kHeadDim);
        const long long t = i / kHeadDim;
        const int h = (int)(t % Hkv);
        const int pos = pos0 + (int)(t / Hkv);
        uint16_t *dst = reinterpret_cast<uint16_t *>(cache + h * head_stride + (long long)(pos / kKvBlock) * kKvBlockBytes);
        dst[is_value ? v_cache_index(pos % kKvBlock, d) : k_cache_index(pos % kKvBlock, d)] = src[i];
    }
}

// ---------------------------------------------------------------------------------------------
// Main kernel.  NQT = number of 16-row query tiles of one launch (rows r = m * G + g, starting at
// row0; rows at or beyond M * G are padding).  More than 64 rows take several launches.
// ---------------------------------------------------------------------------------------------
template <int NQT, int NW>
__global__ __launch_bounds__(NW * 64) void verify_attention_kernel(const AttnParams p) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g4 = lane >> 4, col = lane & 15;
    const int h = blockIdx.y, split = blockIdx.x;
    const int R = p.M * p.G;

    const int b0 = (int)(((long long)p.nblk * split) / p.nsplit);
    const int b1 = (int)(((long long)p.nblk * (split + 1)) / p.nsplit);

    // queries as B operands: lane (query column col, k group g4) holds d = 32 ks + 8 g4 .. + 7
    bf16x8 qb[NQT][4];
    int limit[NQT];                       // last visible position of this lane's query column
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        const int r = p.row0 + 16 * qt + col;
        const int m = r < R ? r / p.G : p.M - 1, g = r < R ? r % p.G : 0;
        limit[qt] = p.L_total - p.M + m;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (r < R)
                v = *reinterpret_cast<const u32x4 *>(p.q + m * p.ldq + ((long long)h * p.G + g) * kHeadDim + 32 * ks + 8 * g4);
            qb[qt][ks] = __builtin_bit_cast(bf16x8, v);
        }
    }

    const u32x4 *kbase = reinterpret_cast<const u32x4 *>(p.kcache + h * p.head_stride) + lane;
    const u32x4 *vbase = reinterpret_cast<const u32x4 *>(p.vcache + h * p.head_stride) + lane;
    auto load_block = [&](int b, u32x4 (&kk)[8], u32x4 (&vv)[8]) {
        const u32x4 *kp = kbase + (long long)b * (kKvBlockBytes / 16);
        const u32x4 *vp = vbase + (long long)b * (kKvBlockBytes / 16);
#pragma unroll
        for (int i = 0; i < 8; ++i) kk[i] = __builtin_nontemporal_load(kp + 64 * i);
#pragma unroll
        for (int i = 0; i < 8; ++i) vv[i] = __builtin_nontemporal_load(vp + 64 * i);
    };

    f32x4 oacc[8][NQT];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) oacc[dt][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrow[NQT], lrow[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) { mrow[qt] = -__builtin_inff(); lrow[qt] = 0.f; }

    // One block of prefetch.  The loads are issued unconditionally (the last iteration fetches its
    // own block once more, a cache hit) so that the compiler can count them: with a conditional
    // prefetch it has to assume the shorter queue and waits for the prefetched block before the
    // current one is used.
    u32x4 kc[8], vc[8];
    int b = b0 + w;
    load_block(min(b, b1 - 1), kc, vc);
    for (; b < b1; b += NW) {
        u32x4 kn[8], vn[8];
        load_block(min(b + NW, b1 - 1), kn, vn);

        const int pos0 = b * kKvBlock;
        const bool edge = pos0 + kKvBlock - 1 > p.L_total - p.M;      // some position may be hidden from some query
        if (edge) {
            // positions at or beyond L_total hold whatever the cache memory held: values there
            // must not reach the product (0 x NaN), so clear their slots
            unsigned int keep[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int oa = pos0 + 4 * g4 + (j & 1) * 2 + (j >> 1) * 16;   // slots 2 (j&1) + 4 (j>>1), and the next one
                keep[j] = (oa < p.L_total ? 0x0000FFFFu : 0u) | (oa + 1 < p.L_total ? 0xFFFF0000u : 0u);
            }
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                vc[dt].x &= keep[0];
                vc[dt].y &= keep[1];
                vc[dt].z &= keep[2];
                vc[dt].w &= keep[3];
            }
        }
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            f32x4 s[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                s[sub] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    s[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kc[sub * 4 + ks]), qb[qt][ks],
                                                                     s[sub], 0, 0, 0);
            }
            if (edge) {
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) {
                    const int pb = pos0 + 16 * sub + 4 * g4;
                    if (pb + 0 > limit[qt]) s[sub].x = -__builtin_inff();
                    if (pb + 1 > limit[qt]) s[sub].y = -__builtin_inff();
                    if (pb + 2 > limit[qt]) s[sub].z = -__builtin_inff();
                    if (pb + 3 > limit[qt]) s[sub].w = -__builtin_inff();
                }
            }
            // running maximum in units of the raw scores; exponentials as exp2(raw * c - max * c) in one
            // fused multiply-add each (c = log2(e) / sqrt(128) > 0 keeps the order)
            float mx = fmaxf(fmaxf(fmaxf(s[0].x, s[0].y), fmaxf(s[0].z, s[0].w)),
                             fmaxf(fmaxf(s[1].x, s[1].y), fmaxf(s[1].z, s[1].w)));
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(mrow[qt], mx);
            const float m_use = m_new == -__builtin_inff() ? 0.f : m_new;     // nothing visible yet
            const float mc = -m_use * p.scale_log2;
            const float alpha = __builtin_amdgcn_exp2f(__builtin_fmaf(mrow[qt], p.scale_log2, mc));   // 0 while mrow is -inf
            mrow[qt] = m_new;
            float pr[8];
            pr[0] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[0].x, p.scale_log2, mc));
            pr[1] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[0].y, p.scale_log2, mc));
            pr[2] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[0].z, p.scale_log2, mc));
            pr[3] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[0].w, p.scale_log2, mc));
            pr[4] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[1].x, p.scale_log2, mc));
            pr[5] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[1].y, p.scale_log2, mc));
            pr[6] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[1].z, p.scale_log2, mc));
            pr[7] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[1].w, p.scale_log2, mc));
            // the probabilities enter the second product as bf16 (hardware conversion, nearest even);
            // the row sum uses the same rounded values so that the weights that are applied sum to one
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            unsigned int pk[4];
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bf16x2 h2 = __builtin_convertvector(f32x2{pr[2 * i], pr[2 * i + 1]}, bf16x2);
                pk[i] = __builtin_bit_cast(unsigned int, h2);
                psum += __uint_as_float(pk[i] << 16) + __uint_as_float(pk[i] & 0xFFFF0000u);
            }
            const u32x4 pb16 = {pk[0], pk[1], pk[2], pk[3]};
            lrow[qt] = lrow[qt] * alpha + psum;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0ull) {        // some row's maximum moved
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) oacc[dt][qt] *= alpha;
            }
#pragma unroll
            for (int dt = 0; dt < 8; ++dt)
                oacc[dt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vc[dt]),
                                                                       __builtin_bit_cast(bf16x8, pb16), oacc[dt][qt], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) { kc[i] = kn[i]; vc[i] = vn[i]; }
    }
    // the four lanes of a query column hold partial row sums; the maxima go on in log2 units
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        lrow[qt] += __shfl_xor(lrow[qt], 16, 64);
        lrow[qt] += __shfl_xor(lrow[qt], 32, 64);
        mrow[qt] *= p.scale_log2;
    }

    // ---- merge the waves through LDS: [NW][NQT][8][64] f32x4 outputs, [NW][NQT][16][2] (max, sum)
    f32x4 *lo = reinterpret_cast<f32x4 *>(lds);
    float *lml = reinterpret_cast<float *>(lds + (size_t)NW * NQT * 8 * 64 * 16);
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) lo[((w * NQT + qt) * 8 + dt) * 64 + lane] = oacc[dt][qt];
        if (g4 == 0) {
            lml[((w * NQT + qt) * 16 + col) * 2 + 0] = mrow[qt];
            lml[((w * NQT + qt) * 16 + col) * 2 + 1] = lrow[qt];
        }
    }
    __syncthreads();
    // wave w merges the output tiles dt = w, w + NW, ...; wave 0 also the (max, sum) pairs
    const long long pbase = ((long long)h * p.nsplit + split) * NQT;
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        float mstar = -__builtin_inff();
        for (int ww = 0; ww < NW; ++ww) mstar = fmaxf(mstar, lml[((ww * NQT + qt) * 16 + col) * 2]);
        const float m_use = mstar == -__builtin_inff() ? 0.f : mstar;
        float f[NW];
        float lsum = 0.f;
        for (int ww = 0; ww < NW; ++ww) {
            f[ww] = exp2f(lml[((ww * NQT + qt) * 16 + col) * 2] - m_use);
            lsum += f[ww] * lml[((ww * NQT + qt) * 16 + col) * 2 + 1];
        }
        for (int dt = w; dt < 8; dt += NW) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            for (int ww = 0; ww < NW; ++ww) acc += lo[((ww * NQT + qt) * 8 + dt) * 64 + lane] * f[ww];
            reinterpret_cast<f32x4 *>(p.part_o)[((pbase + qt) * 8 + dt) * 64 + lane] = acc;
        }
        if (w == 0 && g4 == 0) {
            p.part_ml[((pbase + qt) * 16 + col) * 2 + 0] = mstar;
            p.part_ml[((pbase + qt) * 16 + col) * 2 + 1] = lsum;
        }
    }
}

// Combine the splits: one workgroup of 512 threads per (kv head, query tile, 16-d output tile);
// the 8 waves share the splits (wave g takes splits g, g + 8, ...) and meet twice in LDS: for
// the maximum over all splits, then for the sums (added in wave order: a fixed order).
__global__ __launch_bounds__(512) void attention_merge_kernel(const AttnParams p, int NQT) {
    __shared__ float smax[8][16];
    __shared__ float slsum[8][16];
    __shared__ f32x4 sacc[8][64];
    const int dt = blockIdx.x & 7, qt = (blockIdx.x >> 3) % NQT, h = (blockIdx.x >> 3) / NQT;
    const int sg = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g4 = lane >> 4, col = lane & 15;
    const int r = p.row0 + 16 * qt + col;
    float lmax = -__builtin_inff();
    for (int s = sg; s < p.nsplit; s += 8)
        lmax = fmaxf(lmax, p.part_ml[((((long long)h * p.nsplit + s) * NQT + qt) * 16 + col) * 2]);
    if (g4 == 0) smax[sg][col] = lmax;
    __syncthreads();
    float mstar = smax[0][col];
#pragma unroll
    for (int i = 1; i < 8; ++i) mstar = fmaxf(mstar, smax[i][col]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float lsum = 0.f;
    for (int s = sg; s < p.nsplit; s += 8) {
        const long long pb = ((long long)h * p.nsplit + s) * NQT + qt;
        const float f = exp2f(p.part_ml[(pb * 16 + col) * 2] - mstar);
        lsum += f * p.part_ml[(pb * 16 + col) * 2 + 1];
        acc += reinterpret_cast<const f32x4 *>(p.part_o)[(pb * 8 + dt) * 64 + lane] * f;
    }
    sacc[sg][lane] = acc;
    if (g4 == 0) slsum[sg][col] = lsum;
    __syncthreads();
    if (sg != 0 || r >= p.M * p.G) return;
#pragma unroll
    for (int i = 1; i < 8; ++i) {
        acc += sacc[i][lane];
        lsum += slsum[i][col];
    }
    const float inv = __fdiv_rn(1.0f, lsum);
    const int m = r / p.G, g = r % p.G;
    u32x2 o;
    o.x = float_to_bf16_bits(acc.x * inv) | (float_to_bf16_bits(acc.y * inv) << 16);
    o.y = float_to_bf16_bits(acc.z * inv) | (float_to_bf16_bits(acc.w * inv) << 16);
    *reinterpret_cast<u32x2 *>(p.out + m * p.ldo + ((long long)h * p.G + g) * kHeadDim + 16 * dt + 4 * g4) = o;
}

}  // namespace quasar
