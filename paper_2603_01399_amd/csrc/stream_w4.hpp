// 4-bit group-wise weights x bf16 activations: the weight-streaming contraction with half a
// byte per weight (gfx950).
//
// Packed order: a step is 1056 contiguous bytes, 16 weight rows x one group of 128 input
// channels: 1024 bytes of codes (one wave-wide 128-bit load) followed by the 16 bf16 step
// sizes of the rows for this group.  Lane l = 16*g + i of the load holds row i; its dword j
// (j = 0..3) holds the eight codes of k = 32 j + 8 g + e, e = 0..7, code + 8 in nibble
// (e >> 1) + 4 (e & 1).  With that nibble order, (dword >> 4 t) & 0x000F000F, t = 0..3, or-ed
// with 0x43004300 is a pair of bf16 values 128 + (code + 8) for e = 2 t and 2 t + 1: two
// instructions per pair, no sign handling.  The constant 136 is taken out again inside the
// matrix instruction: the accumulator of a group starts at -136 * (sum of the group's
// activations), computed once per staged chunk in fp32.
//
// Per slot: 4 MFMA (16 rows x 32 k each) into a group accumulator, then four fused
// multiply-adds with the rows' step sizes into the running sums (Eq. 8 inside the group,
// Eq. 10 per group).  Work split, ring discipline and the tile-end sum are those of the
// 8-bit kernel.
#pragma once

#include "stream_gemm.hpp"

namespace quasar {

constexpr int kStepK4 = 128;         // k extent of a 4-bit step = the quantisation group
constexpr int kStepBytes4 = 1056;    // 1024 B of codes + 16 bf16 step sizes
constexpr unsigned int kW4Magic = 0x43004300u;   // bf16 128.0 twice
constexpr float kW4Offset = 136.0f;  // 128 from the magic exponent + 8 from the stored code

typedef const __attribute__((address_space(1))) u32x2 *global_u32x2_ptr;

__device__ __forceinline__ u32x2 ring_refill2(const u32x2 *addr, const u32x2 &used) {
    unsigned long long a = reinterpret_cast<unsigned long long>(addr);
    asm volatile("" : "+v"(a) : "v"(used.x), "v"(used.y));
    return __builtin_nontemporal_load(reinterpret_cast<global_u32x2_ptr>(a));
}

// one dword of eight 4-bit codes -> eight bf16 values 136 + code, in k order.  mask and magic
// arrive in registers (see w4_constants): with literals the compiler needs an AND and an OR
// per pair, with registers it has the three-operand and-or.
__device__ __forceinline__ bf16x8 w4_to_bf16x8(unsigned int w, unsigned int mask, unsigned int magic) {
    u32x4 r;
    r.x = (w & mask) | magic;
    r.y = ((w >> 4) & mask) | magic;
    r.z = ((w >> 8) & mask) | magic;
    r.w = ((w >> 12) & mask) | magic;
    return __builtin_bit_cast(bf16x8, r);
}
// the two constants of w4_to_bf16x8, made opaque to constant folding: the mask in a scalar
// register, the magic pair in a vector register
__device__ __forceinline__ void w4_constants(unsigned int &mask, unsigned int &magic) {
    mask = 0x000F000Fu;
    magic = kW4Magic;
    asm volatile("" : "+s"(mask));
    asm volatile("" : "+v"(magic));
}

// LDS: [activation chunk: [k/8][token] 16 B][group offsets: [step][token] f32x4]
//      [2 x NW staging tiles][tile sums (C > 1)]
// p.xs_bytes covers the first two; p.sc_bytes is 0.
template <int MP, int EPI, int NW, int D>
__global__ __launch_bounds__(NW * 64) void stream_w4_kernel(const GemmParams p) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int NB = (MP == 32) ? 2 : 1;
    constexpr int PPS = 16;                  // 16-byte activation pieces (8 k) per step
    constexpr int LMP = (MP == 8) ? 3 : (MP == 16 ? 4 : 5);
    constexpr int XB = 8;
    constexpr int nthreads = NW * 64;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, mcol = lane & 15;

    const int G = gridDim.x, b = blockIdx.x;
    const int t0 = (int)(((long long)p.T * b) / G);
    const int t1 = (int)(((long long)p.T * (b + 1)) / G);
    const int ntiles = t1 - t0;

    u32x4 *xs = reinterpret_cast<u32x4 *>(lds);                                   // [SC*PPS][MP]
    f32x4 *gofs = reinterpret_cast<f32x4 *>(lds + p.SC * PPS * MP * 16);          // [SC][MP]
    f32x4 *stage = reinterpret_cast<f32x4 *>(lds + p.xs_bytes);                   // [2][NW][NB][64]
    f32x4 *accs = stage + 2 * NW * NB * 64;                                       // [ntiles][NB][64] (C > 1)

    auto x_piece_load = [&](int c, int idx) -> u32x4 {
        const int scc = min(p.SC, p.S - c * p.SC);
        const int npieces = scc * PPS * MP;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (idx < npieces) {
            const int m = idx & (MP - 1), p8 = idx >> LMP;
            if (m < p.M) {
                const long long k = (long long)c * p.SC * kStepK4 + 8ll * p8;
                v = *reinterpret_cast<const u32x4 *>(p.x + m * p.ldx + k);
            }
        }
        return v;
    };
    auto x_stage = [&](int c, int first_batch) {
        const int scc = min(p.SC, p.S - c * p.SC);
        const int npieces = scc * PPS * MP;
        for (int base = first_batch * nthreads * XB; base < npieces; base += nthreads * XB) {
            u32x4 v[XB];
#pragma unroll
            for (int i = 0; i < XB; ++i) v[i] = x_piece_load(c, base + i * nthreads + tid);
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                if (idx < npieces) xs[idx] = v[i];
            }
        }
    };
    // -136 * (sum of a group's activations) per (step of the chunk, token), four copies so that
    // one LDS read fills the accumulator the group's first matrix instruction starts from
    auto group_offsets = [&](int c) {
        const int scc = min(p.SC, p.S - c * p.SC);
        for (int idx = tid; idx < scc * MP; idx += nthreads) {
            const int m = idx & (MP - 1), s = idx >> LMP;
            float sum = 0.f;
#pragma unroll 4
            for (int j = 0; j < PPS; ++j) {
                const u32x4 v = xs[(s * PPS + j) * MP + m];
                sum += __uint_as_float(v.x << 16);
                sum += __uint_as_float(v.x & 0xFFFF0000u);
                sum += __uint_as_float(v.y << 16);
                sum += __uint_as_float(v.y & 0xFFFF0000u);
                sum += __uint_as_float(v.z << 16);
                sum += __uint_as_float(v.z & 0xFFFF0000u);
                sum += __uint_as_float(v.w << 16);
                sum += __uint_as_float(v.w & 0xFFFF0000u);
            }
            const float o = -kW4Offset * sum;
            gofs[idx] = f32x4{o, o, o, o};
        }
    };

    WaveWalk<NW, D> walk{p, w, lane, t0, ntiles};
    typename WaveWalk<NW, D>::Front ld;
    walk.begin(ld);
    // byte address of a slot's step (codes at + 16 lane, step sizes at + 1024 + 8 g); slots
    // without a step read the first bytes of the activations, a line every compute unit holds
    const unsigned char *wbytes = reinterpret_cast<const unsigned char *>(p.w);
    auto slot_base = [&](const typename WaveWalk<NW, D>::Front &f, int &code_off, int &scale_off) {
        const long long step = (long long)(t0 + f.tl) * p.Srow + (long long)f.c * p.SC + f.s_lo + f.si;
        const bool real = walk.real(f);
        code_off = real ? 16 * lane : 0;
        scale_off = real ? 1024 + 8 * g : 0;
        return real ? wbytes + step * kStepBytes4 : reinterpret_cast<const unsigned char *>(p.x);
    };

    // requests in the order they are needed back: first activation batch, then the ring
    u32x4 xfirst[XB];
#pragma unroll
    for (int i = 0; i < XB; ++i) xfirst[i] = x_piece_load(0, i * nthreads + tid);
    u32x4 ring[D];
    u32x2 sring[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        int co, so;
        const unsigned char *base = slot_base(ld, co, so);
        ring[d] = ring_refill(reinterpret_cast<const u32x4 *>(base + co), u32x4{0u, 0u, 0u, 0u});
        sring[d] = ring_refill2(reinterpret_cast<const u32x2 *>(base + so), u32x2{0u, 0u});
        walk.advance(ld);
    }
    {
        const int npieces = min(p.SC, p.S) * PPS * MP;
#pragma unroll
        for (int i = 0; i < XB; ++i) {
            const int idx = i * nthreads + tid;
            if (idx < npieces) xs[idx] = xfirst[i];
        }
        x_stage(0, 1);
        lds_barrier();
        group_offsets(0);
        lds_barrier();
    }

    f32x4 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    float bestv[NB];
    unsigned int besti[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) { bestv[nb] = -__builtin_inff(); besti[nb] = 0x7FFFFFFFu; }
    int parity = 0;
    const int xm = (MP == 8) ? (mcol & 7) : mcol;   // token slot read by this lane
    unsigned int nib_mask, nib_magic;
    w4_constants(nib_mask, nib_magic);

    for (int c = 0; c < p.C; ++c) {
        if (c > 0) {
            // every wave has passed the previous chunk's last tile barrier: the chunk's
            // activations are no longer read
            x_stage(c, 0);
            // full drain: the staging loads are conditional, and without a known-empty load
            // queue here the compiler would fall back to draining the ring on every round
            __builtin_amdgcn_s_waitcnt(0x0F70);
            lds_barrier();
            group_offsets(c);
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
                const u32x4 wv = ring[d];
                u32x2 sv = sring[d];
                if (!valid) sv = u32x2{0u, 0u};      // step sizes 0: the slot contributes nothing
                const int step_in_chunk = valid ? cs.s_lo + si : 0;
                const int piece0 = step_in_chunk * PPS;
                f32x4 accg[NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) accg[nb] = gofs[step_in_chunk * MP + xm + 16 * nb];
                const unsigned int wd[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bf16x8 a = w4_to_bf16x8(wd[j], nib_mask, nib_magic);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const u32x4 bx = xs[(piece0 + 4 * j + g) * MP + xm + 16 * nb];
                        accg[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bx),
                                                                           accg[nb], 0, 0, 0);
                    }
                }
                {
                    int co, so;
                    const unsigned char *base = slot_base(ld, co, so);
                    ring[d] = ring_refill(reinterpret_cast<const u32x4 *>(base + co), wv);
                    sring[d] = ring_refill2(reinterpret_cast<const u32x2 *>(base + so), sv);
                    walk.advance(ld);
                }
                {
                    const float s0 = __uint_as_float(sv.x << 16), s1 = __uint_as_float(sv.x & 0xFFFF0000u);
                    const float s2 = __uint_as_float(sv.y << 16), s3 = __uint_as_float(sv.y & 0xFFFF0000u);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        acc[nb].x = __builtin_fmaf(s0, accg[nb].x, acc[nb].x);
                        acc[nb].y = __builtin_fmaf(s1, accg[nb].y, acc[nb].y);
                        acc[nb].z = __builtin_fmaf(s2, accg[nb].z, acc[nb].z);
                        acc[nb].w = __builtin_fmaf(s3, accg[nb].w, acc[nb].w);
                    }
                }
                if (in_range && si == cs.nsl - 1) {
                    // ---- tile end: cross-wave sum through LDS, fixed order
                    f32x4 *st = stage + (parity * NW) * NB * 64;
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        st[(w * NB + nb) * 64 + lane] = acc[nb];
                        acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                    lds_barrier();
                    if (w == (tl % NW)) {
                        f32x4 rsum[NB];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            rsum[nb] = st[nb * 64 + lane];
#pragma unroll
                            for (int ww = 1; ww < NW; ++ww) rsum[nb] += st[(ww * NB + nb) * 64 + lane];
                            if (p.C > 1) {
                                f32x4 *a = accs + (tl * NB + nb) * 64 + lane;
                                if (c > 0) rsum[nb] += *a;
                                if (c < p.C - 1) *a = rsum[nb];
                            }
                        }
                        if (c == p.C - 1) {
                            const int n0 = (t0 + tl) * kTileRows + 4 * g;
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb) {
                                const int m = mcol + 16 * nb;
                                const float v0 = rsum[nb].x, v1 = rsum[nb].y, v2 = rsum[nb].z, v3 = rsum[nb].w;
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
        // per wave: combine the four k-groups' row subsets, then combine waves, then publish
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
