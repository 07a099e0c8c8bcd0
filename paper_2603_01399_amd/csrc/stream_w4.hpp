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
// A slot of the per-wave sequence is one k-step of a PAIR of neighbouring tiles of the
// workgroup (the second of the pair is a dummy with step sizes 0 when the workgroup's tile
// count is odd): two code loads and two step-size loads, 2 x 4 MFMA (16 rows x 32 k each)
// into two group accumulators that read the same activations from LDS once, then fused
// multiply-adds with the rows' step sizes into the running sums (Eq. 8 inside the group,
// Eq. 10 per group).  Per weight byte that halves the LDS reads, the scalar bookkeeping and
// the tile-end barriers of a one-tile slot; with 4 bits per weight those, not the memory
// system, are what limits the rate.  Addresses advance by constants (no multiplications per
// slot).  Work split over the waves, ring discipline and the fixed-order tile-end sum are
// those of the 8-bit kernel.
#pragma once

#include "stream_gemm.hpp"

namespace quasar {

constexpr int kStepK4 = 128;         // k extent of a 4-bit step = the quantisation group
constexpr int kStepBytes4 = 1056;    // 1024 B of codes + 16 bf16 step sizes
constexpr unsigned int kW4Magic = 0x43004300u;   // bf16 128.0 twice
constexpr float kW4Offset = 136.0f;  // 128 from the magic exponent + 8 from the stored code

typedef const __attribute__((address_space(1))) u32x2 *global_u32x2_ptr;

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

// 64-bit ring refill with a wave-uniform base address (scalar registers) and a per-lane byte
// offset; the address is tied to the registers just consumed, as in ring_refill_at
__device__ __forceinline__ u32x2 ring_refill2_at(unsigned long long base, unsigned int &lane_offset, const u32x2 &used) {
    asm volatile("" : "+v"(lane_offset) : "v"(used.x), "v"(used.y));
    return __builtin_nontemporal_load(reinterpret_cast<global_u32x2_ptr>(base + lane_offset));
}

// LDS: [activation chunk: token rows, token m at m * (row bytes + 16), fetched straight from memory][group
//      offsets: [step][token] f32x4]
//      [PAR x NW x 2 staging tiles][pair sums (C > 1)]
// p.xs_bytes covers the first two; p.sc_bytes is 0.  PAR = 2 staging areas used alternately
// (one barrier per pair) when they fit, else one area and a second barrier.
template <int MP, int EPI, int NW, int D>
__global__ __launch_bounds__(NW * 64) void stream_w4_kernel(const GemmParams p) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int NB = (MP == 32) ? 2 : 1;
    constexpr int PAR = (NB == 1) ? 2 : 1;
    constexpr int PPS = 16;                  // 16-byte activation pieces (8 k) per step
    constexpr int LMP = (MP == 8) ? 3 : (MP == 16 ? 4 : 5);
    constexpr int nthreads = NW * 64;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, mcol = lane & 15;

    const int G = gridDim.x, b = blockIdx.x;
    const int t0 = tile_split(p.T, b, G);
    const int t1 = tile_split(p.T, b + 1, G);
    const int ntiles = t1 - t0;
    const int npairs = (ntiles + 1) >> 1;

    // activations: 16-byte piece p8 (8 k) of token m at m * x_rs + 16 * p8 (the 16-byte skew keeps the tokens of
    // one column in different banks); one direct-to-LDS load instruction moves 1 KB that is contiguous in memory
    // and in LDS - instruction j is 1 KB piece j / MP of token j % MP, wave w takes j = w, w + NW, ...
    const unsigned int x_rs = (unsigned int)(p.SC * kStepK4 * 2 + 16);
    auto xq = [&](int p8, int m) -> u32x4 {
        return *reinterpret_cast<const u32x4 *>(lds + (unsigned int)m * x_rs + (unsigned int)p8 * 16u);
    };
    f32x4 *gofs = reinterpret_cast<f32x4 *>(lds + MP * x_rs);                      // [SC][MP]
    f32x4 *stage = reinterpret_cast<f32x4 *>(lds + p.xs_bytes);                   // [PAR][NW][2][NB][64]
    f32x4 *accs = stage + PAR * NW * 2 * NB * 64;                                 // [npairs][2][NB][64] (C > 1)

    auto x_stage = [&](int c) {
        const unsigned int lds_base = lds_address_of(lds);
        const int rowbytes = min(p.SC, p.S - c * p.SC) * kStepK4 * 2;
        const int ninstr = ((rowbytes + 1023) >> 10) * MP;
        const unsigned long long x0 = reinterpret_cast<unsigned long long>(p.x) + 2ull * (unsigned long long)c * p.SC * kStepK4;
        const unsigned long long ld2 = (unsigned long long)p.ldx * 2ull;
        for (int j = w; j < ninstr; j += NW) {
            const int m = j & (MP - 1), i = j >> LMP;
            const unsigned long long gb = x0 + (unsigned long long)min(m, p.M - 1) * ld2 + (unsigned long long)i * 1024ull;
            const unsigned int glo = __builtin_amdgcn_readfirstlane((unsigned int)gb);
            const unsigned int ghi = __builtin_amdgcn_readfirstlane((unsigned int)(gb >> 32));
            const unsigned long long gbase = ((unsigned long long)ghi << 32) | glo;
            const unsigned int laddr = __builtin_amdgcn_readfirstlane(lds_base + (unsigned int)m * x_rs + (unsigned int)i * 1024u);
            if (i * 1024 + 1024 <= rowbytes) load_to_lds_16(gbase, (unsigned int)lane * 16u, laddr);
            else if (i * 1024 + lane * 16 < rowbytes) load_to_lds_16(gbase, (unsigned int)lane * 16u, laddr);
        }
    };
    // -136 * (sum of a group's activations) per (step of the chunk, token), four copies so that
    // one LDS read fills the accumulator the group's first matrix instruction starts from.
    // Four neighbouring lanes share a (step, token): each sums four of its 16 pieces, two
    // shuffles combine them (a fixed order).
    auto group_offsets = [&](int c) {
        const int scc = min(p.SC, p.S - c * p.SC);
        const int total = ((scc * MP * 4 + nthreads - 1) / nthreads) * nthreads;   // whole waves take the shuffles
        for (int idx4 = tid; idx4 < total; idx4 += nthreads) {
            const int q = idx4 & 3, idx = idx4 >> 2;
            const int m = idx & (MP - 1), s = idx >> LMP;
            float sum = 0.f;
            if (idx < scc * MP) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const u32x4 v = xq(s * PPS + 4 * q + j, m);
                    sum += __uint_as_float(v.x << 16);
                    sum += __uint_as_float(v.x & 0xFFFF0000u);
                    sum += __uint_as_float(v.y << 16);
                    sum += __uint_as_float(v.y & 0xFFFF0000u);
                    sum += __uint_as_float(v.z << 16);
                    sum += __uint_as_float(v.z & 0xFFFF0000u);
                    sum += __uint_as_float(v.w << 16);
                    sum += __uint_as_float(v.w & 0xFFFF0000u);
                }
            }
            sum += __shfl_xor(sum, 1, 64);
            sum += __shfl_xor(sum, 2, 64);
            if (q == 0 && idx < scc * MP) {
                const float o = -kW4Offset * sum;
                gofs[idx] = f32x4{o, o, o, o};
            }
        }
    };

    // ---- load front: the (chunk, pair, step) position the next ring refill belongs to.  The
    // address of tile A's step advances by constants; tile B's step lies one tile (Srow steps)
    // further, or is tile A's again when the pair has no second tile.  Slots without a step
    // (padding, waves without a share) read 16 (8) bytes of the workgroup's own first step, all
    // lanes the same ones: one cache line per wave, in a region the workgroup reads anyway.
    const unsigned long long wbase = reinterpret_cast<unsigned long long>(p.w);
    const unsigned long long idle_addr = wbase + (unsigned long long)t0 * p.Srow * kStepBytes4 + 64u * w;
    const unsigned int tile_bytes = (unsigned int)p.Srow * (unsigned int)kStepBytes4;
    struct LoadFront {
        int c, idx, si, pr, items, padded, nsl;
        bool has;
        unsigned long long addr;
        unsigned int bofs;
    };
    auto lf_slice = [&](LoadFront &f) {
        const int scc = min(p.SC, p.S - f.c * p.SC);
        const int s_lo = (scc * w) / NW;
        const int spw = (scc * (w + 1)) / NW - s_lo;
        f.nsl = max(spw, 1);
        f.has = spw > 0;
        f.items = npairs * f.nsl;
        f.padded = ((f.items + D - 1) / D) * D;
        f.idx = 0; f.si = 0; f.pr = 0;
        f.addr = wbase + ((unsigned long long)t0 * p.Srow + (unsigned long long)f.c * p.SC + s_lo) * kStepBytes4;
        f.bofs = ntiles > 1 ? tile_bytes : 0u;
    };
    auto lf_advance = [&](LoadFront &f) {
        ++f.idx;
        ++f.si;
        f.addr += kStepBytes4;
        if (f.si == f.nsl) {
            f.si = 0;
            ++f.pr;
            f.addr += (unsigned long long)(2 * p.Srow - f.nsl) * kStepBytes4;
            f.bofs = (2 * f.pr + 1 < ntiles) ? tile_bytes : 0u;
        }
        if (f.idx == f.padded) {
            ++f.c;
            if (f.c < p.C) lf_slice(f);
            else { f.items = 0; f.padded = D; f.nsl = 1; f.has = false; f.idx = 0; f.si = 0; f.pr = 0; }
        }
    };
    const unsigned int off_codes = 16u * lane, off_scales = 1024u + 8u * g;

    LoadFront ld;
    ld.c = 0;
    lf_slice(ld);

    // requests in the order they are needed back: the activations (straight into LDS), then the ring
    x_stage(0);
    u32x4 ringA[D], ringB[D];
    u32x2 sclA[D], sclB[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        const bool real = ld.has && ld.idx < ld.items;
        const unsigned long long a = real ? ld.addr : idle_addr;
        const unsigned long long bb = a + (real ? ld.bofs : 0u);
        unsigned int oc = real ? off_codes : 0u, os = real ? off_scales : 0u;
        ringA[d] = ring_refill_at(a, oc, u32x4{0u, 0u, 0u, 0u});
        ringB[d] = ring_refill_at(bb, oc, u32x4{0u, 0u, 0u, 0u});
        sclA[d] = ring_refill2_at(a, os, u32x2{0u, 0u});
        sclB[d] = ring_refill2_at(bb, os, u32x2{0u, 0u});
        lf_advance(ld);
    }
    {
        // loads return in order: once no more than the 4 D ring loads are outstanding, this wave's share of the
        // activations is in LDS
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(4 * D) : "memory");
        lds_barrier();
        group_offsets(0);
        lds_barrier();
    }

    f32x4 accA[NB], accB[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) accA[nb] = accB[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
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
            // every wave has passed the previous chunk's last pair barrier: the chunk's
            // activations are no longer read
            x_stage(c);
            // full drain: the staging loads are conditional, and without a known-empty load
            // queue here the compiler would fall back to draining the ring on every round
            __builtin_amdgcn_s_waitcnt(0x0F70);
            lds_barrier();
            group_offsets(c);
            lds_barrier();
        }
        const int scc = min(p.SC, p.S - c * p.SC);
        const int s_lo = (scc * w) / NW;
        const int spw = (scc * (w + 1)) / NW - s_lo;
        const int nsl = max(spw, 1);
        const bool has = spw > 0;
        const int items = npairs * nsl;
        const int rounds = (items + D - 1) / D;
        int pr = 0, si = 0;
        for (int r = 0; r < rounds; ++r) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const int idx = r * D + d;
                const bool in_range = idx < items;
                const bool valid = in_range && has;
                const bool validB = valid && (2 * pr + 1 < ntiles);
                const u32x4 wA = ringA[d], wB = ringB[d];
                u32x2 svA = sclA[d], svB = sclB[d];
                if (!validB) svB = u32x2{0u, 0u};      // no second tile: step sizes 0, it contributes nothing
                if (valid) {
                    // slots without a step skip the arithmetic (a wave-uniform branch); their loads
                    // below are still issued, one per ring entry and slot
                    const int step_in_chunk = s_lo + si;
                    const int piece0 = step_in_chunk * PPS;
                    f32x4 gA[NB], gB[NB];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) gA[nb] = gB[nb] = gofs[step_in_chunk * MP + xm + 16 * nb];
                    const unsigned int wdA[4] = {wA.x, wA.y, wA.z, wA.w};
                    const unsigned int wdB[4] = {wB.x, wB.y, wB.z, wB.w};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const bf16x8 aA = w4_to_bf16x8(wdA[j], nib_mask, nib_magic);
                        const bf16x8 aB = w4_to_bf16x8(wdB[j], nib_mask, nib_magic);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            const bf16x8 bx = __builtin_bit_cast(bf16x8, xq(piece0 + 4 * j + g, xm + 16 * nb));
                            gA[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aA, bx, gA[nb], 0, 0, 0);
                            gB[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aB, bx, gB[nb], 0, 0, 0);
                        }
                    }
                    const float a0 = __uint_as_float(svA.x << 16), a1 = __uint_as_float(svA.x & 0xFFFF0000u);
                    const float a2 = __uint_as_float(svA.y << 16), a3 = __uint_as_float(svA.y & 0xFFFF0000u);
                    const float b0 = __uint_as_float(svB.x << 16), b1 = __uint_as_float(svB.x & 0xFFFF0000u);
                    const float b2 = __uint_as_float(svB.y << 16), b3 = __uint_as_float(svB.y & 0xFFFF0000u);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        accA[nb].x = __builtin_fmaf(a0, gA[nb].x, accA[nb].x);
                        accA[nb].y = __builtin_fmaf(a1, gA[nb].y, accA[nb].y);
                        accA[nb].z = __builtin_fmaf(a2, gA[nb].z, accA[nb].z);
                        accA[nb].w = __builtin_fmaf(a3, gA[nb].w, accA[nb].w);
                        accB[nb].x = __builtin_fmaf(b0, gB[nb].x, accB[nb].x);
                        accB[nb].y = __builtin_fmaf(b1, gB[nb].y, accB[nb].y);
                        accB[nb].z = __builtin_fmaf(b2, gB[nb].z, accB[nb].z);
                        accB[nb].w = __builtin_fmaf(b3, gB[nb].w, accB[nb].w);
                    }
                }
                {
                    const bool real = ld.has && ld.idx < ld.items;
                    const unsigned long long a = real ? ld.addr : idle_addr;
                    const unsigned long long bb = a + (real ? ld.bofs : 0u);
                    unsigned int oc = real ? off_codes : 0u, os = real ? off_scales : 0u;
                    ringA[d] = ring_refill_at(a, oc, wA);
                    ringB[d] = ring_refill_at(bb, oc, wB);
                    sclA[d] = ring_refill2_at(a, os, svA);
                    sclB[d] = ring_refill2_at(bb, os, svB);
                    lf_advance(ld);
                }
                if (in_range && si == nsl - 1) {
                    // ---- pair end: cross-wave sum through LDS, fixed order
                    if constexpr (PAR == 1) lds_barrier();   // the previous pair's sums have been read
                    f32x4 *st = stage + (parity * NW) * 2 * NB * 64;
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        st[((w * 2 + 0) * NB + nb) * 64 + lane] = accA[nb];
                        st[((w * 2 + 1) * NB + nb) * 64 + lane] = accB[nb];
                        accA[nb] = accB[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                    lds_barrier();
                    if (w == (pr % NW)) {
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const int tl = 2 * pr + h;
                            if (tl < ntiles) {
                                f32x4 rsum[NB];
#pragma unroll
                                for (int nb = 0; nb < NB; ++nb) {
                                    rsum[nb] = st[(h * NB + nb) * 64 + lane];
#pragma unroll
                                    for (int ww = 1; ww < NW; ++ww) rsum[nb] += st[((ww * 2 + h) * NB + nb) * 64 + lane];
                                    if (p.C > 1) {
                                        f32x4 *a = accs + ((pr * 2 + h) * NB + nb) * 64 + lane;
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
                        }
                    }
                    if constexpr (PAR == 2) parity ^= 1;
                }
                if (in_range) {
                    ++si;
                    if (si >= nsl) { si = 0; ++pr; }
                }
            }
        }
    }

    if constexpr (EPI == EPI_ARGMAX) {
        // per wave: combine the four k-groups' row subsets, then combine waves, then publish
        unsigned long long *red = reinterpret_cast<unsigned long long *>(stage);   // [NW][MP]
        lds_barrier();   // all pair-end reads of the staging area are done
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
