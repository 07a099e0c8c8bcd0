// Persistent whole-step kernel (gfx950): a list of linear phases and a final fused
// vocabulary/argmax/acceptance phase executed by one launch of resident workgroups.
//
// Why: a single verification linear streams 4-50 MB, i.e. 1-8 microseconds of HBM time, while
// a kernel boundary costs several microseconds of launch, first-load latency and drain.  Inside
// one persistent kernel the weight stream never stops: weight addresses do not depend on the
// activations, so every wave's load ring runs ahead into the next phase while the workgroups
// meet at a grid barrier and re-stage the new activations.
//
// A phase is a group of linears that share their input (q|k|v, gate|up) and therefore need no
// ordering among themselves; its weight tiles are numbered across the member matrices
// ("segments") and split evenly over the workgroups.
#pragma once

#include "stream_gemm.hpp"

namespace quasar {

constexpr int kMaxSeg = 4;

struct SeqSeg {
    const u32x4 *w;          // packed weights of this member matrix
    const uint16_t *scales;  // [N] (nullptr for bf16 weights)
    uint16_t *y;             // [M, N] output, row stride ldy
    long long ldy;
    int tile_begin;          // index of the segment's first tile inside the phase
    int pad_;
};

struct SeqPhase {
    const uint16_t *x;       // [M, K] input shared by all segments
    long long ldx;
    SeqSeg seg[kMaxSeg];
    int nseg;
    int T;                   // tiles over all segments
    int K, S, SC, C;         // as in GemmParams
    int kind;                // EPI_LINEAR or EPI_ARGMAX (argmax: one segment)
    int sync_before;         // the input is produced by an earlier phase of this launch
    const int32_t *draft;
    int32_t *out_argmax;
    int32_t *out_accept;
    int n_draft;
    int V;
};

typedef const __attribute__((address_space(4))) SeqPhase *const_phase_ptr;   // scalar (constant) loads

// Pointers read out of the phase table are generic; data accesses go through the global
// address space so that they compile to global (not flat) memory instructions.
template <typename T>
__device__ __forceinline__ __attribute__((address_space(1))) T *as_global(T *p) {
    return reinterpret_cast<__attribute__((address_space(1))) T *>(reinterpret_cast<unsigned long long>(p));
}

struct SeqParams {
    const SeqPhase *phases;  // device memory, never written while the kernel runs
    int nphases;
    int M;
    int xs_bytes;            // LDS reserved for activations (max over phases)
    int sc_bytes;            // LDS reserved for row scales (max over phases)
    unsigned int *sync;      // [0] arrival counter (zero at launch), [1] error flag (zero at launch)
    unsigned long long *partial;   // argmax phase: [gridDim.x][MP] packed (logit, index) keys
    unsigned int spin_limit; // bound on barrier polling iterations
};

// Data that crosses a grid barrier inside the launch (outputs of one phase read as the input
// of a later one, argmax partials) is written and read with device-coherent accesses that go
// past the per-XCD L2 caches.  That makes cache write-back / invalidate at the barrier
// unnecessary; on this part those maintenance operations cost more than the barrier itself.
__device__ __forceinline__ void coherent_store_u64(void *p, unsigned long long v) {
    __hip_atomic_store(as_global(static_cast<unsigned long long *>(p)), v, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long coherent_load_u64(const void *p) {
    return __hip_atomic_load(as_global(static_cast<const unsigned long long *>(p)), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u32x4 coherent_load_u32x4(const void *p) {
    const unsigned long long lo = coherent_load_u64(p);
    const unsigned long long hi = coherent_load_u64(static_cast<const unsigned long long *>(p) + 1);
    return u32x4{(unsigned int)lo, (unsigned int)(lo >> 32), (unsigned int)hi, (unsigned int)(hi >> 32)};
}

// All workgroups of the launch meet.  Every wave first waits until its own (coherent) stores
// have been acknowledged, so whatever the workgroup wrote is readable device-wide once the
// arrival counter has been bumped.  Polling is bounded: on timeout the error flag is raised
// and every later barrier falls through, so the grid always drains.
__device__ __forceinline__ void grid_barrier(unsigned int *sync, unsigned int target, unsigned int spin_limit) {
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    lds_barrier();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(as_global(&sync[0]), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned int n = 0;
        while (__hip_atomic_load(as_global(&sync[0]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (__hip_atomic_load(as_global(&sync[1]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            if (++n > spin_limit) {
                __hip_atomic_store(as_global(&sync[1]), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    lds_barrier();
}

template <int MP, bool W16, int NW, int D>
__global__ __launch_bounds__(NW * 64) void stream_sequence_kernel(const SeqParams sp) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int NB = (MP == 32) ? 2 : 1;
    constexpr int PPS = W16 ? 4 : 8;
    constexpr int LMP = (MP == 8) ? 3 : (MP == 16 ? 4 : 5);
    constexpr int KSTEP = W16 ? kStepK16 : kStepK8;
    constexpr int XB = 4;
    constexpr int nthreads = NW * 64;

    static_assert(NW == 16, "the in-kernel second stage of the verify phase assumes 1024 threads");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, mcol = lane & 15;
    const int G = gridDim.x, b = blockIdx.x;
    const int M = sp.M;
    const const_phase_ptr phases = (const_phase_ptr)(unsigned long long)sp.phases;

    u32x4 *xs = reinterpret_cast<u32x4 *>(lds);
    uint16_t *sc_lds = reinterpret_cast<uint16_t *>(lds + sp.xs_bytes);
    f32x4 *stage = reinterpret_cast<f32x4 *>(lds + sp.xs_bytes + sp.sc_bytes);   // [2][NW][NB][64]
    f32x4 *accs = stage + 2 * NW * NB * 64;                                      // [ntiles][NB][64] (C > 1)

    // ---- position in the (phase, chunk, tile, step) sequence of this wave
    struct Front {
        int ph, c, idx, tl, si;          // position
        int t0, ntiles;                  // this workgroup's tile range in phase ph
        int s_lo, spw, nsl, items, padded;
    };
    auto tile_range = [&](const auto &P, int &t0, int &ntiles) {
        t0 = (int)(((long long)P.T * b) / G);
        ntiles = (int)(((long long)P.T * (b + 1)) / G) - t0;
    };
    auto slice = [&](const auto &P, Front &f) {
        const int scc = min(P.SC, P.S - f.c * P.SC);
        f.s_lo = (scc * w) / NW;
        f.spw = (scc * (w + 1)) / NW - f.s_lo;
        f.nsl = max(f.spw, 1);
        f.items = f.ntiles * f.nsl;
        f.padded = ((f.items + D - 1) / D) * D;
    };
    // skip forward over (phase, chunk) pairs that have no slots for this workgroup
    auto settle = [&](Front &f) {
        while (f.ph < sp.nphases) {
            const auto &P = phases[f.ph];
            if (f.c == 0) tile_range(P, f.t0, f.ntiles);
            if (f.c < P.C) {
                slice(P, f);
                if (f.padded > 0) return;
                ++f.c;
            } else {
                ++f.ph;
                f.c = 0;
            }
        }
        f.items = 0; f.padded = 0; f.spw = 0; f.nsl = 1; f.ntiles = 0;
    };
    auto advance = [&](Front &f) {
        ++f.idx;
        ++f.si;
        if (f.si >= f.nsl) { f.si = 0; ++f.tl; }
        if (f.idx >= f.padded && f.ph < sp.nphases) {
            ++f.c; f.idx = 0; f.tl = 0; f.si = 0;
            settle(f);
        }
    };
    auto seg_of = [&](const auto &P, int t) -> int {
        int s = 0;
        if (P.nseg > 1 && t >= P.seg[1].tile_begin) s = 1;
        if (P.nseg > 2 && t >= P.seg[2].tile_begin) s = 2;
        if (P.nseg > 3 && t >= P.seg[3].tile_begin) s = 3;
        return s;
    };
    auto is_real = [&](const Front &f) -> bool {
        return f.ph < sp.nphases && f.idx < f.items && f.si < f.spw;
    };
    auto w_addr = [&](const Front &f) -> const u32x4 * {
        if (!is_real(f)) return reinterpret_cast<const u32x4 *>(phases[0].x);   // one hot line
        const auto &P = phases[f.ph];
        const int t = f.t0 + f.tl;
        const int s = seg_of(P, t);
        const long long step = (long long)(t - P.seg[s].tile_begin) * P.S + (long long)f.c * P.SC + f.s_lo + f.si;
        return P.seg[s].w + step * 64 + lane;
    };

    // ---- staging of one activation chunk and of the row scales of this workgroup's tiles
    auto x_stage = [&](const auto &P, int c) {
        const int scc = min(P.SC, P.S - c * P.SC);
        const int npieces = scc * PPS * MP;
        for (int base = 0; base < npieces; base += nthreads * XB) {
            u32x4 v[XB];
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                v[i] = u32x4{0u, 0u, 0u, 0u};
                if (idx < npieces) {
                    const int m = idx & (MP - 1), p8 = idx >> LMP;
                    if (m < M) {
                        const long long k = (long long)c * P.SC * KSTEP + 8ll * p8;
                        v[i] = coherent_load_u32x4(P.x + m * P.ldx + k);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                if (idx < npieces) xs[idx] = v[i];
            }
        }
    };
    auto scale_stage = [&](const auto &P, int t0, int ntiles) {
        if constexpr (!W16) {
            for (int i = 2 * tid; i < ntiles * kTileRows; i += 2 * nthreads) {
                const int t = t0 + (i >> 4);
                const int s = seg_of(P, t);
                const long long n = (long long)(t - P.seg[s].tile_begin) * kTileRows + (i & 15);
                reinterpret_cast<unsigned int *>(sc_lds)[i >> 1] =
                    *as_global(reinterpret_cast<const unsigned int *>(P.seg[s].scales + n));
            }
        }
    };

    Front ld;
    ld.ph = 0; ld.c = 0; ld.idx = 0; ld.tl = 0; ld.si = 0;
    settle(ld);

    u32x4 ring[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        ring[d] = ring_refill(w_addr(ld), u32x4{0u, 0u, 0u, 0u});
        advance(ld);
    }

    f32x4 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    int parity = 0;
    unsigned int barriers_done = 0;
    const int xm = (MP == 8) ? (mcol & 7) : mcol;

    for (int ph = 0; ph < sp.nphases; ++ph) {
        const auto &P = phases[ph];
        int t0, ntiles;
        tile_range(P, t0, ntiles);
        if (P.sync_before) {
            ++barriers_done;
            grid_barrier(sp.sync, barriers_done * (unsigned int)G, sp.spin_limit);
        } else {
            lds_barrier();   // the previous phase's last epilogue has read its scales
        }
        scale_stage(P, t0, ntiles);
        float bestv[NB];
        unsigned int besti[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) { bestv[nb] = -__builtin_inff(); besti[nb] = 0x7FFFFFFFu; }

        for (int c = 0; c < P.C; ++c) {
            if (ntiles > 0) {
                x_stage(P, c);
            }
            // known-empty load queue: keeps the counted waits of the ring exact (see stream_gemm.hpp)
            __builtin_amdgcn_s_waitcnt(0x0F70);
            lds_barrier();
            Front cs;
            cs.c = c; cs.t0 = t0; cs.ntiles = ntiles;
            slice(P, cs);
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
                    const int piece0 = (valid ? cs.s_lo + si : 0) * PPS;
                    if constexpr (!W16) {
                        const bf16x8 a0 = codes_to_bf16x8(wv.x, wv.y);
                        const bf16x8 a1 = codes_to_bf16x8(wv.z, wv.w);
                        ring[d] = ring_refill(w_addr(ld), wv);
                        advance(ld);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            const u32x4 b0 = xs[(piece0 + 2 * g) * MP + xm + 16 * nb];
                            const u32x4 b1 = xs[(piece0 + 2 * g + 1) * MP + xm + 16 * nb];
                            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, __builtin_bit_cast(bf16x8, b0),
                                                                              acc[nb], 0, 0, 0);
                            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, __builtin_bit_cast(bf16x8, b1),
                                                                              acc[nb], 0, 0, 0);
                        }
                    } else {
                        const bf16x8 a0 = __builtin_bit_cast(bf16x8, wv);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            const u32x4 b0 = xs[(piece0 + g) * MP + xm + 16 * nb];
                            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, __builtin_bit_cast(bf16x8, b0),
                                                                              acc[nb], 0, 0, 0);
                        }
                        ring[d] = ring_refill(w_addr(ld), wv);
                        advance(ld);
                    }
                    if (in_range && si == cs.nsl - 1) {
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
                                if (P.C > 1) {
                                    f32x4 *a = accs + (tl * NB + nb) * 64 + lane;
                                    if (c > 0) rsum[nb] += *a;
                                    if (c < P.C - 1) *a = rsum[nb];
                                }
                            }
                            if (c == P.C - 1) {
                                const int t = t0 + tl;
                                const int s = seg_of(P, t);
                                const int n0 = (t - P.seg[s].tile_begin) * kTileRows + 4 * g;
                                float s4[4] = {1.f, 1.f, 1.f, 1.f};
                                if constexpr (!W16) {
                                    const u32x2 sb =
                                        *reinterpret_cast<const u32x2 *>(sc_lds + tl * kTileRows + 4 * g);
                                    s4[0] = bf16_bits_to_float(sb.x & 0xFFFFu);
                                    s4[1] = bf16_bits_to_float(sb.x >> 16);
                                    s4[2] = bf16_bits_to_float(sb.y & 0xFFFFu);
                                    s4[3] = bf16_bits_to_float(sb.y >> 16);
                                }
#pragma unroll
                                for (int nb = 0; nb < NB; ++nb) {
                                    const int m = mcol + 16 * nb;
                                    const float v0 = rsum[nb].x * s4[0], v1 = rsum[nb].y * s4[1];
                                    const float v2 = rsum[nb].z * s4[2], v3 = rsum[nb].w * s4[3];
                                    if (P.kind == EPI_LINEAR) {
                                        if (m < M) {
                                            u32x2 o;
                                            o.x = float_to_bf16_bits(v0) | (float_to_bf16_bits(v1) << 16);
                                            o.y = float_to_bf16_bits(v2) | (float_to_bf16_bits(v3) << 16);
                                            coherent_store_u64(P.seg[s].y + m * P.seg[s].ldy + n0,
                                                               (unsigned long long)o.x | ((unsigned long long)o.y << 32));
                                        }
                                    } else {
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

        if (P.kind == EPI_ARGMAX) {
            unsigned long long *red = reinterpret_cast<unsigned long long *>(stage);   // [NW][MP]
            lds_barrier();
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
                coherent_store_u64(sp.partial + (long long)b * MP + tid, key);
            }
            ++barriers_done;
            grid_barrier(sp.sync, barriers_done * (unsigned int)G, sp.spin_limit);
            if (b == 0) {
                // second stage on one workgroup: combine the per-workgroup keys, count draft matches
                int32_t *am = reinterpret_cast<int32_t *>(stage);
                const int t32 = tid & 1023;
                const int m = t32 >> 5, sub = t32 & 31;
                unsigned long long key = 0ull;
                if (tid < 1024 && m < M)
                    for (int i = sub; i < G; i += 32) {
                        const unsigned long long o = coherent_load_u64(sp.partial + (long long)i * MP + m);
                        key = o > key ? o : key;
                    }
#pragma unroll
                for (int off = 16; off >= 1; off >>= 1) {
                    const unsigned long long o = shfl_xor_u64(key, off);
                    key = o > key ? o : key;
                }
                if (tid < 1024 && m < M && sub == 0) {
                    unsigned int idx = argmax_key_index(key);
                    if (idx >= (unsigned int)P.V) idx = 0;
                    am[m] = (int32_t)idx;
                    *as_global(P.out_argmax + m) = (int32_t)idx;
                }
                lds_barrier();
                if (tid == 0) {
                    int n = 0;
                    while (n < P.n_draft && am[n] == *as_global(P.draft + n)) ++n;
                    *as_global(P.out_accept) = n;
                }
                lds_barrier();
            }
        }
    }
}

// Clears the two sync words ahead of a sequence launch (a kernel rather than a memset so that
// callers may capture the call sequence in a graph).
__global__ void sequence_reset_kernel(unsigned int *sync) {
    if (threadIdx.x < 2) sync[threadIdx.x] = 0u;
}

}  // namespace quasar
