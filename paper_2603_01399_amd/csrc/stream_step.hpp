// Whole-step kernel with specialised waves (gfx950): the weight stream of a verification step
// (Sec. 3.4, Eq. 11-12: the model's parameters, one byte each, read once per step) executed by
// one persistent launch in which NO wave that streams weights ever waits for anything but its
// own weights and its own activations in LDS.
//
// Why a second form of the whole-step kernel: vector memory loads return to a wave in issue
// order.  A wave that keeps a deep ring of weight loads in flight therefore sees the answer to
// a completion-flag poll, or the activations it asked for, only after everything it requested
// before - up to the whole ring - and a wave that must wait for its stores also waits for its
// ring.  In stream_sequence_kernel every wave both streams and synchronises, so each of the
// four dependent hand-overs of a decoder layer stalls the stream for several memory round trips.
// Here the roles are split inside the workgroup:
//
//   compute waves (kStepNC = 8)  stream weights through a deep register ring (D x 1 KB per
//       wave), convert and multiply; they read activations from LDS and leave one fp32
//       partial tile per K slice in LDS; all their synchronisation is LDS counters.
//   stager (1 wave)  polls the completion flags of exactly those producer tiles a compute
//       wave's K slice depends on and moves that slice of the activations global -> LDS
//       (direct-to-LDS loads), slice by slice, as soon as the slice's producers are done.
//   reducers (2 waves)  sum the partial tiles in fixed order, apply the row step sizes
//       (Eq. 10), store, wait for the store acknowledgement and raise the tile's flag - or keep
//       the running argmax of the vocabulary phase and finish the acceptance count.
//   director (1 wave)  walks the phase table ahead of everybody and leaves each compute wave a
//       ring of 16-byte run descriptors (weight address, steps, position in the chunk), so that
//       the code a compute wave runs between two runs is a few instructions: that code exists once
//       per ring slot in the unrolled loop, and phase-table arithmetic there made the kernel
//       several times larger than the instruction cache.
//
// The K dimension of a tile is cut into kStepNV = 16 slices exactly as in the single-call
// kernels (stream_gemm.hpp) and the partial tiles are summed in slice order, so results are
// bit-identical to those kernels; a compute wave owns two neighbouring slices.
// Tiles are dealt round-robin (workgroup b takes tiles b, b + G, ...), flags are per tile.
#pragma once

#include "stream_sequence.hpp"

namespace quasar {

constexpr int kStepNV = 16;   // K slices (partial sums) per tile
constexpr int kStepNC = 8;    // compute waves
constexpr int kStepVPW = kStepNV / kStepNC;
constexpr int kStepNR = 2;    // reducer waves = staging buffers for partial tiles
constexpr int kStepNS = 2 + kStepNR;   // service waves: stager, reducers, director
constexpr int kStepWaves = kStepNC + kStepNS;
#ifndef STEP_PRIO
#define STEP_PRIO 3
#endif
#ifndef STEP_SLEEP
#define STEP_SLEEP 1
#endif
constexpr int kStepRD = 32;            // descriptors per compute wave's ring
constexpr int kStepCtrlBytes = 1024 + kStepNC * kStepRD * 16;   // control words, argmax keys, descriptor rings

// control block in LDS (32-bit words); everything counts upwards and is never reset
enum {
    CT_READY = 0,                    // [NC] units whose activation slice has been staged for wave w
    CT_FREED = CT_READY + kStepNC,   // [NC] units wave w has finished
    CT_POST = CT_FREED + kStepNC,    // [NR][NV] partial tiles slice v has posted into staging buffer r
    CT_CONS = CT_POST + kStepNR * kStepNV,   // [NR] tiles the reducer has read out of staging buffer r
    CT_RDONE = CT_CONS + kStepNR,    // [NR] tiles reducer r has finished (running sums written)
    CT_ABORT = CT_RDONE + kStepNR,   // a wait timed out: every later wait falls through
    CT_KEYS = CT_ABORT + 1,          // [NR] reducer r has left its argmax keys
    CT_DPROD = CT_KEYS + kStepNR,    // descriptors written per compute wave
    CT_DCONS = CT_DPROD + 1,         // [NC] descriptors compute wave w is done with
    CT_WORDS = CT_DCONS + kStepNC
};
static_assert(CT_WORDS * 4 <= 256, "the control words fit the first 256 bytes of the block");

// Control words are accessed through LDS-address-space pointers (a volatile access through a generic
// pointer would become a flat instruction, which counts as a vector memory operation and would
// make every wait of the weight ring a full drain).  The word is the same for every lane: it is
// read into a scalar so that branches on it are wave-uniform.
typedef __attribute__((address_space(3))) unsigned int lds_u32;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
// descriptor flags: first / last tile of a unit (a K chunk of a phase), end of the sequence
enum { DF_FIRST = 1u, DF_LAST = 2u, DF_END = 4u };
__device__ __forceinline__ unsigned int lds_peek(const lds_u32 *p) {
    return __builtin_amdgcn_readfirstlane(*reinterpret_cast<const volatile lds_u32 *>(p));
}
__device__ __forceinline__ void lds_poke(lds_u32 *p, unsigned int v) {
    *reinterpret_cast<volatile lds_u32 *>(p) = v;
}

__device__ __forceinline__ void lds_drain() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void vmem_drain() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ unsigned int coherent_load_u32(const unsigned int *p) {
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store_u32(unsigned int *p, unsigned int v) {
    __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16 bytes per lane from gbase + lane_offset (gbase wave-uniform), global -> LDS without passing
// through registers; lane i lands at LDS byte address lds_addr + 16 i (wave-uniform, taken from M0).  Written as
// inline assembly on purpose: when the compiler sees a direct-to-LDS load anywhere in a kernel it
// makes every LDS read wait for ALL outstanding vector memory loads (it cannot tell which loads
// write LDS), which would drain the weight ring of the compute waves at every slot.  The waits for
// these loads are therefore explicit (vmem_drain).
__device__ __forceinline__ void load_to_lds_16(unsigned long long gbase, unsigned int lane_offset, unsigned int lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(gbase), "s"(lds_addr)
                 : "memory");   // (M0 is reserved: the compiler keeps nothing in it across statements)
}
__device__ __forceinline__ unsigned int lds_address_of(const unsigned char *p) {
    return __builtin_amdgcn_readfirstlane(
        (unsigned int)(unsigned long long)((const __attribute__((address_space(3))) unsigned char *)p));
}

template <int MP, bool W16, int D>
__global__ __launch_bounds__(kStepWaves * 64) void stream_step_kernel(const SeqParams sp) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int NV = kStepNV, NC = kStepNC, VPW = kStepVPW, NR = kStepNR, RD = kStepRD;
    constexpr int NB = (MP == 32) ? 2 : 1;
    constexpr int PPS = W16 ? 4 : 8;             // 16-byte LDS pieces per step and token
    constexpr int LMP = (MP == 8) ? 3 : (MP == 16 ? 4 : 5);
    constexpr int KSTEP = W16 ? kStepK16 : kStepK8;
    constexpr int XSTEP = PPS * MP * 16;         // LDS bytes of one step of activations
    constexpr int GR = 4;                        // ring slots are refilled in groups of GR
    static_assert(D % GR == 0, "refill groups tile the ring");
    constexpr unsigned int kForever = 0x7FFFFFFFu;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, mcol = lane & 15;
    const int G = gridDim.x, b = blockIdx.x;
    const int M = sp.M;
    const int nph = sp.nphases;
    const const_phase_ptr phases = (const_phase_ptr)(unsigned long long)sp.phases;

    lds_u32 *ctrl = (lds_u32 *)(lds + sp.xs_bytes);
    lds_u32x4 *desc = (lds_u32x4 *)(lds + sp.xs_bytes + 1024);                      // [NC][RD]
    unsigned long long *keys_lds = reinterpret_cast<unsigned long long *>(lds + sp.xs_bytes + 256);   // [NR][32]
    f32x4 *stage = reinterpret_cast<f32x4 *>(lds + sp.xs_bytes + kStepCtrlBytes);   // [NR][NV][NB][64]
    f32x4 *accs = stage + NR * NV * NB * 64;                                        // [tiles][NB][64] (C > 1)

    if (tid < 256) ctrl[tid] = 0u;
    lds_barrier();

    const unsigned int epoch = __builtin_amdgcn_readfirstlane(coherent_load_u32(&sp.sync[2]));
    const unsigned int t_limit = sp.spin_limit;   // ticks of the 100 MHz clock a wait may take

    auto seg_of = [&](const auto &P, int t) -> int {
        int s = 0;
        if (P.nseg > 1 && t >= P.seg[1].tile_begin) s = 1;
        if (P.nseg > 2 && t >= P.seg[2].tile_begin) s = 2;
        if (P.nseg > 3 && t >= P.seg[3].tile_begin) s = 3;
        return s;
    };
    auto tiles_of = [&](const auto &P) -> int { return b < P.T ? (P.T - b + G - 1) / G : 0; };
    // a wait on an LDS word; bounded in time: on expiry the workgroup's abort word is set and every
    // wait of the workgroup falls through from then on, so all waves terminate
    auto lds_wait_ge = [&](const lds_u32 *p, unsigned int need) -> unsigned int {   // returns the ticks waited
        if (lds_peek(p) >= need) return 0u;
        const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
        for (;;) {
            __builtin_amdgcn_s_sleep(STEP_SLEEP);
            const unsigned int dt = (unsigned int)(__builtin_amdgcn_s_memrealtime() - t0);
            if (lds_peek(p) >= need) return dt;
            if (lds_peek(ctrl + CT_ABORT)) return dt;
            if (dt > t_limit) {
                lds_poke(ctrl + CT_ABORT, 1u);
                return dt;
            }
        }
    };
#ifdef STEP_STATS
    unsigned int st_a = 0, st_b = 0, st_c = 0, st_d = 0, st_e = 0, st_f = 0;
    const unsigned long long st_t0 = __builtin_amdgcn_s_memrealtime();
    auto stats_out = [&]() {
        if (lane == 0 && sp.stats) {
            unsigned long long *o = sp.stats + ((long long)b * kStepWaves + w) * 8;
            o[0] = __builtin_amdgcn_s_memrealtime() - st_t0; o[1] = st_a; o[2] = st_b; o[3] = st_c; o[4] = st_d; o[5] = st_e; o[6] = st_f;
        }
    };
#define ST_ADD(var, expr) var += (expr)
#else
    auto stats_out = [&]() {};
#define ST_ADD(var, expr) (void)(expr)
#endif
    // (compute waves issue nothing but weight loads, so the error word in memory is written by the
    // service waves: where their own waits expire, and when they leave)
    auto report_abort = [&]() {
        if (lds_peek(ctrl + CT_ABORT) && lane == 0) coherent_store_u32(&sp.sync[1], 1u);
    };

    if (w < NC) {
        // =================================================================== compute wave
        // Both fronts follow the wave's descriptor ring (written by the director wave): one
        // descriptor per tile of the workgroup, in execution order.
        const lds_u32x4 *my_desc = desc + w * RD;
        const unsigned long long zeros = reinterpret_cast<unsigned long long>(sp.zeros);
        auto desc_read = [&](unsigned int i) -> u32x4 {
            const u32x4 v = *reinterpret_cast<const volatile lds_u32x4 *>(my_desc + (i % RD));
            return u32x4{(unsigned int)__builtin_amdgcn_readfirstlane(v.x), (unsigned int)__builtin_amdgcn_readfirstlane(v.y),
                         (unsigned int)__builtin_amdgcn_readfirstlane(v.z), (unsigned int)__builtin_amdgcn_readfirstlane(v.w)};
        };
        // ---- load front.  It never waits: when the next descriptor has not been written yet (or the
        // sequence is over) the slot loads a block of zeros and is marked in `dummy`; the compute
        // front skips marked slots.
        unsigned int l_i = 0;              // next descriptor to open
        unsigned long long l_base = zeros;
        unsigned int l_inc = 0u, l_left = 0u;
        unsigned int dummy = 0u;           // bit d: ring slot d carries no step
        bool l_over = false;
        auto l_open = [&]() -> bool {      // open the next run with steps; false: none available now
            for (;;) {
                if (l_over || lds_peek(ctrl + CT_DPROD) <= l_i) return false;
                const u32x4 dd = desc_read(l_i);
                if (dd.z >> 16 & DF_END) { l_over = true; return false; }
                ++l_i;
                const unsigned int steps = (dd.y >> 16 & 0xFFu) + (dd.y >> 24);
                if (steps == 0u) continue;
                l_base = ((unsigned long long)(dd.y & 0xFFFFu) << 32) | dd.x;
                l_inc = 1024u;
                l_left = steps;
                return true;
            }
        };
        unsigned int voff = (unsigned int)lane * 16u;
        ST_ADD(st_a, lds_wait_ge(ctrl + CT_DPROD, 1u));  // the first descriptor is worth waiting for
        u32x4 ring[D];
#pragma unroll
        for (int d = 0; d < D; ++d) {
            bool real = l_left > 0u;
            if (!real) real = l_open();
            ring[d] = ring_refill_at(real ? l_base : zeros, voff, u32x4{0u, 0u, 0u, 0u});
            if (real) { l_base += l_inc; --l_left; } else dummy |= 1u << d;
        }

        // ---- compute front: runs of one K slice (two per tile and wave), a partial tile each
        unsigned int c_i = 0xFFFFFFFFu;  // current descriptor = tile sequence number inside the workgroup
        unsigned int c_useq = 0;         // units finished
        unsigned int c_steps_b = 0, c_flags = 0, c_sa = 0, c_steps_a = 0;
        int c_vv = VPW - 1;
        unsigned int c_left = 0u;
        unsigned int c_xoff = 0;
        bool done = false;
        f32x4 acc[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int xm = (MP == 8) ? (mcol & 7) : mcol;
        const unsigned int xlane = (unsigned int)(((W16 ? g : 2 * g) * MP + xm) * 16);

        auto post = [&]() {   // the partial tile of slice VPW * w + c_vv of tile c_i
            f32x4 *st = stage + (((c_i % NR) * NV + (VPW * w + c_vv)) * NB) * 64 + lane;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                st[nb * 64] = acc[nb];
                acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            lds_drain();
            if (lane == 0) lds_poke(ctrl + CT_POST + (c_i % NR) * NV + VPW * w + c_vv, c_i / NR + 1u);
        };
        // move to the next slice that has steps (slices without steps post nothing: the reducer knows)
        auto c_next = [&]() {
            for (;;) {
                if (c_vv == 0) {
                    c_vv = 1;
                    if (c_steps_b > 0u) {
                        c_left = c_steps_b;
                        c_xoff = (c_sa + c_steps_a) * (unsigned int)XSTEP;
                        return;
                    }
                }
                if (c_flags & DF_LAST) {
                    ++c_useq;
                    if (lane == 0) lds_poke(ctrl + CT_FREED + w, c_useq);
                }
                ++c_i;
                if (lane == 0) lds_poke(ctrl + CT_DCONS + w, c_i);
                ST_ADD(st_a, lds_wait_ge(ctrl + CT_DPROD, c_i + 1u));
                const u32x4 dd = desc_read(c_i);
                c_flags = dd.z >> 16;
                if (c_flags & DF_END) { done = true; c_left = 0u; c_flags = 0u; return; }
                c_steps_a = dd.y >> 16 & 0xFFu;
                c_steps_b = dd.y >> 24;
                c_sa = dd.z & 0xFFFFu;
                c_vv = 0;
                if (c_steps_a + c_steps_b > 0u) {
                    if (c_flags & DF_FIRST) ST_ADD(st_b, lds_wait_ge(ctrl + CT_READY + w, c_useq + 1u));
                    // staging buffer c_i % NR is free once the tile that used it before has been read
                    ST_ADD(st_c, lds_wait_ge(ctrl + CT_CONS + (c_i % NR), c_i / NR));
                }
                if (c_steps_a > 0u) {
                    c_left = c_steps_a;
                    c_xoff = c_sa * (unsigned int)XSTEP;
                    return;
                }
            }
        };
        c_next();

        for (;;) {
            if (done) break;
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const u32x4 wv = ring[d];
                if (dummy >> d & 1u) ST_ADD(st_d, 1u);
                if (!(dummy >> d & 1u)) {
                    const unsigned char *xp = lds + (xlane + c_xoff);
                    c_xoff += (unsigned int)XSTEP;
                    bf16x8 a0, a1;
                    if constexpr (!W16) {
                        a0 = codes_to_bf16x8(wv.x, wv.y);
                        a1 = codes_to_bf16x8(wv.z, wv.w);
                    } else {
                        a0 = __builtin_bit_cast(bf16x8, wv);
                    }
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const u32x4 b0 = *reinterpret_cast<const u32x4 *>(xp + nb * 256);
                        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, __builtin_bit_cast(bf16x8, b0), acc[nb], 0, 0, 0);
                        if constexpr (!W16) {
                            const u32x4 b1 = *reinterpret_cast<const u32x4 *>(xp + nb * 256 + MP * 16);
                            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, __builtin_bit_cast(bf16x8, b1), acc[nb], 0, 0, 0);
                        }
                    }
                    if (__builtin_expect(--c_left == 0u, 0)) {
                        post();
                        c_next();
                    }
                }
                if ((d & (GR - 1)) == GR - 1) {
#pragma unroll
                    for (int e = d - (GR - 1); e <= d; ++e) {
                        bool real = l_left > 0u;
                        if (__builtin_expect(!real, 0)) real = l_open();
                        ring[e] = ring_refill_at(real ? l_base : zeros, voff, ring[e]);
                        if (real) { l_base += l_inc; --l_left; dummy &= ~(1u << e); } else dummy |= 1u << e;
                    }
                }
            }
        }
        stats_out();
        return;
    }

    if (w == NC + 1 + NR) {
        // =================================================================== director
        // Writes, for every tile of the workgroup in execution order, one descriptor per compute wave
        // (lane = compute wave): address of the wave's first weight step of the tile, steps of its two
        // K slices, its first step inside the chunk, first / last tile of a unit.
        unsigned int prod = 0;
        const int cw = lane < NC ? lane : NC - 1;
        auto emit = [&](u32x4 dv) {
            // the ring entry is free once every compute wave has moved past the descriptor RD before
            if (prod >= (unsigned int)RD) {
                const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
                for (;;) {
                    const unsigned int seen = *reinterpret_cast<const volatile lds_u32 *>(ctrl + CT_DCONS + cw);
                    if (__builtin_amdgcn_ballot_w64(seen + (unsigned int)RD <= prod) == 0ull) break;
                    if (lds_peek(ctrl + CT_ABORT)) break;
                    if (__builtin_amdgcn_s_memrealtime() - t0 > t_limit) { lds_poke(ctrl + CT_ABORT, 1u); break; }
                    __builtin_amdgcn_s_sleep(STEP_SLEEP);
                }
            }
            if (lane < NC) *(desc + lane * RD + (prod % RD)) = dv;
            lds_drain();
            ++prod;
            if (lane == 0) lds_poke(ctrl + CT_DPROD, prod);
        };
        for (int ph = 0; ph < nph; ++ph) {
            const auto &P = phases[ph];
            const int ntiles = tiles_of(P);
            if (ntiles == 0) continue;
            for (int c = 0; c < P.C; ++c) {
                const int scc = min(P.SC, P.S - c * P.SC);
                const int sa = (scc * (VPW * cw)) / NV, sm = (scc * (VPW * cw + 1)) / NV, se = (scc * (VPW * cw + VPW)) / NV;
                for (int tl = 0; tl < ntiles; ++tl) {
                    const int t = b + tl * G;
                    const int s = seg_of(P, t);
                    const unsigned long long base = reinterpret_cast<unsigned long long>(P.seg[s].w) +
                        ((unsigned long long)(t - P.seg[s].tile_begin) * P.S + (unsigned long long)c * P.SC + sa) * 1024ull;
                    const unsigned int fl = (tl == 0 ? DF_FIRST : 0u) | (tl == ntiles - 1 ? DF_LAST : 0u);
                    emit(u32x4{(unsigned int)base,
                               (unsigned int)(base >> 32) | ((unsigned int)(sm - sa) << 16) | ((unsigned int)(se - sm) << 24),
                               (unsigned int)sa | (fl << 16), 0u});
                }
            }
        }
        emit(u32x4{0u, 0u, DF_END << 16, 0u});
        return;
    }

    __builtin_amdgcn_s_setprio(STEP_PRIO);
    if (w == NC) {
        // =================================================================== stager
        const unsigned int lds_base = lds_address_of(lds);
        unsigned int useq = 0;
        bool aborted = false;
        int prev_scc = 0;            // steps of the previous unit (its slices' LDS byte ranges follow from it)
#ifdef STEP_STATS
        unsigned long long t_prev = 0;
#endif
        for (int ph = 0; ph < nph; ++ph) {
            const auto &P = phases[ph];
            if (tiles_of(P) == 0) continue;
            int nsrc = P.wait == SEQ_WAIT_FLAGS ? (P.src[1].k_hi > P.src[1].k_lo ? 2 : 1) : 0;
            if (nsrc > 0 && !P.fine) {
                // rows of x do not start on cache-line boundaries: a line may only be fetched when
                // everything in it has been produced, so wait for all producer tiles first
                const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
                for (int s = 0; s < nsrc && !aborted; ++s) {
                    const int nfl = (P.src[s].k_hi - P.src[s].k_lo + 15) >> 4;
                    for (int f0 = 0; f0 < nfl && !aborted; f0 += 64) {
                        for (;;) {
                            const unsigned int f = f0 + lane < nfl ? coherent_load_u32(sp.flags + P.src[s].flag0 + f0 + lane) : epoch;
                            if (__builtin_amdgcn_ballot_w64(f != epoch) == 0ull) break;
                            if (lds_peek(ctrl + CT_ABORT) || coherent_load_u32(&sp.sync[1]) != 0u) { aborted = true; break; }
                            if (__builtin_amdgcn_s_memrealtime() - t0 > t_limit) {
                                aborted = true;
                                lds_poke(ctrl + CT_ABORT, 1u);
                                if (lane == 0) coherent_store_u32(&sp.sync[1], 1u);
                                break;
                            }
                            __builtin_amdgcn_s_sleep(STEP_SLEEP);
                        }
                    }
                }
                nsrc = 0;
            }
            // this lane's share of a 64-piece load: row of its token, 8 columns per piece
            const unsigned int x_voff = (unsigned int)min(lane & (MP - 1), M - 1) * (unsigned int)P.ldx * 2u + 16u * (unsigned int)(lane >> LMP);
            for (int c = 0; c < P.C; ++c, ++useq) {
                const int scc = min(P.SC, P.S - c * P.SC);
                const int k0 = c * P.SC * KSTEP;
                unsigned int pending = (1u << NC) - 1u;
                unsigned long long t0 = 0;
                bool timing = false;
                while (pending) {
                    // ---- slices whose LDS bytes nobody reads any more: every compute wave whose slice of
                    // the PREVIOUS unit overlaps them has left that unit (the same wave when K is the same)
                    unsigned int left = 0;
#pragma unroll
                    for (int cw = 0; cw < NC; ++cw)
                        if (aborted || lds_peek(ctrl + CT_FREED + cw) >= useq) left |= 1u << cw;
                    unsigned int cand = 0;
#pragma unroll
                    for (int cw = 0; cw < NC; ++cw) {
                        const int a = (scc * (VPW * cw)) / NV, e = (scc * (VPW * cw + VPW)) / NV;   // in steps
                        unsigned int need = 1u << cw;
#pragma unroll
                        for (int pw = 0; pw < NC; ++pw)
                            if ((prev_scc * (VPW * pw)) / NV < e && (prev_scc * (VPW * pw + VPW)) / NV > a) need |= 1u << pw;
                        if ((pending >> cw & 1u) && (left & need) == need) cand |= 1u << cw;
                    }
                    // ---- of those, the ones whose producers have raised their flags
                    unsigned int go = cand;
                    if (nsrc > 0 && cand && !aborted) {
                        unsigned int fl[NC][2];
#pragma unroll
                        for (int cw = 0; cw < NC; ++cw) {
#pragma unroll
                            for (int s = 0; s < 2; ++s) {
                                fl[cw][s] = epoch;
                                if (s < nsrc && (cand >> cw & 1u)) {
                                    // all columns of every 128-byte line the slice touches
                                    const int ka = (k0 + (scc * (VPW * cw)) / NV * KSTEP) & ~63;
                                    const int kb = (k0 + (scc * (VPW * cw + VPW)) / NV * KSTEP + 63) & ~63;
                                    const int lo = max(ka, P.src[s].k_lo), hi = min(kb, P.src[s].k_hi);
                                    const int fa = P.src[s].flag0 + ((lo - P.src[s].k_lo) >> 4);
                                    const int nf = hi > lo ? ((hi - P.src[s].k_lo + 15) >> 4) - ((lo - P.src[s].k_lo) >> 4) : 0;
                                    // (the host keeps nf <= 64 whenever this path is taken)
                                    if (lane < nf) fl[cw][s] = coherent_load_u32(sp.flags + fa + lane);
                                }
                            }
                        }
                        const unsigned int err = coherent_load_u32(&sp.sync[1]);
#pragma unroll
                        for (int cw = 0; cw < NC; ++cw) {
                            const bool ok = fl[cw][0] == epoch && fl[cw][1] == epoch;
                            if (__builtin_amdgcn_ballot_w64(!ok) != 0ull) go &= ~(1u << cw);
                        }
                        if (err) aborted = true;
                    }
                    if (aborted) go = pending;
                    // ---- move their slices
                    if (go) {
#ifdef STEP_STATS
                        const unsigned long long tl0 = __builtin_amdgcn_s_memrealtime();
#endif
                        if (!aborted) {
                            for (int cw = 0; cw < NC; ++cw) {
                                if (!(go >> cw & 1u)) continue;
                                const int pa = (scc * (VPW * cw)) / NV * (PPS * MP);
                                const int pb = (scc * (VPW * cw + VPW)) / NV * (PPS * MP);
                                // piece i0 + lane: token (lane % MP), columns k0 + 8 (i0 / MP + lane / MP) ..
                                unsigned long long gbase = reinterpret_cast<unsigned long long>(P.x) +
                                                           2ull * (unsigned long long)(k0 + 8 * (pa >> LMP));
                                unsigned int laddr = lds_base + (unsigned int)pa * 16u;
                                for (int i0 = pa; i0 < pb; i0 += 64) {
                                    if (i0 + 64 <= pb) load_to_lds_16(gbase, x_voff, laddr);
                                    else if (i0 + lane < pb) load_to_lds_16(gbase, x_voff, laddr);
                                    gbase += 1024u / MP;   // 64 / MP pieces of 8 columns, 2 bytes each, per token
                                    laddr += 1024u;
                                }
                            }
                            vmem_drain();
                        }
#ifdef STEP_STATS
                        st_c += (unsigned int)(__builtin_amdgcn_s_memrealtime() - tl0);
                        ++st_d;
#endif
                        if (lane == 0) {
                            for (int cw = 0; cw < NC; ++cw)
                                if (go >> cw & 1u) lds_poke(ctrl + CT_READY + cw, useq + 1u);
                        }
                        lds_drain();
                        pending &= ~go;
                        timing = false;
                    } else {
#ifdef STEP_STATS
                        if (timing) { if (cand) st_b += (unsigned int)(__builtin_amdgcn_s_memrealtime() - t_prev); else st_a += (unsigned int)(__builtin_amdgcn_s_memrealtime() - t_prev); }
                        t_prev = __builtin_amdgcn_s_memrealtime();
#endif
                        if (lds_peek(ctrl + CT_ABORT)) aborted = true;
                        if (!timing) { t0 = __builtin_amdgcn_s_memrealtime(); timing = true; }
                        else if (__builtin_amdgcn_s_memrealtime() - t0 > t_limit) {
                            aborted = true;
                            lds_poke(ctrl + CT_ABORT, 1u);
                            if (lane == 0) coherent_store_u32(&sp.sync[1], 1u);
                        }
                        __builtin_amdgcn_s_sleep(STEP_SLEEP);
                    }
                }
                prev_scc = scc;
            }
        }
        report_abort();
        stats_out();
        return;
    }

    // ======================================================================= reducer
    const int r = w - NC - 1;
    float bestv[NB];
    unsigned int besti[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) { bestv[nb] = -__builtin_inff(); besti[nb] = 0x7FFFFFFFu; }
    unsigned int n = 0;          // tile sequence number inside the workgroup
    for (int ph = 0; ph < nph; ++ph) {
        const auto &P = phases[ph];
        const int ntiles = tiles_of(P);
        if (ntiles == 0) continue;
        const int C = P.C;
        for (int c = 0; c < C; ++c) {
            const int scc = min(P.SC, P.S - c * P.SC);
            for (int tl = 0; tl < ntiles; ++tl, ++n) {
                if ((int)(n % NR) != r) continue;
                const bool last = c == C - 1;
                const int t = b + tl * G;
                const int s = seg_of(P, t);
                const int n0 = (t - P.seg[s].tile_begin) * kTileRows + 4 * g;   // this lane's first row in the segment
                u32x2 sb = {0u, 0u};
                if constexpr (!W16) {
                    if (last) sb = *as_global(reinterpret_cast<const u32x2 *>(P.seg[s].scales + n0));
                }
                // slices without steps (fewer than 16 steps in the chunk) post nothing; leaving their
                // zeros out of the sum changes no bit
                unsigned int live = 0;
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    if ((scc * (v + 1)) / NV > (scc * v) / NV) live |= 1u << v;
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    if (live >> v & 1u) ST_ADD(st_a, lds_wait_ge(ctrl + CT_POST + r * NV + v, n / NR + 1u));
                const f32x4 *st = stage + (r * NV * NB) * 64 + lane;
                f32x4 rsum[NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    rsum[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int v = 0; v < NV; ++v)
                        if (live >> v & 1u) rsum[nb] += st[(v * NB + nb) * 64];
                }
                lds_drain();
                if (lane == 0) lds_poke(ctrl + CT_CONS + r, n / NR + 1u);
                if (C > 1) {
                    // running sums over the K chunks; the tile's previous chunk may have been the
                    // other reducer's
                    if (c > 0) {
                        const unsigned int np = n - (unsigned int)ntiles;
                        lds_wait_ge(ctrl + CT_RDONE + (np % NR), np / NR + 1u);
                    }
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        f32x4 *a = accs + (tl * NB + nb) * 64 + lane;
                        if (c > 0) rsum[nb] += *a;
                        if (!last) *a = rsum[nb];
                    }
                    lds_drain();
                }
                if (lane == 0) lds_poke(ctrl + CT_RDONE + r, n / NR + 1u);
                if (!last) continue;
                float s4[4] = {1.f, 1.f, 1.f, 1.f};
                if constexpr (!W16) {
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
                            const unsigned long long lo = float_to_bf16_bits(v0) | (float_to_bf16_bits(v1) << 16);
                            const unsigned long long hi = float_to_bf16_bits(v2) | (float_to_bf16_bits(v3) << 16);
                            coherent_store_u64(P.seg[s].y + m * P.seg[s].ldy + n0, lo | (hi << 32));
                        }
                    } else {
                        if (v0 > bestv[nb]) { bestv[nb] = v0; besti[nb] = n0; }
                        if (v1 > bestv[nb]) { bestv[nb] = v1; besti[nb] = n0 + 1; }
                        if (v2 > bestv[nb]) { bestv[nb] = v2; besti[nb] = n0 + 2; }
                        if (v3 > bestv[nb]) { bestv[nb] = v3; besti[nb] = n0 + 3; }
                    }
                }
                if (P.kind == EPI_LINEAR && P.publish) {
                    // the tile is readable device-wide once its stores have been acknowledged
#ifdef STEP_STATS
                    const unsigned long long ta = __builtin_amdgcn_s_memrealtime();
#endif
                    vmem_drain();
#ifdef STEP_STATS
                    st_b += (unsigned int)(__builtin_amdgcn_s_memrealtime() - ta);
                    ++st_c;
#endif
                    if (lane == 0) coherent_store_u32(sp.flags + P.flag_off + t, epoch);
                }
            }
        }
    }
    // ---- vocabulary phase: workgroup keys, then workgroup 0 combines them and counts the matches
    report_abort();
    stats_out();
    const auto &PV = phases[nph - 1];
    if (PV.kind != EPI_ARGMAX) return;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        unsigned long long key = argmax_key(bestv[nb], besti[nb]);
        unsigned long long o = shfl_xor_u64(key, 16);
        key = o > key ? o : key;
        o = shfl_xor_u64(key, 32);
        key = o > key ? o : key;
        if (g == 0) keys_lds[r * 32 + mcol + 16 * nb] = key;
    }
    lds_drain();
    if (lane == 0) lds_poke(ctrl + CT_KEYS + r, 1u);
    if (r != 0) return;
    for (int rr = 1; rr < NR; ++rr) lds_wait_ge(ctrl + CT_KEYS + rr, 1u);
    unsigned int *head_flags = sp.flags + PV.flag_off;
    if (lane < MP) {
        unsigned long long key = keys_lds[lane];
#pragma unroll
        for (int rr = 1; rr < NR; ++rr) {
            const unsigned long long o = keys_lds[rr * 32 + lane];
            key = o > key ? o : key;
        }
        coherent_store_u64(sp.partial + (long long)b * MP + lane, key);
    }
    vmem_drain();
    if (lane == 0) coherent_store_u32(head_flags + b, epoch);
    if (b != 0) return;
    {   // every workgroup's keys are there
        const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
        for (int i0 = 0; i0 < G; i0 += 64) {
            for (;;) {
                const unsigned int f = i0 + lane < G ? coherent_load_u32(head_flags + i0 + lane) : epoch;
                if (__builtin_amdgcn_ballot_w64(f != epoch) == 0ull) break;
                if (lds_peek(ctrl + CT_ABORT) || coherent_load_u32(&sp.sync[1]) != 0u) break;
                if (__builtin_amdgcn_s_memrealtime() - t0 > t_limit) {
                    if (lane == 0) coherent_store_u32(&sp.sync[1], 1u);
                    break;
                }
                __builtin_amdgcn_s_sleep(STEP_SLEEP);
            }
        }
    }
    // lane = (sub, m): token m, workgroups sub, sub + 64 / MP, ...
    constexpr int SUBS = 64 / MP;
    const int m = lane & (MP - 1), sub = lane >> LMP;
    unsigned long long key = 0ull;
    for (int i0 = sub; i0 < G; i0 += SUBS * 8) {
        unsigned long long o[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + SUBS * u;
            o[u] = i < G ? coherent_load_u64(sp.partial + (long long)i * MP + m) : 0ull;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) key = o[u] > key ? o[u] : key;
    }
#pragma unroll
    for (int off = MP; off < 64; off <<= 1) {
        const unsigned long long o = shfl_xor_u64(key, off);
        key = o > key ? o : key;
    }
    int32_t *am = reinterpret_cast<int32_t *>(keys_lds);
    if (lane < MP) {
        unsigned int idx = argmax_key_index(key);
        if (idx >= (unsigned int)PV.V) idx = 0;
        am[lane] = (int32_t)idx;
        if (lane < M) *as_global(PV.out_argmax + lane) = (int32_t)idx;
    }
    lds_drain();
    if (lane == 0) {
        int na = 0;
        while (na < PV.n_draft && am[na] == *as_global(PV.draft + na)) ++na;
        *as_global(PV.out_accept) = na;
    }
}

}  // namespace quasar
