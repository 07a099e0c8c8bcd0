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
constexpr int kStepNP = 4;    // loader waves
constexpr int kStepCPP = kStepNC / kStepNP;
constexpr int kStepNS = 1 + kStepNR;   // service waves: reducers, director
constexpr int kStepWaves = kStepNC + kStepNP + kStepNS;
constexpr int kStepMaxQueue = 16;      // steps (KB) per compute wave's queue, at most
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
    CT_QHEAD = CT_DCONS + kStepNC,   // [NC] weight steps landed in compute wave w's queue
    CT_QTAIL = CT_QHEAD + kStepNC,   // [NC] weight steps compute wave w has taken out of it
    CT_WORDS = CT_QTAIL + kStepNC
};
static_assert(CT_WORDS * 4 <= 512, "the control words fit the first 512 bytes of the block");

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
__device__ __forceinline__ void load_to_lds_16_nt(unsigned long long gbase, unsigned int lane_offset, unsigned int lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :
                 : "v"(lane_offset), "s"(gbase), "s"(lds_addr)
                 : "memory");
}
// up to four consecutive 1 KB steps, global -> consecutive LDS kilobytes: the instruction offset is added to
// the global AND the LDS address (verified on the device), so one M0 setting serves all of them
__device__ __forceinline__ void load_steps_to_lds_nt(unsigned int n, unsigned long long gbase, unsigned int lane_offset, unsigned int lds_addr) {
    switch (n) {
        case 1: asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" : : "v"(lane_offset), "s"(gbase), "s"(lds_addr) : "memory"); break;
        case 2: asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024 nt" : : "v"(lane_offset), "s"(gbase), "s"(lds_addr) : "memory"); break;
        case 3: asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:2048 nt" : : "v"(lane_offset), "s"(gbase), "s"(lds_addr) : "memory"); break;
        case 4: asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:2048 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:3072 nt" : : "v"(lane_offset), "s"(gbase), "s"(lds_addr) : "memory"); break;
        default: break;
    }
}
// wait until at most n vector memory operations of this wave are outstanding (n is wave-uniform; the
// instruction takes an immediate)
__device__ __forceinline__ void wait_vmcnt_le(unsigned int n) {
    switch (n) {
#define QUASAR_VMCNT_CASE(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
        QUASAR_VMCNT_CASE(0) QUASAR_VMCNT_CASE(1) QUASAR_VMCNT_CASE(2) QUASAR_VMCNT_CASE(3) QUASAR_VMCNT_CASE(4)
        QUASAR_VMCNT_CASE(5) QUASAR_VMCNT_CASE(6) QUASAR_VMCNT_CASE(7) QUASAR_VMCNT_CASE(8) QUASAR_VMCNT_CASE(9)
        QUASAR_VMCNT_CASE(10) QUASAR_VMCNT_CASE(11) QUASAR_VMCNT_CASE(12) QUASAR_VMCNT_CASE(13) QUASAR_VMCNT_CASE(14)
        QUASAR_VMCNT_CASE(15) QUASAR_VMCNT_CASE(16) QUASAR_VMCNT_CASE(17) QUASAR_VMCNT_CASE(18) QUASAR_VMCNT_CASE(19)
        QUASAR_VMCNT_CASE(20) QUASAR_VMCNT_CASE(21) QUASAR_VMCNT_CASE(22) QUASAR_VMCNT_CASE(23) QUASAR_VMCNT_CASE(24)
        QUASAR_VMCNT_CASE(25) QUASAR_VMCNT_CASE(26) QUASAR_VMCNT_CASE(27) QUASAR_VMCNT_CASE(28) QUASAR_VMCNT_CASE(29)
        QUASAR_VMCNT_CASE(30) QUASAR_VMCNT_CASE(31) QUASAR_VMCNT_CASE(32)
#undef QUASAR_VMCNT_CASE
        default: asm volatile("s_waitcnt vmcnt(32)" ::: "memory"); break;
    }
}
__device__ __forceinline__ unsigned int lds_address_of(const unsigned char *p) {
    return __builtin_amdgcn_readfirstlane(
        (unsigned int)(unsigned long long)((const __attribute__((address_space(3))) unsigned char *)p));
}

template <int MP, bool W16, int D>
__global__ __launch_bounds__(kStepWaves * 64) void stream_step_kernel(const SeqParams sp) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int NV = kStepNV, NC = kStepNC, VPW = kStepVPW, NR = kStepNR, RD = kStepRD, NP = kStepNP, CPP = kStepCPP;
    constexpr int LB = 4;                        // loads per compute wave and batch of a loader
    constexpr int NB = (MP == 32) ? 2 : 1;
    constexpr int PPS = W16 ? 4 : 8;             // 16-byte LDS pieces per step and token
    constexpr int LMP = (MP == 8) ? 3 : (MP == 16 ? 4 : 5);
    constexpr int KSTEP = W16 ? kStepK16 : kStepK8;
    constexpr int XSTEP = PPS * MP * 16;         // LDS bytes of one step of activations
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
    unsigned long long *keys_lds = reinterpret_cast<unsigned long long *>(lds + sp.xs_bytes + 512);   // [NR][32]
    // a partial tile: 16 rows x MP tokens fp32; with MP = 8 only the lanes of tokens 0..7 carry one
    constexpr int SL = (MP == 8) ? 32 : NB * 64;       // f32x4 entries per partial tile
    const bool st_lane = MP != 8 || mcol < 8;          // this lane holds part of it ...
    const int st_idx = MP == 8 ? g * 8 + (mcol & 7) : lane;   // ... at this entry (plus 64 per token block)
    f32x4 *stage = reinterpret_cast<f32x4 *>(lds + sp.xs_bytes + kStepCtrlBytes);   // [NR][NV][SL]
    f32x4 *accs = stage + NR * NV * SL;                                             // [tiles][NB][64] (C > 1)
    const int FW = sp.queue_steps;                                                  // steps per compute wave's weight queue
    const unsigned int q_off = (unsigned int)(sp.xs_bytes + kStepCtrlBytes + NR * NV * SL * 16 + sp.acc_bytes);   // [NC][FW] KB

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
        // Follows its descriptor ring (one descriptor per tile of the workgroup, written by the director
        // wave) and takes its weight steps out of its LDS queue, which a loader wave fills.
        const lds_u32x4 *my_desc = desc + w * RD;
        auto desc_read = [&](unsigned int i) -> u32x4 {
            const u32x4 v = *reinterpret_cast<const volatile lds_u32x4 *>(my_desc + (i % RD));
            return u32x4{(unsigned int)__builtin_amdgcn_readfirstlane(v.x), (unsigned int)__builtin_amdgcn_readfirstlane(v.y),
                         (unsigned int)__builtin_amdgcn_readfirstlane(v.z), (unsigned int)__builtin_amdgcn_readfirstlane(v.w)};
        };
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
            f32x4 *st = stage + ((c_i % NR) * NV + (VPW * w + c_vv)) * SL + st_idx;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                if (st_lane) st[nb * 64] = acc[nb];
                acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            lds_drain();
            if (lane == 0) lds_poke(ctrl + CT_POST + (c_i % NR) * NV + VPW * w + c_vv, c_i / NR + 1u);
        };
        // First tile of a unit: bring this wave's K slice of the activations into LDS.  The wave has no
        // other memory traffic of its own, so what it waits for here is exactly its producers and its
        // own loads.  `info`: phase | chunk << 16 | (compute waves whose slice of the previous unit
        // overlaps this slice in LDS) << 24.
        const unsigned int lds_base = lds_address_of(lds);
        auto stage_slice = [&](unsigned int info) {
            const auto &P = phases[info & 0xFFFFu];
            const int c = info >> 16 & 0xFF;
            const unsigned int need = info >> 24;
            const int scc = min(P.SC, P.S - c * P.SC);
            const int k0 = c * P.SC * KSTEP;
            const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
            bool aborted = lds_peek(ctrl + CT_ABORT) != 0u;
            // ---- the LDS bytes are free: the waves that read them in the previous unit have left it
            for (int spin = 0; !aborted; ++spin) {
                static_assert(NC == 8, "the eight counters are read with two 16-byte loads");
                const u32x4 f0 = *reinterpret_cast<const volatile lds_u32x4 *>(ctrl + CT_FREED);
                const u32x4 f1 = *reinterpret_cast<const volatile lds_u32x4 *>(ctrl + CT_FREED + 4);
                const unsigned int fr[NC] = {f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};
                unsigned int left = 0;
#pragma unroll
                for (int cw = 0; cw < NC; ++cw)
                    if ((unsigned int)__builtin_amdgcn_readfirstlane(fr[cw]) >= c_useq) left |= 1u << cw;
                if ((left & need) == need) break;
                __builtin_amdgcn_s_sleep(STEP_SLEEP);
                if (lds_peek(ctrl + CT_ABORT) || (unsigned int)(__builtin_amdgcn_s_memrealtime() - t0) > t_limit) aborted = true;
            }
            // ---- the producers of the slice have raised their flags
            if (P.wait == SEQ_WAIT_FLAGS && !aborted) {
                const int nsrc = P.src[1].k_hi > P.src[1].k_lo ? 2 : 1;
                for (int s = 0; s < nsrc && !aborted; ++s) {
                    int ka = 0, kb = P.K;
                    if (P.fine) {   // all columns of every 128-byte line the slice touches
                        ka = (k0 + (scc * (VPW * w)) / NV * KSTEP) & ~63;
                        kb = (k0 + (scc * (VPW * w + VPW)) / NV * KSTEP + 63) & ~63;
                    }
                    const int lo = max(ka, P.src[s].k_lo), hi = min(kb, P.src[s].k_hi);
                    const int fa = P.src[s].flag0 + ((lo - P.src[s].k_lo) >> 4);
                    const int nf = hi > lo ? ((hi - P.src[s].k_lo + 15) >> 4) - ((lo - P.src[s].k_lo) >> 4) : 0;
                    for (int f0 = 0; f0 < nf && !aborted; f0 += 64) {
                        for (;;) {
                            const unsigned int f = f0 + lane < nf ? coherent_load_u32(sp.flags + fa + f0 + lane) : epoch;
                            const unsigned int err = coherent_load_u32(&sp.sync[1]);
                            if (__builtin_amdgcn_ballot_w64(f != epoch) == 0ull) break;
                            if (err != 0u || lds_peek(ctrl + CT_ABORT) || (unsigned int)(__builtin_amdgcn_s_memrealtime() - t0) > t_limit) { aborted = true; break; }
                            __builtin_amdgcn_s_sleep(STEP_SLEEP);
                        }
                    }
                }
            }
            if (aborted) {
                lds_poke(ctrl + CT_ABORT, 1u);
                if (lane == 0) coherent_store_u32(&sp.sync[1], 1u);
                return;
            }
            // ---- piece i0 + lane: token (lane % MP), columns k0 + 8 (i0 / MP + lane / MP) ..
            const unsigned int x_voff = (unsigned int)min(lane & (MP - 1), M - 1) * (unsigned int)P.ldx * 2u + 16u * (unsigned int)(lane >> LMP);
            const int pa = (scc * (VPW * w)) / NV * (PPS * MP);
            const int pb = (scc * (VPW * w + VPW)) / NV * (PPS * MP);
            unsigned long long gbase = reinterpret_cast<unsigned long long>(P.x) + 2ull * (unsigned long long)(k0 + 8 * (pa >> LMP));
            unsigned int laddr = lds_base + (unsigned int)pa * 16u;
            for (int i0 = pa; i0 < pb; i0 += 64) {
                if (i0 + 64 <= pb) load_to_lds_16(gbase, x_voff, laddr);
                else if (i0 + lane < pb) load_to_lds_16(gbase, x_voff, laddr);
                gbase += 1024u / MP;   // 64 / MP pieces of 8 columns, 2 bytes each, per token
                laddr += 1024u;
            }
            vmem_drain();
            ST_ADD(st_b, (unsigned int)(__builtin_amdgcn_s_memrealtime() - t0));
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
                // one LDS round trip in the usual case: the descriptor together with the two counters
                // that may hold the tile up; the waits below re-read only what was not there yet
                u32x4 dv = *reinterpret_cast<const volatile lds_u32x4 *>(my_desc + (c_i % RD));
                const unsigned int v_prod = *reinterpret_cast<const volatile lds_u32 *>(ctrl + CT_DPROD);
                const unsigned int v_cons = *reinterpret_cast<const volatile lds_u32 *>(ctrl + CT_CONS + (c_i % NR));
                const unsigned int s_prod = __builtin_amdgcn_readfirstlane(v_prod), s_cons = __builtin_amdgcn_readfirstlane(v_cons);
                u32x4 dd = u32x4{(unsigned int)__builtin_amdgcn_readfirstlane(dv.x), (unsigned int)__builtin_amdgcn_readfirstlane(dv.y),
                                 (unsigned int)__builtin_amdgcn_readfirstlane(dv.z), (unsigned int)__builtin_amdgcn_readfirstlane(dv.w)};
                if (s_prod < c_i + 1u) {
                    ST_ADD(st_a, lds_wait_ge(ctrl + CT_DPROD, c_i + 1u));
                    dd = desc_read(c_i);
                }
                c_flags = dd.z >> 16;
                if (c_flags & DF_END) { done = true; c_left = 0u; c_flags = 0u; return; }
                c_steps_a = dd.y >> 16 & 0xFFu;
                c_steps_b = dd.y >> 24;
                c_sa = dd.z & 0xFFFFu;
                c_vv = 0;
                if (c_steps_a + c_steps_b > 0u) {
                    if (c_flags & DF_FIRST) stage_slice(dd.w);
                    // staging buffer c_i % NR is free once the tile that used it before has been read
                    if (s_cons < c_i / NR) ST_ADD(st_c, lds_wait_ge(ctrl + CT_CONS + (c_i % NR), c_i / NR));
                }
                if (c_steps_a > 0u) {
                    c_left = c_steps_a;
                    c_xoff = c_sa * (unsigned int)XSTEP;
                    return;
                }
            }
        };
        c_next();

        const unsigned char *my_q = lds + q_off + (unsigned int)(w * FW) * 1024u + (unsigned int)lane * 16u;
        const unsigned int qmask = (unsigned int)FW - 1u;   // FW is a power of two
        unsigned int taken = 0;          // weight steps taken out of the queue
        unsigned int avail = 0;          // steps known to have landed
        auto fetch = [&](unsigned int step, unsigned int xoff, u32x4 &wv, u32x4 (&bb)[NB][2]) {
            wv = *reinterpret_cast<const u32x4 *>(my_q + (step & qmask) * 1024u);
            const unsigned char *xp = lds + (xlane + xoff);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                bb[nb][0] = *reinterpret_cast<const u32x4 *>(xp + nb * 256);
                if constexpr (!W16) bb[nb][1] = *reinterpret_cast<const u32x4 *>(xp + nb * 256 + MP * 16);
            }
        };
        while (!done) {
            if (avail == 0u) {
                ST_ADD(st_d, lds_wait_ge(ctrl + CT_QHEAD + w, taken + 1u));
                avail = lds_peek(ctrl + CT_QHEAD + w) - taken;
                if (avail == 0u) avail = 1u;   // (only after an abort)
            }
            const unsigned int n = min(avail, c_left);
            // operands of a step are requested from LDS while the step before it is multiplied
#ifdef STEP_STATS
            const unsigned long long ti0 = __builtin_amdgcn_s_memrealtime();
#endif
            u32x4 wv, bb[NB][2];
            fetch(taken, c_xoff, wv, bb);
            for (unsigned int i = 0; i < n; ++i) {
                u32x4 wn = wv, bn[NB][2];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) { bn[nb][0] = bb[nb][0]; bn[nb][1] = bb[nb][1]; }
                if (i + 1u < n) fetch(taken + i + 1u, c_xoff + (i + 1u) * (unsigned int)XSTEP, wn, bn);
                bf16x8 a0, a1;
                if constexpr (!W16) {
                    a0 = codes_to_bf16x8(wv.x, wv.y);
                    a1 = codes_to_bf16x8(wv.z, wv.w);
                } else {
                    a0 = __builtin_bit_cast(bf16x8, wv);
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, __builtin_bit_cast(bf16x8, bb[nb][0]), acc[nb], 0, 0, 0);
                    if constexpr (!W16)
                        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, __builtin_bit_cast(bf16x8, bb[nb][1]), acc[nb], 0, 0, 0);
                }
                wv = wn;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) { bb[nb][0] = bn[nb][0]; bb[nb][1] = bn[nb][1]; }
            }
            taken += n;
            avail -= n;
            c_left -= n;
            c_xoff += n * (unsigned int)XSTEP;
            lds_drain();                 // the queue entries have been read: the loader may reuse them
#ifdef STEP_STATS
            st_e += (unsigned int)(__builtin_amdgcn_s_memrealtime() - ti0);
            st_f += 1u;
#endif
            if (lane == 0) lds_poke(ctrl + CT_QTAIL + w, taken);
            if (c_left == 0u) {
                post();
                c_next();
            }
        }
        stats_out();
        return;
    }

    if (w < NC + NP) {
        // =================================================================== loader
        // Streams the weight steps of its CPP compute waves, in their order, into their LDS queues with
        // direct-to-LDS loads.  It is the only kind of wave that waits for HBM: a compute wave that is
        // held up (activations not there yet) leaves its queue filling, and the queue empties at compute
        // speed afterwards.  Loads go out in batches; a batch is known to have landed (loads return in
        // order) once no more loads are outstanding than were issued after it.
        const int p = w - NC;
        const unsigned int lds_base = lds_address_of(lds);
        const unsigned int voff = (unsigned int)lane * 16u;
        const unsigned int qmask = (unsigned int)FW - 1u;   // FW is a power of two
        static_assert(CPP == 2, "the tails of a loader's compute waves are read with one 8-byte load");
        unsigned int d_i[CPP], left[CPP], issued[CPP], head[CPP];
        unsigned long long base[CPP];
        bool over[CPP];
#pragma unroll
        for (int j = 0; j < CPP; ++j) { d_i[j] = 0; left[j] = 0; issued[j] = 0; head[j] = 0; base[j] = 0; over[j] = false; }
        unsigned int q0 = 0, q1 = 0, q2 = 0;     // batches in flight, oldest first: loads per compute wave, 8 bits each
        int nq = 0;
        unsigned int prod = 0;                   // descriptors known to have been written
        auto total = [](unsigned int q) { return (q & 0xFFu) + (q >> 8 & 0xFFu) + (q >> 16 & 0xFFu) + (q >> 24); };
        for (;;) {
            const u32x2 tv = *reinterpret_cast<const volatile __attribute__((address_space(3))) u32x2 *>(ctrl + CT_QTAIL + p * CPP);
            const unsigned int tails[CPP] = {(unsigned int)__builtin_amdgcn_readfirstlane(tv.x), (unsigned int)__builtin_amdgcn_readfirstlane(tv.y)};
            unsigned int batch = 0;
#pragma unroll
            for (int j = 0; j < CPP; ++j) {
                const int cw = p * CPP + j;
                const unsigned int room = (unsigned int)FW - (issued[j] - tails[j]);
                if (left[j] == 0u && room > 0u && !over[j]) {
                    // open the wave's next run with steps, if its descriptor has been written
                    for (;;) {
                        if (prod <= d_i[j]) prod = lds_peek(ctrl + CT_DPROD);
                        if (prod <= d_i[j]) break;
                        const u32x4 v = *reinterpret_cast<const volatile lds_u32x4 *>(desc + cw * RD + (d_i[j] % RD));
                        const unsigned int dy = __builtin_amdgcn_readfirstlane(v.y), dz = __builtin_amdgcn_readfirstlane(v.z);
                        if (dz >> 16 & DF_END) { over[j] = true; break; }
                        ++d_i[j];
                        left[j] = (dy >> 16 & 0xFFu) + (dy >> 24);
                        base[j] = ((unsigned long long)(dy & 0xFFFFu) << 32) | (unsigned int)__builtin_amdgcn_readfirstlane(v.x);
                        if (left[j]) break;
                    }
                }
                const unsigned int k = min(min(room, left[j]), (unsigned int)LB);
                const unsigned int q_addr = lds_base + q_off + (unsigned int)(cw * FW) * 1024u;
                // (the queue is a ring: up to the wrap, then the rest)
                const unsigned int at = issued[j] & qmask;
                const unsigned int k1 = min(k, (unsigned int)FW - at);
                load_steps_to_lds_nt(k1, base[j], voff, q_addr + at * 1024u);
                load_steps_to_lds_nt(k - k1, base[j] + k1 * 1024ull, voff, q_addr);
                base[j] += k * 1024ull;
                issued[j] += k;
                left[j] -= k;
                batch |= k << (8 * j);
            }
            if (batch) {
                if (nq == 0) q0 = batch; else if (nq == 1) q1 = batch; else q2 = batch;
                ++nq;
            }
            if (nq == 3 || (batch == 0u && nq > 0)) {
                // the oldest batch has landed once only the younger ones are outstanding
#ifdef STEP_STATS
                const unsigned long long tw0 = __builtin_amdgcn_s_memrealtime();
#endif
                wait_vmcnt_le((nq > 1 ? total(q1) : 0u) + (nq > 2 ? total(q2) : 0u));
#ifdef STEP_STATS
                st_a += (unsigned int)(__builtin_amdgcn_s_memrealtime() - tw0);
                st_c += total(q0);
                ++st_d;
#endif
#pragma unroll
                for (int j = 0; j < CPP; ++j) {
                    const unsigned int k = q0 >> (8 * j) & 0xFFu;
                    if (k) {
                        head[j] += k;
                        if (lane == 0) lds_poke(ctrl + CT_QHEAD + p * CPP + j, head[j]);
                    }
                }
                q0 = q1; q1 = q2; q2 = 0;
                --nq;
            } else if (batch == 0u) {
                bool all_over = true;
#pragma unroll
                for (int j = 0; j < CPP; ++j) all_over = all_over && over[j];
                if (all_over || lds_peek(ctrl + CT_ABORT)) break;
#ifdef STEP_STATS
                const unsigned long long ts0 = __builtin_amdgcn_s_memrealtime();
#endif
                __builtin_amdgcn_s_sleep(STEP_SLEEP);
#ifdef STEP_STATS
                st_b += (unsigned int)(__builtin_amdgcn_s_memrealtime() - ts0);
#endif
            }
        }
        stats_out();
        return;
    }

    if (w == NC + NP + NR) {
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
        int prev_scc = 0;            // steps of the previous unit (its slices' LDS ranges follow from it)
        for (int ph = 0; ph < nph; ++ph) {
            const auto &P = phases[ph];
            const int ntiles = tiles_of(P);
            if (ntiles == 0) continue;
            for (int c = 0; c < P.C; ++c) {
                const int scc = min(P.SC, P.S - c * P.SC);
                const int sa = (scc * (VPW * cw)) / NV, sm = (scc * (VPW * cw + 1)) / NV, se = (scc * (VPW * cw + VPW)) / NV;
                // compute waves whose slice of the previous unit overlaps this wave's slice of this one in LDS
                unsigned int need = 0;
#pragma unroll
                for (int pw = 0; pw < NC; ++pw)
                    if ((prev_scc * (VPW * pw)) / NV < se && (prev_scc * (VPW * pw + VPW)) / NV > sa) need |= 1u << pw;
                prev_scc = scc;
                const unsigned int info = (unsigned int)ph | ((unsigned int)c << 16) | (need << 24);
                for (int tl = 0; tl < ntiles; ++tl) {
                    const int t = b + tl * G;
                    const int s = seg_of(P, t);
                    const unsigned long long base = reinterpret_cast<unsigned long long>(P.seg[s].w) +
                        ((unsigned long long)(t - P.seg[s].tile_begin) * P.S + (unsigned long long)c * P.SC + sa) * 1024ull;
                    const unsigned int fl = (tl == 0 ? DF_FIRST : 0u) | (tl == ntiles - 1 ? DF_LAST : 0u);
                    emit(u32x4{(unsigned int)base,
                               (unsigned int)(base >> 32) | ((unsigned int)(sm - sa) << 16) | ((unsigned int)(se - sm) << 24),
                               (unsigned int)sa | (fl << 16), info});
                }
            }
        }
        emit(u32x4{0u, 0u, DF_END << 16, 0u});
        return;
    }

    __builtin_amdgcn_s_setprio(STEP_PRIO);
    // ======================================================================= reducer
    const int r = w - NC - NP;
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
                {   // lane v < 16 watches slice v's counter: one LDS round trip per look
                    const unsigned int need = n / NR + 1u;
                    const bool mine = lane < NV && (live >> lane & 1u);
                    unsigned long long t0 = 0;
                    for (int spin = 0;; ++spin) {
                        const unsigned int seen = *reinterpret_cast<const volatile lds_u32 *>(ctrl + CT_POST + r * NV + (lane & (NV - 1)));
                        if (__builtin_amdgcn_ballot_w64(mine && seen < need) == 0ull) break;
                        if (spin == 0) t0 = __builtin_amdgcn_s_memrealtime();
                        __builtin_amdgcn_s_sleep(STEP_SLEEP);
                        if (lds_peek(ctrl + CT_ABORT)) break;
                        if ((unsigned int)(__builtin_amdgcn_s_memrealtime() - t0) > t_limit) { lds_poke(ctrl + CT_ABORT, 1u); break; }
                    }
                    if (t0) ST_ADD(st_a, (unsigned int)(__builtin_amdgcn_s_memrealtime() - t0));
                }
                const f32x4 *st = stage + (r * NV) * SL + st_idx;
                f32x4 rsum[NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    rsum[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int v = 0; v < NV; ++v)
                        if ((live >> v & 1u) && st_lane) rsum[nb] += st[v * SL + nb * 64];
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
