// Persistent whole-step kernel (gfx950): a list of linear phases and a final fused
// vocabulary/argmax/acceptance phase executed by one launch of resident workgroups.
//
// Why: a single verification linear streams 4-50 MB, i.e. 1-8 microseconds of HBM time, while
// a kernel boundary costs several microseconds of launch, first-load latency and drain.  Inside
// one persistent kernel the weight stream never stops: weight addresses do not depend on the
// activations, so every wave's load ring runs ahead into the following phases while the
// workgroups wait for the activations of the next phase.
//
// A phase is a group of linears that share their input (q|k|v, gate|up) and therefore need no
// ordering among themselves; its weight tiles are numbered across the member matrices
// ("segments") and split evenly over the workgroups.
//
// Each wave walks ONE flat sequence of slots over the whole step:
//     for phase, for K chunk, for tile of this workgroup, for step of this wave's K slice
// (at least one slot per tile so that all waves meet at every tile end; the slots of one
// (phase, chunk) are padded with slots of zeros to a multiple of the refill group, 4).  Slot j
// is loaded into ring[j % D] D - 3 .. D slots before it is consumed, so the ring holds the
// weights of the following phases while the workgroup waits for activations.
#pragma once

#include "stream_w8a8.hpp"

namespace quasar {

constexpr int kMaxSeg = 4;

// How the input of a phase becomes available:
//   NONE     it was there before the launch;
//   FLAGS    it is the write-once output of one or two earlier phases: every workgroup raises a
//            per-phase flag when its share of such a phase is stored, the consumer polls the
//            flags of all workgroups and then reads the data through the caches;
//   BARRIER  anything else (buffers written more than once, write hazards): device-wide barrier.
enum { SEQ_WAIT_NONE = 0, SEQ_WAIT_BARRIER = 1, SEQ_WAIT_FLAGS = 2 };

struct SeqSeg {
    const u32x4 *w;          // packed weights of this member matrix
    const uint16_t *scales;  // [N] (nullptr for bf16 weights)
    uint16_t *y;             // [M, N] output, row stride ldy
    long long ldy;
    int tile_begin;          // index of the segment's first tile inside the phase
    int N;
};

struct SeqPhase {
    const uint16_t *x;       // [M, K] input shared by all segments
    long long ldx;
    SeqSeg seg[kMaxSeg];
    int nseg;
    int T;                   // tiles over all segments
    int K, S, SC, C;         // as in GemmParams
    int kind;                // EPI_LINEAR or EPI_ARGMAX (argmax: one segment)
    int wait;                // SEQ_WAIT_*: how the input becomes available
    const int32_t *draft;
    int32_t *out_argmax;
    int32_t *out_accept;
    int n_draft;
    int V;
    int producer[2];         // SEQ_WAIT_FLAGS: phases whose completion flags gate this input (-1: unused)
    int publish;             // a later phase waits for this phase's flags
    int raw_off;             // W8A8 form: LDS byte offset where the phase's bf16 activations are parked while they
                             // are scanned and quantised out of LDS (0: they are read from memory twice instead)
    const float *smooth;     // W8A8: per-channel smoothing factors of the input ([K], nullptr: none)
    int xs_bytes;            // LDS bytes this phase reserves for activations (a chunk; W8A8: codes, and the parked bf16)
    int sc_bytes;            // LDS bytes for its row scales (+ 256 for the per-token step sizes of the W8A8 form)
    int tile_shift;          // vocabulary split over tile ranges: tiles of the matrix in front of this phase's first (its
                             // weight and scale pointers start there; only the row indices of the argmax need the shift)
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
    int xs_bytes;            // LDS layout before the first phase (each phase then lays the LDS out for itself:
    int sc_bytes;            // activations, scales, cross-wave staging, per-tile sums, in that order)
    unsigned int *sync;      // [0] arrival counter, [1] error flag (both zero at launch), [2] launch epoch,
                             // [8], [9] members of role 0 / 1 so far, [64 + id] workgroups seen on compute unit id
    unsigned int *flags;     // [nphases][gridDim.x]: epoch of the launch in which the workgroup finished the phase
    unsigned long long *partial;   // argmax phase: [gridDim.x][MP] packed (logit, index) keys
    unsigned int spin_limit; // bound on the time one wait may take, in ticks of the 100 MHz constant clock
    const u32x4 *zeros;      // 1 KB of zeros, never written: what a slot without a weight step loads
    unsigned long long *stamps;   // optional (nullptr: none): [nphases][gridDim.x][8] times of the 100 MHz clock at
                                  // which a workgroup [0] began to wait for a phase's input, [1] saw it complete,
                                  // [2] had it staged, [3] had summed its last tile, [4] had its outputs
                                  // acknowledged and its flag raised; untouched where it has no share
};

// Data that crosses from one phase to a later one inside the launch (outputs read as the
// input of a later phase, argmax partials) is written and read with device-coherent accesses
// that go past the per-XCD L2 caches.  That makes cache write-back / invalidate unnecessary;
// on this part those maintenance operations cost more than the barrier itself.
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
// arrival counter has been bumped.  Polling is bounded in TIME (spin_limit ticks of the 100 MHz
// constant clock, measured per wait): on expiry the error flag is raised and every later wait falls
// through, so the grid always drains and a stall cannot last longer than that, whatever a poll costs.
__device__ __forceinline__ void grid_barrier(unsigned int *sync, unsigned int target, unsigned int spin_limit) {
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    lds_barrier();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(as_global(&sync[0]), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();   // 100 MHz, the same on every compute unit
        while (__hip_atomic_load(as_global(&sync[0]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (__hip_atomic_load(as_global(&sync[1]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            if (__builtin_amdgcn_s_memrealtime() - t0 > spin_limit) {
                __hip_atomic_store(as_global(&sync[1]), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
    }
    lds_barrier();
}

// Activation pieces a thread holds per staging batch; ring slots are refilled in groups of kSeqRefillGroup,
// after the group's last slot has been used.
constexpr int kSeqStageBatch = 2;
constexpr int kSeqRefillGroup = 4;

// A8 selects the W8A8 form of the linears: the activations are smoothed and quantised per
// token while they are staged (same arithmetic as stream_w8a8.hpp), the weight step goes
// straight into the int8 matrix core, the cross-wave sums are exact integers.
//
// ROLES == 2 (two workgroups of 8 waves per compute unit): the workgroups of a compute unit take
// the phases in turn.  While one of them waits for the activations of its phase, stages them and
// computes, the other one - whose next phase is the one after - already has its ring full of that
// phase's weights and keeps loading as slots free up, so the memory pipeline has work across the
// hand-over.  A workgroup learns at start which compute unit it runs on and takes the role nobody
// there has yet; roles are capped at half the grid each, so the split is even wherever the
// workgroups land (placement only matters for speed).  Each wave covers the K range that two waves
// of the 16-wave form cover and adds their two partial sums in the same order, so the results are
// the same bits.
constexpr int kSeqCuSlots = 2048;     // distinct compute-unit ids (XCC, shader engine, unit)

template <int MP, bool W16, bool A8, int NW, int D, int ROLES>
__global__ __launch_bounds__(NW * 64, ROLES == 2 ? 4 : 1) void stream_sequence_kernel(const SeqParams sp) {
    extern __shared__ __align__(16) unsigned char lds[];
    static_assert(!(W16 && A8), "the W8A8 form needs int8 weights");
    constexpr int NB = (MP == 32) ? 2 : 1;
    constexpr int PPS = (W16 || A8) ? 4 : 8;   // 16-byte LDS pieces per step and token
    constexpr int LMP = (MP == 8) ? 3 : (MP == 16 ? 4 : 5);
    constexpr int KSTEP = W16 ? kStepK16 : kStepK8;
    // pieces per thread and batch of the staging path through registers (only the barrier-ordered,
    // coherent reads take it; everything else goes straight to LDS): small batches, few registers
    constexpr int XB = kSeqStageBatch;
    constexpr int NPAR = ROLES == 2 ? 1 : 2;   // copies of the cross-wave staging area
    static_assert(ROLES == 1 || ROLES == 2, "one workgroup per compute unit, or two that alternate");
    static_assert((ROLES == 1 && NW == 16) || (ROLES == 2 && NW == 8), "wave count of each form");
    constexpr int GR = kSeqRefillGroup;
    static_assert(GR >= 1 && (GR & (GR - 1)) == 0 && D % GR == 0, "refill groups tile the ring");
    constexpr int nthreads = NW * 64;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, mcol = lane & 15;
    const int G = gridDim.x, b = blockIdx.x;
    const int GW = G / ROLES;          // workgroups that share a phase
    const int M = sp.M;
    const int nph = sp.nphases;
    const const_phase_ptr phases = (const_phase_ptr)(unsigned long long)sp.phases;

    // regions behind the activations; moved at every phase entry to that phase's own sizes
    uint16_t *sc_lds = reinterpret_cast<uint16_t *>(lds + sp.xs_bytes);
    // the last 256 bytes of the scale region: per-token step sizes and maxima of the W8A8 form
    float *tok_dx = reinterpret_cast<float *>(lds + sp.xs_bytes + sp.sc_bytes - 256);                  // [32]
    unsigned int *tok_amax = reinterpret_cast<unsigned int *>(lds + sp.xs_bytes + sp.sc_bytes - 128);  // [32]
    f32x4 *stage = reinterpret_cast<f32x4 *>(lds + sp.xs_bytes + sp.sc_bytes);   // [2][NW][NB][64]
    f32x4 *accs = stage + NPAR * NW * NB * 64;                                   // [ntiles][NB][64] (C > 1)
    auto lay_out = [&](int xs, int sc) {
        sc_lds = reinterpret_cast<uint16_t *>(lds + xs);
        tok_dx = reinterpret_cast<float *>(lds + xs + sc - 256);
        tok_amax = reinterpret_cast<unsigned int *>(lds + xs + sc - 128);
        stage = reinterpret_cast<f32x4 *>(lds + xs + sc);
        accs = stage + NPAR * NW * NB * 64;
    };

    // role (which phases) and rank (which tiles) of this workgroup
    int role = 0, rk = b;
    if constexpr (ROLES == 2) {
        unsigned int *box = reinterpret_cast<unsigned int *>(stage);
        if (tid == 0) {
            const unsigned int cu = __smid() & (unsigned int)(kSeqCuSlots - 1);
            const unsigned int seen = __hip_atomic_fetch_add(as_global(&sp.sync[64 + cu]), 1u, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_AGENT);
            unsigned int r = seen & 1u;
            unsigned int k = __hip_atomic_fetch_add(as_global(&sp.sync[8 + r]), 1u, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
            if (k >= (unsigned int)GW) {       // that role is full: the other one cannot be
                r ^= 1u;
                k = __hip_atomic_fetch_add(as_global(&sp.sync[8 + r]), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            box[0] = r;
            box[1] = k < (unsigned int)GW ? k : 0u;
        }
        lds_barrier();
        role = __builtin_amdgcn_readfirstlane((int)box[0]);
        rk = __builtin_amdgcn_readfirstlane((int)box[1]);
        lds_barrier();
    }
    auto mine = [&](int ph) -> bool { return ROLES == 1 || (ph & 1) == role; };
    auto stamp = [&](int ph, int what) {
        if (sp.stamps && tid == 0)
            *as_global(sp.stamps + ((long long)ph * G + b) * 8 + what) = __builtin_amdgcn_s_memrealtime();
    };

    // Activations produced inside the launch are later read through the caches.  Lines of an
    // earlier launch (same addresses, old values) cannot be hit: the packet processor
    // invalidates the caches when a kernel starts (an explicit invalidate here costs ~25 us).
    const unsigned int epoch = __builtin_amdgcn_readfirstlane(
        __hip_atomic_load(as_global(&sp.sync[2]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));

    auto seg_of = [&](const auto &P, int t) -> int {
        int s = 0;
        if (P.nseg > 1 && t >= P.seg[1].tile_begin) s = 1;
        if (P.nseg > 2 && t >= P.seg[2].tile_begin) s = 2;
        if (P.nseg > 3 && t >= P.seg[3].tile_begin) s = 3;
        return s;
    };

    // ------------------------------------------------------------------ load front
    // A run is this wave's consecutive steps inside one tile: the per-slot path only bumps a
    // scalar address and counts the run down; the phase table is read when a run ends.  Runs
    // without a step (this wave has no share of the K chunk, or the sequence is over) read a
    // block of zeros, so such a slot contributes nothing without any masking.
    constexpr int kForever = 0x7FFFFFFF;
    const unsigned long long zeros = reinterpret_cast<unsigned long long>(sp.zeros);
    int l_ph = 0, l_c = -1, l_tl = 0, l_spw = 0, l_ntiles = 0, l_t0 = 0, l_seg_end = 0, l_s_lo = 0;
    unsigned long long l_stride = 0;   // bytes from one tile to the next
    unsigned long long l_wt = 0;       // this wave's first step in the current tile
    unsigned long long l_base = zeros; // the next slot to load
    unsigned int l_inc = 0;
    int l_left = 1;
    auto l_retile = [&]() {
        const auto &P = phases[l_ph];
        const int t = l_t0 + l_tl;
        const int s = seg_of(P, t);
        l_seg_end = (s + 1 < P.nseg) ? P.seg[s + 1].tile_begin : P.T;
        l_stride = (unsigned long long)P.S * 1024ull;
        l_wt = reinterpret_cast<unsigned long long>(P.seg[s].w) +
               ((unsigned long long)(t - P.seg[s].tile_begin) * P.S + (unsigned long long)l_c * P.SC + l_s_lo) * 1024ull;
    };
    // move to the next (phase, chunk) in which this workgroup has tiles
    auto l_next = [&]() {
        for (;;) {
            ++l_c;
            if (l_ph < nph && l_c >= phases[l_ph].C) { ++l_ph; l_c = 0; }
            if (l_ph >= nph) { l_ntiles = 0; l_spw = 0; return; }
            const auto &P = phases[l_ph];
            l_t0 = (int)(((unsigned int)P.T * (unsigned int)rk) / (unsigned int)GW);   // the host checks T * G < 2^31
            l_ntiles = (int)(((unsigned int)P.T * (unsigned int)(rk + 1)) / (unsigned int)GW) - l_t0;
            if (l_ntiles == 0 || !mine(l_ph)) { l_c = P.C - 1; continue; }
            const int scc = min(P.SC, P.S - l_c * P.SC);
            l_s_lo = (scc * w) / NW;
            l_spw = (scc * (w + 1)) / NW - l_s_lo;
            l_tl = 0;
            l_retile();
            return;
        }
    };
    auto l_run = [&]() {
        if (l_ph < nph && l_spw > 0) { l_base = l_wt; l_inc = 1024u; l_left = l_spw; }
        else { l_base = zeros; l_inc = 0u; l_left = l_ph < nph ? 1 : kForever; }
    };
    // a wave's slots of one (phase, chunk) - a "unit" - are padded with slots of zeros to a
    // multiple of GR, so that every unit starts at the first slot of a refill group
    bool l_in_pad = false;
    auto l_event = [&]() {
        if (l_ph < nph) {
            if (!l_in_pad && ++l_tl < l_ntiles) {
                if (l_t0 + l_tl == l_seg_end) l_retile(); else l_wt += l_stride;
            } else {
                const int pad = l_in_pad ? 0 : (-(l_ntiles * max(l_spw, 1))) & (GR - 1);

                if (pad > 0) {
                    l_in_pad = true;
                    l_base = zeros;
                    l_inc = 0u;
                    l_left = pad;
                    return;
                }
                l_in_pad = false;
                l_next();
            }
        }
        l_run();
    };

    unsigned int voff = (unsigned int)lane * 16u;
    l_next();
    l_run();
    u32x4 ring[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        ring[d] = ring_refill_at(l_base, voff, u32x4{0u, 0u, 0u, 0u});
        l_base += l_inc;
        if (--l_left == 0) l_event();
    }

    // ------------------------------------------------------------------ compute front
    int c_ph = 0, c_c = -1, c_tl = 0, c_nsl = 1, c_ntiles = 0, c_t0 = 0;
    int c_C = 1, c_kind = EPI_LINEAR;
    int c_left = kForever;             // slots to the end of the current tile
    unsigned int c_x0 = 0, c_xinc = 0; // LDS offset of this wave's first step in the chunk; bytes per step
    unsigned int c_xoff = 0;           // LDS offset of the current slot's activations
    // output segment of the current tile, kept in registers so that the tile-end path reads
    // nothing from the phase table
    uint16_t *c_y = nullptr;
    long long c_ldy = 0;
    int c_tb = 0, c_seg_end = 0;
    auto c_reseg = [&]() {
        const auto &P = phases[c_ph];
        const int s = seg_of(P, c_t0 + c_tl);
        c_y = P.seg[s].y;
        c_ldy = P.seg[s].ldy;
        c_tb = P.seg[s].tile_begin - P.tile_shift;
        c_seg_end = (s + 1 < P.nseg) ? P.seg[s + 1].tile_begin : P.T;
    };
    unsigned int barriers_done = 0;
    int parity = 0;
    f32x4 acc[NB];
    [[maybe_unused]] f32x4 acc_lo[NB];   // ROLES == 2: the sum over the first half of this wave's K range
    [[maybe_unused]] int c_h0 = 0, c_half = 0;   // steps in that half; slots until it ends
    i32x4 acci[NB];          // W8A8: exact integer sums
    float bestv[NB];
    unsigned int besti[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc_lo[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
        acci[nb] = i32x4{0, 0, 0, 0};
        bestv[nb] = -__builtin_inff();
        besti[nb] = 0x7FFFFFFFu;
    }
    const int xm = (MP == 8) ? (mcol & 7) : mcol;
    // this lane's B operand inside a step: 8-element piece (W16: g, else 2g and 2g + 1), token xm
    // W8A8: codes as 16-byte pieces [k/16][token]; bf16 activations: token rows (see x_direct), the lane's offset
    // then depends on the phase's row length and is set at its entry
    unsigned int xlane = (unsigned int)((((W16 || A8) ? g : 2 * g) * MP + xm) * 16);
    [[maybe_unused]] unsigned int xrow16 = 0;   // MP = 32: bytes from token m to token m + 16

    // stage one activation chunk.  `coherent` reads go past the L2 (needed when the buffer may
    // have been cached before it was last written: barrier-ordered, reused buffers); otherwise
    // the 32 compute units of an XCD share one fetch of the activations through their L2.
    [[maybe_unused]] const unsigned int lds_base = lds_address_of(lds);
    // bf16 activations, columns k0 .. k0 + ncols - 1 of all tokens, straight into LDS at byte offset `dst`, one
    // token after the other: token m at dst + m * rs (rs = row bytes + 16: the skew keeps the tokens of one column
    // in different banks).  One instruction moves 1 KB that is contiguous in memory AND in LDS - measured on all
    // 256 compute units fetching the same 64 KB: 100 GB/s per compute unit, against 35 GB/s when an instruction
    // gathers 128 bytes from each of eight rows (rows are a multiple of 4 KB apart and meet in one cache channel).
    // Rows past M repeat row M - 1: their results are never used.  Instruction j covers 1 KB piece j / MP of token
    // j % MP (the waves that issue together then read from different rows: measured 0.93 us for 64 KB against
    // 1.03 us with a row after the other, and the index arithmetic needs no division); wave w takes j = w, w + NW, ...
    // The work is split in two: x_plan does the arithmetic (divisions included) and may run while the wave would
    // otherwise idle in front of the phase's wait; x_issue then costs a dozen scalar instructions per load.  (On
    // the hand-over path the sixteen waves of a workgroup execute this code side by side, four to a SIMD, and the
    // youngest wave of a SIMD was found to reach its first load 1.5 us after the flags had been seen.)
    struct XPlan {
        unsigned long long x0, ld2;
        unsigned int rs;
        int count, rowbytes;
    };
    auto x_plan = [&](const auto &P, long long k0, int ncols, unsigned int rs) -> XPlan {
        XPlan pl;
        pl.rowbytes = ncols * 2;
        const int ninstr = ((pl.rowbytes + 1023) >> 10) * MP;
        pl.count = w < ninstr ? (ninstr - w + NW - 1) / NW : 0;
        pl.x0 = reinterpret_cast<unsigned long long>(P.x) + 2ull * (unsigned long long)k0;
        pl.ld2 = (unsigned long long)P.ldx * 2ull;
        pl.rs = rs;
        return pl;
    };
    auto x_issue = [&](const XPlan &pl, unsigned int dst) {
        const unsigned int x_voff = (unsigned int)lane * 16u;
        for (int n = 0; n < pl.count; ++n) {
            const int j = w + n * NW;
            const int m = j & (MP - 1), i = j >> LMP;
            const unsigned long long gb = pl.x0 + (unsigned long long)min(m, M - 1) * pl.ld2 + (unsigned long long)i * 1024ull;
            const unsigned int glo = __builtin_amdgcn_readfirstlane((unsigned int)gb);
            const unsigned int ghi = __builtin_amdgcn_readfirstlane((unsigned int)(gb >> 32));
            const unsigned long long gbase = ((unsigned long long)ghi << 32) | glo;
            const unsigned int laddr = __builtin_amdgcn_readfirstlane(lds_base + dst + (unsigned int)m * pl.rs + (unsigned int)i * 1024u);
            if (i * 1024 + 1024 <= pl.rowbytes) load_to_lds_16(gbase, x_voff, laddr);
            else if (i * 1024 + lane * 16 < pl.rowbytes) load_to_lds_16(gbase, x_voff, laddr);
        }
    };
    auto x_direct = [&](const auto &P, long long k0, int ncols, unsigned int dst, unsigned int rs) {
        x_issue(x_plan(P, k0, ncols, rs), dst);
    };
    auto x_stage = [&](const auto &P, int c, bool coherent) {
        const int scc = min(P.SC, P.S - c * P.SC);
        const int npieces = scc * PPS * MP;
        const unsigned int rs = (unsigned int)(P.SC * KSTEP * 2 + 16);

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
                        if (coherent) v[i] = coherent_load_u32x4(P.x + m * P.ldx + k);
                        else v[i] = *as_global(reinterpret_cast<const u32x4 *>(P.x + m * P.ldx + k));
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                if (idx < npieces)
                    *reinterpret_cast<u32x4 *>(lds + (unsigned int)(idx & (MP - 1)) * rs + (unsigned int)(idx >> LMP) * 16u) = v[i];
            }
        }
    };
    // ---- W8A8 staging (arithmetic of stream_w8a8.hpp).  Every thread always sees the same
    // token, tid % MP.  The activations are read twice (maxima, then codes); the second read
    // hits the caches.
    const int m_own = tid & (MP - 1);
    float a8_inv = 0.f;
    constexpr int AXB = MP == 8 ? 3 : 2;   // pieces per thread and batch (more would spill)
    auto a8_load = [&](const auto &P, long long k, bool coherent) -> u32x4 {
        if (coherent) return coherent_load_u32x4(P.x + m_own * P.ldx + k);
        return *as_global(reinterpret_cast<const u32x4 *>(P.x + m_own * P.ldx + k));
    };
    auto a8_smooth = [&](const auto &P, const u32x4 &v, long long k, float (&xt)[8]) {
        const float *sm = P.smooth;
        if (sm) {
            const f32x4 s0 = *as_global(reinterpret_cast<const f32x4 *>(sm + k));
            const f32x4 s1 = *as_global(reinterpret_cast<const f32x4 *>(sm + k + 4));
            const float sv[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
            smooth_piece(v, nullptr, k, xt);
#pragma unroll
            for (int j = 0; j < 8; ++j) xt[j] = xt[j] * sv[j];
        } else {
            smooth_piece(v, nullptr, k, xt);
        }
    };
    // per-token maxima over the whole K, then step size and its reciprocal
    auto x_scan = [&](const auto &P, bool coherent) {
        if (tid < 32) tok_amax[tid] = 0u;
        lds_barrier();
        const int npieces = (P.K / 8) * MP;
        if (m_own < M) {
            float amax = 0.f;
            for (int base = 0; base < npieces; base += nthreads * AXB) {
                u32x4 v[AXB];
#pragma unroll
                for (int i = 0; i < AXB; ++i) {
                    const int idx = base + i * nthreads + tid;
                    v[i] = u32x4{0u, 0u, 0u, 0u};
                    if (idx < npieces) v[i] = a8_load(P, 8ll * (idx >> LMP), coherent);
                }
#pragma unroll
                for (int i = 0; i < AXB; ++i) {
                    const int idx = base + i * nthreads + tid;
                    if (idx < npieces) {
                        float xt[8];
                        a8_smooth(P, v[i], 8ll * (idx >> LMP), xt);
                        amax = fmaxf(amax, piece_amax(xt));
                    }
                }
            }
            __hip_atomic_fetch_max(&tok_amax[m_own], __float_as_uint(amax), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        lds_barrier();
        const float amax_own = __uint_as_float(tok_amax[m_own]);
        a8_inv = inverse_step_of(amax_own);
        if (tid < MP) tok_dx[tid] = step_of(amax_own);
    };
    // codes of K chunk c -> LDS in B-operand order [k/16][token][16 B]
    auto x_quant = [&](const auto &P, int c, bool coherent) {
        const int scc = min(P.SC, P.S - c * P.SC);
        const int npieces = scc * 8 * MP;
        const long long k0 = (long long)c * P.SC * kStepK8;
        for (int base = 0; base < npieces; base += nthreads * AXB) {
            u32x4 v[AXB];
#pragma unroll
            for (int i = 0; i < AXB; ++i) {
                const int idx = base + i * nthreads + tid;
                v[i] = u32x4{0u, 0u, 0u, 0u};
                if (idx < npieces && m_own < M) v[i] = a8_load(P, k0 + 8ll * (idx >> LMP), coherent);
            }
#pragma unroll
            for (int i = 0; i < AXB; ++i) {
                const int idx = base + i * nthreads + tid;
                if (idx < npieces) {
                    const int p8 = idx >> LMP;
                    u32x2 codes = {0u, 0u};
                    if (m_own < M) {
                        float xt[8];
                        a8_smooth(P, v[i], k0 + 8ll * p8, xt);
                        codes = quantize_piece(xt, a8_inv);
                    }
                    *reinterpret_cast<u32x2 *>(lds + (((p8 >> 1) * MP + m_own) * 16 + 8 * (p8 & 1))) = codes;
                }
            }
        }
    };
    // The same two passes out of LDS (a phase with raw_off != 0: one K chunk, its bf16 activations parked at
    // raw_off by x_direct): one trip to memory instead of two, and the trip needs no registers.
    auto x_scan_quant_lds = [&](const auto &P) {
        if (tid < 32) tok_amax[tid] = 0u;
        lds_barrier();            // (also: the parked activations have landed - the caller waited for its loads)
        const int npieces = (P.K / 8) * MP;
        // this thread's token row of the parked activations (row bytes + 16 apart); piece p8 at 16 * p8
        const unsigned char *raw = lds + P.raw_off + m_own * (P.K * 2 + 16);
        if (m_own < M) {
            float amax = 0.f;
            for (int idx = tid; idx < npieces; idx += nthreads) {
                float xt[8];
                a8_smooth(P, *reinterpret_cast<const u32x4 *>(raw + (idx >> LMP) * 16), 8ll * (idx >> LMP), xt);
                amax = fmaxf(amax, piece_amax(xt));
            }
            __hip_atomic_fetch_max(&tok_amax[m_own], __float_as_uint(amax), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        lds_barrier();
        const float amax_own = __uint_as_float(tok_amax[m_own]);
        a8_inv = inverse_step_of(amax_own);
        if (tid < MP) tok_dx[tid] = step_of(amax_own);
        for (int idx = tid; idx < npieces; idx += nthreads) {
            const int p8 = idx >> LMP;
            u32x2 codes = {0u, 0u};
            if (m_own < M) {
                float xt[8];
                a8_smooth(P, *reinterpret_cast<const u32x4 *>(raw + p8 * 16), 8ll * p8, xt);
                codes = quantize_piece(xt, a8_inv);
            }
            *reinterpret_cast<u32x2 *>(lds + (((p8 >> 1) * MP + m_own) * 16 + 8 * (p8 & 1))) = codes;
        }
    };
    // wait (wave 0 polls, four flags per lane and round trip) until every workgroup has raised
    // its flag for phase `pp` in this launch
    auto flags_wait = [&](int pp) {
        if (w != 0) return;
        const unsigned int *row = sp.flags + (long long)pp * G;   // the first GW entries: ranks of the phase's role
        const unsigned long long t_begin = __builtin_amdgcn_s_memrealtime();
        for (int t0 = 4 * lane; t0 < GW; t0 += 256) {
            for (;;) {
                unsigned int f[4];
                // One 128-bit device-coherent load per lane and poll (the flags are independent words: tearing between
                // them does not matter): a quarter of the requests of four 32-bit loads, measured 0.2 us less from
                // "flag up" to "flag seen".  Load and wait form one statement, so the compiler's count of the ring's
                // outstanding loads is not involved (everything older has landed once this returns).
                if (t0 + 3 < GW) {
                    u32x4 v;
                    asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)"
                                 : "=&v"(v)
                                 : "v"(as_global(row + t0))
                                 : "memory");
                    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        f[i] = t0 + i < GW ? __hip_atomic_load(as_global(row + t0 + i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                          : epoch;
                }
                if (f[0] == epoch && f[1] == epoch && f[2] == epoch && f[3] == epoch) break;
                // (the error word is only read on this path: a load still pending when the loop is left would
                // make the compiler give up counting the ring's outstanding loads and drain it at every slot)
                if (__builtin_amdgcn_s_memrealtime() - t_begin > sp.spin_limit ||
                    __hip_atomic_load(as_global(&sp.sync[1]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                    __hip_atomic_store(as_global(&sp.sync[1]), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
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
    // The same in one load of two scales per thread, which covers all but huge shares (else scale_stage): the
    // member matrix of a thread's row is picked among values held in scalar registers - looking it up in the
    // phase table per lane, as scale_stage does, costs a round trip of its own before the load can be issued.
    // (scale_fetch only requests pair `i` of the workgroup's row scales; scale_put stores what it returned)
    auto scale_fetch = [&](const auto &P, int t0, int ntiles, int i) -> unsigned int {
        unsigned int v = 0u;
        if constexpr (!W16) {
            if (i >= 0 && i < ntiles * (kTileRows / 2)) {
                const int t = t0 + (i >> 3);
                const uint16_t *base = P.seg[0].scales;
                int tb = 0;
                if (P.nseg > 1 && t >= P.seg[1].tile_begin) { base = P.seg[1].scales; tb = P.seg[1].tile_begin; }
                if (P.nseg > 2 && t >= P.seg[2].tile_begin) { base = P.seg[2].scales; tb = P.seg[2].tile_begin; }
                if (P.nseg > 3 && t >= P.seg[3].tile_begin) { base = P.seg[3].scales; tb = P.seg[3].tile_begin; }
                v = *as_global(reinterpret_cast<const unsigned int *>(base + (long long)(t - tb) * kTileRows + ((2 * i) & 15)));
            }
        }
        return v;
    };
    auto scale_put = [&](int ntiles, int i, unsigned int v) {
        if constexpr (!W16) {
            if (i >= 0 && i < ntiles * (kTileRows / 2)) reinterpret_cast<unsigned int *>(sc_lds)[i] = v;
        }
    };
    auto scale_stage_one_trip = [&](const auto &P, int t0, int ntiles) {
        if constexpr (!W16) {
            if (ntiles * (kTileRows / 2) <= nthreads) scale_put(ntiles, tid, scale_fetch(P, t0, ntiles, tid));
            else scale_stage(P, t0, ntiles);
        }
    };
    bool stored = false;   // this wave has output stores in flight
    // end of a phase: raise this workgroup's completion flag if a later phase waits for it
    auto phase_end = [&](int ph) {
        stamp(ph, 3);
        if (!phases[ph].publish) stamp(ph, 4);
        if (phases[ph].publish) {
            // the output stores have been acknowledged before the flag goes up (only waves that
            // stored wait: for the others this would be a wait for their weight loads)
            if (stored) __builtin_amdgcn_s_waitcnt(0x0F70);
            stored = false;
            lds_barrier();
            if (tid == 0)
                __hip_atomic_store(as_global(sp.flags + (long long)ph * G + rk), epoch, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            stamp(ph, 4);
        }
    };
    // after the last phase, if it was the vocabulary phase: publish argmax partials, meet, and
    // let workgroup 0 reduce them and compare with the draft
    auto verify_second_stage = [&]() {
        const auto &P = phases[nph - 1];
        if (P.kind != EPI_ARGMAX) return;
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
            bestv[nb] = -__builtin_inff();
            besti[nb] = 0x7FFFFFFFu;
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
            int32_t *am = reinterpret_cast<int32_t *>(stage);
            const int sub = tid & 31;
            for (int m = tid >> 5; m < MP; m += nthreads / 32) {     // 32 lanes per position
                unsigned long long key = 0ull;
                if (m < M)
                    for (int i0 = sub; i0 < G; i0 += 32 * 8) {
                        unsigned long long o[8];   // eight independent loads in flight per lane
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const int i = i0 + 32 * u;
                            o[u] = i < G ? coherent_load_u64(sp.partial + (long long)i * MP + m) : 0ull;
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) key = o[u] > key ? o[u] : key;
                    }
#pragma unroll
                for (int off = 16; off >= 1; off >>= 1) {
                    const unsigned long long o = shfl_xor_u64(key, off);
                    key = o > key ? o : key;
                }
                if (m < M && sub == 0) {
                    unsigned int idx = argmax_key_index(key);
                    if (idx >= (unsigned int)P.V) idx = 0;
                    am[m] = (int32_t)idx;
                    *as_global(P.out_argmax + m) = (int32_t)idx;
                }
            }
            lds_barrier();
            if (tid == 0) {
                int n = 0;
                while (n < P.n_draft && am[n] == *as_global(P.draft + n)) ++n;
                *as_global(P.out_accept) = n;
            }
            lds_barrier();
        }
    };
    bool nocomp = false;      // padding slots: no arithmetic
    bool sc_early = false;    // the current phase's row scales were requested ahead of its wait
    int unit_left = 0;        // slots (padded) left in the current unit
    // the current (phase, chunk) is done
    auto c_leave = [&]() {
        ++c_c;
        if (c_ph < nph && c_c >= c_C) {
            phase_end(c_ph);
            ++c_ph;
            c_c = 0;
        }
    };
    // this wave's share of chunk c_c of the current phase (registers only: may run ahead of the phase's wait)
    auto chunk_setup = [&](const auto &P) {
        const int scc = min(P.SC, P.S - c_c * P.SC);
        const int s_lo = (scc * w) / NW;
        const int spw = (scc * (w + 1)) / NW - s_lo;
        c_nsl = max(spw, 1);
        if constexpr (ROLES == 2) {
            // the first of the two 16th-parts of the chunk that this wave covers
            c_h0 = (scc * (2 * w + 1)) / (2 * NW) - s_lo;
            c_half = c_h0 > 0 ? c_h0 : kForever;
        }
        if constexpr (A8) {
            c_xinc = spw > 0 ? (unsigned int)(PPS * MP * 16) : 0u;
            c_x0 = spw > 0 ? (unsigned int)s_lo * (unsigned int)(PPS * MP * 16) : 0u;
        } else {
            const unsigned int rs = (unsigned int)(P.SC * KSTEP * 2 + 16);
            xlane = (unsigned int)xm * rs + (unsigned int)((W16 ? g : 2 * g) * 16);
            xrow16 = 16u * rs;
            c_xinc = spw > 0 ? (unsigned int)(KSTEP * 2) : 0u;
            c_x0 = spw > 0 ? (unsigned int)s_lo * (unsigned int)(KSTEP * 2) : 0u;
        }
        c_tl = 0;
        c_left = c_nsl;
        c_xoff = c_x0;
        unit_left = (c_ntiles * c_nsl + GR - 1) & ~(GR - 1);
        nocomp = false;
        c_reseg();
    };
    // enter the next (phase, chunk): take part in the phase's wait, stage scales and
    // activations.  Returns false when the sequence is finished.
    auto c_enter = [&]() -> bool {
        for (;;) {
            if (c_ph >= nph) return false;
            const auto &P = phases[c_ph];
            if (c_c == 0) {
                c_C = P.C;
                c_kind = P.kind;
                c_t0 = (int)(((unsigned int)P.T * (unsigned int)rk) / (unsigned int)GW);
                c_ntiles = (int)(((unsigned int)P.T * (unsigned int)(rk + 1)) / (unsigned int)GW) - c_t0;
                if (P.wait == SEQ_WAIT_BARRIER) {
                    ++barriers_done;
                    grid_barrier(sp.sync, barriers_done * (unsigned int)G, sp.spin_limit);
                }
                if (!mine(c_ph)) {     // the other role's phase: only its device-wide barrier is shared
                    ++c_ph;
                    continue;
                }
                // (this wave has finished everything of the previous phase, its last epilogue included; what the
                // other waves still read of the old layout is read before they pass the barrier below)
                lay_out(P.xs_bytes, P.sc_bytes);
                stamp(c_ph, 0);
            }
            // Everything that needs no memory of the producers is worked out in front of the phase's wait: this
            // wave's share of the chunk and the addresses of its activation loads.  (On the hand-over path the
            // sixteen waves of a workgroup run this scalar code side by side, four to a SIMD; done after the wait,
            // the youngest wave of a SIMD reached its first load 1.5 us after the flags had been seen.)
            if constexpr (!A8) chunk_setup(P);
            const bool direct = !A8 && P.wait != SEQ_WAIT_BARRIER;
            XPlan xpl{};
            if (direct)
                xpl = x_plan(P, (long long)c_c * P.SC * KSTEP, min(P.SC, P.S - c_c * P.SC) * KSTEP,
                             (unsigned int)(P.SC * KSTEP * 2 + 16));
            // (uses that cannot move: without them the compiler sinks these computations, phase-table reads
            // included, behind the wait and into the first tile's epilogue)
            if constexpr (!A8) {
                auto pin = [](unsigned int v) { asm volatile("" ::"s"(v)); };
                pin(c_x0); pin(c_xinc); pin((unsigned int)c_nsl); pin((unsigned int)unit_left);
                pin((unsigned int)c_seg_end); pin((unsigned int)c_tb); pin((unsigned int)c_ldy);
                pin((unsigned int)(unsigned long long)c_y);
                pin((unsigned int)xpl.x0); pin((unsigned int)xpl.ld2); pin((unsigned int)xpl.count);
                pin((unsigned int)xpl.rowbytes); pin(xpl.rs);
                asm volatile("" ::"v"(xlane));
            }
            if (c_c == 0) {
                // The row scales do not depend on anybody either.  While wave 0 polls the producers' flags the other
                // waves request them, and store them once the previous phase's last epilogue has read its own.
                // (Wave 0 takes no part: a load pending across its poll loop would make the compiler stop counting
                // the ring's loads.)
                sc_early = !W16 && !A8 && P.wait == SEQ_WAIT_FLAGS && c_ntiles > 0 &&
                           c_ntiles * (kTileRows / 2) <= nthreads - 64;
                unsigned int sc_pre = 0u;
                if (P.wait != SEQ_WAIT_BARRIER) {
                    if (P.wait == SEQ_WAIT_FLAGS) {
                        if (w == 0) {
                            flags_wait(P.producer[0]);
                            if (P.producer[1] >= 0) flags_wait(P.producer[1]);
                        } else if (sc_early) {
                            sc_pre = scale_fetch(P, c_t0, c_ntiles, tid - 64);
                        }
                    }
                    lds_barrier();   // flags seen by all; the previous phase's last epilogue has read its scales
                }
                // (an explicit wait on every path: the compiler then knows the load queue empty here, whatever path
                // follows; the scales have had the whole flag wait to arrive)
                __builtin_amdgcn_s_waitcnt(0x0F70);
                if (sc_early) scale_put(c_ntiles, tid - 64, sc_pre);
                stamp(c_ph, 1);
                if (c_ntiles == 0) {   // nothing to do here but the waits
                    c_c = c_C - 1;
                    c_leave();
                    continue;
                }
                if constexpr (A8) {
                    if (P.raw_off != 0) {
                        // scales and activations are requested together; everything is waited for once
                        x_direct(P, 0, P.K, (unsigned int)P.raw_off, (unsigned int)(P.K * 2 + 16));
                        scale_stage_one_trip(P, c_t0, c_ntiles);
                        __builtin_amdgcn_s_waitcnt(0x0F70);
                        x_scan_quant_lds(P);
                    } else {
                        scale_stage_one_trip(P, c_t0, c_ntiles);
                        x_scan(P, P.wait == SEQ_WAIT_BARRIER);
                    }
                }
            }
            if constexpr (A8) {
                chunk_setup(P);   // (behind the scan: its registers are not held across it)
                if (P.raw_off == 0) x_quant(P, c_c, P.wait == SEQ_WAIT_BARRIER);
            } else {
                // activations and (where they were not requested ahead) row scales are requested together and waited
                // for once: one round trip, not two (the activations first: they go straight to LDS, so no loaded
                // value is held across their issue loop)
                if (direct) x_issue(xpl, 0u);
                else x_stage(P, c_c, true);
                if (c_c == 0 && !sc_early) scale_stage_one_trip(P, c_t0, c_ntiles);
            }
            // known-empty load queue: keeps the counted waits of the ring exact (see stream_gemm.hpp)
            __builtin_amdgcn_s_waitcnt(0x0F70);
            lds_barrier();
            if (c_c == 0) stamp(c_ph, 2);
            return true;
        }
    };
    // Units start at a group boundary (every GR slots), so the entry code exists D / GR times in the
    // unrolled round.  The end of a run and the end of a tile can fall on any slot and are inlined
    // into every slot of the round (the build raises the compiler's pragma-unroll size limit for
    // this): any other shape - a side exit from the round, or re-entering it through a switch -
    // makes the compiler lose count of the outstanding ring loads and drain the ring.  When the
    // sequence ends in the middle of a round the rest of the round runs without arithmetic and the
    // loop is left at its top.
    const unsigned char *xsb = lds;
    bool done = false;
    c_leave();
    for (;;) {
        if (done) break;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            // ---- group boundary: units begin and end here
            if ((d & (GR - 1)) == 0) {
                if (unit_left == 0 && !c_enter()) {
                    // the sequence is over: the rest of the round runs without arithmetic, the loop is left at its top
                    done = true;
                    nocomp = true;
                    unit_left = kForever & ~(GR - 1);
                }
                if (d == 0 && done) break;
                unit_left -= GR;
            }
            const u32x4 wv = ring[d];
            const unsigned char *xp = xsb + (xlane + c_xoff);
            [[maybe_unused]] const unsigned long long la = l_base;
            bf16x8 a0, a1;
            if constexpr (A8) {
                if constexpr (GR == 1) ring[d] = ring_refill_at(la, voff, wv);
            } else if constexpr (!W16) {
                a0 = codes_to_bf16x8(wv.x, wv.y);
                a1 = codes_to_bf16x8(wv.z, wv.w);
                if constexpr (GR == 1) ring[d] = ring_refill_at(la, voff, wv);
            } else {
                a0 = __builtin_bit_cast(bf16x8, wv);
            }
            if (!nocomp) {
                c_xoff += c_xinc;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const u32x4 b0 = *reinterpret_cast<const u32x4 *>(xp + (A8 ? nb * 256 : nb * xrow16));
                    if constexpr (A8) {
                        acci[nb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, wv),
                                                                         __builtin_bit_cast(i32x4, b0), acci[nb], 0, 0, 0);
                    } else {
                        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, __builtin_bit_cast(bf16x8, b0), acc[nb], 0, 0, 0);
                        if constexpr (!W16) {
                            const u32x4 b1 = *reinterpret_cast<const u32x4 *>(xp + nb * xrow16 + 16);
                            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, __builtin_bit_cast(bf16x8, b1), acc[nb], 0, 0, 0);
                        }
                    }
                }
            }
            if constexpr (GR == 1) {
                if constexpr (W16) ring[d] = ring_refill_at(la, voff, wv);
                l_base += l_inc;
                if (__builtin_expect(--l_left == 0, 0)) l_event();
            }
            if constexpr (ROLES == 2 && !A8) {
                if (!nocomp && __builtin_expect(--c_half == 0, 0)) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        acc_lo[nb] = acc[nb];
                        acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
            if (!nocomp && __builtin_expect(--c_left == 0, 0)) {
                // ---- tile end: cross-wave sum through LDS, fixed order (W8A8: exact integers)
                using acc_t = std::conditional_t<A8, i32x4, f32x4>;
                acc_t *st = reinterpret_cast<acc_t *>(stage) + (parity * NW) * NB * 64;
                if constexpr (NPAR == 1) lds_barrier();   // the previous tile's sums have been read
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    if constexpr (A8) {
                        st[(w * NB + nb) * 64 + lane] = acci[nb];
                        acci[nb] = i32x4{0, 0, 0, 0};
                    } else if constexpr (ROLES == 2) {
                        st[(w * NB + nb) * 64 + lane] = acc_lo[nb] + acc[nb];
                        acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
                        acc_lo[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
                    } else {
                        st[(w * NB + nb) * 64 + lane] = acc[nb];
                        acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                }
                lds_barrier();
                // the epilogue rotates over waves 1..NW-1: wave 0 polls for the next phase's input
                // and should never have to wait for its own stores
                if (w == 1 + (c_tl % (NW - 1))) {
                    stored = true;
                    acc_t rsum[NB];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        if constexpr (ROLES == 2 || A8) {
                            rsum[nb] = st[nb * 64 + lane];
#pragma unroll
                            for (int ww = 1; ww < NW; ++ww) rsum[nb] += st[(ww * NB + nb) * 64 + lane];
                        } else {
                            // pairs of neighbouring waves first, then the pair sums in order
                            rsum[nb] = st[nb * 64 + lane] + st[(NB + nb) * 64 + lane];
#pragma unroll
                            for (int ww = 2; ww < NW; ww += 2)
                                rsum[nb] += st[(ww * NB + nb) * 64 + lane] + st[((ww + 1) * NB + nb) * 64 + lane];
                        }
                        if (c_C > 1) {
                            acc_t *a = reinterpret_cast<acc_t *>(accs) + (c_tl * NB + nb) * 64 + lane;
                            if (c_c > 0) rsum[nb] += *a;
                            if (c_c < c_C - 1) *a = rsum[nb];
                        }
                    }
                    if (c_c == c_C - 1) {
                        const int n0 = (c_t0 + c_tl - c_tb) * kTileRows + 4 * g;
                        float s4[4] = {1.f, 1.f, 1.f, 1.f};
                        if constexpr (!W16) {
                            const u32x2 sb = *reinterpret_cast<const u32x2 *>(sc_lds + c_tl * kTileRows + 4 * g);
                            s4[0] = bf16_bits_to_float(sb.x & 0xFFFFu);
                            s4[1] = bf16_bits_to_float(sb.x >> 16);
                            s4[2] = bf16_bits_to_float(sb.y & 0xFFFFu);
                            s4[3] = bf16_bits_to_float(sb.y >> 16);
                        }
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            const int m = mcol + 16 * nb;
                            float v0, v1, v2, v3;
                            if constexpr (A8) {
                                // Eq. 10: fp32(acc) * (dx * dw), each one fp32 operation
                                const float dxm = tok_dx[m];
                                v0 = (float)rsum[nb].x * (dxm * s4[0]);
                                v1 = (float)rsum[nb].y * (dxm * s4[1]);
                                v2 = (float)rsum[nb].z * (dxm * s4[2]);
                                v3 = (float)rsum[nb].w * (dxm * s4[3]);
                            } else {
                                v0 = rsum[nb].x * s4[0];
                                v1 = rsum[nb].y * s4[1];
                                v2 = rsum[nb].z * s4[2];
                                v3 = rsum[nb].w * s4[3];
                            }
                            if (c_kind == EPI_LINEAR) {
                                if (m < M) {
                                    const unsigned long long lo =
                                        float_to_bf16_bits(v0) | (float_to_bf16_bits(v1) << 16);
                                    const unsigned long long hi =
                                        float_to_bf16_bits(v2) | (float_to_bf16_bits(v3) << 16);
                                    coherent_store_u64(c_y + m * c_ldy + n0, lo | (hi << 32));
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
                if constexpr (NPAR == 2) parity ^= 1;
                if constexpr (ROLES == 2) c_half = c_h0 > 0 ? c_h0 : kForever;
                // advance the compute front; after the unit's last tile only padding is left
                if (++c_tl >= c_ntiles) {
                    nocomp = true;
                    c_leave();
                } else {
                    if (__builtin_expect(c_t0 + c_tl == c_seg_end, 0)) c_reseg();
                    c_left = c_nsl;
                    c_xoff = c_x0;
                }
            }
            // ---- the group's refills, in slot order, once its last slot (and a tile end that fell
            // on it) is done: a load issued while the compute unit's memory pipeline is full blocks
            // the wave at the instruction, so after a wait - ring full, pipeline empty - the landed
            // slots are all used, and a tile's partial sums handed over, before the first refill
            if constexpr (GR > 1) {
                if ((d & (GR - 1)) == GR - 1) {
#pragma unroll
                    for (int e = d - (GR - 1); e <= d; ++e) {
                        ring[e] = ring_refill_at(l_base, voff, ring[e]);
                        l_base += l_inc;
                        if (__builtin_expect(--l_left == 0, 0)) l_event();
                    }
                }
            }
        }
    }
    verify_second_stage();
}

// Runs ahead of every sequence launch: clears the barrier counter and the error flag and
// starts a new epoch for the completion flags (a kernel rather than a memset so that callers
// may capture the call sequence in a graph).
__global__ void sequence_reset_kernel(unsigned int *sync) {
    if (threadIdx.x == 0) {
        sync[0] = 0u;
        sync[1] = 0u;
        sync[2] = sync[2] + 1u;
        sync[8] = 0u;
        sync[9] = 0u;
    }
    for (int i = threadIdx.x; i < kSeqCuSlots; i += blockDim.x) sync[64 + i] = 0u;
}

}  // namespace quasar
