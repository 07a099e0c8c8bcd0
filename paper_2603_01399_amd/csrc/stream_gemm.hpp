// Skinny-M weight-streaming contraction kernels (gfx950).
//
// One workgroup owns a contiguous range of 16-row weight tiles and walks the K
// dimension of every tile with all of its waves: wave w takes the w-th slice of
// the tile's 1 KB "steps", keeps a ring of D 128-bit loads in flight (the ring
// runs ahead across tile and chunk boundaries because weight addresses do not
// depend on the activations), and the per-wave partial tiles are summed through
// LDS in a fixed order.  Activations for the current K chunk sit in LDS in
// operand order.  The packed weight layout makes the whole workgroup stream
// one contiguous address range.
#pragma once

#include "quasar_device.hpp"

namespace quasar {

struct GemmParams {
    const uint16_t *x;       // [M, K] bf16, row stride ldx
    long long ldx;
    const u32x4 *w;          // packed weights, 64 x 16 B per step, steps of a tile contiguous
    const uint16_t *scales;  // [N] bf16 step sizes (nullptr for bf16 weights)
    uint16_t *y;             // [M, N] bf16, row stride ldy          (linear epilogue)
    long long ldy;
    unsigned long long *partial;  // [gridDim.x][MP] packed (logit, index) keys  (argmax epilogue)
    int M, N, K;
    int T;          // number of 16-row tiles
    int S;          // steps per tile (K/64 for int8, K/32 for bf16 weights)
    int SC;         // steps per K chunk (activations of one chunk fit in LDS)
    int C;          // number of K chunks
    int xs_bytes;   // LDS bytes reserved for the activation chunk
    int sc_bytes;   // LDS bytes reserved for the workgroup's row scales
    const float *smooth;   // [K] per-channel smoothing factors of the W8A8 path (nullptr: none)
    int Srow;       // steps per tile in memory (= S unless the workgroup works on a K slice)
    // K split across workgroups (bf16-activation linear only): workgroup b works on K slice
    // b % ksplit of tile group b / ksplit and writes fp32 partial sums, part32[slice][m][n]
    int ksplit;
    int slice_steps;
    float *part32;
    // fused operations around the linear (stream_mfma_kernel with PRE / RES):
    const uint16_t *pre_arg;   // PRE_RMSNORM: gamma [K] bf16
    float eps;                 // PRE_RMSNORM
    const uint16_t *resid;     // RES: residual [M, N] bf16, row stride ldr (may be y itself)
    long long ldr;
};

// Operation applied to the activations while they are staged (the normalisation in front of
// the linears of a decoder block, fused into the linear that consumes its result):
//   PRE_RMSNORM  x^ = bf16( gamma * bf16( x * rsqrt(mean_k x^2 + eps) ) )      (fp32 inside)
// with the bf16 roundings where a bf16 implementation of the block has them.
enum { PRE_NONE = 0, PRE_RMSNORM = 1 };

__device__ __forceinline__ u32x4 pre_rmsnorm_piece(const u32x4 x, const u32x4 gamma, float r) {
    const unsigned int xw[4] = {x.x, x.y, x.z, x.w}, gw[4] = {gamma.x, gamma.y, gamma.z, gamma.w};
    unsigned int o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = bf16_bits_to_float(float_to_bf16_bits(bf16_bits_to_float(xw[i] & 0xFFFFu) * r));
        const float hi = bf16_bits_to_float(float_to_bf16_bits(__uint_as_float(xw[i] & 0xFFFF0000u) * r));
        o[i] = float_to_bf16_bits(lo * bf16_bits_to_float(gw[i] & 0xFFFFu)) |
               (float_to_bf16_bits(hi * __uint_as_float(gw[i] & 0xFFFF0000u)) << 16);
    }
    return u32x4{o[0], o[1], o[2], o[3]};
}
__device__ __forceinline__ float silu_bf16(float g) {
    return bf16_bits_to_float(float_to_bf16_bits(__fdiv_rn(g, 1.0f + __expf(-g))));
}
__device__ __forceinline__ float piece_sumsq(const u32x4 x) {
    const unsigned int xw[4] = {x.x, x.y, x.z, x.w};
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = bf16_bits_to_float(xw[i] & 0xFFFFu), hi = __uint_as_float(xw[i] & 0xFFFF0000u);
        s = __builtin_fmaf(lo, lo, s);
        s = __builtin_fmaf(hi, hi, s);
    }
    return s;
}

// EPI_LOGITS: the linear epilogue with fp32 outputs, part32[m][n] (row stride N): the input of
// the stochastic verification.
// EPI_SWIGLU: the weight rows alternate in blocks of 16 between the gate and the up projection
// (tile 2t = gate rows 16t.., tile 2t+1 = up rows 16t..); the epilogue of an up tile combines it
// with the gate tile before it, y[m][16t + r] = bf16( bf16(silu(bf16(gate))) * bf16(up) ), so the
// two projections never travel through HBM.  Workgroups own whole tile pairs.
enum { EPI_LINEAR = 0, EPI_ARGMAX = 1, EPI_LOGITS = 2, EPI_SWIGLU = 3 };

// ------------------------------------------------------------------------------------
// Per-wave walk over the workgroup's (chunk, tile, step) sequence with a ring of D loads.
//
// Sequence of one wave: for every K chunk c, for every tile of the workgroup, the wave's
// slice of the chunk's steps (at least one slot per tile so that every wave reaches every
// tile-end barrier), padded per chunk to a multiple of D.  Slot j of the sequence is
// loaded into ring[j % D] exactly D slots before it is consumed; slots that carry no
// step (padding, empty slices) load a fixed hot address and contribute zeros.  Every
// iteration issues exactly one load per consumed slot, unconditionally, so the compiler
// can count outstanding loads and never drains the ring.
// ------------------------------------------------------------------------------------
// Ties the address of a ring refill to the registers just consumed: the refill cannot be
// moved above the last read of the slot's old contents, so old and new value share the
// same registers and the ring is never copied (which would drain it) at a loop back-edge.
typedef const __attribute__((address_space(1))) u32x4 *global_u32x4_ptr;

// Ring refill.  The address is tied to the registers just consumed: the load cannot be moved
// above the last read of the slot's old contents, so old and new value share registers and
// the ring is never copied (which would drain it) at a loop back-edge.
__device__ __forceinline__ u32x4 ring_refill(const u32x4 *addr, const u32x4 &used) {
    unsigned long long a = reinterpret_cast<unsigned long long>(addr);
    asm volatile("" : "+v"(a) : "v"(used.x), "v"(used.y), "v"(used.z), "v"(used.w));
    return __builtin_nontemporal_load(reinterpret_cast<global_u32x4_ptr>(a));
}

// The same with a wave-uniform base address (kept in scalar registers) and a per-lane byte
// offset; the tie goes through the offset register.
__device__ __forceinline__ u32x4 ring_refill_at(unsigned long long base, unsigned int &lane_offset, const u32x4 &used) {
    asm volatile("" : "+v"(lane_offset) : "v"(used.x), "v"(used.y), "v"(used.z), "v"(used.w));
    return __builtin_nontemporal_load(reinterpret_cast<global_u32x4_ptr>(base + lane_offset));
}

template <int NW, int D>
struct WaveWalk {
    const GemmParams &p;
    int w, lane, t0, ntiles;

    struct Front { int c, idx, tl, si, s_lo, spw, nsl, items, padded; };

    __device__ __forceinline__ void slice(int c, Front &f) const {
        const int scc = min(p.SC, p.S - c * p.SC);
        f.s_lo = (scc * w) / NW;
        f.spw = (scc * (w + 1)) / NW - f.s_lo;
        f.nsl = max(f.spw, 1);
        f.items = ntiles * f.nsl;
        f.padded = ((f.items + D - 1) / D) * D;
    }
    __device__ __forceinline__ void begin(Front &f) const {
        f.c = 0; f.idx = 0; f.tl = 0; f.si = 0;
        slice(0, f);
    }
    __device__ __forceinline__ void advance(Front &f) const {
        ++f.idx;
        ++f.si;
        if (f.si >= f.nsl) { f.si = 0; ++f.tl; }
        if (f.idx == f.padded) {
            ++f.c; f.idx = 0; f.tl = 0; f.si = 0;
            if (f.c < p.C) slice(f.c, f); else { f.items = 0; f.padded = D; f.spw = 0; f.nsl = 1; }
        }
    }
    __device__ __forceinline__ bool real(const Front &f) const {
        return f.c < p.C && f.idx < f.items && f.si < f.spw;
    }
    // Slots without a step still issue a load (the in-order load counter needs one per slot):
    // every lane reads the first 16 bytes of the activations, a single cache line that every
    // compute unit already holds.
    __device__ __forceinline__ const u32x4 *addr(const Front &f) const {
        const long long step = (long long)(t0 + f.tl) * p.Srow + (long long)f.c * p.SC + f.s_lo + f.si;
        return real(f) ? p.w + step * 64 + lane : reinterpret_cast<const u32x4 *>(p.x);
    }
};

// ------------------------------------------------------------------------------------
// MFMA variant.  A operand = 16 weight rows x 32 k (bf16, converted in registers from the
// int8 codes), B operand = 32 k x 16 tokens from LDS, D = 16 rows x 16 tokens fp32.
// Lane l = 16*g + i holds weight row i, k-group g (A) / token i, k-group g (B) and
// accumulates rows 4g..4g+3 of token i (D).
// LDS: [activation chunk][scales of the workgroup's tiles][2 x NW staging tiles][tile sums]
// ------------------------------------------------------------------------------------
//
// When the activations of the whole K do not fit the LDS, re-staging them chunk by chunk makes
// every workgroup read all of x from the L2 (256 x the bytes) with the weight stream stalled
// meanwhile.  With a workspace the host instead splits K across workgroups (ksplit slices):
// a workgroup stages only its slice of x, once, and writes fp32 partial tiles that
// splitk_finalize_kernel sums in slice order.
template <int MP, bool W16, int EPI, int NW, int D, int PRE = PRE_NONE, bool RES = false>
__global__ __launch_bounds__(NW * 64) void stream_mfma_kernel(const GemmParams p0) {
    extern __shared__ __align__(16) unsigned char lds[];
    GemmParams p = p0;
    int G = gridDim.x, b = blockIdx.x, slice = 0;
    if (p0.ksplit > 1) {
        slice = b % p0.ksplit;
        b = b / p0.ksplit;
        G = G / p0.ksplit;
        const int s0 = slice * p0.slice_steps;
        p.S = min(p0.slice_steps, p0.S - s0);
        p.SC = p.S;
        p.C = 1;
        p.w = p0.w + (long long)s0 * 64;
        p.x = p0.x + (long long)s0 * (W16 ? kStepK16 : kStepK8);
    }
    constexpr int NB = (MP == 32) ? 2 : 1;   // 16-token blocks
    constexpr int PPS = W16 ? 4 : 8;         // 16-byte activation pieces (8 k) per step
    constexpr int LMP = (MP == 8) ? 3 : (MP == 16 ? 4 : 5);
    constexpr int KSTEP = W16 ? kStepK16 : kStepK8;
    // activation pieces per thread per batch (the fused staging operations hold a second
    // operand per piece: half the batch keeps the register count of the plain kernel)
    constexpr int XB = PRE == PRE_NONE ? 8 : 4;
    constexpr int nthreads = NW * 64;
    // Without a fused staging operation the activations go straight from memory into LDS, as token rows: token m
    // at m * rs (rs = a chunk's row bytes + 16: the skew keeps the tokens of one column in different banks).  One
    // load instruction moves 1 KB that is contiguous in memory and in LDS and holds no registers; instruction j is
    // 1 KB piece j / MP of token j % MP, wave w takes j = w, w + NW, ...  (With all compute units fetching the
    // same 64 KB this pattern is 2-3x faster than gathering 128 bytes from each of eight rows per instruction:
    // rows are a multiple of 4 KB apart and meet in one cache channel.)  The fused forms (normalisation while
    // staging) keep the path through registers and the [k/8][token][8] layout.
    constexpr bool ROWS = PRE == PRE_NONE;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, mcol = lane & 15;

    constexpr int TU = EPI == EPI_SWIGLU ? 2 : 1;   // tiles are handed out in units of TU
    const int t0 = TU * tile_split(p.T / TU, b, G);
    const int t1 = TU * tile_split(p.T / TU, b + 1, G);
    const int ntiles = t1 - t0;

    u32x4 *xs = reinterpret_cast<u32x4 *>(lds);                                   // [SC*PPS][MP]
    uint16_t *sc_lds = reinterpret_cast<uint16_t *>(lds + p.xs_bytes);            // [tpw*16]
    f32x4 *stage = reinterpret_cast<f32x4 *>(lds + p.xs_bytes + p.sc_bytes);      // [2][NW][NB][64]
    f32x4 *accs = stage + 2 * NW * NB * 64;                                       // [ntiles][NB][64] (C > 1)
    f32x4 *gate_keep = stage - NB * 64;   // EPI_SWIGLU: the last NB KB of the scale region, [NB][64]

    auto x_piece_load = [&](int c, int idx) -> u32x4 {
        const int scc = min(p.SC, p.S - c * p.SC);
        const int npieces = scc * PPS * MP;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (idx < npieces) {
            const int m = idx & (MP - 1), p8 = idx >> LMP;
            if (m < p.M) {
                const long long k = (long long)c * p.SC * KSTEP + 8ll * p8;
                v = *reinterpret_cast<const u32x4 *>(p.x + m * p.ldx + k);
            }
        }
        return v;
    };
    // second operand of the fused staging operation for the same piece: gamma[k .. k+7]
    auto aux_piece_load = [&](int c, int idx) -> u32x4 {
        const int scc = min(p.SC, p.S - c * p.SC);
        const int npieces = scc * PPS * MP;
        u32x4 v = {0u, 0u, 0u, 0u};
        if constexpr (PRE != PRE_NONE) {
            if (idx < npieces) {
                const int p8 = idx >> LMP;
                const long long k = (long long)c * p.SC * KSTEP + 8ll * p8;
                v = *reinterpret_cast<const u32x4 *>(p.pre_arg + k);
            }
        }
        return v;
    };
    float r_own = 1.f;   // PRE_RMSNORM: rsqrt(mean x^2 + eps) of the token this thread stages
    auto pre_apply = [&](const u32x4 x, const u32x4 aux) -> u32x4 {
        if constexpr (PRE == PRE_RMSNORM) return pre_rmsnorm_piece(x, aux, r_own);
        else return x;
    };
    [[maybe_unused]] const unsigned int x_rs = (unsigned int)(p.SC * KSTEP * 2 + 16);
    [[maybe_unused]] auto x_rows = [&](int c) {
        const unsigned int lds_base = lds_address_of(lds);
        const int rowbytes = min(p.SC, p.S - c * p.SC) * KSTEP * 2;
        const int ninstr = ((rowbytes + 1023) >> 10) * MP;
        const unsigned long long x0 = reinterpret_cast<unsigned long long>(p.x) + 2ull * (unsigned long long)c * p.SC * KSTEP;
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
    auto x_stage = [&](int c, int first_batch) {
        if constexpr (ROWS) {
            x_rows(c);
            return;
        }
        const int scc = min(p.SC, p.S - c * p.SC);
        const int npieces = scc * PPS * MP;
        for (int base = first_batch * nthreads * XB; base < npieces; base += nthreads * XB) {
            u32x4 v[XB];
#pragma unroll
            for (int i = 0; i < XB; ++i) v[i] = x_piece_load(c, base + i * nthreads + tid);
            if constexpr (PRE != PRE_NONE) {
                u32x4 a[XB];
#pragma unroll
                for (int i = 0; i < XB; ++i) a[i] = aux_piece_load(c, base + i * nthreads + tid);
#pragma unroll
                for (int i = 0; i < XB; ++i) v[i] = pre_apply(v[i], a[i]);
            }
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                if (idx < npieces) xs[idx] = v[i];
            }
        }
    };

    WaveWalk<NW, D> walk{p, w, lane, t0, ntiles};
    typename WaveWalk<NW, D>::Front ld;
    walk.begin(ld);

    // requests in the order they are needed back: activations (first batch), scales, weight ring
    u32x4 xfirst[ROWS ? 1 : XB];
    if constexpr (ROWS) {
        x_rows(0);
    } else {
#pragma unroll
        for (int i = 0; i < XB; ++i) xfirst[i] = x_piece_load(0, i * nthreads + tid);
    }
    u32x4 afirst[PRE != PRE_NONE ? XB : 1];
    if constexpr (PRE != PRE_NONE) {
#pragma unroll
        for (int i = 0; i < XB; ++i) afirst[i] = aux_piece_load(0, i * nthreads + tid);
    }
    unsigned int sc_first = 0;
    if constexpr (!W16) {
        if (2 * tid < ntiles * kTileRows)
            sc_first = *reinterpret_cast<const unsigned int *>(p.scales + (long long)t0 * kTileRows + 2 * tid);
    }
    u32x4 ring[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        ring[d] = ring_refill(walk.addr(ld), u32x4{0u, 0u, 0u, 0u});
        walk.advance(ld);
    }
    if constexpr (PRE == PRE_RMSNORM) {
        // sum of squares of this thread's token over the whole K: the first batch is in
        // registers, the rest is read here; then a fixed-order sum over the threads of a token
        const int m_own = tid & (MP - 1);
        const int npieces0 = min(p.SC, p.S) * PPS * MP;
        const int npieces_all = p.S * PPS * MP;
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < XB; ++i)
            if (i * nthreads + tid < npieces0) ss += piece_sumsq(xfirst[i]);
        // pieces of chunk 0 beyond the first batch and of the later chunks (same index space:
        // piece p8 of token m sits at idx = p8 * MP + m whatever the chunking)
        for (int base = 0; base < npieces_all; base += nthreads * XB) {
            u32x4 v[XB];
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = base + i * nthreads + tid;
                v[i] = u32x4{0u, 0u, 0u, 0u};
                const bool held = base == 0 && idx < npieces0;
                if (!held && idx < npieces_all && m_own < p.M)
                    v[i] = *reinterpret_cast<const u32x4 *>(p.x + m_own * p.ldx + 8ll * (idx >> LMP));
            }
#pragma unroll
            for (int i = 0; i < XB; ++i) ss += piece_sumsq(v[i]);
        }
        float *red = reinterpret_cast<float *>(stage);           // [nthreads], then [16 * MP]
        red[tid] = ss;
        lds_barrier();
        if (tid < 16 * MP) {
            const int j = tid >> LMP;
            float a = 0.f;
            for (int q = j; q < nthreads / MP; q += 16) a += red[q * MP + m_own];
            red[nthreads + tid] = a;
        }
        lds_barrier();
        float tot = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) tot += red[nthreads + j * MP + m_own];
        r_own = __fdiv_rn(1.0f, __fsqrt_rn(__fdiv_rn(tot, (float)p.K) + p.eps));
        // the staging loads above are conditional: start the main loop from a known-empty queue
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    {
        if constexpr (!ROWS) {
            const int npieces = min(p.SC, p.S) * PPS * MP;
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int idx = i * nthreads + tid;
                if (idx < npieces) {
                    if constexpr (PRE != PRE_NONE) xs[idx] = pre_apply(xfirst[i], afirst[i]);
                    else xs[idx] = xfirst[i];
                }
            }
        }
        if constexpr (!W16) {
            if (2 * tid < ntiles * kTileRows) reinterpret_cast<unsigned int *>(sc_lds)[tid] = sc_first;
            for (int i = 2 * (tid + nthreads); i < ntiles * kTileRows; i += 2 * nthreads)
                reinterpret_cast<unsigned int *>(sc_lds)[i >> 1] =
                    *reinterpret_cast<const unsigned int *>(p.scales + (long long)t0 * kTileRows + i);
        }
        if constexpr (ROWS) {
            // the direct-to-LDS loads were issued first and loads return in order: once no more than the D ring
            // loads are outstanding, this wave's share of the activations is in LDS
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(D) : "memory");
        } else {
            x_stage(0, 1);
        }
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
    // token rows: this lane's B operand of step s, piece q is at xm * rs + (s * PPS + q) * 16
    [[maybe_unused]] const unsigned char *xrow = lds + (unsigned int)xm * x_rs;

    for (int c = 0; c < p.C; ++c) {
        if (c > 0) {
            // every wave has passed the previous chunk's last tile barrier: the chunk's
            // activations are no longer read
            x_stage(c, 0);
            // full drain: the staging loads are conditional, and without a known-empty load
            // queue here the compiler would fall back to draining the ring on every round
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
                const int piece0 = step_in_chunk * PPS;
                if constexpr (!W16) {
                    const bf16x8 a0 = codes_to_bf16x8(wv.x, wv.y);
                    const bf16x8 a1 = codes_to_bf16x8(wv.z, wv.w);
                    ring[d] = ring_refill(walk.addr(ld), wv);
                    walk.advance(ld);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        u32x4 b0, b1;
                        if constexpr (ROWS) {
                            const unsigned char *q = xrow + (unsigned int)(16 * nb) * x_rs + (unsigned int)(piece0 + 2 * g) * 16u;
                            b0 = *reinterpret_cast<const u32x4 *>(q);
                            b1 = *reinterpret_cast<const u32x4 *>(q + 16);
                        } else {
                            b0 = xs[(piece0 + 2 * g) * MP + xm + 16 * nb];
                            b1 = xs[(piece0 + 2 * g + 1) * MP + xm + 16 * nb];
                        }
                        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, __builtin_bit_cast(bf16x8, b0),
                                                                          acc[nb], 0, 0, 0);
                        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, __builtin_bit_cast(bf16x8, b1),
                                                                          acc[nb], 0, 0, 0);
                    }
                } else {
                    const bf16x8 a0 = __builtin_bit_cast(bf16x8, wv);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        u32x4 b0;
                        if constexpr (ROWS)
                            b0 = *reinterpret_cast<const u32x4 *>(xrow + (unsigned int)(16 * nb) * x_rs +
                                                                  (unsigned int)(piece0 + g) * 16u);
                        else
                            b0 = xs[(piece0 + g) * MP + xm + 16 * nb];
                        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, __builtin_bit_cast(bf16x8, b0),
                                                                          acc[nb], 0, 0, 0);
                    }
                    ring[d] = ring_refill(walk.addr(ld), wv);
                    walk.advance(ld);
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
                            // fixed order: neighbouring waves in pairs, then the pair sums one after the
                            // other (the whole-step kernel's 8-wave form adds each pair inside one wave)
                            rsum[nb] = st[nb * 64 + lane] + st[(NB + nb) * 64 + lane];
#pragma unroll
                            for (int ww = 2; ww < NW; ww += 2)
                                rsum[nb] += st[(ww * NB + nb) * 64 + lane] + st[((ww + 1) * NB + nb) * 64 + lane];
                            if (p.C > 1) {
                                f32x4 *a = accs + (tl * NB + nb) * 64 + lane;
                                if (c > 0) rsum[nb] += *a;
                                if (c < p.C - 1) *a = rsum[nb];
                            }
                        }
                        if (c == p.C - 1) {
                            const int n0 = (t0 + tl) * kTileRows + 4 * g;
                            float s4[4] = {1.f, 1.f, 1.f, 1.f};
                            if constexpr (!W16) {
                                const u32x2 sb = *reinterpret_cast<const u32x2 *>(sc_lds + tl * kTileRows + 4 * g);
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
                                if constexpr (EPI == EPI_SWIGLU) {
                                    // both projections are rounded to bf16 as separate linears would be
                                    const f32x4 r = {bf16_bits_to_float(float_to_bf16_bits(v0)),
                                                     bf16_bits_to_float(float_to_bf16_bits(v1)),
                                                     bf16_bits_to_float(float_to_bf16_bits(v2)),
                                                     bf16_bits_to_float(float_to_bf16_bits(v3))};
                                    if (((t0 + tl) & 1) == 0) {
                                        gate_keep[nb * 64 + lane] = r;      // read by the next tile's reducer, after a barrier
                                    } else if (m < p.M) {
                                        const f32x4 gt = gate_keep[nb * 64 + lane];
                                        u32x2 o;
                                        o.x = float_to_bf16_bits(silu_bf16(gt.x) * r.x) | (float_to_bf16_bits(silu_bf16(gt.y) * r.y) << 16);
                                        o.y = float_to_bf16_bits(silu_bf16(gt.z) * r.z) | (float_to_bf16_bits(silu_bf16(gt.w) * r.w) << 16);
                                        *reinterpret_cast<u32x2 *>(p.y + m * p.ldy + ((t0 + tl) >> 1) * kTileRows + 4 * g) = o;
                                    }
                                } else if constexpr (EPI == EPI_LOGITS) {
                                    if (m < p.M)
                                        *reinterpret_cast<f32x4 *>(p0.part32 + (long long)m * p.N + n0) =
                                            f32x4{v0, v1, v2, v3};
                                } else if constexpr (EPI == EPI_LINEAR) {
                                    if (m < p.M) {
                                        if (p0.ksplit > 1) {
                                            *reinterpret_cast<f32x4 *>(p0.part32 + ((long long)slice * p.M + m) * p.N + n0) =
                                                rsum[nb];
                                        } else if constexpr (RES) {
                                            // y = bf16( bf16(linear) + residual ), as a bf16 block computes it
                                            const u32x2 rr = *reinterpret_cast<const u32x2 *>(p.resid + m * p.ldr + n0);
                                            const float r0 = bf16_bits_to_float(float_to_bf16_bits(v0)) + bf16_bits_to_float(rr.x & 0xFFFFu);
                                            const float r1 = bf16_bits_to_float(float_to_bf16_bits(v1)) + __uint_as_float(rr.x & 0xFFFF0000u);
                                            const float r2 = bf16_bits_to_float(float_to_bf16_bits(v2)) + bf16_bits_to_float(rr.y & 0xFFFFu);
                                            const float r3 = bf16_bits_to_float(float_to_bf16_bits(v3)) + __uint_as_float(rr.y & 0xFFFF0000u);
                                            u32x2 o;
                                            o.x = float_to_bf16_bits(r0) | (float_to_bf16_bits(r1) << 16);
                                            o.y = float_to_bf16_bits(r2) | (float_to_bf16_bits(r3) << 16);
                                            *reinterpret_cast<u32x2 *>(p.y + m * p.ldy + n0) = o;
                                        } else {
                                            u32x2 o;
                                            o.x = float_to_bf16_bits(v0) | (float_to_bf16_bits(v1) << 16);
                                            o.y = float_to_bf16_bits(v2) | (float_to_bf16_bits(v3) << 16);
                                            *reinterpret_cast<u32x2 *>(p.y + m * p.ldy + n0) = o;
                                        }
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

// ------------------------------------------------------------------------------------
// VALU variant for M <= 4: fp32 FMA dot products, no matrix cores.  Lane l = 16*g + i holds
// 16 consecutive k of weight row i per step; activations sit in LDS as fp32 [M][Kchunk]
// (all lanes of a k-group read the same address: a broadcast).  The k-groups of a lane
// row are combined with cross-lane shuffles, the waves through LDS.
// ------------------------------------------------------------------------------------
template <int MV, int NW, int D>
__global__ __launch_bounds__(NW * 64) void stream_valu_kernel(const GemmParams p) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int nthreads = NW * 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, i16 = lane & 15;

    const int G = gridDim.x, b = blockIdx.x;
    const int t0 = tile_split(p.T, b, G);
    const int t1 = tile_split(p.T, b + 1, G);
    const int ntiles = t1 - t0;
    const int kc_max = p.SC * kStepK8;

    float *xs = reinterpret_cast<float *>(lds);                                   // [MV][kc_max]
    uint16_t *sc_lds = reinterpret_cast<uint16_t *>(lds + p.xs_bytes);            // [tpw*16]
    float *stage = reinterpret_cast<float *>(lds + p.xs_bytes + p.sc_bytes);      // [2][NW][MV][16]
    float *accs = stage + 2 * NW * MV * 16;                                       // [ntiles][MV][16]

    auto x_stage = [&](int c) {
        const int scc = min(p.SC, p.S - c * p.SC);
        const int kc8 = scc * (kStepK8 / 8);         // 8 bf16 per piece
        const int npieces = kc8 * MV;
        for (int idx = tid; idx < npieces; idx += nthreads) {
            const int m = idx / kc8, p8 = idx - m * kc8;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (m < p.M)
                v = *reinterpret_cast<const u32x4 *>(p.x + m * p.ldx + (long long)c * p.SC * kStepK8 + 8 * p8);
            f32x4 lo, hi;
            lo.x = __uint_as_float(v.x << 16); lo.y = __uint_as_float(v.x & 0xFFFF0000u);
            lo.z = __uint_as_float(v.y << 16); lo.w = __uint_as_float(v.y & 0xFFFF0000u);
            hi.x = __uint_as_float(v.z << 16); hi.y = __uint_as_float(v.z & 0xFFFF0000u);
            hi.z = __uint_as_float(v.w << 16); hi.w = __uint_as_float(v.w & 0xFFFF0000u);
            f32x4 *dst = reinterpret_cast<f32x4 *>(xs + m * kc_max + 8 * p8);
            dst[0] = lo;
            dst[1] = hi;
        }
    };

    WaveWalk<NW, D> walk{p, w, lane, t0, ntiles};
    typename WaveWalk<NW, D>::Front ld;
    walk.begin(ld);

    for (int i = 2 * tid; i < ntiles * kTileRows; i += 2 * nthreads)
        reinterpret_cast<unsigned int *>(sc_lds)[i >> 1] =
            *reinterpret_cast<const unsigned int *>(p.scales + (long long)t0 * kTileRows + i);
    x_stage(0);
    u32x4 ring[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        ring[d] = ring_refill(walk.addr(ld), u32x4{0u, 0u, 0u, 0u});
        walk.advance(ld);
    }
    lds_barrier();

    float acc[MV];
#pragma unroll
    for (int m = 0; m < MV; ++m) acc[m] = 0.f;
    int parity = 0;

    for (int c = 0; c < p.C; ++c) {
        if (c > 0) {
            x_stage(c);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), as in the MFMA kernel
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
                float wf[16];
                const unsigned int wd[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    wf[4 * q + 0] = (float)(signed char)(wd[q] & 0xff);
                    wf[4 * q + 1] = (float)(signed char)((wd[q] >> 8) & 0xff);
                    wf[4 * q + 2] = (float)(signed char)((wd[q] >> 16) & 0xff);
                    wf[4 * q + 3] = (float)(signed char)(wd[q] >> 24);
                }
                ring[d] = ring_refill(walk.addr(ld), wv);
                walk.advance(ld);
                const int k0 = (valid ? cs.s_lo + si : 0) * kStepK8 + 16 * g;
#pragma unroll
                for (int m = 0; m < MV; ++m) {
                    const f32x4 *xp = reinterpret_cast<const f32x4 *>(xs + m * kc_max + k0);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x4 xv = xp[q];
                        acc[m] = __builtin_fmaf(wf[4 * q + 0], xv.x, acc[m]);
                        acc[m] = __builtin_fmaf(wf[4 * q + 1], xv.y, acc[m]);
                        acc[m] = __builtin_fmaf(wf[4 * q + 2], xv.z, acc[m]);
                        acc[m] = __builtin_fmaf(wf[4 * q + 3], xv.w, acc[m]);
                    }
                }
                if (in_range && si == cs.nsl - 1) {
                    float *st = stage + parity * NW * MV * 16;
#pragma unroll
                    for (int m = 0; m < MV; ++m) {
                        float v = acc[m];
                        v += __shfl_xor(v, 16, 64);
                        v += __shfl_xor(v, 32, 64);
                        if (g == 0) st[(w * MV + m) * 16 + i16] = v;
                        acc[m] = 0.f;
                    }
                    lds_barrier();
                    if (w == (tl % NW) && lane < MV * 16) {
                        const int m = lane >> 4;
                        float rsum = st[m * 16 + i16];
#pragma unroll
                        for (int ww = 1; ww < NW; ++ww) rsum += st[(ww * MV + m) * 16 + i16];
                        if (p.C > 1) {
                            float *a = accs + (tl * MV + m) * 16 + i16;
                            if (c > 0) rsum += *a;
                            if (c < p.C - 1) *a = rsum;
                        }
                        if (c == p.C - 1 && m < p.M) {
                            const int n = (t0 + tl) * kTileRows + i16;
                            const float v = rsum * bf16_bits_to_float(sc_lds[tl * kTileRows + i16]);
                            p.y[m * p.ldy + n] = (uint16_t)float_to_bf16_bits(v);
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
}

// ------------------------------------------------------------------------------------
// Second stage of the fused verify: combine the per-workgroup keys, then count leading
// draft matches.  One workgroup of 1024 threads, 32 threads per token position.
// ------------------------------------------------------------------------------------
// y[m, n] = bf16( (sum over K slices, in slice order, of part32[slice][m][n]) * delta_n ).
// One thread per four consecutive outputs of a token.
template <bool W16>
__global__ __launch_bounds__(256) void splitk_finalize_kernel(const float *part32, int ksplit, int M, int N,
                                                              const uint16_t *scales, uint16_t *y, long long ldy) {
    const long long q = (long long)blockIdx.x * 256 + threadIdx.x;
    const int nq = N / 4;
    if (q >= (long long)M * nq) return;
    const int m = (int)(q / nq), n0 = (int)(q % nq) * 4;
    f32x4 acc = *reinterpret_cast<const f32x4 *>(part32 + (long long)m * N + n0);
    for (int sl = 1; sl < ksplit; ++sl)
        acc += *reinterpret_cast<const f32x4 *>(part32 + ((long long)sl * M + m) * N + n0);
    float s4[4] = {1.f, 1.f, 1.f, 1.f};
    if constexpr (!W16) {
        const u32x2 sb = *reinterpret_cast<const u32x2 *>(scales + n0);
        s4[0] = bf16_bits_to_float(sb.x & 0xFFFFu);
        s4[1] = bf16_bits_to_float(sb.x >> 16);
        s4[2] = bf16_bits_to_float(sb.y & 0xFFFFu);
        s4[3] = bf16_bits_to_float(sb.y >> 16);
    }
    u32x2 o;
    o.x = float_to_bf16_bits(acc.x * s4[0]) | (float_to_bf16_bits(acc.y * s4[1]) << 16);
    o.y = float_to_bf16_bits(acc.z * s4[2]) | (float_to_bf16_bits(acc.w * s4[3]) << 16);
    *reinterpret_cast<u32x2 *>(y + m * ldy + n0) = o;
}

__global__ __launch_bounds__(1024) void verify_finalize_kernel(const unsigned long long *partial, int nparts,
                                                               int MP, int M, int V, const int32_t *draft,
                                                               int n_draft, int32_t *out_argmax,
                                                               int32_t *out_accept) {
    __shared__ int32_t am[32];
    const int tid = threadIdx.x;
    const int m = tid >> 5, sub = tid & 31;
    unsigned long long key = 0ull;
    if (m < M)
        for (int i = sub; i < nparts; i += 32) {
            const unsigned long long o = partial[(long long)i * MP + m];
            key = o > key ? o : key;
        }
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) {
        const unsigned long long o = shfl_xor_u64(key, off);
        key = o > key ? o : key;
    }
    if (m < M && sub == 0) {
        unsigned int idx = argmax_key_index(key);
        if (idx >= (unsigned int)V) idx = 0;   // only reachable with non-finite logits
        am[m] = (int32_t)idx;
        out_argmax[m] = (int32_t)idx;
    }
    __syncthreads();
    if (tid == 0) {
        int n = 0;
        while (n < n_draft && am[n] == draft[n]) ++n;
        out_accept[0] = n;
    }
}

}  // namespace quasar
