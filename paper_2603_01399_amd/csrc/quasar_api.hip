// C-ABI entry points of the verification library: host-side validation, launch planning
// and kernel dispatch.  Everything that touches data runs in the HIP kernels included below.
#include "../../include/quasar.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <utility>
#include <vector>

#include "pack.hpp"
#include "probe.hpp"
#include "stream_gemm.hpp"
#include "stream_sequence.hpp"
#include "sample.hpp"
#include "stream_w8a8.hpp"
#include "stream_w4.hpp"
#include "drafter.hpp"
#include "attention.hpp"

using namespace quasar;

namespace {

constexpr int kMaxLds = 160 * 1024;          // gfx950 LDS per compute unit
constexpr int kSingleChunkX = 128 * 1024;    // activation bytes allowed when K needs no chunking
constexpr int kMultiChunkX = 96 * 1024;      // activation bytes per chunk otherwise
constexpr int kMinLds = 82 * 1024;           // > half the LDS: at most one workgroup per compute unit
constexpr int kMaxGrid = 4096;               // bound on workgroups (sizes the argmax partials)

std::atomic<int> g_path{QUASAR_PATH_AUTO};
std::atomic<int> g_tune_nw{16};
std::atomic<int> g_tune_d{4};
std::atomic<int> g_tune_wgs{1};

struct EnvInit {
    EnvInit() {
        const char *e = std::getenv("QUASAR_FORCE_PATH");
        if (e) {
            if (!std::strcmp(e, "valu")) g_path = QUASAR_PATH_VALU;
            else if (!std::strcmp(e, "mfma")) g_path = QUASAR_PATH_MFMA;
        }
        const char *t = std::getenv("QUASAR_TUNE_NW");
        if (t) { const int v = std::atoi(t); if (v == 8 || v == 16) g_tune_nw = v; }
        const char *g = std::getenv("QUASAR_TUNE_WGS");
        if (g) { const int v = std::atoi(g); if (v >= 1 && v <= 8) g_tune_wgs = v; }
    }
} g_env_init;

int device_cus() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int v = cached[dev].load();
    if (v == 0) {
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        cached[dev] = v;
    }
    return v;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_mnk(int64_t M, int64_t N, int64_t K) {
    if (M < 1 || M > 32) return QUASAR_ERR_SHAPE;
    if (K < 64 || K % 64 != 0 || K > (1 << 24)) return QUASAR_ERR_SHAPE;
    if (N < 16 || N % 16 != 0 || N > (1 << 26)) return QUASAR_ERR_SHAPE;
    return QUASAR_OK;
}

struct Plan {
    int S, SC, C, xs_bytes, sc_bytes, lds_bytes, grid;
};

constexpr int kMaxTilesPerWg = 512;   // bounds the per-workgroup scale table in LDS (16 KB)

// K chunking shared by the single-call kernels and the whole-step kernel (identical chunks
// give identical fp32 summation order, hence identical bits): one chunk if the activations
// fit beside the staging area, otherwise equal chunks that leave room for scales and sums.
void choose_chunks(int S, int x_bytes_per_step, int stage_bytes, int &SC, int &C) {
    int single = kMaxLds - stage_bytes - 8 * 1024;
    if (single > kSingleChunkX) single = kSingleChunkX;
    int multi = kMaxLds - stage_bytes - 32 * 1024;
    if (multi > kMultiChunkX) multi = kMultiChunkX;
    const long long xall = (long long)S * x_bytes_per_step;
    if (xall <= single) {
        C = 1;
        SC = S;
        return;
    }
    int per = multi / x_bytes_per_step;   // steps per chunk that fit
    if (per < 1) per = 1;
    C = (S + per - 1) / per;
    SC = (S + C - 1) / C;
    C = (S + SC - 1) / SC;
}

// x_bytes_per_step: LDS bytes one step of activations occupies; unit_bytes: LDS bytes of one
// tile accumulator / staging slot per wave; with_scales: reserve the row-scale table.
Plan make_plan(int T, int S, int x_bytes_per_step, int unit_bytes, int NW, bool with_scales, int grid_want = 0) {
    Plan pl{};
    pl.S = S;
    choose_chunks(S, x_bytes_per_step, 2 * NW * unit_bytes, pl.SC, pl.C);
    // (+ 512: activations kept as token rows lie 16 bytes further apart than their length, at most 32 rows)
    pl.xs_bytes = pl.SC * x_bytes_per_step + 512;
    const int stage = 2 * NW * unit_bytes;
    int grid = grid_want > 0 ? grid_want : device_cus() * g_tune_wgs.load();
    if (grid > T) grid = T;
    // tiles per workgroup are bounded by the LDS left for the scale table and, when K is
    // chunked, the per-tile running sums
    const int per_tile = (with_scales ? kTileRows * 2 : 0) + (pl.C > 1 ? unit_bytes : 0);
    int tpw_max = kMaxTilesPerWg;
    if (per_tile > 0) {
        const int room = kMaxLds - pl.xs_bytes - stage - 64;
        const int fit = room / per_tile;
        if (fit < tpw_max) tpw_max = fit;
    }
    if (tpw_max < 1) tpw_max = 1;
    const int need = (T + tpw_max - 1) / tpw_max;
    if (grid < need) grid = need;
    pl.grid = grid;
    const int tpw = (T + grid - 1) / grid;
    pl.sc_bytes = with_scales ? ((tpw * kTileRows * 2 + 15) / 16) * 16 : 0;
    pl.lds_bytes = pl.xs_bytes + pl.sc_bytes + stage + (pl.C > 1 ? tpw * unit_bytes : 0);
    if (pl.lds_bytes < kMinLds && g_tune_wgs.load() == 1) pl.lds_bytes = kMinLds;
    return pl;
}

// Kernels that use more than the default dynamic LDS limit need a one-time opt-in per
// function (and per device); remember which ones have had it.
bool allow_large_lds(const void *fn) {
    static std::mutex mu;
    static std::vector<std::pair<const void *, int>> done;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    std::lock_guard<std::mutex> lock(mu);
    for (const auto &e : done)
        if (e.first == fn && e.second == dev) return true;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) != hipSuccess) return false;
    done.emplace_back(fn, dev);
    return true;
}

template <typename KernelT>
int launch(KernelT kernel, int grid, int block, int lds_bytes, hipStream_t stream, const GemmParams &p) {
    if (lds_bytes > kMaxLds) return QUASAR_ERR_SHAPE;
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return QUASAR_ERR_HIP;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(block), lds_bytes, stream, p);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

// K split across workgroups for the bf16-activation linear: how many slices (1 = no split) and
// steps per slice, such that the activations of one slice fit the LDS in one piece.
void splitk_shape(int M, int S, bool w16, int &ksplit, int &slice_steps) {
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    const int NB = MP == 32 ? 2 : 1;
    const int xbps = (w16 ? 64 : 128) * MP;
    int SC = 0, C = 0;
    choose_chunks(S, xbps, 2 * 16 * NB * 1024, SC, C);
    ksplit = 1;
    slice_steps = S;
    if (C <= 1) return;
    int single = kMaxLds - 2 * 16 * NB * 1024 - 8 * 1024;
    if (single > kSingleChunkX) single = kSingleChunkX;
    int per = single / xbps;
    if (per < 1) per = 1;
    ksplit = (S + per - 1) / per;
    slice_steps = (S + ksplit - 1) / ksplit;          // equal slices ...
    // ... in whole multiples of 16 steps where that is possible: the 16 waves of a workgroup share
    // a slice's steps, and a ragged share leaves some of them idle at every tile
    const int up = (slice_steps + 15) / 16 * 16;
    if (up <= per) slice_steps = up;
    else if (MP < 32 && slice_steps >= 16) slice_steps -= slice_steps % 16;
    ksplit = (S + slice_steps - 1) / slice_steps;
}
size_t splitk_bytes(int M, int N, int ksplit) { return ksplit > 1 ? (size_t)ksplit * M * N * sizeof(float) : 0; }

template <bool W16, int EPI>
int launch_mfma(const GemmParams &base, int M, hipStream_t stream, int *grid_out, void *workspace = nullptr,
                size_t workspace_bytes = 0) {
    GemmParams p = base;
    p.Srow = p.S;
    p.ksplit = 1;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    const int NB = MP == 32 ? 2 : 1;
    const int NW = g_tune_nw.load();
    Plan pl = make_plan(p.T, p.S, (W16 ? 64 : 128) * MP, NB * 1024, NW, !W16);
    int launch_grid = pl.grid;
    if (EPI == EPI_LINEAR && pl.C > 1 && NW == 16 && workspace && aligned(workspace, 16)) {
        int ksplit = 1, slice_steps = p.S;
        splitk_shape(M, p.S, W16, ksplit, slice_steps);
        const int groups = device_cus() / ksplit;
        if (ksplit > 1 && groups >= 1 && workspace_bytes >= splitk_bytes(M, p.N, ksplit)) {
            const Plan ps = make_plan(p.T, slice_steps, (W16 ? 64 : 128) * MP, NB * 1024, NW, !W16, groups);
            if (ps.C == 1 && (long long)ps.grid * ksplit <= kMaxGrid) {
                pl = ps;
                p.ksplit = ksplit;
                p.slice_steps = slice_steps;
                p.part32 = static_cast<float *>(workspace);
                launch_grid = ps.grid * ksplit;
            }
        }
    }
    if (launch_grid > kMaxGrid) return QUASAR_ERR_SHAPE;
    p.SC = pl.SC;
    p.C = pl.C;
    p.xs_bytes = pl.xs_bytes;
    p.sc_bytes = pl.sc_bytes;
    if (grid_out) *grid_out = launch_grid;
    const int DD = g_tune_d.load();
#define QUASAR_LAUNCH(MPV)                                                                                   \
    (NW == 16 ? (DD == 8 ? launch(stream_mfma_kernel<MPV, W16, EPI, 16, 8>, launch_grid, 1024, pl.lds_bytes, stream, p) \
                         : launch(stream_mfma_kernel<MPV, W16, EPI, 16, 4>, launch_grid, 1024, pl.lds_bytes, stream, p)) \
              : (DD == 8 ? launch(stream_mfma_kernel<MPV, W16, EPI, 8, 8>, launch_grid, 512, pl.lds_bytes, stream, p)    \
                         : launch(stream_mfma_kernel<MPV, W16, EPI, 8, 4>, launch_grid, 512, pl.lds_bytes, stream, p)))
    int rc;
    if (MP == 8) rc = QUASAR_LAUNCH(8);
    else if (MP == 16) rc = QUASAR_LAUNCH(16);
    else rc = QUASAR_LAUNCH(32);
#undef QUASAR_LAUNCH
    if (rc != QUASAR_OK || p.ksplit == 1) return rc;
    const long long quads = (long long)M * (p.N / 4);
    hipLaunchKernelGGL(splitk_finalize_kernel<W16>, dim3((unsigned int)((quads + 255) / 256)), dim3(256), 0, stream,
                       p.part32, p.ksplit, M, p.N, p.scales, p.y, p.ldy);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

int launch_valu(const GemmParams &base, int M, hipStream_t stream) {
    GemmParams p = base;
    p.Srow = p.S;
    p.ksplit = 1;
    const int MV = M <= 1 ? 1 : (M <= 2 ? 2 : 4);
    const int NW = 8;
    const Plan pl = make_plan(p.T, p.S, MV * kStepK8 * 4, MV * 64, NW, true);
    p.SC = pl.SC;
    p.C = pl.C;
    p.xs_bytes = pl.xs_bytes;
    p.sc_bytes = pl.sc_bytes;
    if (MV == 1) return launch(stream_valu_kernel<1, 8, 8>, pl.grid, 512, pl.lds_bytes, stream, p);
    if (MV == 2) return launch(stream_valu_kernel<2, 8, 8>, pl.grid, 512, pl.lds_bytes, stream, p);
    return launch(stream_valu_kernel<4, 8, 8>, pl.grid, 512, pl.lds_bytes, stream, p);
}

template <bool W16>
int linear_impl(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const void *wp, const uint16_t *scales,
                int64_t N, uint16_t *y, int64_t ldy, void *workspace, size_t workspace_bytes, void *stream) {
    if (!x || !wp || !y || (!W16 && !scales)) return QUASAR_ERR_NULL;
    if (const int e = check_mnk(M, N, K)) return e;
    if (ldx < K || ldy < N || ldx % 8 || ldy % 8) return QUASAR_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(wp, 16) || (!W16 && !aligned(scales, 8)))
        return QUASAR_ERR_ALIGN;
    GemmParams p{};
    p.x = x; p.ldx = ldx; p.w = static_cast<const u32x4 *>(wp); p.scales = scales;
    p.y = y; p.ldy = ldy; p.partial = nullptr;
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.T = (int)(N / kTileRows);
    p.S = (int)(K / (W16 ? kStepK16 : kStepK8));
    const int path = g_path.load();
    if (!W16 && M <= 4 && path == QUASAR_PATH_VALU) return launch_valu(p, (int)M, static_cast<hipStream_t>(stream));
    return launch_mfma<W16, EPI_LINEAR>(p, (int)M, static_cast<hipStream_t>(stream), nullptr, workspace,
                                        workspace_bytes);
}

template <bool W16>
int verify_impl(const uint16_t *h, int64_t M, int64_t K, int64_t ldh, const void *wp, const uint16_t *scales,
                int64_t V, const int32_t *draft, int64_t n_draft, int32_t *out_argmax, int32_t *out_accept,
                void *workspace, size_t workspace_bytes, void *stream) {
    if (!h || !wp || !out_argmax || !out_accept || (!W16 && !scales)) return QUASAR_ERR_NULL;
    if (n_draft > 0 && !draft) return QUASAR_ERR_NULL;
    if (const int e = check_mnk(M, V, K)) return e;
    if (V > 0x7FFFFFF0ll) return QUASAR_ERR_SHAPE;
    if (n_draft < 0 || n_draft > M) return QUASAR_ERR_SHAPE;
    if (ldh < K || ldh % 8) return QUASAR_ERR_SHAPE;
    if (!aligned(h, 16) || !aligned(wp, 16) || (!W16 && !aligned(scales, 8))) return QUASAR_ERR_ALIGN;
    if (!workspace || workspace_bytes < quasar_workspace_bytes(M, V, K)) return QUASAR_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return QUASAR_ERR_ALIGN;
    GemmParams p{};
    p.x = h; p.ldx = ldh; p.w = static_cast<const u32x4 *>(wp); p.scales = scales;
    p.y = nullptr; p.ldy = 0; p.partial = static_cast<unsigned long long *>(workspace);
    p.M = (int)M; p.N = (int)V; p.K = (int)K;
    p.T = (int)(V / kTileRows);
    p.S = (int)(K / (W16 ? kStepK16 : kStepK8));
    hipStream_t st = static_cast<hipStream_t>(stream);
    int grid = 0;
    if (const int e = launch_mfma<W16, EPI_ARGMAX>(p, (int)M, st, &grid)) return e;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    hipLaunchKernelGGL(verify_finalize_kernel, dim3(1), dim3(1024), 0, st, p.partial, grid, MP, (int)M, (int)V,
                       draft, (int)n_draft, out_argmax, out_accept);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

// Argmax partials of quasar_lmhead_verify_static: part of the device image, one copy per GPU.
constexpr size_t kStaticPartialWords = (size_t)kMaxGrid * 32u;
static __device__ __align__(256) unsigned long long g_verify_scratch[kStaticPartialWords];

// Device address of g_verify_scratch on the current device (looked up once per device; the
// array's name is only a host-side handle and must never be passed to a kernel).
int static_scratch(unsigned long long **out) {
    static std::atomic<unsigned long long *> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return QUASAR_ERR_HIP;
    unsigned long long *ptr = cached[dev].load();
    if (!ptr) {
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(g_verify_scratch)) != hipSuccess || !sym) {
            (void)hipGetLastError();
            return QUASAR_ERR_HIP;
        }
        ptr = static_cast<unsigned long long *>(sym);
        cached[dev] = ptr;
    }
    *out = ptr;
    return QUASAR_OK;
}

}  // namespace

extern "C" {

const char *quasar_status_string(int status) {
    switch (status) {
        case QUASAR_OK: return "ok";
        case QUASAR_ERR_NULL: return "null pointer";
        case QUASAR_ERR_SHAPE: return "shape or stride outside limits";
        case QUASAR_ERR_ALIGN: return "misaligned pointer";
        case QUASAR_ERR_WORKSPACE: return "workspace missing or too small";
        case QUASAR_ERR_DTYPE: return "unknown dtype or path";
        case QUASAR_ERR_HIP: return "HIP runtime error at launch";
        default: return "unknown status";
    }
}

int quasar_version(void) { return 100; }

int quasar_set_path(int path) {
    if (path != QUASAR_PATH_AUTO && path != QUASAR_PATH_VALU && path != QUASAR_PATH_MFMA) return QUASAR_ERR_DTYPE;
    g_path = path;
    return QUASAR_OK;
}
int quasar_get_path(void) { return g_path.load(); }

int quasar_set_tuning(int waves, int wgs_per_cu, int depth) {
    if ((waves != 8 && waves != 16) || wgs_per_cu < 1 || wgs_per_cu > 8 || (depth != 4 && depth != 8))
        return QUASAR_ERR_SHAPE;
    g_tune_nw = waves;
    g_tune_wgs = wgs_per_cu;
    g_tune_d = depth;
    return QUASAR_OK;
}

size_t quasar_packed_bytes(int64_t N, int64_t K) {
    if (N < 16 || N % 16 || K < 64 || K % 64) return 0;
    return (size_t)N * (size_t)K;
}
size_t quasar_packed_bytes_bf16(int64_t N, int64_t K) {
    if (N < 16 || N % 16 || K < 64 || K % 64) return 0;
    return (size_t)N * (size_t)K * 2u;
}
size_t quasar_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (check_mnk(M, N, K)) return 0;
    size_t need = (size_t)kMaxGrid * 32u * sizeof(unsigned long long);    // argmax partials
    // fp32 partial sums when K is split across workgroups (int8 or bf16 weights, whichever needs more)
    for (int w16 = 0; w16 < 2; ++w16) {
        int ksplit = 1, slice_steps = 0;
        splitk_shape((int)M, (int)(K / (w16 ? kStepK16 : kStepK8)), w16 != 0, ksplit, slice_steps);
        const size_t sk = splitk_bytes((int)M, (int)N, ksplit);
        if (sk > need) need = sk;
    }
    return need;
}

int quasar_quantize_weights_smoothed(const void *w, int w_dtype, int64_t N, int64_t K, int64_t ldw,
                                     const float *smooth, int8_t *wq_packed, uint16_t *scales_bf16,
                                     void *hip_stream) {
    if (!w || !wq_packed || !scales_bf16) return QUASAR_ERR_NULL;
    if (w_dtype != QUASAR_F32 && w_dtype != QUASAR_BF16) return QUASAR_ERR_DTYPE;
    if (const int e = check_mnk(1, N, K)) return e;
    if (ldw < K) return QUASAR_ERR_SHAPE;
    if (!aligned(wq_packed, 16) || !aligned(scales_bf16, 2) || !aligned(w, w_dtype == QUASAR_F32 ? 4 : 2) ||
        !aligned(smooth, 4))
        return QUASAR_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int T = (int)(N / kTileRows);
    if (w_dtype == QUASAR_F32)
        hipLaunchKernelGGL(quantize_pack_kernel<false>, dim3(T), dim3(256), 0, st, w, (long long)ldw, (int)N, (int)K,
                           smooth, reinterpret_cast<u32x4 *>(wq_packed), scales_bf16);
    else
        hipLaunchKernelGGL(quantize_pack_kernel<true>, dim3(T), dim3(256), 0, st, w, (long long)ldw, (int)N, (int)K,
                           smooth, reinterpret_cast<u32x4 *>(wq_packed), scales_bf16);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

int quasar_quantize_weights(const void *w, int w_dtype, int64_t N, int64_t K, int64_t ldw, int8_t *wq_packed,
                            uint16_t *scales_bf16, void *hip_stream) {
    return quasar_quantize_weights_smoothed(w, w_dtype, N, K, ldw, nullptr, wq_packed, scales_bf16, hip_stream);
}

int quasar_unpack_weights(const int8_t *wq_packed, int64_t N, int64_t K, int8_t *q_rowmajor, void *hip_stream) {
    if (!wq_packed || !q_rowmajor) return QUASAR_ERR_NULL;
    if (const int e = check_mnk(1, N, K)) return e;
    if (!aligned(wq_packed, 16) || !aligned(q_rowmajor, 16)) return QUASAR_ERR_ALIGN;
    const long long nslots = (long long)N * K / 16;
    const int grid = (int)((nslots + 255) / 256 > 65535 ? 65535 : (nslots + 255) / 256);
    hipLaunchKernelGGL(unpack_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<const u32x4 *>(wq_packed), (int)N, (int)K, q_rowmajor);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

int quasar_w8_linear(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const int8_t *wq_packed,
                     const uint16_t *scales_bf16, int64_t N, uint16_t *y, int64_t ldy, void *workspace,
                     size_t workspace_bytes, void *hip_stream) {
    return linear_impl<false>(x, M, K, ldx, wq_packed, scales_bf16, N, y, ldy, workspace, workspace_bytes, hip_stream);
}

int quasar_lmhead_verify(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh, const int8_t *wq_packed,
                         const uint16_t *scales_bf16, int64_t V, const int32_t *draft_ids, int64_t n_draft,
                         int32_t *out_argmax, int32_t *out_accept_len, void *workspace, size_t workspace_bytes,
                         void *hip_stream) {
    return verify_impl<false>(hidden, M, K, ldh, wq_packed, scales_bf16, V, draft_ids, n_draft, out_argmax,
                              out_accept_len, workspace, workspace_bytes, hip_stream);
}

int quasar_lmhead_verify_static(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh, const int8_t *wq_packed,
                                const uint16_t *scales_bf16, int64_t V, const int32_t *draft_ids, int64_t n_draft,
                                int32_t *out_argmax, int32_t *out_accept_len, void *hip_stream) {
    if (const int e = check_mnk(M, V, K)) return e;                  // M <= 32: 32 slots per workgroup suffice
    unsigned long long *scratch = nullptr;
    if (const int e = static_scratch(&scratch)) return e;
    // verify_impl refuses launches of more than kMaxGrid workgroups before anything runs, which
    // is what the array is sized for
    return verify_impl<false>(hidden, M, K, ldh, wq_packed, scales_bf16, V, draft_ids, n_draft, out_argmax,
                              out_accept_len, scratch, kStaticPartialWords * sizeof(unsigned long long), hip_stream);
}

int quasar_pack_bf16_weights(const void *w, int w_dtype, int64_t N, int64_t K, int64_t ldw, uint16_t *w_packed,
                             void *hip_stream) {
    if (!w || !w_packed) return QUASAR_ERR_NULL;
    if (w_dtype != QUASAR_F32 && w_dtype != QUASAR_BF16) return QUASAR_ERR_DTYPE;
    if (const int e = check_mnk(1, N, K)) return e;
    if (ldw < K) return QUASAR_ERR_SHAPE;
    if (!aligned(w_packed, 16)) return QUASAR_ERR_ALIGN;
    const long long nslots = (long long)N * K / 8;
    const int grid = (int)((nslots + 255) / 256 > 65535 ? 65535 : (nslots + 255) / 256);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (w_dtype == QUASAR_F32)
        hipLaunchKernelGGL(pack_bf16_kernel<false>, dim3(grid), dim3(256), 0, st, w, (long long)ldw, (int)N, (int)K,
                           reinterpret_cast<u32x4 *>(w_packed));
    else
        hipLaunchKernelGGL(pack_bf16_kernel<true>, dim3(grid), dim3(256), 0, st, w, (long long)ldw, (int)N, (int)K,
                           reinterpret_cast<u32x4 *>(w_packed));
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

int quasar_bf16_linear(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const uint16_t *w_packed, int64_t N,
                       uint16_t *y, int64_t ldy, void *workspace, size_t workspace_bytes, void *hip_stream) {
    return linear_impl<true>(x, M, K, ldx, w_packed, nullptr, N, y, ldy, workspace, workspace_bytes, hip_stream);
}

int quasar_bf16_lmhead_verify(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh, const uint16_t *w_packed,
                              int64_t V, const int32_t *draft_ids, int64_t n_draft, int32_t *out_argmax,
                              int32_t *out_accept_len, void *workspace, size_t workspace_bytes, void *hip_stream) {
    return verify_impl<true>(hidden, M, K, ldh, w_packed, nullptr, V, draft_ids, n_draft, out_argmax, out_accept_len,
                             workspace, workspace_bytes, hip_stream);
}

int quasar_read_stream(const void *src, size_t bytes, void *sink, void *hip_stream) {
    if (!src || !sink) return QUASAR_ERR_NULL;
    if (bytes < 1024 || bytes % 1024) return QUASAR_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(sink, 4)) return QUASAR_ERR_ALIGN;
    const long long nsteps = (long long)(bytes / 1024);
    long long grid = (long long)device_cus() * g_tune_wgs.load();
    if (grid > nsteps) grid = nsteps;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (g_tune_nw.load() == 16)
        hipLaunchKernelGGL((read_stream_kernel<16, 8>), dim3((int)grid), dim3(1024), 0, st,
                           static_cast<const u32x4 *>(src), nsteps, static_cast<unsigned int *>(sink));
    else
        hipLaunchKernelGGL((read_stream_kernel<8, 16>), dim3((int)grid), dim3(512), 0, st,
                           static_cast<const u32x4 *>(src), nsteps, static_cast<unsigned int *>(sink));
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

int quasar_copy_stream(void *dst, const void *src, size_t bytes, void *hip_stream) {
    if (!src || !dst) return QUASAR_ERR_NULL;
    if (bytes < 16 || bytes % 16) return QUASAR_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(dst, 16)) return QUASAR_ERR_ALIGN;
    const long long n16 = (long long)(bytes / 16);
    long long grid = (n16 + 255) / 256;
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(copy_stream_kernel, dim3((int)grid), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), n16);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------
// Whole-step sequences
// ------------------------------------------------------------------------------------------
namespace {

constexpr int kSeqWaves = 16;
constexpr int kSeqDepth = 8;
// the form with two alternating workgroups per compute unit (M <= 8): waves, ring depth, and the LDS
// bytes that let exactly two such workgroups share a compute unit
constexpr int kSeqWaves2 = 8;
constexpr int kSeqDepth2 = 12;
constexpr int kSeqMaxLds2 = 80 * 1024 - 1280;
constexpr int kSeqMinLds2 = 56 * 1024;
std::atomic<int> g_seq_form{0};          // 0: choose; 1 or 2: workgroups per compute unit wanted
constexpr int kSeqMagic = 0x51534551;   // "QSEQ"
// Bound on any single wait inside the whole-step launch: 200 ms of the 100 MHz constant clock.  A step takes
// about 2 ms; a wait that long means a workgroup is not running at all, and the launch then ends with the
// error word set instead of holding the device.
constexpr unsigned int kSeqSpinLimit = 20000000u;

struct SeqHandle {   // lives in quasar_sequence::words
    int magic, nphases, M, MP, w16, xs_bytes, sc_bytes, lds_bytes, grid, has_verify, n_linears, a8;
    int n_barriers, n_flag_waits, roles;
};
static_assert(sizeof(SeqHandle) <= sizeof(quasar_sequence), "handle must fit");

struct Range { uintptr_t lo, hi; };
bool overlaps(const Range &a, const Range &b) { return a.lo < b.hi && b.lo < a.hi; }

// Chunking of one phase for a fixed grid; returns false if it cannot fit the LDS.
bool plan_phase(SeqPhase &ph, int MP, bool w16, bool a8, int G, int &xs_bytes, int &sc_bytes, int &acc_bytes) {
    const int NB = MP == 32 ? 2 : 1;
    // bytes of LDS one step of activations takes: bf16 (64 k per int8 step, 32 per bf16 step) or int8 codes
    const int x_bytes_per_step = ((w16 || a8) ? 64 : 128) * MP;
    choose_chunks(ph.S, x_bytes_per_step, 2 * kSeqWaves * NB * 1024, ph.SC, ph.C);
    const int tpw = (ph.T + G - 1) / G;
    // (bf16 activations lie in LDS as token rows 16 bytes further apart than their length)
    xs_bytes = ph.SC * x_bytes_per_step + (a8 ? 0 : MP * 16);
    // row scales, then 256 bytes for the per-token step sizes of the W8A8 form
    sc_bytes = (w16 ? 0 : ((tpw * kTileRows * 2 + 15) / 16) * 16) + 256;
    acc_bytes = ph.C > 1 ? tpw * NB * 1024 : 0;
    return true;
}

// The vocabulary projection with fp32 outputs (input of the stochastic verification): the
// int8-weight streaming kernel in its default shape, logits to part32[m][n].
int launch_logits(const GemmParams &base, int M, hipStream_t stream) {
    GemmParams p = base;
    p.Srow = p.S;
    p.ksplit = 1;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    const int NB = MP == 32 ? 2 : 1;
    const Plan pl = make_plan(p.T, p.S, 128 * MP, NB * 1024, 16, true);
    if (pl.grid > kMaxGrid) return QUASAR_ERR_SHAPE;
    p.SC = pl.SC;
    p.C = pl.C;
    p.xs_bytes = pl.xs_bytes;
    p.sc_bytes = pl.sc_bytes;
    if (MP == 8) return launch(stream_mfma_kernel<8, false, EPI_LOGITS, 16, 4>, pl.grid, 1024, pl.lds_bytes, stream, p);
    if (MP == 16) return launch(stream_mfma_kernel<16, false, EPI_LOGITS, 16, 4>, pl.grid, 1024, pl.lds_bytes, stream, p);
    return launch(stream_mfma_kernel<32, false, EPI_LOGITS, 16, 4>, pl.grid, 1024, pl.lds_bytes, stream, p);
}

template <int EPI>
int launch_w8a8(const GemmParams &base, int M, hipStream_t stream, int *grid_out) {
    GemmParams p = base;
    p.Srow = p.S;
    p.ksplit = 1;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    const int NB = MP == 32 ? 2 : 1;
    // int8 codes: 64 bytes of LDS per token and step; 256 bytes more for the per-token steps
    Plan pl = make_plan(p.T, p.S, 64 * MP, NB * 1024, 16, true);
    if (pl.grid > kMaxGrid) return QUASAR_ERR_SHAPE;
    p.SC = pl.SC;
    p.C = pl.C;
    p.xs_bytes = pl.xs_bytes;
    p.sc_bytes = pl.sc_bytes + 256;
    const int lds = pl.lds_bytes + 256;
    if (grid_out) *grid_out = pl.grid;
    if (MP == 8) return launch(stream_w8a8_kernel<8, EPI, 16, 8>, pl.grid, 1024, lds, stream, p);
    if (MP == 16) return launch(stream_w8a8_kernel<16, EPI, 16, 8>, pl.grid, 1024, lds, stream, p);
    return launch(stream_w8a8_kernel<32, EPI, 16, 8>, pl.grid, 1024, lds, stream, p);
}

// The int8 linear with the block's surrounding operations fused in: default launch shape, K in
// chunks when the activations do not fit the LDS (no split across workgroups).  The gate/up form
// hands tiles out in pairs and keeps NB KB of the scale region for the gate tile of a pair.
template <int EPI, int PRE, bool RES>
int launch_fused(const GemmParams &base, int M, hipStream_t stream) {
    GemmParams p = base;
    p.Srow = p.S;
    p.ksplit = 1;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    const int NB = MP == 32 ? 2 : 1;
    Plan pl = make_plan(p.T, p.S, 128 * MP, NB * 1024, 16, true);
    int lds = pl.lds_bytes;
    int sc_bytes = pl.sc_bytes;
    if (EPI == EPI_SWIGLU) {
        // whole pairs per workgroup: up to one tile more than an even split, and the kept gate tile
        const int pairs = p.T / 2;
        if (pl.grid > pairs) pl.grid = pairs;
        const int tpw = 2 * ((pairs + pl.grid - 1) / pl.grid);
        sc_bytes = ((tpw * kTileRows * 2 + 15) / 16) * 16 + NB * 1024;
        lds = pl.xs_bytes + sc_bytes + 2 * 16 * NB * 1024 + (pl.C > 1 ? tpw * NB * 1024 : 0);
        if (lds < kMinLds) lds = kMinLds;
    }
    if (pl.grid > kMaxGrid || pl.grid < 1 || lds > kMaxLds) return QUASAR_ERR_SHAPE;
    p.SC = pl.SC;
    p.C = pl.C;
    p.xs_bytes = pl.xs_bytes;
    p.sc_bytes = sc_bytes;
    if (MP == 8)
        return launch(stream_mfma_kernel<8, false, EPI, 16, 4, PRE, RES>, pl.grid, 1024, lds, stream, p);
    if (MP == 16)
        return launch(stream_mfma_kernel<16, false, EPI, 16, 4, PRE, RES>, pl.grid, 1024, lds, stream, p);
    return launch(stream_mfma_kernel<32, false, EPI, 16, 4, PRE, RES>, pl.grid, 1024, lds, stream, p);
}

std::atomic<int> g_w4_nw{16};
std::atomic<int> g_w4_d{2};

int check_mnk_w4(int64_t M, int64_t N, int64_t K) {
    if (const int e = check_mnk(M, N, K)) return e;
    return K % kStepK4 ? QUASAR_ERR_SHAPE : QUASAR_OK;
}

// LDS plan of the 4-bit kernel: activations of a K chunk (+ one f32x4 group offset per step and
// token), staging for the pair-end sums, running pair sums when K is chunked.  When the running
// sums of a workgroup's tiles leave too little room for activations the tiles are spread over more
// workgroups than compute units.
struct PlanW4 { int SC, C, xs_bytes, lds_bytes, grid; };
bool plan_w4(int T, int S, int MP, int NW, PlanW4 &pl) {
    const int NB = MP == 32 ? 2 : 1;
    const int PAR = NB == 1 ? 2 : 1;
    const int stage = PAR * NW * 2 * NB * 1024;
    const int xps = 272 * MP;
    int grid = device_cus();
    if (grid > T) grid = T;
    // (+ 512: the activations lie in LDS as token rows 16 bytes further apart than their length, at most 32 rows)
    if ((long long)S * xps + 512 + stage + 64 <= kMaxLds) {
        pl.SC = S;
        pl.C = 1;
        pl.xs_bytes = S * xps + 512;
        pl.lds_bytes = pl.xs_bytes + stage;
    } else {
        const int want = S < 8 ? S : 8;      // steps per chunk worth having
        for (;;) {
            const int tpw = (T + grid - 1) / grid;
            const int sums = ((tpw + 1) / 2) * 2 * NB * 1024;
            const int per = (kMaxLds - stage - sums - 64 - 512) / xps;
            const bool can_grow = grid < T && grid * 2 <= kMaxGrid;
            if (per >= want || (per >= 1 && !can_grow)) {
                pl.C = (S + per - 1) / per;
                pl.SC = (S + pl.C - 1) / pl.C;
                pl.C = (S + pl.SC - 1) / pl.SC;
                pl.xs_bytes = pl.SC * xps + 512;
                pl.lds_bytes = pl.xs_bytes + stage + sums;
                break;
            }
            if (!can_grow) return false;
            grid = grid * 2 > T ? T : grid * 2;
        }
    }
    if (pl.lds_bytes < kMinLds) pl.lds_bytes = kMinLds;
    pl.grid = grid;
    return true;
}

template <int EPI>
int launch_w4(const GemmParams &base, int M, hipStream_t stream, int *grid_out) {
    GemmParams p = base;
    p.Srow = p.S;
    p.ksplit = 1;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    const int NW = g_w4_nw.load(), DD = g_w4_d.load();
    PlanW4 pl{};
    if (!plan_w4(p.T, p.S, MP, NW, pl) || pl.grid > kMaxGrid) return QUASAR_ERR_SHAPE;
    p.SC = pl.SC;
    p.C = pl.C;
    p.xs_bytes = pl.xs_bytes;
    p.sc_bytes = 0;
    if (grid_out) *grid_out = pl.grid;
#define QUASAR_LAUNCH_W4(MPV)                                                                              \
    (NW == 16 ? (DD == 4 ? launch(stream_w4_kernel<MPV, EPI, 16, 4>, pl.grid, 1024, pl.lds_bytes, stream, p) \
                         : launch(stream_w4_kernel<MPV, EPI, 16, 2>, pl.grid, 1024, pl.lds_bytes, stream, p)) \
              : (DD == 8 ? launch(stream_w4_kernel<MPV, EPI, 8, 8>, pl.grid, 512, pl.lds_bytes, stream, p)   \
                         : launch(stream_w4_kernel<MPV, EPI, 8, 4>, pl.grid, 512, pl.lds_bytes, stream, p)))
    if (MP == 8) return QUASAR_LAUNCH_W4(8);
    if (MP == 16) return QUASAR_LAUNCH_W4(16);
    return QUASAR_LAUNCH_W4(32);
#undef QUASAR_LAUNCH_W4
}

template <int MP, bool W16, bool A8, int ROLES>
int launch_sequence(const SeqHandle &h, const SeqParams &sp, hipStream_t st) {
    constexpr int NW = ROLES == 2 ? kSeqWaves2 : kSeqWaves;
    auto kernel = stream_sequence_kernel<MP, W16, A8, NW, (ROLES == 2 ? kSeqDepth2 : kSeqDepth), ROLES>;
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return QUASAR_ERR_HIP;
    hipLaunchKernelGGL(sequence_reset_kernel, dim3(1), dim3(256), 0, st, sp.sync);
    // Plain launch: every workgroup is resident by construction (grid = ROLES workgroups per compute
    // unit, and that many fit each; checked when the sequence is prepared); a cooperative launch
    // would add ~20 us.
    hipLaunchKernelGGL(kernel, dim3(h.grid), dim3(NW * 64), (unsigned int)h.lds_bytes, st, sp);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

// Workgroups of this kernel shape that fit one compute unit (0 on error).
template <int MP, bool W16, bool A8, int ROLES>
int sequence_residency(int lds_bytes) {
    constexpr int NW = ROLES == 2 ? kSeqWaves2 : kSeqWaves;
    auto kernel = stream_sequence_kernel<MP, W16, A8, NW, (ROLES == 2 ? kSeqDepth2 : kSeqDepth), ROLES>;
    if (!allow_large_lds(reinterpret_cast<const void *>(kernel))) return 0;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, NW * 64, (size_t)lds_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return per_cu;
}
template <int ROLES>
int sequence_residency_of(int MP, bool w16, bool a8, int lds_bytes) {
    if constexpr (ROLES == 2) {
        if (MP != 8) return 0;
        return w16 ? sequence_residency<8, true, false, 2>(lds_bytes)
                   : (a8 ? sequence_residency<8, false, true, 2>(lds_bytes) : sequence_residency<8, false, false, 2>(lds_bytes));
    } else {
        if (w16) return MP == 8 ? sequence_residency<8, true, false, 1>(lds_bytes)
                                : (MP == 16 ? sequence_residency<16, true, false, 1>(lds_bytes) : sequence_residency<32, true, false, 1>(lds_bytes));
        if (a8) return MP == 8 ? sequence_residency<8, false, true, 1>(lds_bytes)
                               : (MP == 16 ? sequence_residency<16, false, true, 1>(lds_bytes) : sequence_residency<32, false, true, 1>(lds_bytes));
        return MP == 8 ? sequence_residency<8, false, false, 1>(lds_bytes)
                       : (MP == 16 ? sequence_residency<16, false, false, 1>(lds_bytes) : sequence_residency<32, false, false, 1>(lds_bytes));
    }
}

}  // namespace

extern "C" {

constexpr size_t kSeqZeroBytes = 1024;
// A vocabulary phase whose per-tile running sums do not fit the LDS is split into several phases over tile ranges:
// room for that many more table entries and flag rows than there are linears
constexpr int kSeqExtraPhases = 16;
constexpr size_t seq_table_phases(int64_t n_linears) { return (size_t)(n_linears + 1 + kSeqExtraPhases); }

size_t quasar_sequence_plan_bytes(int64_t n_linears) {
    if (n_linears < 0 || n_linears > (1 << 20)) return 0;
    return seq_table_phases(n_linears) * sizeof(SeqPhase) + kSeqZeroBytes;   // phase table, block of zeros
}

// workspace: [sync words, then one counter per compute-unit id][argmax partials][completion flags: (n_linears + 1 + spare) x grid]
constexpr size_t kSeqHeaderBytes = 16 * 1024;
static_assert((64 + kSeqCuSlots) * sizeof(unsigned int) <= kSeqHeaderBytes, "header holds the counters");
constexpr size_t kSeqPartialBytes = (size_t)kMaxGrid * 32u * sizeof(unsigned long long);

size_t quasar_sequence_workspace_bytes(int64_t n_linears, int64_t M) {
    if (M < 1 || M > 32 || n_linears < 0 || n_linears > (1 << 20)) return 0;
    return kSeqHeaderBytes + kSeqPartialBytes + seq_table_phases(n_linears) * kMaxGrid * sizeof(unsigned int);
}

static int sequence_prepare_impl(const quasar_linear_desc *linears, int64_t n_linears, const float *const *smooth,
                                 const quasar_verify_desc *verify, const float *verify_smooth, bool a8, int64_t M,
                                 void *plan_device, size_t plan_bytes, void *workspace, size_t workspace_bytes,
                                 quasar_sequence *seq) {
    if (!seq || !plan_device || !workspace || (n_linears > 0 && !linears)) return QUASAR_ERR_NULL;
    if (workspace_bytes < quasar_sequence_workspace_bytes(n_linears, M) || !aligned(workspace, 16))
        return QUASAR_ERR_WORKSPACE;
    if (n_linears < 0 || (n_linears == 0 && !verify)) return QUASAR_ERR_SHAPE;
    if (M < 1 || M > 32) return QUASAR_ERR_SHAPE;
    if (plan_bytes < quasar_sequence_plan_bytes(n_linears)) return QUASAR_ERR_WORKSPACE;
    if (!aligned(plan_device, 16)) return QUASAR_ERR_ALIGN;
    const bool w16 = n_linears > 0 ? linears[0].scales == nullptr : verify->scales == nullptr;
    if (a8 && w16) return QUASAR_ERR_DTYPE;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    const int NB = MP == 32 ? 2 : 1;
    const int G = device_cus();          // workgroups that share a phase (the grid is G times the workgroups per unit)
    if (2 * G > kMaxGrid) return QUASAR_ERR_SHAPE;

    std::vector<SeqPhase> phases;
    // every output written so far in the sequence: (range, phase, segment, N, ldy, pointer)
    struct Out { Range r; int ph, seg; long long N, ldy; const uint16_t *y; int writes; };
    std::vector<Out> outs;
    std::vector<Range> reads, writes;     // since the last device-wide barrier
    // every cache line read so far in the launch (never cleared): a line that some compute unit has
    // already fetched may sit in a cache with its old contents, so an input that is written inside the
    // launch AFTER one of its lines was read must be re-read past the caches (barrier form)
    struct LineRead { Range r; int ph; };
    std::vector<LineRead> lines_read;
    auto lines = [](const Range &r) { return Range{r.lo & ~(uintptr_t)127, (r.hi + 127) & ~(uintptr_t)127}; };
    // How does a phase reading `xr` (and writing `yrs`) have to wait?  (see SEQ_WAIT_* in
    // stream_sequence.hpp)  Writes that clash with anything touched since the last barrier, or
    // inputs in buffers written more than once, need the barrier; inputs that are write-once
    // outputs of at most two earlier phases are gated by those phases' completion flags.
    auto classify = [&](const Range &xr, const std::vector<Range> &yrs, int producers[2]) -> int {
        producers[0] = producers[1] = -1;
        bool write_clash = false, raw = false;
        for (const Range &y : yrs) {
            for (const Range &wr : writes) if (overlaps(y, wr)) write_clash = true;
            for (const Range &rd : reads) if (overlaps(y, rd)) write_clash = true;
        }
        for (const Range &wr : writes) if (overlaps(xr, wr)) raw = true;
        // a line of this input that an earlier phase read no later than the phase that (re)wrote it
        for (const Out &o : outs) {
            if (!overlaps(lines(xr), lines(o.r))) continue;
            for (const LineRead &lr : lines_read)
                if (lr.ph <= o.ph && overlaps(lines(xr), lr.r) && overlaps(lines(o.r), lr.r)) write_clash = true;
        }
        if (write_clash) return SEQ_WAIT_BARRIER;
        if (!raw) return SEQ_WAIT_NONE;
        int n = 0;
        for (const Out &o : outs) {
            if (!overlaps(xr, o.r)) continue;
            if (o.writes != 1) return SEQ_WAIT_BARRIER;
            if (n > 0 && producers[0] == o.ph) continue;
            if (n > 1 && producers[1] == o.ph) continue;
            if (n == 2) return SEQ_WAIT_BARRIER;
            producers[n++] = o.ph;
        }
        return n > 0 ? SEQ_WAIT_FLAGS : SEQ_WAIT_BARRIER;
    };
    auto note_output = [&](const Range &yr, int ph, int seg, long long N, long long ldy, const uint16_t *y) {
        int n = 1;
        for (Out &o : outs)
            if (overlaps(o.r, yr)) { ++o.writes; n = o.writes; }
        outs.push_back(Out{yr, ph, seg, N, ldy, y, n});
    };
    for (int64_t i = 0; i < n_linears; ++i) {
        const quasar_linear_desc &d = linears[i];
        if (!d.x || !d.w_packed || !d.y) return QUASAR_ERR_NULL;
        if ((d.scales == nullptr) != w16) return QUASAR_ERR_DTYPE;
        if (const int e = check_mnk(M, d.N, d.K)) return e;
        if (d.ldx < d.K || d.ldy < d.N || d.ldx % 8 || d.ldy % 8) return QUASAR_ERR_SHAPE;
        if (!aligned(d.x, 16) || !aligned(d.y, 16) || !aligned(d.w_packed, 16) || (!w16 && !aligned(d.scales, 8)))
            return QUASAR_ERR_ALIGN;
        const Range xr{reinterpret_cast<uintptr_t>(d.x), reinterpret_cast<uintptr_t>(d.x + (M - 1) * d.ldx + d.K)};
        const Range yr{reinterpret_cast<uintptr_t>(d.y), reinterpret_cast<uintptr_t>(d.y + (M - 1) * d.ldy + d.N)};
        if (overlaps(xr, yr)) return QUASAR_ERR_SHAPE;    // in-place is not supported
        const float *sm = (a8 && smooth) ? smooth[i] : nullptr;
        if (!aligned(sm, 16)) return QUASAR_ERR_ALIGN;
        // join the previous phase when it reads the same input (smoothed the same way) and nothing
        // orders the two
        if (!phases.empty()) {
            SeqPhase &p = phases.back();
            if (p.kind == EPI_LINEAR && p.nseg < kMaxSeg && p.x == d.x && p.ldx == d.ldx && p.K == (int)d.K &&
                p.smooth == sm) {
                bool clash = false;
                // (the shared input is already waited for by the phase being joined)
                for (const Range &wr : writes) if (overlaps(yr, wr)) clash = true;
                for (const Range &rd : reads) if (overlaps(yr, rd)) clash = true;
                for (const Out &o : outs) if (overlaps(o.r, yr)) clash = true;   // keeps outputs single-assignment
                if (!clash) {
                    SeqSeg &sg = p.seg[p.nseg];
                    sg.w = static_cast<const u32x4 *>(d.w_packed); sg.scales = d.scales; sg.y = d.y; sg.ldy = d.ldy;
                    sg.tile_begin = p.T; sg.N = (int)d.N;
                    p.T += (int)(d.N / kTileRows);
                    note_output(yr, (int)phases.size() - 1, p.nseg, d.N, d.ldy, d.y);
                    ++p.nseg;
                    writes.push_back(yr);
                    continue;
                }
            }
        }
        SeqPhase p{};
        p.smooth = sm;
        p.x = d.x; p.ldx = d.ldx; p.nseg = 1; p.K = (int)d.K;
        p.S = (int)(d.K / (w16 ? kStepK16 : kStepK8));
        p.T = (int)(d.N / kTileRows);
        p.kind = EPI_LINEAR;
        p.seg[0].w = static_cast<const u32x4 *>(d.w_packed); p.seg[0].scales = d.scales; p.seg[0].y = d.y;
        p.seg[0].ldy = d.ldy; p.seg[0].tile_begin = 0; p.seg[0].N = (int)d.N;
        p.producer[0] = p.producer[1] = -1;
        p.wait = phases.empty() ? SEQ_WAIT_NONE : classify(xr, {yr}, p.producer);
        if (p.wait == SEQ_WAIT_BARRIER) { reads.clear(); writes.clear(); }
        reads.push_back(xr);
        lines_read.push_back(LineRead{lines(xr), (int)phases.size()});
        writes.push_back(yr);
        note_output(yr, (int)phases.size(), 0, d.N, d.ldy, d.y);
        phases.push_back(p);
    }
    // an output that turned out to be written again later must not be gated by flags
    for (SeqPhase &p : phases) {
        if (p.wait != SEQ_WAIT_FLAGS) continue;
        for (const Out &o : outs)
            if ((o.ph == p.producer[0] || o.ph == p.producer[1]) && o.writes > 1) p.wait = SEQ_WAIT_BARRIER;
    }
    if (verify) {
        const quasar_verify_desc &v = *verify;
        if (!v.hidden || !v.w_packed || !v.out_argmax || !v.out_accept_len) return QUASAR_ERR_NULL;
        if (v.n_draft > 0 && !v.draft_ids) return QUASAR_ERR_NULL;
        if ((v.scales == nullptr) != w16) return QUASAR_ERR_DTYPE;
        if (const int e = check_mnk(M, v.V, v.K)) return e;
        if (v.V > 0x7FFFFFF0ll || v.n_draft < 0 || v.n_draft > M || v.ldh < v.K || v.ldh % 8) return QUASAR_ERR_SHAPE;
        if (!aligned(v.hidden, 16) || !aligned(v.w_packed, 16) || (!w16 && !aligned(v.scales, 8))) return QUASAR_ERR_ALIGN;
        if (!aligned(verify_smooth, 16)) return QUASAR_ERR_ALIGN;
        SeqPhase p{};
        p.smooth = a8 ? verify_smooth : nullptr;
        p.x = v.hidden; p.ldx = v.ldh; p.nseg = 1; p.K = (int)v.K;
        p.S = (int)(v.K / (w16 ? kStepK16 : kStepK8));
        p.T = (int)(v.V / kTileRows);
        p.kind = EPI_ARGMAX;
        p.seg[0].w = static_cast<const u32x4 *>(v.w_packed); p.seg[0].scales = v.scales; p.seg[0].y = nullptr;
        p.seg[0].ldy = 0; p.seg[0].tile_begin = 0; p.seg[0].N = (int)v.V;
        p.draft = v.draft_ids; p.n_draft = (int)v.n_draft; p.out_argmax = v.out_argmax; p.out_accept = v.out_accept_len;
        p.V = (int)v.V;
        const Range xr{reinterpret_cast<uintptr_t>(v.hidden), reinterpret_cast<uintptr_t>(v.hidden + (M - 1) * v.ldh + v.K)};
        p.producer[0] = p.producer[1] = -1;
        p.wait = phases.empty() ? SEQ_WAIT_NONE : classify(xr, {}, p.producer);
        // When K is chunked every tile of a workgroup keeps a running sum in LDS.  If the vocabulary's share of
        // tiles does not fit beside the activations, the phase is split into phases over tile ranges that do:
        // weight and scale pointers advanced to the range, the row indices of the argmax shifted by as much,
        // the running argmax carried in registers from one to the next; the later ones find their input already
        // there.
        {
            int xs = 0, sc = 0, ac = 0;
            SeqPhase probe = p;
            plan_phase(probe, MP, w16, a8, G, xs, sc, ac);
            const int stage_all = 2 * kSeqWaves * NB * 1024;
            int part = p.T;
            if (xs + sc + stage_all + ac > kMaxLds) {
                const int per_tile = kTileRows * 2 + NB * 1024;
                const int room = kMaxLds - xs - stage_all - 256 - 64;
                const int tpw = room / per_tile;
                if (tpw < 1) return QUASAR_ERR_SHAPE;
                part = tpw * G;
            }
            const int nsub = (p.T + part - 1) / part;
            if (nsub > kSeqExtraPhases + 1) return QUASAR_ERR_SHAPE;
            const int T_all = p.T;
            for (int j = 0; j < nsub; ++j) {
                SeqPhase q = p;
                q.T = T_all - j * part < part ? T_all - j * part : part;
                q.tile_shift = j * part;
                q.seg[0].w = p.seg[0].w + (size_t)j * part * p.S * 64;
                if (p.seg[0].scales) q.seg[0].scales = p.seg[0].scales + (size_t)j * part * kTileRows;
                if (j > 0) { q.wait = SEQ_WAIT_NONE; q.producer[0] = q.producer[1] = -1; }
                phases.push_back(q);
            }
        }
    }
    for (SeqPhase &p : phases) {
        if (p.wait != SEQ_WAIT_FLAGS) { p.producer[0] = p.producer[1] = -1; continue; }
        phases[p.producer[0]].publish = 1;
        if (p.producer[1] >= 0) phases[p.producer[1]].publish = 1;
    }

    // LDS of a phase: activations (a K chunk), row scales, the cross-wave staging area, per-tile running sums
    // when K is chunked.  Every phase lays the LDS out for itself; the launch reserves the largest total.
    std::vector<int> acc_of(phases.size());
    const int stage1 = 2 * kSeqWaves * NB * 1024, stage2 = kSeqWaves2 * NB * 1024;
    for (size_t i = 0; i < phases.size(); ++i) {
        SeqPhase &p = phases[i];
        if ((long long)p.T * (G + 1) >= (1ll << 31)) return QUASAR_ERR_SHAPE;   // the kernel splits tiles in 32 bits
        int xs, sc, ac;
        plan_phase(p, MP, w16, a8, G, xs, sc, ac);
        p.xs_bytes = xs;
        p.sc_bytes = sc;
        p.raw_off = 0;
        acc_of[i] = ac;
        if (xs + sc + stage1 + ac > kMaxLds) return QUASAR_ERR_SHAPE;
        // W8A8: a phase whose activations take one chunk and need no cache-bypassing reads parks them in LDS
        // as bf16 (twice the bytes of its codes, behind them) and scans and quantises them there - one trip to
        // memory on the hand-over path instead of two - if the LDS has room for that.
        if (a8 && p.C == 1 && p.wait != SEQ_WAIT_BARRIER && 3 * xs + MP * 16 + sc + stage1 + ac <= kMaxLds) {
            p.raw_off = xs;
            p.xs_bytes = 3 * xs + MP * 16;   // (parked as token rows 16 bytes further apart than their length)
        }
    }
    auto lds_need = [&](int stage_bytes) {
        int most = 0;
        for (size_t i = 0; i < phases.size(); ++i) {
            const int n = phases[i].xs_bytes + phases[i].sc_bytes + stage_bytes + acc_of[i];
            if (n > most) most = n;
        }
        return most;
    };
    // One workgroup of 16 waves per compute unit, or two alternating ones of 8.  Measured on the 36-layer
    // step: the alternating form is ~15% faster when the phases do not wait for each other (while one
    // workgroup stages its activations the other streams) and ~25% slower on a chain of dependent phases
    // (every hand-over costs the same round trips, and half the waves then work through each phase).  So it
    // is chosen when at most a quarter of the phases wait, the shape allows it (M <= 8, everything fits
    // half the LDS with the K chunks that the single calls use - about 64 KB of activations, K <= 4096 for
    // bf16 activations - and two such workgroups are resident together), or when it is asked for.
    int n_waits = 0;
    for (const SeqPhase &p : phases) n_waits += p.wait != SEQ_WAIT_NONE;
    const int form = g_seq_form.load();
    const bool want2 = form == 2 || (form == 0 && 4 * n_waits <= (int)phases.size() && phases.size() >= 2);
    int roles = 1;
    int lds = lds_need(stage1);
    if (MP == 8 && want2) {
        int lds2 = lds_need(stage2);
        if (lds2 < kSeqMinLds2) lds2 = kSeqMinLds2;
        if (lds2 <= kSeqMaxLds2 && sequence_residency_of<2>(MP, w16, a8, lds2) >= 2) {
            roles = 2;
            lds = lds2;
        } else if (form == 2) {
            return QUASAR_ERR_SHAPE;
        }
    } else if (form == 2) {
        return QUASAR_ERR_SHAPE;
    }
    if (lds > kMaxLds) return QUASAR_ERR_SHAPE;
    if (hipMemcpy(plan_device, phases.data(), phases.size() * sizeof(SeqPhase), hipMemcpyHostToDevice) != hipSuccess)
        return QUASAR_ERR_HIP;
    if (hipMemset(static_cast<unsigned char *>(plan_device) + seq_table_phases(n_linears) * sizeof(SeqPhase), 0,
                  kSeqZeroBytes) != hipSuccess)
        return QUASAR_ERR_HIP;
    // epoch and completion flags start from zero (the first launch runs in epoch 1)
    if (hipMemset(workspace, 0, quasar_sequence_workspace_bytes(n_linears, M)) != hipSuccess) return QUASAR_ERR_HIP;
    if (hipDeviceSynchronize() != hipSuccess) return QUASAR_ERR_HIP;
    SeqHandle h{};
    h.magic = kSeqMagic; h.nphases = (int)phases.size(); h.M = (int)M; h.MP = MP; h.w16 = w16 ? 1 : 0;
    h.xs_bytes = 0; h.sc_bytes = 256;      // layout before the first phase (the kernel's start-up scratch sits in the staging area)
    h.lds_bytes = (roles == 1 && lds < kMinLds) ? kMinLds : lds;
    h.grid = G * roles; h.roles = roles;
    h.has_verify = verify ? 1 : 0; h.n_linears = (int)n_linears; h.a8 = a8 ? 1 : 0;
    h.n_barriers = 0; h.n_flag_waits = 0;
    for (const SeqPhase &p : phases) {
        if (p.wait == SEQ_WAIT_BARRIER) ++h.n_barriers;
        if (p.wait == SEQ_WAIT_FLAGS) ++h.n_flag_waits;
    }
    // The launch relies on every workgroup being resident at once (they wait for each other).
    if (roles == 1 && sequence_residency_of<1>(MP, w16, a8, h.lds_bytes) < 1) return QUASAR_ERR_HIP;
    std::memset(seq, 0, sizeof(*seq));
    std::memcpy(seq, &h, sizeof(h));
    return QUASAR_OK;
}

int quasar_sequence_prepare(const quasar_linear_desc *linears, int64_t n_linears, const quasar_verify_desc *verify,
                            int64_t M, void *plan_device, size_t plan_bytes, void *workspace, size_t workspace_bytes,
                            quasar_sequence *seq) {
    return sequence_prepare_impl(linears, n_linears, nullptr, verify, nullptr, false, M, plan_device, plan_bytes,
                                 workspace, workspace_bytes, seq);
}

int quasar_sequence_prepare_w8a8(const quasar_linear_desc *linears, int64_t n_linears, const float *const *smooth,
                                 const quasar_verify_desc *verify, const float *verify_smooth, int64_t M,
                                 void *plan_device, size_t plan_bytes, void *workspace, size_t workspace_bytes,
                                 quasar_sequence *seq) {
    return sequence_prepare_impl(linears, n_linears, smooth, verify, verify_smooth, true, M, plan_device, plan_bytes,
                                 workspace, workspace_bytes, seq);
}

static int sequence_run_impl(const quasar_sequence *seq, const void *plan_device, void *workspace, size_t workspace_bytes,
                             uint64_t *stamps, size_t stamps_bytes, void *hip_stream) {
    if (!seq || !plan_device || !workspace) return QUASAR_ERR_NULL;
    SeqHandle h;
    std::memcpy(&h, seq, sizeof(h));
    if (h.magic != kSeqMagic || h.nphases < 1) return QUASAR_ERR_SHAPE;
    if (workspace_bytes < quasar_sequence_workspace_bytes(h.n_linears, h.M)) return QUASAR_ERR_WORKSPACE;
    if (!aligned(workspace, 16) || !aligned(plan_device, 16)) return QUASAR_ERR_ALIGN;
    if ((h.roles != 1 && h.roles != 2) || h.grid != device_cus() * h.roles) return QUASAR_ERR_SHAPE;   // prepared for another device
    SeqParams sp{};
    sp.phases = static_cast<const SeqPhase *>(plan_device);
    sp.nphases = h.nphases; sp.M = h.M; sp.xs_bytes = h.xs_bytes; sp.sc_bytes = h.sc_bytes;
    sp.sync = static_cast<unsigned int *>(workspace);
    sp.partial = reinterpret_cast<unsigned long long *>(static_cast<unsigned char *>(workspace) + kSeqHeaderBytes);
    sp.flags = reinterpret_cast<unsigned int *>(static_cast<unsigned char *>(workspace) + kSeqHeaderBytes + kSeqPartialBytes);
    sp.spin_limit = kSeqSpinLimit;
    sp.stamps = nullptr;
    if (stamps) {
        if (stamps_bytes < (size_t)h.nphases * h.grid * 8 * sizeof(uint64_t)) return QUASAR_ERR_WORKSPACE;
        if (!aligned(stamps, 8)) return QUASAR_ERR_ALIGN;
        sp.stamps = reinterpret_cast<unsigned long long *>(stamps);
    }
    sp.zeros = reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(plan_device) +
                                               seq_table_phases(h.n_linears) * sizeof(SeqPhase));
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (h.roles == 2) {
        if (h.MP != 8) return QUASAR_ERR_SHAPE;
        if (h.w16) return launch_sequence<8, true, false, 2>(h, sp, st);
        if (h.a8) return launch_sequence<8, false, true, 2>(h, sp, st);
        return launch_sequence<8, false, false, 2>(h, sp, st);
    }
    if (h.w16) {
        if (h.MP == 8) return launch_sequence<8, true, false, 1>(h, sp, st);
        if (h.MP == 16) return launch_sequence<16, true, false, 1>(h, sp, st);
        return launch_sequence<32, true, false, 1>(h, sp, st);
    }
    if (h.a8) {
        if (h.MP == 8) return launch_sequence<8, false, true, 1>(h, sp, st);
        if (h.MP == 16) return launch_sequence<16, false, true, 1>(h, sp, st);
        return launch_sequence<32, false, true, 1>(h, sp, st);
    }
    if (h.MP == 8) return launch_sequence<8, false, false, 1>(h, sp, st);
    if (h.MP == 16) return launch_sequence<16, false, false, 1>(h, sp, st);
    return launch_sequence<32, false, false, 1>(h, sp, st);
}

int quasar_sequence_run(const quasar_sequence *seq, const void *plan_device, void *workspace, size_t workspace_bytes,
                        void *hip_stream) {
    return sequence_run_impl(seq, plan_device, workspace, workspace_bytes, nullptr, 0, hip_stream);
}

size_t quasar_sequence_stamps_bytes(const quasar_sequence *seq) {
    if (!seq) return 0;
    SeqHandle h;
    std::memcpy(&h, seq, sizeof(h));
    if (h.magic != kSeqMagic) return 0;
    return (size_t)h.nphases * h.grid * 8 * sizeof(uint64_t);
}

int quasar_sequence_run_stamped(const quasar_sequence *seq, const void *plan_device, void *workspace,
                                size_t workspace_bytes, uint64_t *stamps, size_t stamps_bytes, void *hip_stream) {
    if (!stamps) return QUASAR_ERR_NULL;
    return sequence_run_impl(seq, plan_device, workspace, workspace_bytes, stamps, stamps_bytes, hip_stream);
}

int quasar_set_sequence_form(int workgroups_per_cu) {
    if (workgroups_per_cu < 0 || workgroups_per_cu > 2) return QUASAR_ERR_SHAPE;
    g_seq_form = workgroups_per_cu;
    return QUASAR_OK;
}

int quasar_quantize_activations(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const float *smooth,
                                int8_t *xq, float *dx, void *hip_stream) {
    if (!x || !xq || !dx) return QUASAR_ERR_NULL;
    if (const int e = check_mnk(M, 16, K)) return e;
    if (ldx < K || ldx % 8) return QUASAR_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(xq, 8) || !aligned(dx, 4) || !aligned(smooth, 16)) return QUASAR_ERR_ALIGN;
    hipLaunchKernelGGL(quantize_activations_kernel, dim3((unsigned int)M), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), x, (long long)ldx, (int)K, smooth, xq, dx);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

int quasar_w8a8_linear(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const float *smooth,
                       const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t N, uint16_t *y, int64_t ldy,
                       void *workspace, size_t workspace_bytes, void *hip_stream) {
    (void)workspace; (void)workspace_bytes;
    if (!x || !wq_packed || !scales_bf16 || !y) return QUASAR_ERR_NULL;
    if (const int e = check_mnk(M, N, K)) return e;
    if (ldx < K || ldy < N || ldx % 8 || ldy % 8) return QUASAR_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(wq_packed, 16) || !aligned(scales_bf16, 8) ||
        !aligned(smooth, 16))
        return QUASAR_ERR_ALIGN;
    GemmParams p{};
    p.x = x; p.ldx = ldx; p.w = reinterpret_cast<const u32x4 *>(wq_packed); p.scales = scales_bf16;
    p.y = y; p.ldy = ldy; p.partial = nullptr; p.smooth = smooth;
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.T = (int)(N / kTileRows);
    p.S = (int)(K / kStepK8);
    return launch_w8a8<EPI_LINEAR>(p, (int)M, static_cast<hipStream_t>(hip_stream), nullptr);
}

int quasar_w8a8_lmhead_verify(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh, const float *smooth,
                              const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t V,
                              const int32_t *draft_ids, int64_t n_draft, int32_t *out_argmax,
                              int32_t *out_accept_len, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!hidden || !wq_packed || !scales_bf16 || !out_argmax || !out_accept_len) return QUASAR_ERR_NULL;
    if (n_draft > 0 && !draft_ids) return QUASAR_ERR_NULL;
    if (const int e = check_mnk(M, V, K)) return e;
    if (V > 0x7FFFFFF0ll) return QUASAR_ERR_SHAPE;
    if (n_draft < 0 || n_draft > M) return QUASAR_ERR_SHAPE;
    if (ldh < K || ldh % 8) return QUASAR_ERR_SHAPE;
    if (!aligned(hidden, 16) || !aligned(wq_packed, 16) || !aligned(scales_bf16, 8) || !aligned(smooth, 16))
        return QUASAR_ERR_ALIGN;
    if (!workspace || workspace_bytes < quasar_workspace_bytes(M, V, K)) return QUASAR_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return QUASAR_ERR_ALIGN;
    GemmParams p{};
    p.x = hidden; p.ldx = ldh; p.w = reinterpret_cast<const u32x4 *>(wq_packed); p.scales = scales_bf16;
    p.y = nullptr; p.ldy = 0; p.partial = static_cast<unsigned long long *>(workspace); p.smooth = smooth;
    p.M = (int)M; p.N = (int)V; p.K = (int)K;
    p.T = (int)(V / kTileRows);
    p.S = (int)(K / kStepK8);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int grid = 0;
    if (const int e = launch_w8a8<EPI_ARGMAX>(p, (int)M, st, &grid)) return e;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    hipLaunchKernelGGL(verify_finalize_kernel, dim3(1), dim3(1024), 0, st, p.partial, grid, MP, (int)M, (int)V,
                       draft_ids, (int)n_draft, out_argmax, out_accept_len);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

size_t quasar_sample_workspace_bytes(int64_t M, int64_t V) {
    if (M < 1 || M > 32 || V < 16 || V % 16 || V > 0x7FFFFFF0ll) return 0;
    // logits, per-(position, vocabulary block) softmax statistics
    return (size_t)M * (size_t)V * sizeof(float) + 32u * (size_t)kSampleBlocks * 2u * sizeof(float);
}

int quasar_lmhead_verify_sample(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh, const int8_t *wq_packed,
                                const uint16_t *scales_bf16, int64_t V, const int32_t *draft_ids, int64_t n_draft,
                                float temperature, const float *u_accept, const float *u_sample,
                                int32_t *out_accept_len, int32_t *out_next_token, float *out_p_draft,
                                void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!hidden || !wq_packed || !scales_bf16 || !u_sample || !out_accept_len || !out_next_token)
        return QUASAR_ERR_NULL;
    if (n_draft > 0 && (!draft_ids || !u_accept)) return QUASAR_ERR_NULL;
    if (const int e = check_mnk(M, V, K)) return e;
    if (V > 0x7FFFFFF0ll) return QUASAR_ERR_SHAPE;
    if (n_draft < 0 || n_draft > M - 1) return QUASAR_ERR_SHAPE;     // the bonus token needs one position more
    if (!(temperature > 0.f) || !(temperature < 3.0e38f)) return QUASAR_ERR_SHAPE;
    if (ldh < K || ldh % 8) return QUASAR_ERR_SHAPE;
    if (!aligned(hidden, 16) || !aligned(wq_packed, 16) || !aligned(scales_bf16, 8) || !aligned(u_accept, 4) ||
        !aligned(u_sample, 4) || !aligned(out_p_draft, 4))
        return QUASAR_ERR_ALIGN;
    if (!workspace || workspace_bytes < quasar_sample_workspace_bytes(M, V)) return QUASAR_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return QUASAR_ERR_ALIGN;
    float *logits = static_cast<float *>(workspace);
    float *stats = logits + (size_t)M * (size_t)V;
    GemmParams p{};
    p.x = hidden; p.ldx = ldh; p.w = reinterpret_cast<const u32x4 *>(wq_packed); p.scales = scales_bf16;
    p.y = nullptr; p.ldy = 0; p.partial = nullptr; p.part32 = logits;
    p.M = (int)M; p.N = (int)V; p.K = (int)K;
    p.T = (int)(V / kTileRows);
    p.S = (int)(K / kStepK8);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (const int e = launch_logits(p, (int)M, st)) return e;
    const float inv_t = 1.0f / temperature;
    hipLaunchKernelGGL(softmax_partial_kernel, dim3(kSampleBlocks, (unsigned int)M), dim3(256), 0, st, logits, (int)V,
                       inv_t, stats);
    hipLaunchKernelGGL(speculative_sample_kernel, dim3(1), dim3(1024), 0, st, logits, (int)V, (int)M, inv_t, draft_ids,
                       (int)n_draft, u_accept, u_sample, stats, out_accept_len, out_next_token, out_p_draft);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

/* ---- 4-bit group-wise weights ---- */

size_t quasar_w4_packed_bytes(int64_t N, int64_t K) {
    if (check_mnk_w4(1, N, K)) return 0;
    return (size_t)(N / kTileRows) * (size_t)(K / kStepK4) * (size_t)kStepBytes4;
}

/* waves per workgroup and ring depth (in slots of two steps): (16, 4), (16, 2), (8, 8) or (8, 4) */
int quasar_set_tuning_w4(int waves, int depth) {
    if (!((waves == 16 && (depth == 4 || depth == 2)) || (waves == 8 && (depth == 8 || depth == 4))))
        return QUASAR_ERR_SHAPE;
    g_w4_nw = waves;
    g_w4_d = depth;
    return QUASAR_OK;
}

int quasar_quantize_weights_w4(const void *w, int w_dtype, int64_t N, int64_t K, int64_t ldw, void *w4_packed,
                               void *hip_stream) {
    if (!w || !w4_packed) return QUASAR_ERR_NULL;
    if (w_dtype != QUASAR_F32 && w_dtype != QUASAR_BF16) return QUASAR_ERR_DTYPE;
    if (const int e = check_mnk_w4(1, N, K)) return e;
    if (ldw < K) return QUASAR_ERR_SHAPE;
    if (!aligned(w4_packed, 16) || !aligned(w, w_dtype == QUASAR_F32 ? 4 : 2)) return QUASAR_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int T = (int)(N / kTileRows);
    if (w_dtype == QUASAR_F32)
        hipLaunchKernelGGL(quantize_pack_w4_kernel<false>, dim3(T), dim3(256), 0, st, w, (long long)ldw, (int)N, (int)K,
                           static_cast<unsigned char *>(w4_packed));
    else
        hipLaunchKernelGGL(quantize_pack_w4_kernel<true>, dim3(T), dim3(256), 0, st, w, (long long)ldw, (int)N, (int)K,
                           static_cast<unsigned char *>(w4_packed));
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

int quasar_unpack_weights_w4(const void *w4_packed, int64_t N, int64_t K, int8_t *q_rowmajor, uint16_t *scales_bf16,
                             void *hip_stream) {
    if (!w4_packed || !q_rowmajor || !scales_bf16) return QUASAR_ERR_NULL;
    if (const int e = check_mnk_w4(1, N, K)) return e;
    if (!aligned(w4_packed, 16) || !aligned(q_rowmajor, 8) || !aligned(scales_bf16, 2)) return QUASAR_ERR_ALIGN;
    const long long nwords = (long long)N * K / 8;
    const int grid = (int)((nwords + 255) / 256 > 65535 ? 65535 : (nwords + 255) / 256);
    hipLaunchKernelGGL(unpack_w4_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const unsigned char *>(w4_packed), (int)N, (int)K, q_rowmajor, scales_bf16);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

int quasar_w4_linear(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const void *w4_packed, int64_t N,
                     uint16_t *y, int64_t ldy, void *hip_stream) {
    if (!x || !w4_packed || !y) return QUASAR_ERR_NULL;
    if (const int e = check_mnk_w4(M, N, K)) return e;
    if (ldx < K || ldy < N || ldx % 8 || ldy % 8) return QUASAR_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(w4_packed, 16)) return QUASAR_ERR_ALIGN;
    GemmParams p{};
    p.x = x; p.ldx = ldx; p.w = static_cast<const u32x4 *>(w4_packed); p.scales = nullptr;
    p.y = y; p.ldy = ldy; p.partial = nullptr;
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.T = (int)(N / kTileRows);
    p.S = (int)(K / kStepK4);
    return launch_w4<EPI_LINEAR>(p, (int)M, static_cast<hipStream_t>(hip_stream), nullptr);
}

int quasar_w4_lmhead_verify(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh, const void *w4_packed,
                            int64_t V, const int32_t *draft_ids, int64_t n_draft, int32_t *out_argmax,
                            int32_t *out_accept_len, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!hidden || !w4_packed || !out_argmax || !out_accept_len) return QUASAR_ERR_NULL;
    if (n_draft > 0 && !draft_ids) return QUASAR_ERR_NULL;
    if (const int e = check_mnk_w4(M, V, K)) return e;
    if (V > 0x7FFFFFF0ll) return QUASAR_ERR_SHAPE;
    if (n_draft < 0 || n_draft > M) return QUASAR_ERR_SHAPE;
    if (ldh < K || ldh % 8) return QUASAR_ERR_SHAPE;
    if (!aligned(hidden, 16) || !aligned(w4_packed, 16)) return QUASAR_ERR_ALIGN;
    if (!workspace || workspace_bytes < quasar_workspace_bytes(M, V, K)) return QUASAR_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return QUASAR_ERR_ALIGN;
    GemmParams p{};
    p.x = hidden; p.ldx = ldh; p.w = static_cast<const u32x4 *>(w4_packed); p.scales = nullptr;
    p.y = nullptr; p.ldy = 0; p.partial = static_cast<unsigned long long *>(workspace);
    p.M = (int)M; p.N = (int)V; p.K = (int)K;
    p.T = (int)(V / kTileRows);
    p.S = (int)(K / kStepK4);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int grid = 0;
    if (const int e = launch_w4<EPI_ARGMAX>(p, (int)M, st, &grid)) return e;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    hipLaunchKernelGGL(verify_finalize_kernel, dim3(1), dim3(1024), 0, st, p.partial, grid, MP, (int)M, (int)V,
                       draft_ids, (int)n_draft, out_argmax, out_accept_len);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}


/* ---- int8 linears with the decoder block's surrounding operations fused in ---- */

int quasar_w8_linear_fused(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const uint16_t *gamma, float eps,
                           const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t N, const uint16_t *residual,
                           int64_t ldr, uint16_t *y, int64_t ldy, void *hip_stream) {
    if (!x || !wq_packed || !scales_bf16 || !y) return QUASAR_ERR_NULL;
    if (const int e = check_mnk(M, N, K)) return e;
    if (ldx < K || ldy < N || ldx % 8 || ldy % 8) return QUASAR_ERR_SHAPE;
    if (gamma && !(eps >= 0.f && eps < 1.0f)) return QUASAR_ERR_SHAPE;
    if (residual && (ldr < N || ldr % 4)) return QUASAR_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(wq_packed, 16) || !aligned(scales_bf16, 8) ||
        !aligned(gamma, 16) || !aligned(residual, 8))
        return QUASAR_ERR_ALIGN;
    GemmParams p{};
    p.x = x; p.ldx = ldx; p.w = reinterpret_cast<const u32x4 *>(wq_packed); p.scales = scales_bf16;
    p.y = y; p.ldy = ldy; p.partial = nullptr;
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.T = (int)(N / kTileRows);
    p.S = (int)(K / kStepK8);
    p.pre_arg = gamma; p.eps = eps; p.resid = residual; p.ldr = ldr;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int m = (int)M;
    if (gamma)
        return residual ? launch_fused<EPI_LINEAR, PRE_RMSNORM, true>(p, m, st)
                        : launch_fused<EPI_LINEAR, PRE_RMSNORM, false>(p, m, st);
    return residual ? launch_fused<EPI_LINEAR, PRE_NONE, true>(p, m, st)
                    : launch_fused<EPI_LINEAR, PRE_NONE, false>(p, m, st);
}

int quasar_w8_gateup_swiglu(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const uint16_t *gamma, float eps,
                            const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t I, uint16_t *y, int64_t ldy,
                            void *hip_stream) {
    if (!x || !wq_packed || !scales_bf16 || !y) return QUASAR_ERR_NULL;
    if (I < 16 || I % 16 || I > (1 << 25)) return QUASAR_ERR_SHAPE;
    if (const int e = check_mnk(M, 2 * I, K)) return e;
    if (ldx < K || ldy < I || ldx % 8 || ldy % 4) return QUASAR_ERR_SHAPE;
    if (gamma && !(eps >= 0.f && eps < 1.0f)) return QUASAR_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(y, 8) || !aligned(wq_packed, 16) || !aligned(scales_bf16, 8) || !aligned(gamma, 16))
        return QUASAR_ERR_ALIGN;
    GemmParams p{};
    p.x = x; p.ldx = ldx; p.w = reinterpret_cast<const u32x4 *>(wq_packed); p.scales = scales_bf16;
    p.y = y; p.ldy = ldy; p.partial = nullptr;
    p.M = (int)M; p.N = (int)(2 * I); p.K = (int)K;
    p.T = (int)(2 * I / kTileRows);
    p.S = (int)(K / kStepK8);
    p.pre_arg = gamma; p.eps = eps;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return gamma ? launch_fused<EPI_SWIGLU, PRE_RMSNORM, false>(p, (int)M, st)
                 : launch_fused<EPI_SWIGLU, PRE_NONE, false>(p, (int)M, st);
}

/* ---- attention of a verification step ---- */

namespace {
constexpr int kAttnWaves = 4;
struct AttnShape { int NQT, nblk, nsplit; };
bool attn_shape(int64_t M, int64_t Hq, int64_t Hkv, int64_t L_total, AttnShape &a) {
    if (M < 1 || M > 32 || Hkv < 1 || Hkv > 1024 || Hq < Hkv || Hq % Hkv || Hq > 4096) return false;
    if (L_total < M || L_total > (1 << 24)) return false;
    const int64_t R = M * (Hq / Hkv);
    if (R > 1024) return false;
    a.NQT = R <= 32 ? 2 : 4;                                       // rows per launch: 32 or 64
    a.nblk = (int)((L_total + kKvBlock - 1) / kKvBlock);
    int64_t cap = (int64_t)device_cus() / Hkv;                     // one workgroup per compute unit in total
    if (cap < 1) cap = 1;
    int64_t ns = a.nblk / kAttnWaves;
    if (ns < 1) ns = 1;
    a.nsplit = (int)(ns < cap ? ns : cap);
    return true;
}
int64_t cache_blocks(int64_t max_len) { return (max_len + kKvBlock - 1) / kKvBlock; }
}  // namespace

size_t quasar_kv_cache_bytes(int64_t n_kv_heads, int64_t max_len) {
    if (n_kv_heads < 1 || n_kv_heads > 1024 || max_len < 1 || max_len > (1 << 24)) return 0;
    return 2u * (size_t)n_kv_heads * (size_t)cache_blocks(max_len) * (size_t)kKvBlockBytes;
}

int quasar_kv_cache_fill(const uint16_t *k, const uint16_t *v, int64_t n, int64_t n_kv_heads, int64_t pos0,
                         void *kv_cache, int64_t max_len, void *hip_stream) {
    if (!k || !v || !kv_cache) return QUASAR_ERR_NULL;
    if (!quasar_kv_cache_bytes(n_kv_heads, max_len) || n < 1 || pos0 < 0 || pos0 + n > max_len) return QUASAR_ERR_SHAPE;
    if (!aligned(kv_cache, 16) || !aligned(k, 2) || !aligned(v, 2)) return QUASAR_ERR_ALIGN;
    const long long head_stride = (long long)cache_blocks(max_len) * kKvBlockBytes;
    unsigned char *kc = static_cast<unsigned char *>(kv_cache), *vc = kc + n_kv_heads * head_stride;
    const long long ne = (long long)n * n_kv_heads * kHeadDim;
    const int grid = (int)((ne + 255) / 256 > 4096 ? 4096 : (ne + 255) / 256);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(kv_cache_fill_kernel, dim3(grid), dim3(256), 0, st, k, ne, (int)n_kv_heads, (int)pos0, kc, head_stride, 0);
    hipLaunchKernelGGL(kv_cache_fill_kernel, dim3(grid), dim3(256), 0, st, v, ne, (int)n_kv_heads, (int)pos0, vc, head_stride, 1);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

int quasar_attn_prepare(const uint16_t *qkv, int64_t M, int64_t ld, int64_t n_q_heads, int64_t n_kv_heads, int64_t L,
                        const uint16_t *q_gamma, const uint16_t *k_gamma, float eps, float rope_theta, uint16_t *q_out,
                        int64_t ldq, void *kv_cache, int64_t max_len, void *hip_stream) {
    if (!qkv || !q_gamma || !k_gamma || !q_out || !kv_cache) return QUASAR_ERR_NULL;
    AttnShape a{};
    if (L < 0 || !attn_shape(M, n_q_heads, n_kv_heads, L + M, a)) return QUASAR_ERR_SHAPE;
    if (!quasar_kv_cache_bytes(n_kv_heads, max_len) || L + M > max_len) return QUASAR_ERR_SHAPE;
    if (ld < (n_q_heads + 2 * n_kv_heads) * kHeadDim || ldq < n_q_heads * kHeadDim) return QUASAR_ERR_SHAPE;
    if (!(eps >= 0.f && eps < 1.f) || !(rope_theta > 1.f) || !(rope_theta < 1e30f)) return QUASAR_ERR_SHAPE;
    if (!aligned(qkv, 2) || !aligned(q_out, 2) || !aligned(kv_cache, 16)) return QUASAR_ERR_ALIGN;
    const long long head_stride = (long long)cache_blocks(max_len) * kKvBlockBytes;
    unsigned char *kc = static_cast<unsigned char *>(kv_cache), *vc = kc + n_kv_heads * head_stride;
    hipLaunchKernelGGL(attn_prepare_kernel, dim3((unsigned int)(M * (n_q_heads + 2 * n_kv_heads))), dim3(64), 0,
                       static_cast<hipStream_t>(hip_stream), qkv, (long long)ld, (int)M, (int)n_q_heads, (int)n_kv_heads,
                       (int)L, q_gamma, k_gamma, eps, std::log2((double)rope_theta), q_out, (long long)ldq, kc, vc,
                       head_stride);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
}

size_t quasar_attention_workspace_bytes(int64_t M, int64_t n_q_heads, int64_t n_kv_heads, int64_t L_total) {
    AttnShape a{};
    if (!attn_shape(M, n_q_heads, n_kv_heads, L_total, a)) return 0;
    return (size_t)n_kv_heads * a.nsplit * a.NQT * (8 * 64 * 16 + 16 * 2 * 4);
}

int quasar_verify_attention(const uint16_t *q, int64_t M, int64_t ldq, int64_t n_q_heads, int64_t n_kv_heads,
                            const void *kv_cache, int64_t max_len, int64_t L_total, uint16_t *out, int64_t ldo,
                            void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!q || !kv_cache || !out) return QUASAR_ERR_NULL;
    AttnShape a{};
    if (!attn_shape(M, n_q_heads, n_kv_heads, L_total, a)) return QUASAR_ERR_SHAPE;
    if (!quasar_kv_cache_bytes(n_kv_heads, max_len) || L_total > max_len) return QUASAR_ERR_SHAPE;
    if (ldq < n_q_heads * kHeadDim || ldo < n_q_heads * kHeadDim || ldq % 8 || ldo % 4) return QUASAR_ERR_SHAPE;
    if (!aligned(q, 16) || !aligned(out, 8) || !aligned(kv_cache, 16)) return QUASAR_ERR_ALIGN;
    if (!workspace || workspace_bytes < quasar_attention_workspace_bytes(M, n_q_heads, n_kv_heads, L_total))
        return QUASAR_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return QUASAR_ERR_ALIGN;
    AttnParams p{};
    const long long head_stride = (long long)cache_blocks(max_len) * kKvBlockBytes;
    p.q = q; p.ldq = ldq;
    p.kcache = static_cast<const unsigned char *>(kv_cache);
    p.vcache = p.kcache + n_kv_heads * head_stride;
    p.head_stride = head_stride;
    p.out = out; p.ldo = ldo;
    p.part_o = static_cast<float *>(workspace);
    p.part_ml = p.part_o + (size_t)n_kv_heads * a.nsplit * a.NQT * 8 * 64 * 4;
    p.M = (int)M; p.G = (int)(n_q_heads / n_kv_heads); p.Hkv = (int)n_kv_heads;
    p.L_total = (int)L_total; p.nblk = a.nblk; p.nsplit = a.nsplit;
    p.scale_log2 = 1.4426950408889634f / 11.313708498984761f;      // log2(e) / sqrt(128)
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int lds = kAttnWaves * a.NQT * (8 * 64 * 16 + 16 * 2 * 4);
    const dim3 grid((unsigned int)a.nsplit, (unsigned int)n_kv_heads);
    const int R = (int)(M * (n_q_heads / n_kv_heads));
    for (int row0 = 0; row0 < R; row0 += 16 * a.NQT) {             // 64 query rows per pass over the cache
        p.row0 = row0;
        if (a.NQT == 2) {
            auto kern = verify_attention_kernel<2, kAttnWaves>;
            if (!allow_large_lds(reinterpret_cast<const void *>(kern))) return QUASAR_ERR_HIP;
            hipLaunchKernelGGL(kern, grid, dim3(kAttnWaves * 64), lds, st, p);
        } else {
            auto kern = verify_attention_kernel<4, kAttnWaves>;
            if (!allow_large_lds(reinterpret_cast<const void *>(kern))) return QUASAR_ERR_HIP;
            hipLaunchKernelGGL(kern, grid, dim3(kAttnWaves * 64), lds, st, p);
        }
        if (hipGetLastError() != hipSuccess) return QUASAR_ERR_HIP;
        hipLaunchKernelGGL(attention_merge_kernel, dim3((unsigned int)(n_kv_heads * a.NQT * 8)), dim3(512), 0, st, p, a.NQT);
        if (hipGetLastError() != hipSuccess) return QUASAR_ERR_HIP;
    }
    return QUASAR_OK;
}

/* ---- prompt-lookup n-gram drafter (host side) ---- */

struct quasar_drafter {
    NgramDrafter impl;
    quasar_drafter(int k_min, int k_max, int64_t cap) : impl(k_min, k_max, cap) {}
};

quasar_drafter *quasar_drafter_create(int k_min, int k_max, int64_t capacity_hint) {
    if (k_min < 1 || k_max < k_min || k_max > 64 || capacity_hint < 0) return nullptr;
    try {
        return new quasar_drafter(k_min, k_max, capacity_hint);
    } catch (...) {
        return nullptr;
    }
}

void quasar_drafter_destroy(quasar_drafter *d) { delete d; }

int quasar_drafter_append(quasar_drafter *d, const int32_t *tokens, int64_t n) {
    if (!d || (n > 0 && !tokens)) return QUASAR_ERR_NULL;
    if (n < 0 || d->impl.length() + n > (int64_t(1) << 31)) return QUASAR_ERR_SHAPE;
    try {
        d->impl.append(tokens, n);
    } catch (...) {
        return QUASAR_ERR_WORKSPACE;
    }
    return QUASAR_OK;
}

int64_t quasar_drafter_length(const quasar_drafter *d) { return d ? d->impl.length() : -1; }

int quasar_drafter_propose(const quasar_drafter *d, int64_t gamma, int32_t *out_draft, int64_t *out_n_draft,
                           int *out_lookup_len) {
    if (!d || !out_draft || !out_n_draft) return QUASAR_ERR_NULL;
    if (gamma < 1) return QUASAR_ERR_SHAPE;
    *out_n_draft = d->impl.propose(gamma, out_draft, out_lookup_len);
    return QUASAR_OK;
}

}  // extern "C"
