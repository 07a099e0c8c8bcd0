// C-ABI entry points of the verification library: host-side validation, launch planning
// and kernel dispatch.  Everything that touches data runs in the HIP kernels included below.
#include "../../include/quasar.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <utility>
#include <vector>

#include "pack.hpp"
#include "probe.hpp"
#include "stream_gemm.hpp"

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

// x_bytes_per_step: LDS bytes one step of activations occupies; unit_bytes: LDS bytes of one
// tile accumulator / staging slot per wave; with_scales: reserve the row-scale table.
Plan make_plan(int T, int S, int x_bytes_per_step, int unit_bytes, int NW, bool with_scales) {
    Plan pl{};
    pl.S = S;
    const long long xall = (long long)S * x_bytes_per_step;
    if (xall <= kSingleChunkX) {
        pl.C = 1;
        pl.SC = S;
    } else {
        const int per = kMultiChunkX / x_bytes_per_step;   // steps per chunk that fit
        pl.C = (S + per - 1) / per;
        pl.SC = (S + pl.C - 1) / pl.C;
        pl.C = (S + pl.SC - 1) / pl.SC;
    }
    pl.xs_bytes = pl.SC * x_bytes_per_step;
    const int stage = 2 * NW * unit_bytes;
    int grid = device_cus() * g_tune_wgs.load();
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

template <bool W16, int EPI>
int launch_mfma(const GemmParams &base, int M, hipStream_t stream, int *grid_out) {
    GemmParams p = base;
    const int MP = M <= 8 ? 8 : (M <= 16 ? 16 : 32);
    const int NB = MP == 32 ? 2 : 1;
    const int NW = g_tune_nw.load();
    const Plan pl = make_plan(p.T, p.S, (W16 ? 64 : 128) * MP, NB * 1024, NW, !W16);
    if (pl.grid > kMaxGrid) return QUASAR_ERR_SHAPE;
    p.SC = pl.SC;
    p.C = pl.C;
    p.xs_bytes = pl.xs_bytes;
    p.sc_bytes = pl.sc_bytes;
    if (grid_out) *grid_out = pl.grid;
    const int DD = g_tune_d.load();
#define QUASAR_LAUNCH(MPV)                                                                                   \
    (NW == 16 ? (DD == 8 ? launch(stream_mfma_kernel<MPV, W16, EPI, 16, 8>, pl.grid, 1024, pl.lds_bytes, stream, p) \
                         : launch(stream_mfma_kernel<MPV, W16, EPI, 16, 4>, pl.grid, 1024, pl.lds_bytes, stream, p)) \
              : (DD == 8 ? launch(stream_mfma_kernel<MPV, W16, EPI, 8, 8>, pl.grid, 512, pl.lds_bytes, stream, p)    \
                         : launch(stream_mfma_kernel<MPV, W16, EPI, 8, 4>, pl.grid, 512, pl.lds_bytes, stream, p)))
    if (MP == 8) return QUASAR_LAUNCH(8);
    if (MP == 16) return QUASAR_LAUNCH(16);
    return QUASAR_LAUNCH(32);
#undef QUASAR_LAUNCH
}

int launch_valu(const GemmParams &base, int M, hipStream_t stream) {
    GemmParams p = base;
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
                int64_t N, uint16_t *y, int64_t ldy, void *stream) {
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
    return launch_mfma<W16, EPI_LINEAR>(p, (int)M, static_cast<hipStream_t>(stream), nullptr);
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

/* development knob, not part of the documented contract: waves per workgroup (8 or 16) and
 * workgroups per compute unit (1..8) used by the streaming kernels */
int quasar_set_tuning(int waves, int wgs_per_cu, int depth) {
    if ((waves != 8 && waves != 16) || wgs_per_cu < 1 || wgs_per_cu > 8 || (depth != 4 && depth != 8))
        return QUASAR_ERR_DTYPE;
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
    return (size_t)kMaxGrid * 32u * sizeof(unsigned long long);
}

int quasar_quantize_weights(const void *w, int w_dtype, int64_t N, int64_t K, int64_t ldw, int8_t *wq_packed,
                            uint16_t *scales_bf16, void *hip_stream) {
    if (!w || !wq_packed || !scales_bf16) return QUASAR_ERR_NULL;
    if (w_dtype != QUASAR_F32 && w_dtype != QUASAR_BF16) return QUASAR_ERR_DTYPE;
    if (const int e = check_mnk(1, N, K)) return e;
    if (ldw < K) return QUASAR_ERR_SHAPE;
    if (!aligned(wq_packed, 16) || !aligned(scales_bf16, 2) || !aligned(w, w_dtype == QUASAR_F32 ? 4 : 2))
        return QUASAR_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int T = (int)(N / kTileRows);
    if (w_dtype == QUASAR_F32)
        hipLaunchKernelGGL(quantize_pack_kernel<false>, dim3(T), dim3(256), 0, st, w, (long long)ldw, (int)N, (int)K,
                           reinterpret_cast<u32x4 *>(wq_packed), scales_bf16);
    else
        hipLaunchKernelGGL(quantize_pack_kernel<true>, dim3(T), dim3(256), 0, st, w, (long long)ldw, (int)N, (int)K,
                           reinterpret_cast<u32x4 *>(wq_packed), scales_bf16);
    return hipGetLastError() == hipSuccess ? QUASAR_OK : QUASAR_ERR_HIP;
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
    (void)workspace; (void)workspace_bytes;
    return linear_impl<false>(x, M, K, ldx, wq_packed, scales_bf16, N, y, ldy, hip_stream);
}

int quasar_lmhead_verify(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh, const int8_t *wq_packed,
                         const uint16_t *scales_bf16, int64_t V, const int32_t *draft_ids, int64_t n_draft,
                         int32_t *out_argmax, int32_t *out_accept_len, void *workspace, size_t workspace_bytes,
                         void *hip_stream) {
    return verify_impl<false>(hidden, M, K, ldh, wq_packed, scales_bf16, V, draft_ids, n_draft, out_argmax,
                              out_accept_len, workspace, workspace_bytes, hip_stream);
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
    (void)workspace; (void)workspace_bytes;
    return linear_impl<true>(x, M, K, ldx, w_packed, nullptr, N, y, ldy, hip_stream);
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
