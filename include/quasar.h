/*
 * quasar.h - C ABI of the int8 weight-streaming verification library for MI355X (gfx950).
 *
 * The library covers the memory-bound part of one verification step of
 * self-speculative decoding with a quantised verifier: every linear layer of the
 * target model applied to the M = gamma + 1 candidate positions, and the final
 * vocabulary projection followed by the acceptance decision.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or retains them.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *     Calls validate their arguments on the host, enqueue their kernels on that
 *     stream and return without waiting.  The returned status covers argument
 *     and launch errors only, not faults that surface later on the stream.
 *   - bf16 values are passed as uint16_t bit patterns.
 *   - Outputs are fully overwritten.  Workspace contents need not be
 *     initialised and are undefined afterwards.
 *   - Shape limits (checked, QUASAR_ERR_SHAPE otherwise):
 *         1 <= M <= 32,  K >= 64 and K % 64 == 0,  N >= 16 and N % 16 == 0,
 *         row strides (ldx, ldy, ldh, ldw) >= the row length; ldx, ldy, ldh % 8 == 0.
 *   - Alignment (checked, QUASAR_ERR_ALIGN otherwise): x, y, hidden, packed
 *     weights 16 bytes; scales 8 bytes; workspace 16 bytes.
 *   - Non-finite inputs give unspecified values but never a fault.
 *   - Concurrent calls on different streams are safe as long as they do not
 *     share output or workspace buffers.
 */
#ifndef QUASAR_H_
#define QUASAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum quasar_status {
    QUASAR_OK = 0,
    QUASAR_ERR_NULL = 1,       /* a required pointer is NULL */
    QUASAR_ERR_SHAPE = 2,      /* a size or stride is outside the documented limits */
    QUASAR_ERR_ALIGN = 3,      /* a pointer is not aligned as documented */
    QUASAR_ERR_WORKSPACE = 4,  /* workspace missing or smaller than quasar_workspace_bytes */
    QUASAR_ERR_DTYPE = 5,      /* unknown quasar_dtype / quasar_path value */
    QUASAR_ERR_HIP = 6         /* the HIP runtime reported an error at launch */
} quasar_status;

typedef enum quasar_dtype { QUASAR_F32 = 0, QUASAR_BF16 = 1 } quasar_dtype;

/* Contraction variant used by quasar_w8_linear (for A/B measurements). */
typedef enum quasar_path {
    QUASAR_PATH_AUTO = 0,  /* library's choice by M */
    QUASAR_PATH_VALU = 1,  /* fp32 FMA dot products on the vector ALUs, M <= 4 only */
    QUASAR_PATH_MFMA = 2   /* bf16 matrix-core tiles */
} quasar_path;

const char *quasar_status_string(int status);
int quasar_version(void);

/* Process-wide override of the contraction variant (host argument, not thread-safe
 * against concurrent calls).  Also settable through the environment variable
 * QUASAR_FORCE_PATH={auto,valu,mfma}, read when the library is loaded.
 * QUASAR_PATH_VALU with M > 4 falls back to MFMA.  Returns QUASAR_ERR_DTYPE for
 * an unknown value. */
int quasar_set_path(int path);
int quasar_get_path(void);

/* Development knobs (no passage of the paper stands behind them; process-wide, not thread-safe,
 * meant for launch-shape sweeps in the benchmark, never needed for correct results):
 *   quasar_set_tuning      waves per workgroup (8 or 16), workgroups per compute unit (1..8) and
 *                          load-ring depth (4 or 8) of the single-call int8 / bf16 kernels; the
 *                          first two can also be preset through the environment variables
 *                          QUASAR_TUNE_NW and QUASAR_TUNE_WGS, read when the library is loaded;
 *   quasar_set_tuning_w4   waves per workgroup and ring depth of the 4-bit kernel;
 *   quasar_set_sequence_form   workgroups per compute unit of the whole-step launch for sequences
 *                          prepared afterwards: 0 lets quasar_sequence_prepare choose (two alternating
 *                          workgroups of 8 waves when at most a quarter of the phases wait for an
 *                          earlier one, M <= 8 and the shapes fit half the LDS; else one of 16 waves),
 *                          1 or 2 asks for that form (2 makes prepare fail with QUASAR_ERR_SHAPE
 *                          where it does not fit).  Results are the same bits in both forms.
 * Each returns QUASAR_ERR_SHAPE for a value outside the stated set. */
int quasar_set_tuning(int waves, int wgs_per_cu, int depth);
int quasar_set_tuning_w4(int waves, int depth);
int quasar_set_sequence_form(int workgroups_per_cu);

/* Bytes of the packed int8 / packed bf16 weight buffer for an [N, K] matrix.
 * Int8: exactly one byte per parameter (the 2x footprint reduction of Sec. 3.3,
 * "Offline Weight Preparation"); bf16: two.  0 if the shape is invalid. */
size_t quasar_packed_bytes(int64_t N, int64_t K);
size_t quasar_packed_bytes_bf16(int64_t N, int64_t K);

/* Workspace bytes for quasar_*_lmhead_verify (per-workgroup argmax partials, always needed
 * there) and for the linear entry points.  A linear works without a workspace (NULL); given
 * one of at least this size, shapes whose activations do not fit the on-chip memory in one
 * piece (large M x K) split K across workgroups through fp32 partial sums in the workspace
 * instead of re-reading the activations chunk by chunk - same result up to fp32 summation
 * order, several times faster.  The workspace is scratch: undefined on entry and on exit. */
size_t quasar_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * Offline weight preparation (Sec. 3.2 Eq. 6: symmetric uniform quantisation
 * W_int8 = Q(W, delta_w); Sec. 3.3 "Offline Weight Preparation").
 *   w            device, [N, K] row-major, row stride ldw elements, fp32 or bf16
 *   wq_packed    device out, quasar_packed_bytes(N, K) bytes, tile order (opaque;
 *                quasar_unpack_weights recovers row-major codes)
 *   scales_bf16  device out, [N] bf16: delta_n = bf16(max_k|W[n,k]| / 127)
 * Per output row: q = clamp(rint(W / delta_n), -127, 127), rint = half to even,
 * quotient in fp32.  A row whose step rounds to zero gets delta = 0, q = 0.
 */
int quasar_quantize_weights(const void *w, int w_dtype, int64_t N, int64_t K, int64_t ldw,
                            int8_t *wq_packed, uint16_t *scales_bf16, void *hip_stream);

/* Inverse of the packing permutation: packed -> q[N, K] row-major int8 (device). */
int quasar_unpack_weights(const int8_t *wq_packed, int64_t N, int64_t K,
                          int8_t *q_rowmajor, void *hip_stream);

/*
 * Quantised linear layer of the verifier (Sec. 3.2 Eq. 8 integer-code matmul,
 * Sec. 3.3 Eq. 10 dequantisation), activations kept in bf16:
 *     y[m, n] = bf16( ( sum_k x[m, k] * q[n, k] ) * delta_n ),  fp32 accumulation.
 *   x  device [M, K] bf16, row stride ldx        y  device out [M, N] bf16, row stride ldy
 *   wq_packed / scales_bf16 as produced by quasar_quantize_weights
 *   workspace may be NULL; see quasar_workspace_bytes for what a workspace buys.
 * Weight bytes are read from HBM exactly once (the 1-byte-per-parameter term of
 * Eq. 12).
 */
int quasar_w8_linear(const uint16_t *x, int64_t M, int64_t K, int64_t ldx,
                     const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t N,
                     uint16_t *y, int64_t ldy,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Vocabulary projection fused with the acceptance decision (Sec. 3.1 Eq. 2 in
 * its temperature-0, deterministic-drafter case; Sec. 3.3 "Lossless Rejection
 * Sampling"): logits[m, v] as in quasar_w8_linear but compared in fp32 without
 * rounding to bf16 and never written to memory;
 *     out_argmax[m]     = smallest v attaining max_v logits[m, v]        (M values)
 *     out_accept_len[0] = number of leading i < n_draft with out_argmax[i] == draft_ids[i]
 * so the token to emit after the accepted prefix is out_argmax[out_accept_len].
 *   hidden device [M, K] bf16 (row stride ldh); draft_ids device [n_draft] int32,
 *   0 <= n_draft <= M (may be NULL when n_draft == 0); ids outside [0, V) never match.
 *   workspace: device, >= quasar_workspace_bytes(M, V, K) bytes.
 */
int quasar_lmhead_verify(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh,
                         const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t V,
                         const int32_t *draft_ids, int64_t n_draft,
                         int32_t *out_argmax, int32_t *out_accept_len,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * quasar_lmhead_verify for callers that cannot allocate or carry a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as quasar_lmhead_verify, without the workspace pair: the per-workgroup
 * argmax partials live in a 1 MiB array that is part of the library's device image (4096
 * workgroups x 32 positions x 8 bytes, which covers every shape quasar_lmhead_verify
 * accepts: M <= 32 and at most 4096 workgroups; anything beyond that is refused with
 * QUASAR_ERR_SHAPE before any launch).  The call allocates and frees nothing.  Each GPU
 * holds one copy of the array until the process ends, and every call on that GPU uses it:
 * calls that overlap on one GPU (different streams, different threads) race on it and must
 * be serialised by the caller.  Nothing in it needs clearing between calls: each launch
 * writes every slot that it later reads.
 */
int quasar_lmhead_verify_static(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh,
                                const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t V,
                                const int32_t *draft_ids, int64_t n_draft,
                                int32_t *out_argmax, int32_t *out_accept_len, void *hip_stream);

/*
 * Full-precision comparison point (Sec. 3.4 Eq. 11: two bytes per parameter):
 * the same kernels streaming bf16 weights.  quasar_pack_bf16_weights converts
 * (fp32 -> bf16 round-to-nearest-even, or copies bf16) into the tile order.
 */
int quasar_pack_bf16_weights(const void *w, int w_dtype, int64_t N, int64_t K, int64_t ldw,
                             uint16_t *w_packed, void *hip_stream);
int quasar_bf16_linear(const uint16_t *x, int64_t M, int64_t K, int64_t ldx,
                       const uint16_t *w_packed, int64_t N,
                       uint16_t *y, int64_t ldy,
                       void *workspace, size_t workspace_bytes, void *hip_stream);
int quasar_bf16_lmhead_verify(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh,
                              const uint16_t *w_packed, int64_t V,
                              const int32_t *draft_ids, int64_t n_draft,
                              int32_t *out_argmax, int32_t *out_accept_len,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Whole-step execution: the linears of a verification pass (and optionally the final
 * vocabulary projection + acceptance) run as ONE persistent launch, so that the weight
 * stream of Sec. 3.4 (Eq. 12: one byte per parameter over the whole model) is not interrupted
 * at every layer boundary.  Results are bit-identical to calling quasar_w8_linear /
 * quasar_lmhead_verify one by one in list order with no workspace given to quasar_w8_linear
 * (a workspace lets it split K across workgroups, which sums in another order) and the
 * single-call kernels in their default shape (16 waves per workgroup).
 *
 * Linears are described on the HOST; consecutive entries that read the same x (q|k|v, gate|up)
 * are executed together.  An entry whose input is the output of earlier entries waits for
 * those entries only (per-workgroup completion flags) provided every buffer involved is
 * written once per step; buffers that are written more than once per step (ping-pong reuse)
 * or partially overwritten are ordered by a device-wide barrier instead, which is slower.
 * All entries use the same M and the same weight type: int8 (scales != NULL) or packed bf16
 * (scales == NULL).
 *
 * quasar_sequence_prepare (offline and synchronous: copies a small table to plan_device and
 * clears the workspace) fills the host handle `seq`; quasar_sequence_run enqueues one step.
 * The workspace (device, >= quasar_sequence_workspace_bytes(n_linears, M)) belongs to this
 * sequence from prepare on: it holds barrier words, completion flags and argmax partials and
 * must not be shared or modified between steps.  After a step its second 32-bit word is
 * non-zero if a wait timed out (results then invalid).
 * The launch needs every workgroup resident at once: do not run other kernels concurrently
 * on the same device while a step is in flight.
 */
typedef struct quasar_linear_desc {
    const uint16_t *x;        /* device [M, K] bf16, row stride ldx */
    int64_t ldx;
    const void *w_packed;     /* device, from quasar_quantize_weights or quasar_pack_bf16_weights */
    const uint16_t *scales;   /* device [N] bf16, or NULL for bf16 weights */
    uint16_t *y;              /* device [M, N] bf16, row stride ldy */
    int64_t ldy;
    int64_t N, K;
} quasar_linear_desc;

typedef struct quasar_verify_desc {
    const uint16_t *hidden;   /* device [M, K] bf16, row stride ldh */
    int64_t ldh;
    const void *w_packed;
    const uint16_t *scales;   /* NULL for bf16 weights */
    int64_t V, K;
    const int32_t *draft_ids; /* device [n_draft] */
    int64_t n_draft;
    int32_t *out_argmax;      /* device [M] */
    int32_t *out_accept_len;  /* device [1] */
} quasar_verify_desc;

typedef struct quasar_sequence { int32_t words[16]; } quasar_sequence;

size_t quasar_sequence_plan_bytes(int64_t n_linears);
size_t quasar_sequence_workspace_bytes(int64_t n_linears, int64_t M);
int quasar_sequence_prepare(const quasar_linear_desc *linears, int64_t n_linears,
                            const quasar_verify_desc *verify /* may be NULL */, int64_t M,
                            void *plan_device, size_t plan_bytes,
                            void *workspace, size_t workspace_bytes, quasar_sequence *seq);
int quasar_sequence_run(const quasar_sequence *seq, const void *plan_device,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Profiling aid (no passage of the paper stands behind it): quasar_sequence_run that also records
 * when each workgroup passed the hand-over points of each phase, for a per-phase timeline of
 * the launch.  stamps: device, quasar_sequence_stamps_bytes(seq) bytes, laid out
 * [phase][workgroup][8] uint64 readings of the GPU's 100 MHz constant clock:
 *   [0] began to wait for the phase's input      [1] saw the input complete
 *   [2] had the input staged in LDS              [3] had summed its last tile
 *   [4] had its outputs acknowledged and its completion flag raised      [5..7] unused
 * Entries of workgroups without a share in a phase are left as they were (clear the buffer
 * first).  Results are those of quasar_sequence_run; the stamps cost a few stores per phase.
 */
size_t quasar_sequence_stamps_bytes(const quasar_sequence *seq);
int quasar_sequence_run_stamped(const quasar_sequence *seq, const void *plan_device,
                                void *workspace, size_t workspace_bytes,
                                uint64_t *stamps, size_t stamps_bytes, void *hip_stream);

/*
 * ---- W8A8 form: int8 codes on both sides (Sec. 3.2 "Smoothing Transformation" and
 * "Quantized Inference"; Sec. 3.3 "Online Activation Smoothing and Quantization",
 * "INT8 Gemm and Dequantization", Eq. 10) ----
 *
 * `smooth` is the per-input-channel factor vector s of the smoothing transformation:
 * device, [K] fp32, 16-byte aligned, or NULL for none.  Offline the weights take
 * W diag(s)^-1, online the activations take X (.) s; calibrating s is not part of this
 * library.  Every floating-point step that decides a code or the result bits is one IEEE
 * fp32 operation (round to nearest even), in this order:
 *     x~[m,k] = float(x[m,k]) * s[k]
 *     amax_m = max_k |x~[m,k]|;  dx_m = amax_m / 127;  inv_m = 127 / amax_m
 *     x^[m,k] = clamp(rint(x~[m,k] * inv_m), -127, 127)        (a zero row: dx = 0, codes 0)
 *     acc[m,n] = sum_k x^[m,k] * q[n,k]                        (int32, exact)
 *     y[m,n]  = bf16( float(acc[m,n]) * (dx_m * dw_n) )
 * so results are reproducible bit for bit.  Non-finite inputs give unspecified values.
 */

/* Offline weight preparation with the smoothing divide (Sec. 3.3 "Offline Weight
 * Preparation": W_int8 = Q(W diag(s)^-1)): as quasar_quantize_weights, applied to
 * fp32(W[n,k] / s[k]).  smooth NULL = quasar_quantize_weights. */
int quasar_quantize_weights_smoothed(const void *w, int w_dtype, int64_t N, int64_t K, int64_t ldw,
                                     const float *smooth, int8_t *wq_packed, uint16_t *scales_bf16,
                                     void *hip_stream);

/* The activation quantiser on its own (Sec. 3.3 "Online Activation Smoothing and
 * Quantization", X_int8 = Q(X (.) s, delta_x)), one step size per token.
 *   x     device, [M, K] bf16, row stride ldx (multiple of 8), 16-byte aligned
 *   xq    device out, [M, K] int8 row-major, 8-byte aligned
 *   dx    device out, [M] fp32 step sizes
 * The fused entry points below run the same arithmetic internally; this one makes the
 * codes observable. */
int quasar_quantize_activations(const uint16_t *x, int64_t M, int64_t K, int64_t ldx,
                                const float *smooth, int8_t *xq, float *dx, void *hip_stream);

/* W8A8 linear layer: activation smoothing + quantisation, int8 x int8 matrix-core
 * contraction with int32 sums, dequantisation by (delta_w . delta_x) (Eq. 10), one launch.
 * Arguments as quasar_w8_linear plus `smooth`; workspace unused (may be NULL). */
int quasar_w8a8_linear(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const float *smooth,
                       const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t N,
                       uint16_t *y, int64_t ldy,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* W8A8 vocabulary projection fused with the acceptance decision (Eq. 10 logits kept in
 * fp32, then Eq. 2 at temperature 0 as in quasar_lmhead_verify).  Arguments as
 * quasar_lmhead_verify plus `smooth`. */
int quasar_w8a8_lmhead_verify(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh,
                              const float *smooth,
                              const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t V,
                              const int32_t *draft_ids, int64_t n_draft,
                              int32_t *out_argmax, int32_t *out_accept_len,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* The whole-step launch in the W8A8 form: as quasar_sequence_prepare, every linear and the
 * vocabulary phase computed as quasar_w8a8_linear / quasar_w8a8_lmhead_verify compute them
 * (same bits).  smooth: host array of n_linears device pointers ([K_i] fp32 each, entries or
 * the array itself may be NULL); verify_smooth likewise for the vocabulary phase.  Linears
 * that share their input share a phase only if they also share the smoothing vector.
 * quasar_sequence_run runs the prepared handle. */
int quasar_sequence_prepare_w8a8(const quasar_linear_desc *linears, int64_t n_linears,
                                 const float *const *smooth,
                                 const quasar_verify_desc *verify /* may be NULL */,
                                 const float *verify_smooth, int64_t M,
                                 void *plan_device, size_t plan_bytes,
                                 void *workspace, size_t workspace_bytes, quasar_sequence *seq);

/*
 * ---- Stochastic verification, temperature T > 0 (Sec. 3.1: accept candidate i iff
 * r < min(1, p/q), on rejection resample from norm(max(0, p - q)); Sec. 3.3 "Lossless
 * Rejection Sampling": p is the softmax of the dequantised logits) ----
 *
 * The drafter is deterministic (prompt-lookup n-gram, as in the paper's experiments): q is a
 * point mass on the proposed token, so candidate i is accepted iff u_accept[i] < p_i(x~_i), and
 * the corrective token at the first rejected position n is drawn from p_n with the rejected
 * token's mass removed.  If all n_draft candidates are accepted the bonus token is drawn from
 * p at position n_draft, hence n_draft <= M - 1.  The draw is the inverse CDF in vocabulary
 * order with u_sample[n]: token = min{ v : C(v) > u * C(V-1) }.
 *   hidden, wq_packed, scales_bf16, V, draft_ids   as quasar_lmhead_verify
 *   temperature     T > 0; p = softmax(logits / T), logits and softmax in fp32
 *   u_accept        device [n_draft] fp32 in [0, 1): the r of the acceptance tests
 *   u_sample        device [M] fp32 in [0, 1): entry n is used for the draw at position n
 *   out_accept_len  device [1]: number of leading accepted candidates
 *   out_next_token  device [1]: corrective or bonus token
 *   out_p_draft     device [n_draft] fp32 or NULL: p_i(x~_i)
 *   workspace       quasar_sample_workspace_bytes(M, V) bytes (the [M, V] fp32 logits live there)
 * Three launches: the weight stream with fp32 outputs, softmax statistics per position, the
 * decision.  int8 weights with bf16 activations only.
 */
size_t quasar_sample_workspace_bytes(int64_t M, int64_t V);
int quasar_lmhead_verify_sample(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh,
                                const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t V,
                                const int32_t *draft_ids, int64_t n_draft, float temperature,
                                const float *u_accept, const float *u_sample,
                                int32_t *out_accept_len, int32_t *out_next_token, float *out_p_draft,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * ---- 4-bit group-wise weights (Sec. 6 names lower-bit weights as the way to cut the
 * verification traffic further; the quantiser is Eq. 6 at b = 4, the product Eq. 8 inside a
 * group of input channels and Eq. 10 per group) ----
 *
 * One step size per output row and per group of 128 consecutive input channels:
 *   delta[n, g] = bf16( fp32(max_{k in g} |W[n,k]|) / 7 ),
 *   q[n, k]     = clamp( rint( fp32(W[n,k]) / delta[n, k/128] ), -7, 7 )   (fp32 division,
 *                 round half to even; a group whose step size rounds to 0 gets all-zero codes),
 *   y[m, n]     = bf16( sum_g delta[n, g] * sum_{k in g} x[m, k] * q[n, k] )   (fp32 sums).
 * Codes and step sizes live in ONE packed buffer of quasar_w4_packed_bytes(N, K) bytes
 * (N*K/2 bytes of codes + 2 bytes per row and group, interleaved so that a workgroup streams one
 * contiguous range); K must be a multiple of 128, N of 16, other limits as quasar_w8_linear.
 * Activations stay in bf16.  The accepted tolerance of the linear outputs is that of
 * quasar_w8_linear; argmax and accepted length are exact outside logit ties.
 */
size_t quasar_w4_packed_bytes(int64_t N, int64_t K);   /* 0 on invalid shapes */

/* Offline preparation: quantise w[N, K] (device, row stride ldw elements, QUASAR_F32 or
 * QUASAR_BF16) into w4_packed (device, 16-byte aligned, quasar_w4_packed_bytes(N, K) bytes). */
int quasar_quantize_weights_w4(const void *w, int w_dtype, int64_t N, int64_t K, int64_t ldw,
                               void *w4_packed, void *hip_stream);

/* Inverse of the packing, for checking: codes to q_rowmajor (device int8 [N, K], 8-byte
 * aligned), step sizes to scales_bf16 (device [N, K/128]). */
int quasar_unpack_weights_w4(const void *w4_packed, int64_t N, int64_t K,
                             int8_t *q_rowmajor, uint16_t *scales_bf16, void *hip_stream);

/* y[M, N] (bf16, row stride ldy) from x[M, K] (bf16, row stride ldx) and packed 4-bit weights;
 * arguments, alignment and errors as quasar_w8_linear (no workspace: K is never split across
 * workgroups here). */
int quasar_w4_linear(const uint16_t *x, int64_t M, int64_t K, int64_t ldx,
                     const void *w4_packed, int64_t N,
                     uint16_t *y, int64_t ldy, void *hip_stream);

/* Vocabulary projection with 4-bit weights fused with the greedy acceptance decision (Eq. 2 at
 * temperature 0); arguments and workspace as quasar_lmhead_verify. */
int quasar_w4_lmhead_verify(const uint16_t *hidden, int64_t M, int64_t K, int64_t ldh,
                            const void *w4_packed, int64_t V,
                            const int32_t *draft_ids, int64_t n_draft,
                            int32_t *out_argmax, int32_t *out_accept_len,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * ---- The int8 linears with the decoder block's surrounding operations fused in (the rest of
 * the verification forward around the quantised matmuls of Sec. 3.3: the paper changes the
 * linears only, the block is the target model's own) ----
 *
 * Every rounding to bf16 sits where a bf16 implementation of the block has one; arithmetic
 * inside is fp32.  The linears are quasar_w8_linear's (same packed weights, same tolerance).
 *
 * quasar_w8_linear_fused:    y = [residual +] W8( [RMSNorm](x) )
 *   gamma     device [K] bf16, 16-byte aligned, or NULL (no normalisation).  With gamma the kernel
 *             stages bf16( gamma[k] * bf16( x[m,k] * rsqrt(mean_k x[m,:]^2 + eps) ) ) instead of x, so the
 *             normalised activations never travel through HBM; eps in [0, 1)
 *   residual  device [M, N] bf16, row stride ldr, or NULL; if given, y = bf16( bf16(linear) + residual ),
 *             and y may be the residual buffer itself
 *   other arguments, alignment and errors as quasar_w8_linear (K is never split across workgroups)
 *
 * quasar_w8_gateup_swiglu:   y[M, I] = bf16( bf16(silu(gate)) * up ),  gate / up = bf16( W8_gate/up( [RMSNorm](x) ) ),
 *   silu(g) = g / (1 + exp(-g)).  The two projections share ONE weight matrix of 2 I rows whose rows
 *   alternate in blocks of 16: rows 32 t .. 32 t + 15 are gate rows 16 t .. 16 t + 15, rows 32 t + 16 .. 32 t + 31
 *   the up rows of the same indices (quantise that matrix with quasar_quantize_weights; per-row step
 *   sizes are unaffected by the order).  The gated product is formed in the epilogue of the kernel:
 *   the projections themselves never travel through HBM.  I a multiple of 16; y row stride ldy >= I,
 *   a multiple of 4; other arguments as above.
 */
int quasar_w8_linear_fused(const uint16_t *x, int64_t M, int64_t K, int64_t ldx,
                           const uint16_t *gamma, float eps,
                           const int8_t *wq_packed, const uint16_t *scales_bf16, int64_t N,
                           const uint16_t *residual, int64_t ldr,
                           uint16_t *y, int64_t ldy, void *hip_stream);
int quasar_w8_gateup_swiglu(const uint16_t *x, int64_t M, int64_t K, int64_t ldx,
                            const uint16_t *gamma, float eps,
                            const int8_t *wq_packed_interleaved, const uint16_t *scales_bf16_interleaved,
                            int64_t I, uint16_t *y, int64_t ldy, void *hip_stream);

/*
 * ---- Attention of a verification step (Sec. 3.1: the gamma + 1 positions are verified in one
 * forward pass; the attention of that pass is the target model's own: grouped-query attention
 * with a key/value cache, per-head RMSNorm of queries and keys, rotary position embedding;
 * head dimension 128) ----
 *
 * The key/value cache of a layer is ONE device buffer of quasar_kv_cache_bytes(n_kv_heads, max_len)
 * bytes, 16-byte aligned, in a layout private to the library (blocks of 32 positions in
 * matrix-core operand order); it need not be initialised.  Positions are written by
 * quasar_attn_prepare (the M new positions of a step) or quasar_kv_cache_fill (plain
 * [n, n_kv_heads, 128] bf16 keys and values, already normalised and rotated, to positions
 * pos0 .. pos0 + n - 1, e.g. a prompt).
 *
 * quasar_attn_prepare: qkv is the fused projection output [M, (n_q_heads + 2 n_kv_heads) * 128] bf16
 *   (query heads, then key heads, then value heads; row stride ld).  Queries and keys:
 *   n = bf16( gamma * bf16( x * rsqrt(mean_head x^2 + eps) ) ) per head, then the rotary embedding at
 *   position L + m in the rotate-half convention with angles (L + m) * rope_theta^(-2 i / 128), one
 *   rounding to bf16.  Queries go to q_out [M, n_q_heads * 128] (row stride ldq); keys and values
 *   (values unchanged) into the cache at positions L .. L + M - 1.  L + M <= max_len.
 *
 * quasar_verify_attention: out[m, h, :] = softmax_j( q[m, h, :] . k[j, h / G, :] / sqrt(128) ) v[j, h / G, :]
 *   over the cached positions j <= L_total - M + m (the M queries are the last M cached positions,
 *   causal among themselves), G = n_q_heads / n_kv_heads (64 query rows m * G + g per pass over the
 *   cache; more rows take more passes); probabilities enter the
 *   second product as bf16, sums are fp32, one rounding of the output to bf16.  q as written by
 *   quasar_attn_prepare (16-byte aligned, ldq a multiple of 8); out [M, n_q_heads * 128] bf16, row
 *   stride ldo a multiple of 4; workspace: quasar_attention_workspace_bytes(M, n_q_heads, n_kv_heads, L_total)
 *   bytes (partial results of the splits over the positions).  Two launches per pass.
 */
size_t quasar_kv_cache_bytes(int64_t n_kv_heads, int64_t max_len);   /* 0 on invalid arguments */
int quasar_kv_cache_fill(const uint16_t *k, const uint16_t *v, int64_t n, int64_t n_kv_heads, int64_t pos0,
                         void *kv_cache, int64_t max_len, void *hip_stream);
int quasar_attn_prepare(const uint16_t *qkv, int64_t M, int64_t ld, int64_t n_q_heads, int64_t n_kv_heads,
                        int64_t L, const uint16_t *q_gamma, const uint16_t *k_gamma, float eps, float rope_theta,
                        uint16_t *q_out, int64_t ldq, void *kv_cache, int64_t max_len, void *hip_stream);
size_t quasar_attention_workspace_bytes(int64_t M, int64_t n_q_heads, int64_t n_kv_heads, int64_t L_total);
int quasar_verify_attention(const uint16_t *q, int64_t M, int64_t ldq, int64_t n_q_heads, int64_t n_kv_heads,
                            const void *kv_cache, int64_t max_len, int64_t L_total,
                            uint16_t *out, int64_t ldo, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * ---- Prompt-lookup n-gram drafter (Sec. 2: drafts by n-gram matching against the context;
 * Sec. 4 "Implementation Details": lookup length adjusted dynamically between a minimum and a
 * maximum, 1 and 4 in the paper; Sec. 4.4: range (K_min, K_max), gamma speculative tokens) ----
 *
 * HOST code and HOST pointers throughout; no GPU work, no stream.  The context (prompt plus
 * accepted tokens) only grows.  A proposal tries the lookup lengths from k_max down to k_min;
 * for a length k the pattern is the last k tokens, a match is an earlier start s < n - k with the
 * same k tokens (it may overlap the pattern), the most recent match of the first length that
 * has one is taken, and the draft is the up to gamma tokens that followed it (cut at the end of
 * the context).  No match: n_draft = 0.  An object is not safe for concurrent calls.
 *   quasar_drafter_create   NULL on invalid arguments (1 <= k_min <= k_max <= 64) or out of memory;
 *                           capacity_hint = expected context length (0 if unknown)
 *   quasar_drafter_append   extends the context by n tokens (copied)
 *   quasar_drafter_propose  out_draft: host [gamma]; *out_n_draft tokens written;
 *                           *out_lookup_len (may be NULL) = the length that matched, 0 if none
 */
typedef struct quasar_drafter quasar_drafter;
quasar_drafter *quasar_drafter_create(int k_min, int k_max, int64_t capacity_hint);
void quasar_drafter_destroy(quasar_drafter *drafter);
int quasar_drafter_append(quasar_drafter *drafter, const int32_t *tokens, int64_t n);
int64_t quasar_drafter_length(const quasar_drafter *drafter);   /* -1 for NULL */
int quasar_drafter_propose(const quasar_drafter *drafter, int64_t gamma, int32_t *out_draft,
                           int64_t *out_n_draft, int *out_lookup_len);

/*
 * Measurement helpers (the bandwidth term of Eq. 11-12 measured directly).
 * quasar_read_stream reads `bytes` (multiple of 16) from `src` with the same
 * load pattern as the linear kernels and writes one checksum word per workgroup
 * into sink (device, >= 8192 bytes).  quasar_copy_stream copies `bytes`
 * (multiple of 16) from src to dst; it is the plain copy kernel of known size
 * used to calibrate hardware byte counters.
 */
int quasar_read_stream(const void *src, size_t bytes, void *sink, void *hip_stream);
int quasar_copy_stream(void *dst, const void *src, size_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* QUASAR_H_ */
