/*
 * Second, independent form of the CPU oracle: naive C loops (TEST INFRASTRUCTURE ONLY).
 *
 * Same definitions as the numpy oracle, written without any library routine so
 * that the two can be checked against each other:
 *   - symmetric per-output-row int8 quantisation (Eq. 6; offline weight
 *     preparation of Sec. 3.3),
 *   - integer-code matmul then rescale by the row step size (Eq. 8, Eq. 10)
 *     with bf16 activations, accumulated in double,
 *   - vocabulary projection + first-index argmax + count of leading draft
 *     matches (Eq. 2 at temperature 0).
 * No blocking, no reordering: the k loop runs 0..K-1 for every output.
 * The product library never links or loads this file.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static double bf16_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static uint16_t float_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return 0x7FC0; /* NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* W[N,K] fp32 row-major (row stride ldw) -> q[N,K] int8 row-major, delta[N] bf16 bits */
void qref_quantize(const float *w, int64_t N, int64_t K, int64_t ldw,
                   int8_t *q, uint16_t *delta_bits) {
    for (int64_t n = 0; n < N; ++n) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float a = fabsf(w[n * ldw + k]);
            if (a > amax) amax = a;
        }
        volatile float step = amax / 127.0f;           /* fp32 quotient */
        uint16_t sb = float_to_bf16_rne(step);
        float s = (float)bf16_to_double(sb);
        if (!(s > 0.0f)) {
            delta_bits[n] = 0;
            for (int64_t k = 0; k < K; ++k) q[n * K + k] = 0;
            continue;
        }
        delta_bits[n] = sb;
        for (int64_t k = 0; k < K; ++k) {
            volatile float ratio = w[n * ldw + k] / s; /* fp32 quotient decides the code */
            float r = nearbyintf(ratio);               /* default mode: half to even */
            if (r > 127.0f) r = 127.0f;
            if (r < -127.0f) r = -127.0f;
            q[n * K + k] = (int8_t)r;
        }
    }
}

/* y[M,N] double = (sum_k x[m,k]*q[n,k]) * delta[n] */
void qref_w8_linear(const uint16_t *x_bits, int64_t M, int64_t K,
                    const int8_t *q, const uint16_t *delta_bits, int64_t N, double *y) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += bf16_to_double(x_bits[m * K + k]) * (double)q[n * K + k];
            y[m * N + n] = acc * bf16_to_double(delta_bits[n]);
        }
}

/* y[M,N] double = sum_k x[m,k]*w[n,k], both bf16 */
void qref_bf16_linear(const uint16_t *x_bits, int64_t M, int64_t K,
                      const uint16_t *w_bits, int64_t N, double *y) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += bf16_to_double(x_bits[m * K + k]) * bf16_to_double(w_bits[n * K + k]);
            y[m * N + n] = acc;
        }
}

/* argmax[m] = first index of the row maximum of the logits; returns accepted length */
int32_t qref_lmhead_verify(const uint16_t *h_bits, int64_t M, int64_t K,
                           const int8_t *q, const uint16_t *delta_bits, int64_t V,
                           const int32_t *draft, int64_t n_draft, int32_t *argmax_out) {
    for (int64_t m = 0; m < M; ++m) {
        double best = -INFINITY;
        int64_t arg = 0;
        for (int64_t v = 0; v < V; ++v) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += bf16_to_double(h_bits[m * K + k]) * (double)q[v * K + k];
            double lg = acc * bf16_to_double(delta_bits[v]);
            if (lg > best) { best = lg; arg = v; }
        }
        argmax_out[m] = (int32_t)arg;
    }
    int32_t n_acc = 0;
    for (int64_t i = 0; i < n_draft && i < M; ++i) {
        if (argmax_out[i] != draft[i]) break;
        ++n_acc;
    }
    return n_acc;
}

/* ---------------------------------------------------------------------------------------
 * W8A8 form (Sec. 3.2 "Quantized Inference"; Sec. 3.3 online activation smoothing and
 * quantisation, INT8 gemm and dequantisation, Eq. 10).  One IEEE fp32 operation per step,
 * in the order of the numpy form; integer products summed in 64-bit and checked to fit
 * int32 by the caller.
 * ------------------------------------------------------------------------------------- */
static float bf16_to_float(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* x[M,K] bf16 (+ optional s[K] fp32) -> xq[M,K] int8, dx[M] fp32 */
void qref_quantize_activations(const uint16_t *x_bits, int64_t M, int64_t K, const float *smooth,
                               int8_t *xq, float *dx) {
    for (int64_t m = 0; m < M; ++m) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            volatile float xt = bf16_to_float(x_bits[m * K + k]);
            if (smooth) xt = xt * smooth[k];
            float a = fabsf(xt);
            if (a > amax) amax = a;
        }
        if (!(amax > 0.0f)) {
            dx[m] = 0.0f;
            for (int64_t k = 0; k < K; ++k) xq[m * K + k] = 0;
            continue;
        }
        volatile float step = amax / 127.0f;
        volatile float inv = 127.0f / amax;
        dx[m] = step;
        for (int64_t k = 0; k < K; ++k) {
            volatile float xt = bf16_to_float(x_bits[m * K + k]);
            if (smooth) xt = xt * smooth[k];
            volatile float pr = xt * inv;
            float r = nearbyintf(pr);
            if (r > 127.0f) r = 127.0f;
            if (r < -127.0f) r = -127.0f;
            xq[m * K + k] = (int8_t)r;
        }
    }
}

/* logits[M,N] fp32 = fp32(sum_k xq*q) * (dx[m] * dw[n]); returns 0, or 1 if a sum left int32 */
int32_t qref_w8a8_logits(const int8_t *xq, const float *dx, int64_t M, int64_t K,
                         const int8_t *q, const uint16_t *dw_bits, int64_t N, float *out) {
    int32_t overflow = 0;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k) acc += (int64_t)xq[m * K + k] * (int64_t)q[n * K + k];
            if (acc > 2147483647LL || acc < -2147483648LL) overflow = 1;
            volatile float scale = dx[m] * bf16_to_float(dw_bits[n]);
            volatile float a = (float)(int32_t)acc;
            volatile float y = a * scale;
            out[m * N + n] = y;
        }
    return overflow;
}

uint16_t qref_float_to_bf16(float f) { return float_to_bf16_rne(f); }
