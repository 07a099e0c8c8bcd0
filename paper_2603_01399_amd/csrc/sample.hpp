// Stochastic verification at temperature T > 0 on the fp32 logits of the M positions (gfx950):
// softmax statistics per position, the acceptance test r < min(1, p/q) against a deterministic
// drafter (q is a point mass on the proposed token), and the draw of the corrective or bonus
// token by inverse CDF in vocabulary order (Sec. 3.1, the acceptance and resampling rules;
// Sec. 3.3 "Lossless Rejection Sampling").  The logits come from the streaming kernel's fp32
// epilogue: [M, V] fp32 is a few MB beside the hundreds of MB of weights it was computed from.
//
// Two kernels.  softmax_partial_kernel spreads the exponentials over the whole chip: the
// vocabulary is cut into kSampleBlocks contiguous blocks, one workgroup per (block, position)
// leaves that block's (max, sum of exp(z - max)).  speculative_sample_kernel (one workgroup)
// merges them, takes the acceptance decisions, locates the block in which the draw falls from
// the block masses and resolves the draw inside that block only.
#pragma once

#include "quasar_device.hpp"

namespace quasar {

constexpr int kSampleBlocks = 32;

// (max, sum of exp(z - max)) pairs combine associatively
__device__ __forceinline__ void softmax_merge(float &m, float &s, float m2, float s2) {
    if (!(m2 > -__builtin_inff())) return;
    const float mm = fmaxf(m, m2);
    s = s * expf(m - mm) + s2 * expf(m2 - mm);
    m = mm;
}

__device__ __forceinline__ int sample_block_quads(int V) { return (V / 4 + kSampleBlocks - 1) / kSampleBlocks; }

// grid (kSampleBlocks, M), 256 threads.  partial[(m * kSampleBlocks + b) * 2] = max of z over the
// block, [.. + 1] = sum of exp(z - max); z = logit * inv_t.  V is a multiple of 16: rows are read
// as 16-byte quads.
__global__ __launch_bounds__(256) void softmax_partial_kernel(const float *logits, int V, float inv_t,
                                                             float *partial) {
    __shared__ float sm[4], ss[4];
    const int b = blockIdx.x, m = blockIdx.y, tid = threadIdx.x;
    const f32x4 *row4 = reinterpret_cast<const f32x4 *>(logits + (long long)m * V);
    const int qc = sample_block_quads(V);
    const int q_lo = min(V / 4, b * qc), q_hi = min(V / 4, q_lo + qc);
    float mx = -__builtin_inff(), s = 0.f;
    for (int q0 = q_lo + tid; q0 < q_hi; q0 += 256 * 4) {
        f32x4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = q0 + 256 * j;
            v[j] = q < q_hi ? row4[q] : f32x4{-__builtin_inff(), -__builtin_inff(), -__builtin_inff(), -__builtin_inff()};
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float z4[4] = {v[j].x * inv_t, v[j].y * inv_t, v[j].z * inv_t, v[j].w * inv_t};
            const float zm = fmaxf(fmaxf(z4[0], z4[1]), fmaxf(z4[2], z4[3]));
            if (zm > mx) {
                s = s * expf(mx - zm);
                mx = zm;
            }
            if (zm > -__builtin_inff())
                s += (expf(z4[0] - mx) + expf(z4[1] - mx)) + (expf(z4[2] - mx) + expf(z4[3] - mx));
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float m2 = __shfl_xor(mx, off, 64), s2 = __shfl_xor(s, off, 64);
        softmax_merge(mx, s, m2, s2);
    }
    if ((tid & 63) == 0) { sm[tid >> 6] = mx; ss[tid >> 6] = s; }
    __syncthreads();
    if (tid == 0) {
        float M0 = sm[0], S0 = ss[0];
        for (int w = 1; w < 4; ++w) softmax_merge(M0, S0, sm[w], ss[w]);
        partial[((long long)m * kSampleBlocks + b) * 2] = M0;
        partial[((long long)m * kSampleBlocks + b) * 2 + 1] = S0;
    }
}

// One workgroup of 1024 threads.
__global__ __launch_bounds__(1024) void speculative_sample_kernel(const float *logits, int V, int M, float inv_t,
                                                                 const int32_t *draft, int n_draft,
                                                                 const float *u_accept, const float *u_sample,
                                                                 const float *partial, int32_t *out_accept,
                                                                 int32_t *out_token, float *out_p_draft) {
    __shared__ float pos_max[32], pos_sum[32], pos_pd[32], pos_zd[32], pos_ua[32], pos_us[32];
    __shared__ float part[1024];
    __shared__ float wave_tot[16];
    __shared__ int pos_s, blk_s, chunk_s;
    __shared__ float target_s;
    __shared__ float blk_stat[32 * kSampleBlocks * 2];
    const int tid = threadIdx.x;
    // the block statistics and the proposed tokens' logits come in with one round trip
    for (int i = tid; i < M * kSampleBlocks * 2; i += 1024) blk_stat[i] = partial[i];
    float zd = -__builtin_inff();
    if (tid < n_draft) {
        const int d = draft[tid];
        if (d >= 0 && d < V) zd = logits[(long long)tid * V + d] * inv_t;
        pos_ua[tid] = u_accept[tid];
    }
    if (tid < M) pos_us[tid] = u_sample[tid];
    __syncthreads();
    // per position: merge the block statistics in block order; p of the proposed token
    if (tid < M) {
        float mx = -__builtin_inff(), s = 0.f;
        for (int b = 0; b < kSampleBlocks; ++b)
            softmax_merge(mx, s, blk_stat[(tid * kSampleBlocks + b) * 2], blk_stat[(tid * kSampleBlocks + b) * 2 + 1]);
        float pd = 0.f;
        if (tid < n_draft) {
            if (zd > -__builtin_inff()) pd = expf(zd - mx) / s;
            if (out_p_draft) out_p_draft[tid] = pd;
        }
        pos_zd[tid] = zd;
        pos_max[tid] = mx;
        pos_sum[tid] = s;
        pos_pd[tid] = pd;
    }
    __syncthreads();
    if (tid == 0) {
        int n = 0;
        while (n < n_draft && pos_ua[n] < fminf(1.f, pos_pd[n])) ++n;    // q(x~) = 1
        pos_s = n;
        out_accept[0] = n;
        // the draw at position n: masses of the blocks, the rejected token's mass removed
        // (max(0, p - q) is 0 on the proposed token and p elsewhere)
        const float mx = pos_max[n];
        const int banned = n < n_draft ? draft[n] : -1;
        const bool ban = banned >= 0 && banned < V;
        const float ban_mass = ban ? expf(pos_zd[n] - mx) : 0.f;
        const int ban_blk = ban ? (banned / 4) / sample_block_quads(V) : -1;
        float bm[kSampleBlocks];
        float total = 0.f;
        for (int b = 0; b < kSampleBlocks; ++b) {
            const float pm = blk_stat[(n * kSampleBlocks + b) * 2];
            float v = pm > -__builtin_inff() ? blk_stat[(n * kSampleBlocks + b) * 2 + 1] * expf(pm - mx) : 0.f;
            if (b == ban_blk) v = fmaxf(0.f, v - ban_mass);
            bm[b] = v;
            total += v;
        }
        float target = pos_us[n] * total;
        if (!(target < total)) target = total * (1.f - 1.f / 16777216.f);     // u * total rounded up to the total
        float run = 0.f;
        int blk = kSampleBlocks - 1;
        for (int b = 0; b < kSampleBlocks; ++b) {
            if (run + bm[b] > target) { blk = b; break; }
            run += bm[b];
        }
        // blocks after the last one with mass cannot be chosen; if rounding walked past, step back
        while (blk > 0 && !(bm[blk] > 0.f)) { --blk; run -= bm[blk]; }
        blk_s = blk;
        target_s = target - run;            // what is left to cover inside the block
        chunk_s = 1023;
    }
    __syncthreads();
    const int pos = pos_s, blk = blk_s;
    const float *row = logits + (long long)pos * V;
    const float mx = pos_max[pos];
    const int banned = pos < n_draft ? draft[pos] : -1;
    // inside the block: contiguous stretches of quads per thread, prefix sums in vocabulary order
    const int qc = sample_block_quads(V);
    const int q_lo = min(V / 4, blk * qc), q_hi = min(V / 4, q_lo + qc);
    const int per = (q_hi - q_lo + 1023) / 1024;                  // quads per thread
    const int a0 = min(q_hi, q_lo + tid * per), a1 = min(q_hi, a0 + per);
    const f32x4 *row4 = reinterpret_cast<const f32x4 *>(row);
    float sum = 0.f;
    for (int q = a0; q < a1; ++q) {
        const f32x4 v = row4[q];
        const float z4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (4 * q + e != banned) sum += expf(z4[e] * inv_t - mx);
    }
    float incl = sum;
    const int lane = tid & 63, wv = tid >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    float base = 0.f, total = 0.f;
    for (int i = 0; i < 16; ++i) {
        if (i < wv) base += wave_tot[i];
        total += wave_tot[i];
    }
    incl += base;
    part[tid] = incl;
    float target = target_s;
    if (!(target < total)) target = total * (1.f - 1.f / 16777216.f);   // block mass and in-block sum differ by rounding
    if (target < 0.f) target = 0.f;
    __syncthreads();
    if (incl > target && (tid == 0 || !(part[tid - 1] > target))) chunk_s = tid;
    __syncthreads();
    if (tid == chunk_s) {
        float run = tid > 0 ? part[tid - 1] : 0.f;
        int tok = -1, last = -1;
        for (int q = a0; q < a1 && tok < 0; ++q) {
            const f32x4 v = row4[q];
            const float z4[4] = {v.x, v.y, v.z, v.w};
            for (int e = 0; e < 4; ++e) {
                if (4 * q + e == banned) continue;
                const float ex = expf(z4[e] * inv_t - mx);
                if (ex > 0.f) last = 4 * q + e;
                run += ex;
                if (run > target) { tok = 4 * q + e; break; }
            }
        }
        if (tok < 0) tok = last;            // rounding at the very end of the stretch
        if (tok < 0) tok = a1 > a0 ? 4 * a1 - 1 : V - 1;
        out_token[0] = tok;
    }
}

}  // namespace quasar
