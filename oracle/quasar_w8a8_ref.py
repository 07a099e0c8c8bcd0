"""CPU oracle for the W8A8 form of the quantized verifier (TEST INFRASTRUCTURE ONLY).

Plain numpy, no blocking, no fusion.  Nothing in the product path imports this
file and this file imports nothing from the product path.

The passages followed (Sec. 3.2 "Smoothing Transformation" and "Quantized
Inference"; Sec. 3.3 "Offline Weight Preparation", "Online Activation Smoothing
and Quantization", "INT8 Gemm and Dequantization"):

* ``smooth_weights``          W~ = W diag(s)^-1, applied offline before the weight
                              quantiser (Sec. 3.3, offline weight preparation).
* ``quantize_activations``    X^ = Q(X (.) s, delta_x): the element-wise smoothing
                              multiply and the symmetric 8-bit quantiser, one step
                              size per token (Sec. 3.3, online activation smoothing
                              and quantisation).
* ``w8a8_accumulate``         Y_INT32 = W^ x X^, integer products summed in int32.
* ``w8a8_linear``             Y = Y_INT32 . (delta_w . delta_x) rounded to bf16 (Eq. 10).
* ``w8a8_lmhead_verify``      the same projection onto the vocabulary, logits left in
                              fp32, then the temperature-0 acceptance test (Eq. 2 with a
                              deterministic drafter).

Precision.  The paper fixes INT8 operands, INT32 accumulation and a BF16 result.
Every floating-point step in between decides either an integer code or the bits
of the result, so each is pinned to ONE IEEE fp32 operation, rounded to nearest
even, in the order written below; numpy's float32 arithmetic performs exactly
these single operations.  The readings (per-token step size, reciprocal form of
the quantiser, grouping of the two step sizes) are listed in the design
document and restated next to the code.

bf16 values travel as uint16 bit patterns (see quasar_ref.py).
"""
from __future__ import annotations

import numpy as np

QMAX = 127
_F32 = np.float32


def _bf16_bits_to_f32(bits) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _f32_to_bf16_bits(a) -> np.ndarray:
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    u = a32.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    out = (((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) & np.uint64(0xFFFF)).astype(np.uint16)
    return np.where(np.isnan(a32), np.uint16(0x7FC0), out).astype(np.uint16)


def smooth_weights(w, s) -> np.ndarray:
    """W~[n, k] = fp32( W[n, k] / s[k] ): the weight side of the smoothing identity
    Y = (W diag(s)^-1)(diag(s) X) with the online convention X~ = X (.) s."""
    w32 = np.ascontiguousarray(w, dtype=np.float32)
    s32 = np.ascontiguousarray(s, dtype=np.float32)
    if w32.ndim != 2 or s32.shape != (w32.shape[1],):
        raise ValueError("w must be [N, K] and s [K]")
    return (w32 / s32[None, :]).astype(np.float32)


def quantize_activations(x_bits, smooth=None):
    """Per token m (row of x[M, K], bf16):
        x~[m, k] = fp32(x[m, k]) * s[k]                  (one fp32 multiply; s absent: x~ = x)
        amax_m   = max_k |x~[m, k]|
        dx_m     = amax_m / 127                          (fp32 division; the step size)
        inv_m    = 127 / amax_m                          (fp32 division; its reciprocal)
        x^[m, k] = clamp( rint( x~[m, k] * inv_m ), -127, 127 )   (fp32 multiply, half to even)
    A row of zeros gets dx = 0 and all-zero codes.
    Returns (x^ int8 [M, K], dx float32 [M]).
    """
    x32 = _bf16_bits_to_f32(x_bits)
    if x32.ndim != 2:
        raise ValueError("x must be [M, K]")
    if smooth is not None:
        s32 = np.ascontiguousarray(smooth, dtype=np.float32)
        if s32.shape != (x32.shape[1],):
            raise ValueError("smooth must be [K]")
        xt = (x32 * s32[None, :]).astype(np.float32)
    else:
        xt = x32
    M, K = xt.shape
    amax = np.max(np.abs(xt), axis=1).astype(np.float32) if K else np.zeros(M, np.float32)
    live = amax > 0
    dx = np.zeros(M, dtype=np.float32)
    xq = np.zeros((M, K), dtype=np.int8)
    if np.any(live):
        dx[live] = (amax[live] / _F32(QMAX)).astype(np.float32)
        inv = (_F32(QMAX) / amax[live]).astype(np.float32)
        prod = (xt[live] * inv[:, None]).astype(np.float32)
        xq[live] = np.clip(np.rint(prod), -QMAX, QMAX).astype(np.int8)
    return xq, dx


def w8a8_accumulate(xq, q) -> np.ndarray:
    """acc[m, n] = sum_k x^[m, k] * q[n, k], exact; must fit int32 (it does for
    K <= 133000 since every product is at most 127 * 127).

    The sum is taken by the fp64 matrix product: every product is an integer below 2^14
    and every partial sum an integer below 2^31 * ... < 2^53, so no rounding can occur in
    any summation order (pinned against pure-Python integer sums in the tests)."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    q = np.ascontiguousarray(q, dtype=np.int8)
    if xq.ndim != 2 or q.ndim != 2 or xq.shape[1] != q.shape[1]:
        raise ValueError("shape mismatch: xq[M,K], q[N,K]")
    if xq.shape[1] > 2 ** 38:
        raise OverflowError("K too large for exact fp64 summation")
    acc = xq.astype(np.float64) @ q.astype(np.float64).T
    if acc.size and (acc.max() > 2**31 - 1 or acc.min() < -2**31):
        raise OverflowError("int32 accumulator overflow")
    return acc.astype(np.int64).astype(np.int32)


def w8a8_scale(dw_bits, dx) -> np.ndarray:
    """The factor of Eq. 10, (delta_w . delta_x), as one fp32 product per (m, n)."""
    dw = _bf16_bits_to_f32(dw_bits)
    return (np.asarray(dx, dtype=np.float32)[:, None] * dw[None, :]).astype(np.float32)


def w8a8_logits(x_bits, q, dw_bits, smooth=None) -> np.ndarray:
    """fp32 [M, N]: fp32(acc) * (dw * dx); int32 -> fp32 conversion rounds to nearest even."""
    xq, dx = quantize_activations(x_bits, smooth)
    acc = w8a8_accumulate(xq, q)
    return (acc.astype(np.float32) * w8a8_scale(dw_bits, dx)).astype(np.float32)


def w8a8_linear(x_bits, q, dw_bits, smooth=None) -> np.ndarray:
    """bf16 bits [M, N] of Eq. 10."""
    return _f32_to_bf16_bits(w8a8_logits(x_bits, q, dw_bits, smooth))


def w8a8_lmhead_verify(h_bits, q, dw_bits, draft, smooth=None, *, rows_per_block: int = 8192):
    """argmax over the vocabulary of the fp32 logits (first index on ties), then the
    count of leading draft tokens that equal it.  Blocked over vocabulary rows only
    to bound memory; the result does not depend on the block size."""
    xq, dx = quantize_activations(h_bits, smooth)
    M = xq.shape[0]
    V = q.shape[0]
    best = np.full(M, -np.inf, dtype=np.float32)
    arg = np.zeros(M, dtype=np.int64)
    for v0 in range(0, V, rows_per_block):
        v1 = min(V, v0 + rows_per_block)
        acc = w8a8_accumulate(xq, q[v0:v1])
        lg = (acc.astype(np.float32) * w8a8_scale(dw_bits[v0:v1], dx)).astype(np.float32)
        loc = np.argmax(lg, axis=1)                      # first index of the block maximum
        val = lg[np.arange(M), loc]
        upd = val > best                                 # strictly greater: earlier block wins ties
        best = np.where(upd, val, best)
        arg = np.where(upd, loc + v0, arg)
    draft = np.asarray(draft, dtype=np.int64).reshape(-1)
    n_acc = 0
    for i in range(min(draft.size, M)):
        if arg[i] != draft[i]:
            break
        n_acc += 1
    return arg.astype(np.int32), n_acc
