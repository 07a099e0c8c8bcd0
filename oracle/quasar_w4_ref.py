"""CPU oracle for the 4-bit-weight form of the verification path (TEST INFRASTRUCTURE ONLY).

Plain numpy, fp64 arithmetic, no blocking beyond bounding memory.  Nothing in the product path
imports this file and this file imports nothing from the product path.

The paper names 4-bit weights as the direction that cuts the weight traffic of verification
further (Sec. 6, future work); it gives no formulas of its own for them.  What is written out
here is the paper's own quantiser and matmul at b = 4:

* ``quantize_weights_w4``  the symmetric uniform quantiser Q(W, delta) of Eq. 6 with a 4-bit
                           signed code range, one step size per output row AND per group of
                           ``group`` consecutive input channels (a single step size per row is
                           too coarse for 15 levels; group = K gives the per-row form back).
* ``w4_linear``            Eq. 8 inside a group (sum of code x activation), Eq. 10 per group
                           (times the group's step size), summed over the groups; activations
                           stay in bf16 as in the 8-bit path.
* ``w4_lmhead_verify``     vocabulary projection with such weights + the greedy acceptance
                           rule of Eq. 2 at temperature 0.

Readings: the code range is [-7, 7] (symmetric, -8 never produced, as -128 is not in the 8-bit
path); delta = bf16(fp32(amax) / fp32(7)) is stored as bf16; the code is
clamp(rint(fp32(w) / fp32(delta))) with the quotient an IEEE fp32 division (the precision the
device decides it in) and rint = round half to even; a group whose step size rounds to zero
gets delta = 0 and all-zero codes.  bf16 values travel as uint16 bit patterns.
"""
from __future__ import annotations

import numpy as np

QMAX4 = 7
GROUP = 128


def _f32_to_bf16_bits(a) -> np.ndarray:
    """fp32 -> bf16 bits, round to nearest even (inputs here are finite)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    return (r & np.uint64(0xFFFF)).astype(np.uint16)


def _bf16_bits_to_f64(bits) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def quantize_weights_w4(w, group: int = GROUP):
    """Symmetric 4-bit quantisation of W[N, K], one step size per (row, group of `group` k).

    Returns (q int8 [N, K] with values in [-7, 7], delta as uint16 bf16 bits [N, K // group]).
    """
    w32 = np.ascontiguousarray(w, dtype=np.float32)
    if w32.ndim != 2 or group < 1 or w32.shape[1] % group:
        raise ValueError("w must be [N, K] with K a multiple of the group size")
    N, K = w32.shape
    G = K // group
    wg = w32.reshape(N, G, group)
    amax = np.max(np.abs(wg), axis=2).astype(np.float32)
    step32 = (amax / np.float32(QMAX4)).astype(np.float32)
    s_bits = _f32_to_bf16_bits(step32).reshape(N, G)
    s32 = _bf16_bits_to_f64(s_bits).astype(np.float32)
    live = s32 > 0
    q = np.zeros((N, G, group), dtype=np.int8)
    safe = np.where(live, s32, np.float32(1.0))
    ratio = (wg / safe[:, :, None]).astype(np.float32)              # fp32 division
    code = np.clip(np.rint(ratio), -QMAX4, QMAX4).astype(np.int8)
    q[live] = code[live]
    s_bits = np.where(live, s_bits, np.uint16(0)).astype(np.uint16)
    return q.reshape(N, K), s_bits


def dequantize_w4(q, s_bits, group: int = GROUP) -> np.ndarray:
    """W_hat[n, k] = q[n, k] * delta[n, k // group], exact in fp64."""
    q = np.asarray(q)
    N, K = q.shape
    s = _bf16_bits_to_f64(s_bits).reshape(N, K // group)
    return q.astype(np.float64) * np.repeat(s, group, axis=1)


def w4_linear(x_bits, q, s_bits, group: int = GROUP, rows_per_block: int = 4096) -> np.ndarray:
    """y[m, n] = sum_g delta[n, g] * ( sum_{k in group g} x[m, k] * q[n, k] ), fp64, unrounded.

    x_bits: uint16 bf16 bits [M, K]; q: int8 [N, K]; s_bits: uint16 [N, K // group].
    Rows are visited in blocks only to bound memory.
    """
    x = _bf16_bits_to_f64(x_bits)
    q = np.asarray(q)
    if x.ndim != 2 or q.ndim != 2 or x.shape[1] != q.shape[1] or q.shape[1] % group:
        raise ValueError("shape mismatch: x[M,K], q[N,K], K a multiple of the group size")
    M, K = x.shape
    N = q.shape[0]
    G = K // group
    s = _bf16_bits_to_f64(s_bits).reshape(N, G)
    xg = x.reshape(M, G, group)
    y = np.zeros((M, N))
    for n0 in range(0, N, rows_per_block):
        n1 = min(N, n0 + rows_per_block)
        qg = q[n0:n1].astype(np.float64).reshape(n1 - n0, G, group)
        inner = np.einsum("mgk,ngk->mng", xg, qg)                   # Eq. 8 inside each group
        y[:, n0:n1] = np.einsum("mng,ng->mn", inner, s[n0:n1])      # Eq. 10 per group, then the sum
    return y


def w4_lmhead_verify(h_bits, q, s_bits, draft, group: int = GROUP):
    """Vocabulary projection with 4-bit weights, per-position argmax (lowest index on ties),
    accepted length = number of leading candidates equal to the argmax of their position.

    Returns dict(argmax int64 [M], n_acc int, top1 [M], top2 [M], maxabs [M])."""
    lg = w4_linear(h_bits, q, s_bits, group)
    M = lg.shape[0]
    arg = np.argmax(lg, axis=1).astype(np.int64)                    # first maximum
    top1 = lg[np.arange(M), arg]
    rest = lg.copy()
    rest[np.arange(M), arg] = -np.inf
    top2 = rest.max(axis=1) if lg.shape[1] > 1 else np.full(M, -np.inf)
    draft = np.asarray(draft, dtype=np.int64).reshape(-1)
    if draft.size > M:
        raise ValueError("n_draft must not exceed M")
    n_acc = 0
    for i in range(draft.size):
        if arg[i] != draft[i]:
            break
        n_acc += 1
    return {"argmax": arg, "n_acc": n_acc, "top1": top1, "top2": top2, "maxabs": np.abs(lg).max(axis=1)}
