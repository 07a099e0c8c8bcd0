"""CPU oracle for the quantized verification path (TEST INFRASTRUCTURE ONLY).

Plain numpy, fp64 arithmetic, no blocking, no fusion.  Nothing in the product
path imports this file and this file imports nothing from the product path; the
only callers are the tests, the smoke check and the benchmark's cpu_baseline leg.

What is defined here, and the passage of the paper each part follows:

* ``quantize_weights``   symmetric uniform quantisation Q(W, delta_w) of the weight
                         matrix, done offline (Sec. 3.2 "Quantized Inference",
                         Eq. 6; Sec. 3.3 "Offline Weight Preparation").
* ``w8_linear``          the quantised matmul followed by the dequantisation
                         rescale (Eq. 8 and Eq. 10), with the activations kept in
                         bf16 (the W8A16 reading; delta_x = 1).
* ``bf16_linear``        the full-precision comparison point of Eq. 11 (weights
                         held in bf16, 2 bytes each).
* ``lmhead_verify``      final projection to the vocabulary and the acceptance
                         test of Eq. 2 in its temperature-0 / deterministic
                         drafter special case: a candidate is kept iff it is the
                         argmax of the target logits; the count of leading kept
                         candidates is the accepted length (Sec. 3.1, Sec. 3.3
                         "Lossless Rejection Sampling").

Readings taken where the paper is silent (granularity, step-size formula,
rounding mode, scale dtype, tie-break) are listed in the repository's design
document; they are restated next to the code that uses them.

bf16 values travel as uint16 bit patterns so that both sides of a parity test
consume the very same bits.
"""
from __future__ import annotations

import numpy as np

QMAX = 127  # symmetric code range is [-127, 127]; -128 is never produced


# --------------------------------------------------------------------------
# bf16 <-> float helpers (bit-level, round-to-nearest-even)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a) -> np.ndarray:
    """Round fp32 values to bf16 (nearest, ties to even); returns uint16 bits.

    bf16 is the top half of an IEEE fp32 word, so rounding adds half an ulp of
    the kept part (0x7FFF plus the lowest kept bit) and drops the low 16 bits.
    NaN keeps a quiet-NaN pattern.
    """
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    u = a32.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = (u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    out = (r & np.uint64(0xFFFF)).astype(np.uint16)
    nan = np.isnan(a32)
    if np.any(nan):
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f64(bits) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    u = b.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(a) -> np.ndarray:
    """Round fp64 values to bf16, nearest-even, in ONE rounding step.

    Used for the expected bf16 output of a linear layer: the exact (fp64) value
    is rounded straight to 8 significant bits, without passing through fp32.
    Works on the fp64 bit pattern: bf16 keeps the sign, an 8-bit exponent and 7
    fraction bits.  Values are assumed finite and inside bf16's normal range or
    zero (test inputs never leave it).
    """
    a64 = np.ascontiguousarray(a, dtype=np.float64)
    out = np.zeros(a64.shape, dtype=np.uint16)
    nz = a64 != 0.0
    if not np.any(nz):
        return np.where(np.signbit(a64), np.uint16(0x8000), out).astype(np.uint16)
    m, e = np.frexp(np.abs(a64))          # |a| = m * 2**e, m in [0.5, 1)
    # 8 significant bits: scale mantissa to [128, 256) and round half-even
    sig = np.rint(m * 256.0)              # np.rint is round-half-even
    e = np.where(sig == 256.0, e + 1, e)
    sig = np.where(sig == 256.0, 128.0, sig)
    biased = (e - 1) + 127                # value = (sig/128) * 2**(e-1)
    if np.any(nz & ((biased <= 0) | (biased >= 255))):
        raise ValueError("f64_to_bf16_bits: value outside bf16 normal range")
    frac = (sig - 128.0).astype(np.int64)
    word = (biased.astype(np.int64) << 7) | frac
    word = np.where(nz, word, 0)
    word = word | np.where(np.signbit(a64), 0x8000, 0)
    return word.astype(np.uint16)


# --------------------------------------------------------------------------
# O1  weight quantisation  (Eq. 6; offline weight preparation, Sec. 3.3)
# --------------------------------------------------------------------------
def quantize_weights(w):
    """Symmetric int8 quantisation of W[N, K], one step size per output row.

    Reading (the paper gives Q(W, delta) without its constants): per output
    channel n,
        amax_n  = max_k |W[n, k]|
        delta_n = bf16( fp32(amax_n) / fp32(127) )        (stored scale, bf16)
        q[n, k] = clamp( rint( fp32(W[n,k]) / fp32(delta_n) ), -127, 127 )
    with rint = round half to even.  The quotient that decides the integer code
    is an IEEE fp32 division (the precision the device kernel decides it in), so
    the codes are comparable bit for bit.  A row whose step size rounds to zero
    gets delta = 0 and all-zero codes.

    Returns (q int8 [N, K] row-major, delta as uint16 bf16 bits [N]).
    """
    w32 = np.ascontiguousarray(w, dtype=np.float32)
    if w32.ndim != 2:
        raise ValueError("w must be [N, K]")
    amax = np.max(np.abs(w32), axis=1) if w32.shape[1] else np.zeros(w32.shape[0], np.float32)
    step32 = (amax.astype(np.float32) / np.float32(QMAX)).astype(np.float32)
    s_bits = f32_to_bf16_bits(step32)
    s32 = bf16_bits_to_f64(s_bits).astype(np.float32)      # exact: bf16 -> fp32
    q = np.zeros(w32.shape, dtype=np.int8)
    live = s32 > 0
    if np.any(live):
        ratio = (w32[live] / s32[live, None]).astype(np.float32)   # fp32 division
        code = np.clip(np.rint(ratio), -QMAX, QMAX)
        q[live] = code.astype(np.int8)
    s_bits = np.where(live, s_bits, np.uint16(0)).astype(np.uint16)
    return q, s_bits


def dequantize(q, s_bits) -> np.ndarray:
    """W_hat[n, k] = q[n, k] * delta_n in fp64 (exact: 8-bit by 8-bit significands)."""
    return q.astype(np.float64) * bf16_bits_to_f64(s_bits)[:, None]


# --------------------------------------------------------------------------
# O2  quantised linear  (Eq. 8 then Eq. 10, activations left in bf16)
# --------------------------------------------------------------------------
def w8_linear(x_bits, q, s_bits) -> np.ndarray:
    """y[m, n] = ( sum_k x[m, k] * q[n, k] ) * delta_n, everything in fp64.

    x_bits: uint16 bf16 bits [M, K]; q: int8 [N, K]; s_bits: uint16 [N].
    The integer-code product is summed first (Eq. 8) and the per-row step size
    applied afterwards (Eq. 10), the order the paper states.
    Returns fp64 [M, N] (unrounded).
    """
    x = bf16_bits_to_f64(x_bits)
    if x.ndim != 2 or q.ndim != 2 or x.shape[1] != q.shape[1]:
        raise ValueError("shape mismatch: x[M,K], q[N,K]")
    acc = x @ q.astype(np.float64).T
    return acc * bf16_bits_to_f64(s_bits)[None, :]


def bf16_linear(x_bits, w_bits) -> np.ndarray:
    """Full-precision comparison point: y = x . W^T with W held in bf16 (Eq. 11)."""
    x = bf16_bits_to_f64(x_bits)
    w = bf16_bits_to_f64(w_bits)
    return x @ w.T


def rel_maxabs_err(y_test, y_ref) -> float:
    """max|y_test - y_ref| / max|y_ref|  (the linear-output acceptance measure)."""
    y_ref = np.asarray(y_ref, dtype=np.float64)
    d = np.max(np.abs(np.asarray(y_test, dtype=np.float64) - y_ref)) if y_ref.size else 0.0
    den = np.max(np.abs(y_ref)) if y_ref.size else 0.0
    return float(d / den) if den > 0 else float(d)


# --------------------------------------------------------------------------
# O3  LM head + greedy acceptance  (Eq. 2 at temperature 0)
# --------------------------------------------------------------------------
def lmhead_verify(h_bits, q, s_bits, draft, *, rows_per_block: int = 8192,
                  weights_are_bf16: bool = False):
    """Vocabulary projection, per-position argmax, accepted length.

    logit[m, v] is ``w8_linear`` (or ``bf16_linear``) applied to the vocabulary
    matrix.  Position i's logits judge candidate token draft[i]; the candidate is
    kept iff it equals the smallest index attaining the row maximum (with a
    deterministic drafter the ratio test of Eq. 2 accepts exactly the argmax).
    The accepted length is the number of leading kept candidates; the token at
    the first rejected position (or the bonus position after a full match) is
    argmax[n_acc].

    Vocabulary rows are visited in blocks only to bound memory; each logit is
    still one plain fp64 dot product.

    Returns dict(argmax int64 [M], n_acc int, top1 [M], top2 [M], maxabs [M]).
    top2 is the largest logit at any OTHER index (equal to top1 on an exact tie).
    """
    x = bf16_bits_to_f64(h_bits)
    M = x.shape[0]
    V = q.shape[0]
    best = np.full(M, -np.inf)
    second = np.full(M, -np.inf)
    arg = np.zeros(M, dtype=np.int64)
    maxabs = np.zeros(M)
    for v0 in range(0, V, rows_per_block):
        v1 = min(V, v0 + rows_per_block)
        if weights_are_bf16:
            lg = x @ bf16_bits_to_f64(q[v0:v1]).T
        else:
            lg = (x @ q[v0:v1].astype(np.float64).T) * bf16_bits_to_f64(s_bits[v0:v1])[None, :]
        maxabs = np.maximum(maxabs, np.max(np.abs(lg), axis=1))
        for m in range(M):
            row = lg[m]
            j = int(np.argmax(row))          # numpy returns the first maximum
            b1 = row[j]
            if row.size > 1:
                tmp = row.copy()
                tmp[j] = -np.inf
                b2 = float(np.max(tmp))
            else:
                b2 = -np.inf
            if b1 > best[m]:                 # strict: earlier block wins ties
                second[m] = max(best[m], b2)
                best[m] = b1
                arg[m] = v0 + j
            else:
                second[m] = max(second[m], b1)
    draft = np.asarray(draft, dtype=np.int64).reshape(-1)
    if draft.size > M:
        raise ValueError("n_draft must not exceed M")
    n_acc = 0
    for i in range(draft.size):
        if arg[i] == draft[i]:
            n_acc += 1
        else:
            break
    return {"argmax": arg, "n_acc": n_acc, "top1": best, "top2": second, "maxabs": maxabs}


def accepted_length(argmax, draft) -> int:
    """Number of leading positions i with argmax[i] == draft[i] (Eq. 2, T = 0)."""
    n = 0
    for a, d in zip(list(argmax), list(draft)):
        if int(a) != int(d):
            break
        n += 1
    return n
