"""Pins for the W8A8 oracle: closed forms, exact rational arithmetic, brute force in pure
Python integers, invariants, the quantisation error bound against the real-valued
product, and the independent naive-C form.  No GPU, and no expected value comes from the
HIP path.
"""
import struct
from fractions import Fraction

import numpy as np
import pytest

from oracle import quasar_ref as ref
from oracle import quasar_w8a8_ref as a8
from paper_2603_01399_amd import synth


def bits(x):
    return synth.to_bf16_bits(np.asarray(x, dtype=np.float32))


def f32(v):
    """Round a Python number (int, float or Fraction) to fp32, nearest even, through the C library."""
    return struct.unpack("f", struct.pack("f", float(v)))[0]


def bf16_of_f32(v):
    """bf16 bits of an fp32 number by exact rational comparison (no shared helper)."""
    if v == 0:
        return 0
    u = struct.unpack("I", struct.pack("f", v))[0]
    lo, hi = u & 0xFFFF0000, (u & 0xFFFF0000) + 0x10000
    flo = Fraction(struct.unpack("f", struct.pack("I", lo))[0])
    fhi = Fraction(struct.unpack("f", struct.pack("I", hi))[0])
    x = Fraction(v)
    dl, dh = abs(x - flo), abs(fhi - x)
    if dl < dh:
        return lo >> 16
    if dh < dl:
        return hi >> 16
    return (lo >> 16) if ((lo >> 16) & 1) == 0 else (hi >> 16)


# ------------------------------------------------------------ activation quantiser
def test_activation_codes_closed_forms():
    # amax = 127 -> dx = 1, inv = 1: integer inputs are their own codes
    row = np.array([[127, -127, 1, 0, -64, 33, 2, -5]], dtype=np.float32)
    xq, dx = a8.quantize_activations(bits(row))
    assert dx[0] == 1.0
    assert np.array_equal(xq[0], row[0].astype(np.int8))
    # the largest magnitude always maps to +-127, whatever the scale
    r = np.random.Generator(np.random.Philox(5))
    x = r.standard_normal((16, 256)).astype(np.float32) * np.exp2(r.integers(-20, 20, (16, 1))).astype(np.float32)
    xb = bits(x)
    xq, dx = a8.quantize_activations(xb)
    xr = ref.bf16_bits_to_f64(xb)
    j = np.argmax(np.abs(xr), axis=1)
    assert np.array_equal(np.abs(xq[np.arange(16), j]), np.full(16, 127))
    assert np.abs(xq.astype(int)).max() <= 127
    # the step size is the fp32 quotient amax / 127
    for m in range(16):
        assert dx[m] == f32(Fraction(f32(np.abs(xr[m]).max())) / 127)


def test_activation_zero_row_and_power_of_two_invariance():
    x = np.zeros((3, 64), dtype=np.float32)
    x[1, 5] = 0.375
    x[2] = np.linspace(-1, 1, 64)
    xb = bits(x)
    xq, dx = a8.quantize_activations(xb)
    assert dx[0] == 0 and not xq[0].any()
    assert xq[1, 5] == 127 and np.count_nonzero(xq[1]) == 1
    # scaling a row by 2^p scales the step and keeps the codes
    xq2, dx2 = a8.quantize_activations(bits(ref.bf16_bits_to_f64(xb) * 2.0 ** 9))
    assert np.array_equal(xq2, xq)
    assert np.array_equal(dx2, dx * np.float32(2.0 ** 9))


def test_activation_codes_match_exact_rational_rule():
    """Re-derive every code with exact rationals: code = rint(fp32(x~ * inv)), inv = fp32(127/amax)."""
    r = np.random.Generator(np.random.Philox(6))
    x = r.standard_normal((3, 96)).astype(np.float32)
    s = np.exp2(r.uniform(-2, 2, 96)).astype(np.float32)
    xb = bits(x)
    xq, dx = a8.quantize_activations(xb, s)
    xv = ref.bf16_bits_to_f64(xb)
    for m in range(3):
        xt = [f32(Fraction(xv[m, k]) * Fraction(float(s[k]))) for k in range(96)]
        amax = max(abs(v) for v in xt)
        inv = f32(Fraction(127) / Fraction(amax))
        assert dx[m] == f32(Fraction(amax) / 127)
        for k in range(96):
            p = Fraction(f32(Fraction(xt[k]) * Fraction(inv)))
            fl = p.numerator // p.denominator
            rem = p - fl
            code = fl + (1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2) else 0)
            assert xq[m, k] == max(-127, min(127, code)), (m, k)


def test_activation_error_bound_and_smoothing_identity():
    r = np.random.Generator(np.random.Philox(7))
    x = r.standard_normal((8, 512)).astype(np.float32)
    xb = bits(x)
    ones = np.ones(512, dtype=np.float32)
    a, da = a8.quantize_activations(xb)
    b, db = a8.quantize_activations(xb, ones)
    assert np.array_equal(a, b) and np.array_equal(da, db)
    # |x~ - dx * code| <= dx/2 up to the fp32 rounding of inv and of the product
    xv = ref.bf16_bits_to_f64(xb)
    err = np.abs(xv - a.astype(np.float64) * da[:, None].astype(np.float64))
    assert np.all(err <= 0.5 * da[:, None] * (1 + 1e-5) + 1e-12)
    # smoothing by s then quantising equals quantising the pre-multiplied (fp32) activations
    s = np.exp2(r.integers(-3, 4, 512)).astype(np.float32)       # powers of two: x*s is a bf16 number
    c, dc = a8.quantize_activations(xb, s)
    d, dd = a8.quantize_activations(bits(xv * s))
    assert np.array_equal(c, d) and np.array_equal(dc, dd)


def test_smooth_weights_identity_in_exact_arithmetic():
    # (W diag(s)^-1)(diag(s) x) = W x when s is a power of two (both divisions exact)
    r = np.random.Generator(np.random.Philox(8))
    w = r.standard_normal((12, 40)).astype(np.float32)
    s = np.exp2(r.integers(-4, 5, 40)).astype(np.float32)
    x = r.standard_normal(40).astype(np.float32)
    wt = a8.smooth_weights(w, s)
    assert np.array_equal(wt.astype(np.float64) * s.astype(np.float64), w.astype(np.float64))
    assert np.allclose(wt.astype(np.float64) @ (x.astype(np.float64) * s), w.astype(np.float64) @ x, rtol=1e-12)
    # general s: one fp32 division per element
    s2 = r.uniform(0.5, 2.0, 40).astype(np.float32)
    wt2 = a8.smooth_weights(w, s2)
    for n, k in [(0, 0), (3, 7), (11, 39)]:
        assert wt2[n, k] == f32(Fraction(float(w[n, k])) / Fraction(float(s2[k])))


# ------------------------------------------------------------ integer matmul + dequantisation
def test_accumulate_brute_force_python_ints():
    r = np.random.Generator(np.random.Philox(9))
    xq = r.integers(-127, 128, (5, 37)).astype(np.int8)
    q = r.integers(-127, 128, (11, 37)).astype(np.int8)
    acc = a8.w8a8_accumulate(xq, q)
    for m in range(5):
        for n in range(11):
            assert int(acc[m, n]) == sum(int(xq[m, k]) * int(q[n, k]) for k in range(37))
    # a transposed operand or a dropped term would break this
    assert acc.dtype == np.int32
    with pytest.raises(ValueError):
        a8.w8a8_accumulate(xq, q[:, :36])


def test_accumulate_overflow_is_detected():
    K = 133200                                  # 127 * 127 * K > 2^31 - 1
    xq = np.full((1, K), 127, dtype=np.int8)
    q = np.full((1, K), 127, dtype=np.int8)
    with pytest.raises(OverflowError):
        a8.w8a8_accumulate(xq, q)


def test_linear_bits_against_rational_arithmetic():
    """Each output re-derived with Fractions: fp32(acc) * fp32(dx*dw) -> fp32 -> bf16."""
    r = np.random.Generator(np.random.Philox(10))
    M, K, N = 3, 64, 9
    xb = bits(r.standard_normal((M, K)).astype(np.float32) * 3)
    w = (r.standard_normal((N, K)) * 0.02).astype(np.float32)
    q, dwb = ref.quantize_weights(w)
    y = a8.w8a8_linear(xb, q, dwb)
    xq, dx = a8.quantize_activations(xb)
    dw = ref.bf16_bits_to_f64(dwb)
    for m in range(M):
        for n in range(N):
            acc = sum(int(xq[m, k]) * int(q[n, k]) for k in range(K))
            scale = f32(Fraction(float(dx[m])) * Fraction(float(dw[n])))
            val = f32(Fraction(f32(acc)) * Fraction(scale))
            assert int(y[m, n]) == bf16_of_f32(val), (m, n)


def test_int32_to_fp32_conversion_rounds_to_even():
    # acc = 2^24 + 1 is not an fp32 number: it must round to 2^24 (even), 2^24 + 3 to 2^24 + 4
    for acc_want, f_want in [(2 ** 24 + 1, 2.0 ** 24), (2 ** 24 + 3, 2.0 ** 24 + 4)]:
        K = 1100
        xq = np.zeros((1, K), dtype=np.int8)
        q = np.zeros((1, K), dtype=np.int8)
        full, rest = divmod(acc_want, 127 * 127)
        xq[0, :full] = 127
        q[0, :full] = 127
        a, bq = divmod(rest, 127)
        xq[0, full] = 127
        q[0, full] = a
        xq[0, full + 1] = bq
        q[0, full + 1] = 1
        assert int(a8.w8a8_accumulate(xq, q)[0, 0]) == acc_want
        dwb = bits(np.array([1.0], dtype=np.float32))
        lg = (a8.w8a8_accumulate(xq, q).astype(np.float32) * a8.w8a8_scale(dwb, np.array([1.0], np.float32)))
        assert float(lg[0, 0]) == f_want


def test_w8a8_within_quantisation_error_bound_of_real_product():
    """|y - W~ x~| <= sum_k ( |w~| dx/2 + |x~| dw/2 + dx dw/4 ) + rounding: the bound the
    method's two quantisers imply; a wrong scale grouping or a missing step size fails it."""
    r = np.random.Generator(np.random.Philox(12))
    M, K, N = 8, 1024, 48
    x = r.standard_normal((M, K)).astype(np.float32)
    w = (r.standard_normal((N, K)) * 0.02).astype(np.float32)
    s = np.exp2(r.uniform(-1, 1, K)).astype(np.float32)
    xb = bits(x)
    wt = a8.smooth_weights(w, s)
    q, dwb = ref.quantize_weights(wt)
    lg = a8.w8a8_logits(xb, q, dwb, s).astype(np.float64)
    xt = (ref.bf16_bits_to_f64(xb).astype(np.float32) * s).astype(np.float64)
    exact = xt @ wt.astype(np.float64).T
    _, dx = a8.quantize_activations(xb, s)
    dw = ref.bf16_bits_to_f64(dwb)
    bound = (np.abs(wt).sum(axis=1)[None, :] * dx[:, None] / 2 + np.abs(xt).sum(axis=1)[:, None] * dw[None, :] / 2
             + K * dx[:, None] * dw[None, :] / 4)
    # bf16 step sizes are themselves rounded (<= 2^-9 relative): widen the weight term accordingly
    bound = bound * 1.01 + 1e-6 * np.abs(exact)
    assert np.all(np.abs(lg - exact) <= bound)
    # and it is not vacuous: the smoothing identity holds to fp32 accuracy, the error is real but small
    plain = ref.bf16_bits_to_f64(xb) @ w.astype(np.float64).T
    assert np.abs(exact - plain).max() <= 1e-4 * np.abs(plain).max()
    assert 1e-4 < np.abs(lg - exact).max() / np.abs(exact).max() < 2e-2


def test_identity_weights_return_dequantised_activations():
    K = 64
    w = np.eye(K, dtype=np.float32)
    q, dwb = ref.quantize_weights(w)             # codes 127 on the diagonal, dw = bf16(1/127)
    r = np.random.Generator(np.random.Philox(13))
    xb = bits(r.standard_normal((4, K)).astype(np.float32))
    xq, dx = a8.quantize_activations(xb)
    lg = a8.w8a8_logits(xb, q, dwb)
    dw = np.float32(ref.bf16_bits_to_f64(dwb)[0])
    want = (xq.astype(np.float32) * np.float32(127)) * (dx[:, None] * dw)
    assert np.array_equal(lg, want.astype(np.float32))


# ------------------------------------------------------------ verification
def test_lmhead_verify_planted_and_ties():
    r = np.random.Generator(np.random.Philox(14))
    M, K, V = 6, 128, 700
    xb = bits(r.standard_normal((M, K)).astype(np.float32))
    w = (r.standard_normal((V, K)) * 0.02).astype(np.float32)
    q, dwb = ref.quantize_weights(w)
    lg = a8.w8a8_logits(xb, q, dwb)
    want = np.argmax(lg, axis=1)
    for j in (0, 3, 5):
        draft = want[:5].copy()
        if j < 5:
            draft[j] = (draft[j] + 1) % V
        arg, n = a8.w8a8_lmhead_verify(xb, q, dwb, draft, rows_per_block=97)
        assert np.array_equal(arg, want)
        assert n == j
    # exact ties: duplicate the winning row later in the vocabulary -> the first index wins
    q2 = np.concatenate([q, q[want[0]:want[0] + 1]], axis=0)
    d2 = np.concatenate([dwb, dwb[want[0]:want[0] + 1]])
    arg, _ = a8.w8a8_lmhead_verify(xb, q2, d2, [], rows_per_block=64)
    assert arg[0] == want[0]
    # block size does not matter
    a1, n1 = a8.w8a8_lmhead_verify(xb, q, dwb, want[:5], rows_per_block=1)
    a2, n2 = a8.w8a8_lmhead_verify(xb, q, dwb, want[:5], rows_per_block=10 ** 6)
    assert np.array_equal(a1, a2) and n1 == n2 == 5


# ------------------------------------------------------------ independent C form
def test_c_form_agrees_bit_for_bit(cref):
    r = np.random.Generator(np.random.Philox(15))
    M, K, N = 7, 320, 45
    xb = bits(r.standard_normal((M, K)).astype(np.float32) * np.exp2(r.integers(-6, 6, (M, 1))).astype(np.float32))
    xb[2] = 0
    s = r.uniform(0.25, 4.0, K).astype(np.float32)
    w = (r.standard_normal((N, K)) * 0.02).astype(np.float32)
    q, dwb = ref.quantize_weights(w)
    for smooth in (None, s):
        xq, dx = a8.quantize_activations(xb, smooth)
        cq, cdx = cref.quantize_activations(xb, smooth)
        assert np.array_equal(xq, cq)
        assert np.array_equal(dx.view(np.uint32), cdx.view(np.uint32))
        lg = a8.w8a8_logits(xb, q, dwb, smooth)
        clg = cref.w8a8_logits(cq, cdx, q, dwb)
        assert np.array_equal(lg.view(np.uint32), clg.view(np.uint32))
