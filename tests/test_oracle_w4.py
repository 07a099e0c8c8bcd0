"""Pins for the 4-bit-weight oracle: a hand-worked example in exact rationals, error bounds of the
quantiser, structure (groups are independent, the largest element of a group gets +-7),
invariances, brute force in exact rational arithmetic for the grouped matmul, reduction to the
8-bit routine when one group spans the row, and the acceptance rule.  No GPU."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import quasar_ref as ref
from oracle import quasar_w4_ref as w4


def bf16_fraction(bits) -> Fraction:
    """Exact value of a (normal, finite) bf16 bit pattern, without numpy float arithmetic."""
    bits = int(bits)
    sign = -1 if bits & 0x8000 else 1
    e = (bits >> 7) & 0xFF
    f = bits & 0x7F
    if e == 0 and f == 0:
        return Fraction(0)
    assert 0 < e < 255
    return sign * Fraction(128 + f, 128) * Fraction(2) ** (e - 127)


def test_worked_example_in_exact_rationals():
    """Row (0.7, -0.33, 0.1, 0 | 0.021, 0.01, -0.04, 0.03), groups of 4.
    Group 0: amax 0.7, 0.7/7 = 0.1 -> bf16 0x3DCD = 0.10009765625; codes 0.7/d = 6.993 -> 7,
    -0.33/d = -3.297 -> -3, 0.1/d = 0.999 -> 1, 0 -> 0.
    Group 1: amax 0.04, 0.04/7 = 0.0057142... -> bf16 0x3BBB = 0.005706787109375; codes
    0.021/d = 3.680 -> 4, 0.01/d = 1.752 -> 2, -0.04/d = -7.009 -> -7, 0.03/d = 5.257 -> 5."""
    w = np.array([[0.7, -0.33, 0.1, 0.0, 0.021, 0.01, -0.04, 0.03]], dtype=np.float32)
    q, s = w4.quantize_weights_w4(w, group=4)
    assert s.tolist() == [[0x3DCD, 0x3BBB]]
    assert bf16_fraction(0x3DCD) == Fraction(205, 2048) and bf16_fraction(0x3BBB) == Fraction(187, 32768)
    assert q.tolist() == [[7, -3, 1, 0, 4, 2, -7, 5]]
    # the same codes from exact rational arithmetic on the fp32 inputs (none is near a rounding tie)
    for g in range(2):
        d = bf16_fraction(s[0, g])
        for k in range(4):
            r = Fraction(float(w[0, 4 * g + k])) / d
            want = max(-7, min(7, round(r)))
            assert abs(r - round(r)) < Fraction(2, 5)
            assert q[0, 4 * g + k] == want


def test_quantiser_error_bound_and_code_range():
    r = np.random.Generator(np.random.Philox(41))
    w = (r.standard_normal((48, 512)) * 0.02).astype(np.float32)
    w[3, 128:256] = 0.0                                     # an all-zero group
    w[5, 7] = 0.5                                           # an outlier only hurts its own group
    q, s = w4.quantize_weights_w4(w, group=128)
    assert q.dtype == np.int8 and q.min() >= -7 and q.max() <= 7
    d = ref.bf16_bits_to_f64(s)                              # [N, G]
    wh = w4.dequantize_w4(q, s, 128)
    err = np.abs(wh - w.astype(np.float64)).reshape(48, 4, 128)
    amax = np.abs(w).reshape(48, 4, 128).max(axis=2)
    # half a step, plus what rounding the step to bf16 (relative 2^-9) can add at the clamped end
    assert np.all(err <= 0.5 * d[:, :, None] + amax[:, :, None] * 2.0 ** -8 + 1e-12)
    # the step is amax/7 to bf16 precision, and the largest element of every live group gets +-7
    live = amax > 0
    assert np.all(np.abs(d[live] * 7 / amax[live] - 1) <= 2.0 ** -8)
    assert np.all(np.abs(q).reshape(48, 4, 128).max(axis=2)[live] == 7)
    assert np.all(q[3, 128:256] == 0) and s[3, 1] == 0
    # the outlier's group is coarse, the neighbouring group of the same row is not
    assert d[5, 0] > 5 * d[5, 1]


def test_groups_are_independent_and_scale_invariance():
    r = np.random.Generator(np.random.Philox(42))
    w = (r.standard_normal((16, 256)) * 0.05).astype(np.float32)
    q, s = w4.quantize_weights_w4(w, group=64)
    for g in range(4):
        qg, sg = w4.quantize_weights_w4(w[:, 64 * g:64 * (g + 1)], group=64)
        assert np.array_equal(qg, q[:, 64 * g:64 * (g + 1)]) and np.array_equal(sg[:, 0], s[:, g])
    # powers of two move the step and leave the codes alone; the sign flips the codes
    q2, s2 = w4.quantize_weights_w4(w * np.float32(8.0), group=64)
    assert np.array_equal(q2, q) and np.allclose(ref.bf16_bits_to_f64(s2), 8.0 * ref.bf16_bits_to_f64(s), rtol=0, atol=0)
    q3, s3 = w4.quantize_weights_w4(-w, group=64)
    assert np.array_equal(q3, -q) and np.array_equal(s3, s)
    with pytest.raises(ValueError):
        w4.quantize_weights_w4(w, group=48)


def test_rounding_is_half_to_even_and_clamped():
    # step exactly 1 (amax = 7): 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, -3.5 -> -4; 7 stays 7
    w = np.array([[7.0, 0.5, 1.5, 2.5, -3.5, -0.5, 6.5, -6.5]], dtype=np.float32)
    q, s = w4.quantize_weights_w4(w, group=8)
    assert ref.bf16_bits_to_f64(s)[0, 0] == 1.0
    assert q.tolist() == [[7, 0, 2, 2, -4, 0, 6, -6]]
    # a step rounded DOWN to bf16 makes amax/step exceed 7: the clamp holds it at 7
    w = np.array([[0.7, -0.7, 0.0, 0.0]], dtype=np.float32)
    w[0, 0] = np.float32(7 * 1.00390625)                     # 7 * (1 + 2^-8): step rounds to even, down to 1.0
    w[0, 1] = -w[0, 0]
    q, s = w4.quantize_weights_w4(w, group=4)
    assert ref.bf16_bits_to_f64(s)[0, 0] == 1.0 and q.tolist() == [[7, -7, 0, 0]]


def test_linear_brute_force_exact_rationals():
    r = np.random.Generator(np.random.Philox(43))
    M, N, K, group = 3, 5, 24, 8
    x_bits = ref.f32_to_bf16_bits(r.standard_normal((M, K)).astype(np.float32))
    q = r.integers(-7, 8, size=(N, K)).astype(np.int8)
    s_bits = ref.f32_to_bf16_bits((r.random((N, K // group)) * 0.01 + 0.001).astype(np.float32))
    y = w4.w4_linear(x_bits, q, s_bits, group)
    for m in range(M):
        for n in range(N):
            tot = Fraction(0)
            for g in range(K // group):
                inner = sum(bf16_fraction(x_bits[m, k]) * int(q[n, k]) for k in range(group * g, group * (g + 1)))
                tot += bf16_fraction(s_bits[n, g]) * inner
            assert abs(Fraction(float(y[m, n])) - tot) <= abs(tot) * Fraction(1, 10 ** 13) + Fraction(1, 10 ** 18)


def test_linear_special_cases():
    r = np.random.Generator(np.random.Philox(44))
    M, N, K, group = 4, 32, 256, 64
    x_bits = ref.f32_to_bf16_bits(r.standard_normal((M, K)).astype(np.float32))
    w = (r.standard_normal((N, K)) * 0.02).astype(np.float32)
    q, s_bits = w4.quantize_weights_w4(w, group)
    y = w4.w4_linear(x_bits, q, s_bits, group)
    # (a) the same number as x . W_hat^T with the weights dequantised first
    x = ref.bf16_bits_to_f64(x_bits)
    assert np.allclose(y, x @ w4.dequantize_w4(q, s_bits, group).T, rtol=1e-12, atol=1e-15)
    # (b) one group spanning the whole row is the per-row rule of the 8-bit routine
    q1, s1 = w4.quantize_weights_w4(w, K)
    assert np.allclose(w4.w4_linear(x_bits, q1, s1, K), ref.w8_linear(x_bits, q1, s1[:, 0]), rtol=1e-13, atol=0)
    # (c) a one-hot activation picks out one dequantised column; zero activations give zero
    e = np.zeros((1, K), dtype=np.float32)
    e[0, 70] = 1.0
    col = w4.w4_linear(ref.f32_to_bf16_bits(e), q, s_bits, group)[0]
    assert np.array_equal(col, q[:, 70].astype(np.float64) * ref.bf16_bits_to_f64(s_bits)[:, 70 // group])
    assert not w4.w4_linear(ref.f32_to_bf16_bits(np.zeros((2, K), np.float32)), q, s_bits, group).any()
    # (d) close to the unquantised product: 15 levels per group of 64 give a few per cent rms
    exact = x @ w.astype(np.float64).T
    rms = np.sqrt(np.mean((y - exact) ** 2) / np.mean(exact ** 2))
    assert 0.01 < rms < 0.2
    # (e) blocks of rows only bound memory
    assert np.array_equal(w4.w4_linear(x_bits, q, s_bits, group, rows_per_block=5), y)


def test_lmhead_verify_planted_and_ties():
    r = np.random.Generator(np.random.Philox(45))
    M, V, K, group = 6, 96, 128, 32
    h = r.standard_normal((M, K)).astype(np.float32)
    h_bits = ref.f32_to_bf16_bits(h)
    hb = ref.bf16_bits_to_f64(h_bits)
    w = (r.standard_normal((V, K)) * 0.02).astype(np.float32)
    target = np.array([5, 17, 40, 41, 77, 90])
    for i, t in enumerate(target):
        w[t] += (8.0 / np.dot(hb[i], hb[i])) * hb[i].astype(np.float32)
    q, s = w4.quantize_weights_w4(w, group)
    for j in range(M):
        draft = target[:M - 1].copy()
        if j < M - 1:
            draft[j] = (draft[j] + 1) % V
        res = w4.w4_lmhead_verify(h_bits, q, s, draft, group)
        assert np.array_equal(res["argmax"], target) and res["n_acc"] == min(j, M - 1)
        assert np.all(res["top1"] - res["top2"] > 1.0)
    assert w4.w4_lmhead_verify(h_bits, q, s, [], group)["n_acc"] == 0
    # identical rows tie: the lower index wins; all-zero hidden states give index 0
    q[60] = q[17]
    s[60] = s[17]
    q[3] = q[17]
    s[3] = s[17]
    res = w4.w4_lmhead_verify(h_bits, q, s, [], group)
    assert res["argmax"][1] == 3 and res["top1"][1] == res["top2"][1]
    z = w4.w4_lmhead_verify(np.zeros((2, K), np.uint16), q, s, [0, 0], group)
    assert z["argmax"].tolist() == [0, 0] and z["n_acc"] == 2
    with pytest.raises(ValueError):
        w4.w4_lmhead_verify(h_bits, q, s, np.zeros(M + 1), group)
