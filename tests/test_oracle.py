"""Pins for the CPU oracle: closed forms, exact integer arithmetic, brute force,
invariants and the independent naive-C form.  None of these need a GPU and none
of the expected values comes from the HIP path.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import quasar_ref as ref
from paper_2603_01399_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bits(x):
    return synth.to_bf16_bits(np.asarray(x, dtype=np.float32))


# ---------------------------------------------------------------- bf16 helpers
def _golden_bf16():
    out = []
    with open(os.path.join(GOLD, "bf16_closed_forms.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                expr, hx = line.split()
                out.append((expr, int(hx, 16)))
    return out


@pytest.mark.parametrize("expr,want", _golden_bf16())
def test_bf16_rounding_closed_forms(expr, want):
    val = float(eval(expr, {"__builtins__": {}}, {}))
    got32 = int(ref.f32_to_bf16_bits(np.array([val], dtype=np.float32))[0])
    got64 = int(ref.f64_to_bf16_bits(np.array([val], dtype=np.float64))[0])
    # 1/127 is not an fp32 number: the fp32 route rounds twice, both land on the same code here
    assert got32 == want
    assert got64 == want


def test_bf16_rounding_matches_torch_conversion():
    r = np.random.Generator(np.random.Philox(11))
    a = (r.standard_normal(200000) * np.exp2(r.integers(-30, 30, 200000))).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ref.f32_to_bf16_bits(a), want)
    # fp64 route agrees whenever the input is an fp32 number (single rounding either way)
    assert np.array_equal(ref.f64_to_bf16_bits(a.astype(np.float64)), want)
    # widening is exact
    back = ref.bf16_bits_to_f64(want)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy())


def test_f64_to_bf16_single_rounding_differs_from_double_rounding():
    # 1 + 2^-8 + 2^-40 is above the bf16 midpoint; via fp32 it first collapses onto the midpoint
    v = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert int(ref.f64_to_bf16_bits(np.array([v]))[0]) == 0x3F81
    assert int(ref.f32_to_bf16_bits(np.array([v], dtype=np.float32))[0]) == 0x3F80


# ---------------------------------------------------------------- O1 quantise
def test_quantize_unit_row_closed_form():
    w = np.zeros((3, 8), dtype=np.float32)
    w[0, 0] = 1.0                     # delta = bf16(1/127) = 0x3C01, code 127
    w[1, 3] = -127.0 * 2.0 ** -5      # delta = 2^-5 exactly
    q, s = ref.quantize_weights(w)
    assert s[0] == 0x3C01 and q[0, 0] == 127 and np.count_nonzero(q[0]) == 1
    assert ref.bf16_bits_to_f64(s[1:2])[0] == 2.0 ** -5 and q[1, 3] == -127
    assert s[2] == 0 and not q[2].any()          # zero row -> (0, 0)


def test_quantize_integer_rows_are_reproduced_exactly():
    _, w, wi, exps = synth.integer_case(2, 64, 256, seed=3, row_exponents=True)
    q, s = ref.quantize_weights(w)
    assert np.array_equal(q.astype(np.int64), wi)
    assert np.array_equal(ref.bf16_bits_to_f64(s), np.exp2(exps.astype(np.float64)))


def test_quantize_rounding_mode_is_half_even():
    w = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, 3.5, 126.5]], dtype=np.float32)
    q, s = ref.quantize_weights(w)
    assert ref.bf16_bits_to_f64(s)[0] == 1.0
    assert q[0].tolist() == [127, 0, 2, 2, 0, -2, 4, 126]


def test_quantize_error_bound_range_symmetry_scaling():
    w = synth.normal_weights(96, 512, seed=synth.seed_for(1, 0, 7))
    q, s = ref.quantize_weights(w)
    sd = ref.bf16_bits_to_f64(s)
    err = np.abs(w.astype(np.float64) - ref.dequantize(q, s))
    assert np.all(err <= sd[:, None] / 2 * (1 + 1e-6))        # |W - q*delta| <= delta/2
    assert np.all(np.max(np.abs(q.astype(np.int32)), axis=1) == 127)
    assert q.min() >= -127
    q2, s2 = ref.quantize_weights(-w)
    assert np.array_equal(q2, -q) and np.array_equal(s2, s)   # Q(-W) = -Q(W)
    q3, s3 = ref.quantize_weights(w * np.float32(8.0))
    assert np.array_equal(q3, q)                              # power-of-two row scaling
    assert np.array_equal(ref.bf16_bits_to_f64(s3), 8.0 * sd)
    # step size is bf16(amax/127) to within one bf16 rounding of the exact quotient
    exact = np.max(np.abs(w), axis=1).astype(np.float64) / 127.0
    assert np.all(np.abs(sd - exact) <= exact * 2.0 ** -8)


def test_quantize_matches_naive_c(cref):
    w = synth.normal_weights(40, 192, seed=77)
    w[5] = 0
    q, s = ref.quantize_weights(w)
    qc, sc = cref.quantize(w)
    assert np.array_equal(q, qc) and np.array_equal(s, sc)


# ---------------------------------------------------------------- O2 linear
def _exact_int_linear(xi, wi):
    M, K = xi.shape
    N = wi.shape[0]
    out = [[sum(int(xi[m, k]) * int(wi[n, k]) for k in range(K)) for n in range(N)] for m in range(M)]
    return np.array(out, dtype=object)


def test_linear_integer_inputs_exact_vs_bigint():
    xb, w, wi, exps = synth.integer_case(3, 24, 192, seed=9, row_exponents=True)
    q, s = ref.quantize_weights(w)
    y = ref.w8_linear(xb, q, s)
    xi = ref.bf16_bits_to_f64(xb).astype(np.int64)
    want = _exact_int_linear(xi, wi)
    for m in range(3):
        for n in range(24):
            assert Fraction(float(y[m, n])) == Fraction(int(want[m, n])) * Fraction(2) ** int(exps[n])


def test_linear_identity_onehot_permutation():
    K = 64
    xb = synth.activations_bf16(5, K, seed=21)
    x = ref.bf16_bits_to_f64(xb)
    eye = np.eye(K, dtype=np.float32)
    q, s = ref.quantize_weights(eye)
    y = ref.w8_linear(xb, q, s)
    # dequantised identity is 127*bf16(1/127) = 0.99994: y equals x after bf16 rounding
    assert np.array_equal(ref.f64_to_bf16_bits(y), xb)
    assert np.allclose(y, x * (127 * ref.bf16_bits_to_f64(np.array([0x3C01], np.uint16))[0]), rtol=0, atol=0)
    # one-hot rows gather columns (transposition or a wrong index would show here)
    sel = np.array([7, 0, 63, 7, 31])
    oh = np.zeros((5, K), dtype=np.float32)
    oh[np.arange(5), sel] = 127.0
    q, s = ref.quantize_weights(oh)
    y = ref.w8_linear(xb, q, s)
    assert y.shape == (5, 5)
    assert np.array_equal(y, 127.0 * x[:, sel])
    # permuting weight rows permutes output columns
    w = synth.normal_weights(48, K, seed=5)
    q, s = ref.quantize_weights(w)
    p = np.random.Generator(np.random.Philox(1)).permutation(48)
    assert np.array_equal(ref.w8_linear(xb, q[p], s[p]), ref.w8_linear(xb, q, s)[:, p])


def test_linear_bruteforce_python_and_c(cref):
    M, N, K = 3, 20, 96
    xb = synth.activations_bf16(M, K, seed=31)
    w = synth.normal_weights(N, K, seed=32)
    q, s = ref.quantize_weights(w)
    y = ref.w8_linear(xb, q, s)
    x = ref.bf16_bits_to_f64(xb)
    sd = ref.bf16_bits_to_f64(s)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                acc += Fraction(float(x[m, k])) * int(q[n, k])
            want = float(acc * Fraction(float(sd[n])))
            assert abs(y[m, n] - want) <= 1e-12 * max(1.0, abs(want))
    yc = cref.w8_linear(xb, q, s)
    assert np.max(np.abs(yc - y)) <= 1e-12 * np.max(np.abs(y))
    # summation order does not matter at fp64 resolution
    yr = ref.w8_linear(xb[:, ::-1].copy(), q[:, ::-1].copy(), s)
    assert np.max(np.abs(yr - y)) <= 1e-12 * np.max(np.abs(y))
    # linearity in x on exactly representable inputs
    xi, _, _, _ = synth.integer_case(M, N, K, seed=33)
    y1 = ref.w8_linear(xi, q, s)
    two = synth.to_bf16_bits(2.0 * ref.bf16_bits_to_f64(xi).astype(np.float32))
    assert np.array_equal(ref.w8_linear(two, q, s), 2.0 * y1)


def test_linear_quantisation_noise_vs_unquantised():
    # sanity, not parity: rounding noise of the codes is uniform(+-delta/2) per weight
    M, N, K = 8, 256, 1024
    xb = synth.activations_bf16(M, K, seed=synth.seed_for(1))
    w = synth.normal_weights(N, K, seed=synth.seed_for(1, 0, 1))
    q, s = ref.quantize_weights(w)
    y = ref.w8_linear(xb, q, s)
    y0 = ref.bf16_bits_to_f64(xb) @ w.astype(np.float64).T
    rms = np.sqrt(np.mean((y - y0) ** 2) / np.mean(y0 ** 2))
    assert 0.002 < rms < 0.03


def test_bf16_linear_bruteforce(cref):
    M, N, K = 2, 9, 64
    xb = synth.activations_bf16(M, K, seed=41)
    wb = synth.to_bf16_bits(synth.normal_weights(N, K, seed=42))
    y = ref.bf16_linear(xb, wb)
    x = ref.bf16_bits_to_f64(xb)
    w = ref.bf16_bits_to_f64(wb)
    for m in range(M):
        for n in range(N):
            want = float(sum(Fraction(float(x[m, k])) * Fraction(float(w[n, k])) for k in range(K)))
            assert abs(y[m, n] - want) <= 1e-13
    assert np.max(np.abs(cref.bf16_linear(xb, wb) - y)) <= 1e-13


def test_rel_maxabs_err_definition():
    assert ref.rel_maxabs_err(np.array([1.0, -4.0]), np.array([1.5, -4.0])) == 0.5 / 4.0


# ---------------------------------------------------------------- O3 verify
def _verify_case(M, V, K, j, seed):
    h = synth.activations_bf16(M, K, seed=seed)
    w = synth.normal_weights(V, K, seed=seed + 1)
    t = synth.distinct_targets(M, V, seed=seed + 2)
    synth.plant_targets(w, h, t)
    d = synth.draft_with_matches(t, j, V, M - 1)
    return h, w, t, d


@pytest.mark.parametrize("j", [0, 1, 3, 7])
def test_verify_planted_targets_and_accept_length(j, cref):
    M, V, K = 8, 1000, 256
    h, w, t, d = _verify_case(M, V, K, j, seed=500)
    q, s = ref.quantize_weights(w)
    out = ref.lmhead_verify(h, q, s, d, rows_per_block=333)   # ragged blocks on purpose
    assert np.array_equal(out["argmax"], t)
    assert out["n_acc"] == j
    assert np.all(out["top1"] - out["top2"] > 1e-2 * out["maxabs"])
    # brute force: full logits, plain argmax
    lg = ref.w8_linear(h, q, s)
    assert np.array_equal(np.argmax(lg, axis=1), out["argmax"])
    srt = np.sort(lg, axis=1)
    assert np.allclose(out["top1"], srt[:, -1], rtol=0, atol=0)
    assert np.allclose(out["top2"], srt[:, -2], rtol=0, atol=0)
    assert np.allclose(out["maxabs"], np.max(np.abs(lg), axis=1), rtol=0, atol=0)
    arg_c, n_c = cref.lmhead_verify(h, q, s, d)
    assert np.array_equal(arg_c, t) and n_c == j


def test_verify_monotone_in_planted_matches():
    M, V, K = 8, 400, 128
    h, w, t, _ = _verify_case(M, V, K, 0, seed=600)
    q, s = ref.quantize_weights(w)
    got = [ref.lmhead_verify(h, q, s, synth.draft_with_matches(t, j, V, M - 1))["n_acc"] for j in range(M)]
    assert got == list(range(M))
    assert ref.lmhead_verify(h, q, s, np.zeros(0, np.int32))["n_acc"] == 0


def test_verify_ties_take_lowest_index_and_zero_hidden(cref):
    M, V, K = 4, 64, 64
    h = synth.activations_bf16(M, K, seed=700)
    w = synth.normal_weights(V, K, seed=701)
    t = np.array([40, 41, 42, 43])
    synth.plant_targets(w, h, t)
    w[10] = w[40]                       # identical rows: the lower index must win
    q, s = ref.quantize_weights(w)
    out = ref.lmhead_verify(h, q, s, np.array([10, 41, 42], np.int32), rows_per_block=16)
    assert out["argmax"].tolist() == [10, 41, 42, 43]
    assert out["top1"][0] == out["top2"][0]
    assert out["n_acc"] == 3
    arg_c, n_c = cref.lmhead_verify(h, q, s, np.array([10, 41, 42], np.int32))
    assert arg_c.tolist() == [10, 41, 42, 43] and n_c == 3
    z = np.zeros((M, K), dtype=np.uint16)
    out0 = ref.lmhead_verify(z, q, s, np.array([0, 0, 5], np.int32))
    assert out0["argmax"].tolist() == [0, 0, 0, 0] and out0["n_acc"] == 2


def test_verify_bf16_weights_variant():
    M, V, K = 4, 300, 128
    h, w, t, d = _verify_case(M, V, K, 2, seed=800)
    wb = synth.to_bf16_bits(w)
    out = ref.lmhead_verify(h, wb, None, d, rows_per_block=77, weights_are_bf16=True)
    lg = ref.bf16_linear(h, wb)
    assert np.array_equal(out["argmax"], np.argmax(lg, axis=1))
    assert np.array_equal(out["argmax"], t) and out["n_acc"] == 2


def test_accepted_length_definition():
    assert ref.accepted_length([5, 6, 7, 8], [5, 6, 9]) == 2
    assert ref.accepted_length([5, 6, 7, 8], [5, 6, 7]) == 3
    assert ref.accepted_length([5, 6, 7, 8], [4, 6, 7]) == 0
    assert ref.accepted_length([5], []) == 0


# ---------------------------------------------------------------- byte counts (Eq. 11-12)
def test_weight_bytes_fixture_matches_latency_model():
    with open(os.path.join(GOLD, "weight_bytes.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    shapes = {n: (k, o) for n, k, o in synth.QWEN3_8B_LAYER}
    shapes["lm_head"] = (synth.QWEN3_8B_HIDDEN, synth.QWEN3_VOCAB)
    for name, dout, din, b8, b16 in rows:
        k, o = shapes[name]
        assert (int(dout), int(din)) == (o, k)
        assert int(b8) == o * k * 1 and int(b16) == o * k * 2
    layer = sum(k * o for _, k, o in synth.QWEN3_8B_LAYER)
    assert layer == 192937984
    assert 36 * layer + synth.QWEN3_VOCAB * 4096 == 7568097280
