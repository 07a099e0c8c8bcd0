"""GPU parity for the 4-bit group-wise weight path through the C-ABI against the CPU oracle.
Codes and step sizes are bit-exact; argmax and accepted length are exact on planted cases and on
exact ties; bf16 linear outputs are held to max|y_gpu - y_ref| / max|y_ref| <= 1e-2 (the bar of
the 8-bit path) and, as the arithmetic predicts (fp32 sums, one bf16 rounding), 4e-3 in
practice."""
import numpy as np
import pytest
import torch

from oracle import quasar_ref as ref
from oracle import quasar_w4_ref as w4
from paper_2603_01399_amd import synth
from gpu_util import bf16_to_dev, bf16_to_host, f32_to_dev, i32_to_dev

pytestmark = pytest.mark.gpu

TOL = 1e-2
TOL_EXPECTED = 4e-3
GROUP = 128


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_01399_amd import binding
    return binding


def say(*a):
    print(*a, flush=True)


def quantize_both(qb, w):
    q_ref, s_ref = w4.quantize_weights_w4(w, GROUP)
    return q_ref, s_ref, qb.quantize_weights_w4(f32_to_dev(w))


# ------------------------------------------------------------------ quantise / pack
@pytest.mark.parametrize("N,K,seed", [(16, 128, 1), (48, 384, 2), (1024, 1024, 3), (80, 4096, 4), (4096, 256, 5)])
def test_quantize_w4_bit_exact(qb, N, K, seed):
    say("w4 quantize", N, K, seed)
    w = synth.normal_weights(N, K, seed=synth.seed_for(8, 0, seed))
    if N >= 48:
        w[5, :128] = 0.0                               # zero group -> delta 0, codes 0
        w[7] *= np.float32(2.0 ** -20)                 # tiny row
        w[9] = np.round(w[9] * 300)                    # integer-valued row with ties after scaling
        w[11, 3] = 0.5                                 # an outlier
    q_ref, s_ref, wp = quantize_both(qb, w)
    assert wp.numel() == qb.w4_packed_bytes(N, K) == N * K // 2 + 2 * N * (K // GROUP)
    q_gpu, s_gpu = qb.unpack_weights_w4(wp, N, K)
    assert np.array_equal(bf16_to_host(s_gpu), s_ref)
    assert np.array_equal(q_gpu.cpu().numpy(), q_ref)


def test_quantize_w4_ties_bf16_and_strided_source(qb):
    say("w4 quantize ties")
    w = np.zeros((16, 128), dtype=np.float32)
    w[0, :8] = [7.0, 0.5, 1.5, 2.5, -0.5, -1.5, 3.5, 6.5]
    w[1, 0] = 1.0
    q_ref, s_ref, wp = quantize_both(qb, w)
    q_gpu, s_gpu = qb.unpack_weights_w4(wp, 16, 128)
    assert q_gpu.cpu().numpy()[0, :8].tolist() == [7, 0, 2, 2, 0, -2, 4, 6]
    assert np.array_equal(q_gpu.cpu().numpy(), q_ref) and np.array_equal(bf16_to_host(s_gpu), s_ref)
    # bf16 source weights: same result as quantising their fp32 widening
    wb = synth.to_bf16_bits(synth.normal_weights(64, 256, seed=77))
    w32 = ref.bf16_bits_to_f64(wb).astype(np.float32)
    q_ref, s_ref = w4.quantize_weights_w4(w32, GROUP)
    q_gpu, s_gpu = qb.unpack_weights_w4(qb.quantize_weights_w4(bf16_to_dev(wb)), 64, 256)
    assert np.array_equal(q_gpu.cpu().numpy(), q_ref) and np.array_equal(bf16_to_host(s_gpu), s_ref)
    # strided source
    w = synth.normal_weights(32, 384, seed=88)
    q_ref, s_ref = w4.quantize_weights_w4(w[:, :256], GROUP)
    q_gpu, s_gpu = qb.unpack_weights_w4(qb.quantize_weights_w4(f32_to_dev(w)[:, :256]), 32, 256)
    assert np.array_equal(q_gpu.cpu().numpy(), q_ref) and np.array_equal(bf16_to_host(s_gpu), s_ref)


# ------------------------------------------------------------------ linear
def integer_case_w4(M, N, K, seed):
    """Integer activations in [-8, 8] and integer weights in [-7, 7] with a +-7 in every group
    and a power-of-two factor per (row, group): codes, step sizes and every sum are exact."""
    r = np.random.Generator(np.random.Philox(seed))
    xi = r.integers(-8, 9, size=(M, K))
    wi = r.integers(-7, 8, size=(N, K))
    G = K // GROUP
    cols = r.integers(0, GROUP, size=(N, G))
    for g in range(G):
        wi[np.arange(N), g * GROUP + cols[:, g]] = 7 * (r.integers(0, 2, size=N) * 2 - 1)
    exps = r.integers(-5, 3, size=(N, G))
    w = (wi.astype(np.float64) * np.repeat(np.exp2(exps.astype(np.float64)), GROUP, axis=1)).astype(np.float32)
    return synth.to_bf16_bits(xi.astype(np.float32)), w, wi


@pytest.mark.parametrize("M", [1, 3, 8, 9, 16, 17, 32])
@pytest.mark.parametrize("N,K", [(48, 256), (256, 1024), (64, 4096 + 128)])
def test_w4_linear_integer_inputs_bit_exact(qb, M, N, K):
    say("w4 linear int", M, N, K)
    xb, w, wi = integer_case_w4(M, N, K, seed=2000 + M)
    q_ref, s_ref, wp = quantize_both(qb, w)
    assert np.array_equal(q_ref, wi)
    want = ref.f64_to_bf16_bits(w4.w4_linear(xb, q_ref, s_ref, GROUP))    # exact sums, one rounding
    got = bf16_to_host(qb.w4_linear(bf16_to_dev(xb), wp, N))
    assert np.array_equal(got, want)


SHAPES_RANDOM = [
    (8, 1024, 1024),
    (1, 4096, 4096), (4, 1024, 4096), (8, 4096, 4096), (16, 4096, 4096),
    (8, 12288, 4096), (8, 4096, 12288), (16, 4096, 12288), (32, 4096, 12288),     # chunked K
    (5, 16 * 37, 128 * 5), (12, 16 * 300 + 16, 128 * 9), (32, 1024, 5120), (27, 16 * 513, 256),
    (8, 5120, 25600), (32, 16 * 700, 8192),
]


@pytest.mark.parametrize("M,N,K", SHAPES_RANDOM)
def test_w4_linear_random(qb, M, N, K):
    say("w4 linear", M, N, K)
    xb = synth.activations_bf16(M, K, seed=synth.seed_for(8, 1, M + N % 97 + K % 89))
    w = synth.normal_weights(N, K, seed=synth.seed_for(8, 2, M + N % 97 + K % 89))
    q_ref, s_ref, wp = quantize_both(qb, w)
    y_ref = w4.w4_linear(xb, q_ref, s_ref, GROUP)
    y = ref.bf16_bits_to_f64(bf16_to_host(qb.w4_linear(bf16_to_dev(xb), wp, N)))
    err = ref.rel_maxabs_err(y, y_ref)
    say("   rel err", err)
    assert err <= TOL
    assert err <= TOL_EXPECTED


def test_w4_linear_offset_activations_and_outliers(qb):
    """The kernel removes a constant of 136 per code through the sum of a group's activations:
    activations with a large common sign or single huge entries are where that would show."""
    say("w4 linear offsets")
    M, N, K = 8, 512, 2048
    r = np.random.Generator(np.random.Philox(31))
    x = r.standard_normal((M, K)).astype(np.float32)
    x[0] += 4.0                                         # all positive: the offsets are large
    x[1] = np.abs(x[1]) * -3.0
    x[2, 100] = 900.0                                   # outliers
    x[3, ::128] = -250.0
    x[4] *= 1e-3
    xb = synth.to_bf16_bits(x)
    w = synth.normal_weights(N, K, seed=32)
    q_ref, s_ref, wp = quantize_both(qb, w)
    y_ref = w4.w4_linear(xb, q_ref, s_ref, GROUP)
    y = ref.bf16_bits_to_f64(bf16_to_host(qb.w4_linear(bf16_to_dev(xb), wp, N)))
    for m in range(M):                                  # per token, so a small row is not hidden by a big one
        assert ref.rel_maxabs_err(y[m], y_ref[m]) <= TOL_EXPECTED, m


def test_w4_linear_strided_and_repeatable(qb):
    say("w4 linear strided")
    M, N, K = 8, 1024, 2048
    xb = synth.activations_bf16(M, K + 64, seed=41)
    w = synth.normal_weights(N, K, seed=42)
    q_ref, s_ref, wp = quantize_both(qb, w)
    x_dev = bf16_to_dev(xb)[:, :K]                      # row stride K + 64
    y_buf = torch.zeros((M, N + 32), dtype=torch.bfloat16, device="cuda")
    y = qb.w4_linear(x_dev, wp, N, y=y_buf[:, :N])
    got = bf16_to_host(y_buf)
    assert not got[:, N:].any()                         # nothing written past N
    y_ref = w4.w4_linear(xb[:, :K], q_ref, s_ref, GROUP)
    assert ref.rel_maxabs_err(ref.bf16_bits_to_f64(got[:, :N]), y_ref) <= TOL_EXPECTED
    again = bf16_to_host(qb.w4_linear(x_dev.contiguous(), wp, N))
    assert np.array_equal(again, got[:, :N])            # same bits run to run and for any stride


# ------------------------------------------------------------------ vocabulary verify
@pytest.mark.parametrize("M,V,K", [(8, 4096, 512), (5, 16 * 333, 256), (16, 8192, 1024), (32, 2048, 256), (1, 1024, 128)])
def test_w4_lmhead_verify_planted(qb, M, V, K):
    say("w4 verify", M, V, K)
    h = synth.activations_bf16(M, K, seed=synth.seed_for(8, 3, M))
    w = synth.normal_weights(V, K, seed=synth.seed_for(8, 4, M))
    targets = synth.distinct_targets(M, V, seed=synth.seed_for(8, 5, M))
    synth.plant_targets(w, h, targets)
    q_ref, s_ref, wp = quantize_both(qb, w)
    ws = qb.make_workspace(M, V, K)
    for j in sorted({0, M // 2, M}):
        draft = synth.draft_with_matches(targets, j, V, M)
        want = w4.w4_lmhead_verify(h, q_ref, s_ref, draft, GROUP)
        assert np.array_equal(want["argmax"], targets) and want["n_acc"] == j
        assert np.all(want["top1"] - want["top2"] > 1e-2 * want["maxabs"])
        am, acc = qb.w4_lmhead_verify(bf16_to_dev(h), wp, V, i32_to_dev(draft), ws)
        assert np.array_equal(am.cpu().numpy(), targets) and int(acc.cpu()[0]) == j
    am, acc = qb.w4_lmhead_verify(bf16_to_dev(h), wp, V, None, ws)
    assert np.array_equal(am.cpu().numpy(), targets) and int(acc.cpu()[0]) == 0


def test_w4_lmhead_verify_ties_and_zero_hidden(qb):
    say("w4 verify ties")
    M, V, K = 4, 1024, 256
    h = synth.activations_bf16(M, K, seed=51)
    w = synth.normal_weights(V, K, seed=52)
    targets = np.array([700, 33, 900, 512])
    synth.plant_targets(w, h, targets)
    w[20] = w[700]                                       # identical rows: exact ties, lower index wins
    w[999] = w[33]
    q_ref, s_ref, wp = quantize_both(qb, w)
    want = w4.w4_lmhead_verify(h, q_ref, s_ref, [20, 33, 900], GROUP)
    assert want["argmax"].tolist() == [20, 33, 900, 512] and want["n_acc"] == 3
    ws = qb.make_workspace(M, V, K)
    am, acc = qb.w4_lmhead_verify(bf16_to_dev(h), wp, V, i32_to_dev([20, 33, 900]), ws)
    assert am.cpu().numpy().tolist() == [20, 33, 900, 512] and int(acc.cpu()[0]) == 3
    z = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    am, acc = qb.w4_lmhead_verify(z, wp, V, i32_to_dev([0, 0, 1]), ws)
    assert am.cpu().numpy().tolist() == [0, 0, 0, 0] and int(acc.cpu()[0]) == 2


def test_w4_argument_errors(qb):
    say("w4 argument errors")
    assert qb.w4_packed_bytes(16, 64) == 0 and qb.w4_packed_bytes(8, 128) == 0
    x = torch.zeros((4, 192), dtype=torch.bfloat16, device="cuda")
    wp = torch.zeros(1056 * 4, dtype=torch.uint8, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.w4_linear(x, wp, 16)                                              # K not a multiple of 128
    with pytest.raises(qb.QuasarError):
        qb.quantize_weights_w4(torch.zeros((16, 192), device="cuda"))         # K not a multiple of 128
    x = torch.zeros((33, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.w4_linear(x, wp, 16)                                              # M > 32
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.w4_linear(x, wp[8:8 + 1056], 16)                                  # misaligned weights
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.w4_lmhead_verify(x, wp, 16, None, small)                          # workspace too small
