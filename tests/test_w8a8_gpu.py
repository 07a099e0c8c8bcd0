"""GPU parity for the W8A8 entry points, through the C-ABI, against the CPU oracle.  Every
step of this path is pinned to single IEEE fp32 operations and exact integer sums, so the
bar is bit-exact everywhere: activation codes and step sizes, smoothed weight codes, the
bf16 output bits, the argmax and the accepted length."""
import numpy as np
import pytest
import torch

from oracle import quasar_ref as ref
from oracle import quasar_w8a8_ref as a8
from paper_2603_01399_amd import synth
from gpu_util import bf16_to_dev, bf16_to_host, f32_to_dev, i32_to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_01399_amd import binding
    return binding


def say(*a):
    print(*a, flush=True)


def smooth_vector(K, seed):
    r = np.random.Generator(np.random.Philox(seed))
    return np.exp2(r.uniform(-2.0, 2.0, K)).astype(np.float32)


def activations(M, K, seed, outliers=True):
    """N(0,1) activations with a few outlier channels and per-token magnitudes spread over
    several binades, as LLM hidden states have; one token of zeros when there is room."""
    xb = synth.activations_bf16(M, K, seed=seed)
    x = ref.bf16_bits_to_f64(xb).astype(np.float32)
    r = np.random.Generator(np.random.Philox(seed + 1))
    if outliers:
        ch = r.choice(K, size=max(1, K // 256), replace=False)
        x[:, ch] *= np.float32(40.0)
    x *= np.exp2(r.integers(-3, 4, (M, 1))).astype(np.float32)
    if M >= 3:
        x[2] = 0.0
    return synth.to_bf16_bits(x)


# ------------------------------------------------------------------ activation quantiser
@pytest.mark.parametrize("M,K,seed,smoothed", [(1, 64, 1, False), (3, 192, 2, True), (8, 1024, 3, False),
                                               (8, 4096, 4, True), (16, 4096, 5, True), (32, 12288, 6, False)])
def test_activation_codes_bit_exact(qb, M, K, seed, smoothed):
    say("quantize_activations", M, K, seed, smoothed)
    xb = activations(M, K, synth.seed_for(6, 0, seed))
    s = smooth_vector(K, 900 + seed) if smoothed else None
    xq_ref, dx_ref = a8.quantize_activations(xb, s)
    xq, dx = qb.quantize_activations(bf16_to_dev(xb), None if s is None else f32_to_dev(s))
    assert np.array_equal(dx.cpu().numpy().view(np.uint32), dx_ref.view(np.uint32))
    assert np.array_equal(xq.cpu().numpy(), xq_ref)


def test_activation_quantiser_strided_and_ties(qb):
    say("quantize_activations strided/ties")
    xb = activations(8, 320, 77)
    big = bf16_to_dev(xb)
    xq, dx = qb.quantize_activations(big[:, :256])
    xq_ref, dx_ref = a8.quantize_activations(xb[:, :256])
    assert np.array_equal(xq.cpu().numpy(), xq_ref) and np.array_equal(dx.cpu().numpy(), dx_ref)
    # amax = 127: codes are the values; halves round to even
    row = np.zeros((1, 64), dtype=np.float32)
    row[0, :8] = [127.0, 0.5, 1.5, 2.5, -0.5, -1.5, 3.5, 126.5]
    xq, dx = qb.quantize_activations(bf16_to_dev(synth.to_bf16_bits(row)))
    assert xq.cpu().numpy()[0, :8].tolist() == [127, 0, 2, 2, 0, -2, 4, 126]   # 126.5 is a bf16 number
    assert float(dx.cpu()[0]) == 1.0


# ------------------------------------------------------------------ smoothed weight preparation
@pytest.mark.parametrize("N,K,seed", [(16, 64, 1), (48, 192, 2), (1024, 1024, 3)])
def test_smoothed_weight_codes_bit_exact(qb, N, K, seed):
    say("quantize_weights_smoothed", N, K, seed)
    w = synth.normal_weights(N, K, seed=synth.seed_for(6, 1, seed))
    s = smooth_vector(K, 700 + seed)
    q_ref, d_ref = ref.quantize_weights(a8.smooth_weights(w, s))
    wq, sc = qb.quantize_weights_smoothed(f32_to_dev(w), f32_to_dev(s))
    assert np.array_equal(bf16_to_host(sc), d_ref)
    assert np.array_equal(qb.unpack_weights(wq, N, K).cpu().numpy(), q_ref)
    # no vector: the plain quantiser
    wq0, sc0 = qb.quantize_weights_smoothed(f32_to_dev(w), None)
    q0, d0 = ref.quantize_weights(w)
    assert np.array_equal(bf16_to_host(sc0), d0)
    assert np.array_equal(qb.unpack_weights(wq0, N, K).cpu().numpy(), q0)


# ------------------------------------------------------------------ linear
def linear_case(qb, M, N, K, seed, smoothed):
    w = synth.normal_weights(N, K, seed=synth.seed_for(6, 2, seed))
    xb = activations(M, K, synth.seed_for(6, 3, seed))
    s = smooth_vector(K, 500 + seed) if smoothed else None
    wt = a8.smooth_weights(w, s) if smoothed else w
    q_ref, d_ref = ref.quantize_weights(wt)
    s_dev = None if s is None else f32_to_dev(s)
    wq, sc = qb.quantize_weights_smoothed(f32_to_dev(w), s_dev)
    return xb, s, s_dev, q_ref, d_ref, wq, sc


@pytest.mark.parametrize("M,N,K,seed,smoothed", [
    (8, 1024, 1024, 1, False),       # small configuration
    (1, 16, 64, 2, False),           # smallest legal shape
    (5, 48, 192, 3, True),           # ragged everything: fewer steps than waves
    (8, 4096, 4096, 4, True),        # one tile per workgroup, several steps per wave
    (16, 4096 + 16 * 37, 1024, 5, False),   # uneven tiles per workgroup
    (8, 1024, 12288, 6, True),       # long K, one chunk in int8
    (32, 512, 8192, 7, False),       # K chunked in LDS
    (32, 256, 25600, 8, True),       # the longest K of the larger model, chunked
])
def test_w8a8_linear_bit_exact(qb, M, N, K, seed, smoothed):
    say("w8a8_linear", M, N, K, seed, smoothed)
    xb, s, s_dev, q_ref, d_ref, wq, sc = linear_case(qb, M, N, K, seed, smoothed)
    y_ref = a8.w8a8_linear(xb, q_ref, d_ref, s)
    y = qb.w8a8_linear(bf16_to_dev(xb), wq, sc, N, smooth=s_dev)
    got = bf16_to_host(y)
    assert got.shape == y_ref.shape
    bad = np.argwhere(got != y_ref)
    assert bad.size == 0, (bad[:5], got[tuple(bad[0])], y_ref[tuple(bad[0])])


def test_w8a8_linear_strided_and_repeatable(qb):
    say("w8a8_linear strided")
    M, N, K = 8, 256, 512
    xb, s, s_dev, q_ref, d_ref, wq, sc = linear_case(qb, M, N, K, 21, True)
    big = torch.zeros((M, K + 64), dtype=torch.bfloat16, device="cuda")
    big[:, :K] = bf16_to_dev(xb)
    ybig = torch.full((M, N + 32), 7.0, dtype=torch.bfloat16, device="cuda")
    qb.w8a8_linear(big[:, :K], wq, sc, N, smooth=s_dev, y=ybig[:, :N])
    y_ref = a8.w8a8_linear(xb, q_ref, d_ref, s)
    assert np.array_equal(bf16_to_host(ybig[:, :N]), y_ref)
    assert torch.all(ybig[:, N:] == 7.0)             # nothing written past N
    y2 = qb.w8a8_linear(big[:, :K], wq, sc, N, smooth=s_dev)
    assert np.array_equal(bf16_to_host(y2), y_ref)


def test_w8a8_integer_case_exact_sums(qb):
    """Activations that are their own codes (amax = 127, dx = 1) and unit weight steps:
    the output is the integer dot product itself, beyond 2^24 it rounds like int -> fp32."""
    say("w8a8 integer case")
    M, N, K = 4, 32, 2048
    r = np.random.Generator(np.random.Philox(31))
    x = r.integers(-127, 128, (M, K)).astype(np.float32)
    x[:, 0] = 127
    x[3] = 127                                          # all-127 token: |acc| up to 127*127*2048 > 2^24
    w = r.integers(-127, 128, (N, K)).astype(np.float32)
    w[:, 1] = 127
    w[5] = 127
    xb = synth.to_bf16_bits(x)
    q_ref, d_ref = ref.quantize_weights(w)              # dw = bf16(1) = 1
    assert np.all(ref.bf16_bits_to_f64(d_ref) == 1.0) and np.array_equal(q_ref, w.astype(np.int8))
    wq, sc = qb.quantize_weights(f32_to_dev(w))
    y = bf16_to_host(qb.w8a8_linear(bf16_to_dev(xb), wq, sc, N))
    acc = x.astype(np.int64) @ w.astype(np.int64).T
    want = ref.f32_to_bf16_bits(acc.astype(np.float32))
    assert np.array_equal(y, want)
    assert np.array_equal(y, a8.w8a8_linear(xb, q_ref, d_ref))


# ------------------------------------------------------------------ verification
@pytest.mark.parametrize("M,V,K,seed,smoothed", [(8, 4096, 1024, 1, False), (8, 16 * 1001, 512, 2, True),
                                                 (16, 8192, 4096, 3, True), (32, 2048, 8192, 4, False)])
def test_w8a8_verify_exact(qb, M, V, K, seed, smoothed):
    say("w8a8_lmhead_verify", M, V, K, seed, smoothed)
    xb, s, s_dev, q_ref, d_ref, wq, sc = linear_case(qb, M, V, K, 40 + seed, smoothed)
    want, _ = a8.w8a8_lmhead_verify(xb, q_ref, d_ref, [], s)
    ws = qb.make_workspace(M, V, K)
    for j in (0, M // 2, M - 1):
        draft = want[:M - 1].copy()
        if j < M - 1:
            draft[j] = (draft[j] + 1) % V
        am, acc = qb.w8a8_lmhead_verify(bf16_to_dev(xb), wq, sc, V, i32_to_dev(draft), ws, smooth=s_dev)
        assert np.array_equal(am.cpu().numpy(), want)
        assert int(acc.cpu()[0]) == j
        _, n_ref = a8.w8a8_lmhead_verify(xb, q_ref, d_ref, draft, s)
        assert n_ref == j


def test_w8a8_verify_ties_take_lowest_index(qb):
    say("w8a8 verify ties")
    M, V, K = 8, 4096, 256
    w = synth.normal_weights(V, K, seed=91)
    w[3000] = w[17]
    w[2000] = w[17]                                     # three identical rows
    xb = activations(M, K, 92)
    q_ref, d_ref = ref.quantize_weights(w)
    # make the triple the winner for every token: scale it up
    w[[17, 2000, 3000]] *= 0  # placeholder rows, rebuilt below
    x = ref.bf16_bits_to_f64(xb)
    w[17] = w[2000] = w[3000] = (x[0] / np.abs(x[0]).max() * 0.5).astype(np.float32)
    q_ref, d_ref = ref.quantize_weights(w)
    want, _ = a8.w8a8_lmhead_verify(xb, q_ref, d_ref, [])
    assert want[0] == 17
    wq, sc = qb.quantize_weights(f32_to_dev(w))
    ws = qb.make_workspace(M, V, K)
    am, _ = qb.w8a8_lmhead_verify(bf16_to_dev(xb), wq, sc, V, None, ws)
    assert np.array_equal(am.cpu().numpy(), want)


def test_w8a8_argument_errors(qb):
    say("w8a8 argument errors")
    x = torch.zeros((8, 128), dtype=torch.bfloat16, device="cuda")
    wq = torch.zeros(16 * 128, dtype=torch.int8, device="cuda")
    sc = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.w8a8_linear(x, wq, sc, 24)                     # N not a multiple of 16
    x33 = torch.zeros((33, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.w8a8_linear(x33, wq, sc, 16)                   # M > 32
    with pytest.raises(ValueError):
        qb.w8a8_linear(x, wq, sc, 16, smooth=torch.ones(64, device="cuda"))
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.w8a8_lmhead_verify(x, wq, sc, 16, None, small)  # workspace too small


# ------------------------------------------------------------------ whole step in one launch, W8A8 form
def _chain_case(qb, M, dims, seed, smoothed, with_head, V=2048):
    """A chain of linears (each reads its predecessor's output; the two middle ones share
    their input, as q|k or gate|up do), optionally closed by the vocabulary phase."""
    r = np.random.Generator(np.random.Philox(seed))
    xb0 = activations(M, dims[0], synth.seed_for(6, 7, seed))
    layers = []                                   # (K, N, q_ref, d_ref, wq, sc, smooth_host, smooth_dev, src)
    src = -1                                      # -1: the external input
    for i in range(len(dims) - 1):
        K, N = dims[i], dims[i + 1]
        for rep in range(2 if i == 1 else 1):     # second stage: two linears on the same input
            w = synth.normal_weights(N, K, seed=synth.seed_for(6, 8, 10 * seed + 2 * i + rep)) * np.float32(4.0)
            s = smooth_vector(K, 300 + seed + i) if smoothed else None
            wt = a8.smooth_weights(w, s) if smoothed else w
            q_ref, d_ref = ref.quantize_weights(wt)
            s_dev = None if s is None else f32_to_dev(s)
            wq, sc = qb.quantize_weights_smoothed(f32_to_dev(w), s_dev)
            layers.append([K, N, q_ref, d_ref, wq, sc, s, s_dev, src])
        src = len(layers) - 1                     # the next stage reads the last linear of this one
    head = None
    if with_head:
        K = dims[-1]
        w = synth.normal_weights(V, K, seed=synth.seed_for(6, 9, seed))
        s = smooth_vector(K, 400 + seed) if smoothed else None
        q_ref, d_ref = ref.quantize_weights(a8.smooth_weights(w, s) if smoothed else w)
        s_dev = None if s is None else f32_to_dev(s)
        wq, sc = qb.quantize_weights_smoothed(f32_to_dev(w), s_dev)
        head = (V, q_ref, d_ref, wq, sc, s, s_dev)
    return xb0, layers, head


@pytest.mark.parametrize("M,dims,seed,smoothed,with_head", [
    (8, (1024, 1024, 512, 1024), 1, False, False),
    (8, (4096, 4096, 1024, 4096), 2, True, True),
    (5, (192, 256, 64, 128), 3, True, True),          # fewer steps than waves, ragged M
    (16, (2048, 12288, 1024, 2048), 4, False, True),  # long K in the third stage
    (32, (8192, 512, 8192, 256), 5, True, False),     # K chunked in LDS
])
def test_w8a8_sequence_bit_exact(qb, M, dims, seed, smoothed, with_head):
    say("w8a8 sequence", M, dims, seed, smoothed, with_head)
    xb0, layers, head = _chain_case(qb, M, dims, seed, smoothed, with_head)
    # oracle chain
    outs_ref = []
    for K, N, q_ref, d_ref, wq, sc, s, s_dev, src in layers:
        xin = xb0 if src < 0 else outs_ref[src]
        outs_ref.append(a8.w8a8_linear(xin, q_ref, d_ref, s))
    # device chain in one launch; every buffer written once
    x0 = bf16_to_dev(xb0)
    ys = [torch.empty((M, L[1]), dtype=torch.bfloat16, device="cuda") for L in layers]
    lin = [(x0 if L[8] < 0 else ys[L[8]], L[4], L[5], L[1], ys[i]) for i, L in enumerate(layers)]
    verify = None
    draft = None
    if head is not None:
        V, q_ref, d_ref, wq, sc, s, s_dev = head
        want, _ = a8.w8a8_lmhead_verify(outs_ref[-1], q_ref, d_ref, [], s)
        draft = want[:M - 1].copy()
        j = (M - 1) // 2
        draft[j] = (draft[j] + 1) % V
        oa = torch.empty(M, dtype=torch.int32, device="cuda")
        oc = torch.empty(1, dtype=torch.int32, device="cuda")
        verify = (ys[-1], wq, sc, V, i32_to_dev(draft), oa, oc)
    seq = qb.Sequence(lin, verify=verify, w8a8=True, smooth=[L[7] for L in layers] if smoothed else None,
                      verify_smooth=head[6] if head is not None else None)
    assert seq.n_barriers == 0
    for _ in range(2):                             # the second run reuses flags of a new epoch
        for y in ys:
            y.fill_(float("nan"))
        seq.run()
        torch.cuda.synchronize()
        assert not seq.timed_out()
        for i, y in enumerate(ys):
            assert np.array_equal(bf16_to_host(y), outs_ref[i]), i
        if head is not None:
            assert np.array_equal(oa.cpu().numpy(), want)
            assert int(oc.cpu()[0]) == j
    # the same bits as the single calls
    for i, L in enumerate(layers):
        xin = x0 if L[8] < 0 else ys[L[8]]
        y1 = qb.w8a8_linear(xin, L[4], L[5], L[1], smooth=L[7])
        assert torch.equal(y1.view(torch.int16), ys[i].view(torch.int16))


def test_w8a8_sequence_argument_errors(qb):
    say("w8a8 sequence argument errors")
    x = torch.zeros((8, 128), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    wq = torch.zeros(64 * 128, dtype=torch.int8, device="cuda")
    sc = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):
        qb.Sequence([(x, wq, sc, 64, y)], w8a8=True, smooth=[None, None])
    with pytest.raises(ValueError):
        qb.Sequence([(x, wq, sc, 64, y)], smooth=[None])
    wp = torch.zeros(64 * 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.Sequence([(x, wp, None, 64, y)], w8a8=True)      # bf16 weights have no W8A8 form
