"""GPU parity for the int8 linears with the block operations fused in (RMSNorm while the
activations are staged, residual or the SwiGLU product in the epilogue) through the C-ABI against
the CPU oracle.
The device takes the normalisation and the sigmoid in fp32, the oracle in fp64, so single bf16
values of the staged activations may differ by one unit in the last place; the outputs are held
to the bar of the plain linear (max|y_gpu - y_ref| <= 1e-2 max|y_ref|) and to 6e-3 in practice
(the residual form adds one more bf16 rounding of the output)."""
import numpy as np
import pytest
import torch

from oracle import quasar_layer_ref as lr
from oracle import quasar_ref as ref
from paper_2603_01399_amd import synth
from gpu_util import bf16_to_dev, bf16_to_host, f32_to_dev

pytestmark = pytest.mark.gpu
TOL = 1e-2
TOL_EXPECTED = 6e-3


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_01399_amd import binding
    return binding


def say(*a):
    print(*a, flush=True)


def case(qb, M, N, K, seed):
    xb = synth.activations_bf16(M, K, seed=synth.seed_for(10, 0, seed))
    rb = synth.activations_bf16(M, N, seed=synth.seed_for(10, 2, seed))
    r = np.random.Generator(np.random.Philox(synth.seed_for(10, 3, seed)))
    gb = synth.to_bf16_bits((1.0 + 0.2 * r.standard_normal(K)).astype(np.float32))
    w = synth.normal_weights(N, K, seed=synth.seed_for(10, 4, seed))
    q, s = ref.quantize_weights(w)
    wq, sc = qb.quantize_weights(f32_to_dev(w))
    return xb, rb, gb, q, s, wq, sc


def err(y_dev, want_bits):
    return ref.rel_maxabs_err(ref.bf16_bits_to_f64(bf16_to_host(y_dev)), ref.bf16_bits_to_f64(want_bits))


SHAPES = [(8, 1024, 1024), (1, 256, 512), (5, 16 * 37, 64 * 9), (8, 4096, 4096), (16, 4096, 4096), (8, 4096, 12288),
          (32, 1024, 4096), (27, 16 * 300, 64 * 21), (8, 12288, 4096)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_fused_linear_all_forms(qb, M, N, K):
    say("fused linear", M, N, K)
    xb, rb, gb, q, s, wq, sc = case(qb, M, N, K, M + N % 97 + K % 89)
    x, res, gamma = bf16_to_dev(xb), bf16_to_dev(rb), bf16_to_dev(gb)
    # no normalisation, no residual: the plain linear's bits
    plain = qb.w8_linear_fused(x, wq, sc, N)
    assert np.array_equal(bf16_to_host(plain), bf16_to_host(qb.w8_linear(x, wq, sc, N)))
    forms = {
        "rmsnorm": (dict(gamma=gamma, eps=1e-6), dict(gamma_bits=gb, eps=1e-6)),
        "residual": (dict(residual=res), dict(residual_bits=rb)),
        "rmsnorm+residual": (dict(gamma=gamma, eps=1e-5, residual=res), dict(gamma_bits=gb, eps=1e-5, residual_bits=rb)),
    }
    for name, (dev_kw, ref_kw) in forms.items():
        y = qb.w8_linear_fused(x, wq, sc, N, **dev_kw)
        torch.cuda.synchronize()
        e = err(y, lr.fused_linear(xb, q, s, **ref_kw))
        say("   ", name, "rel err", e)
        assert e <= TOL and e <= TOL_EXPECTED, name


GATEUP = [(8, 512, 1024), (1, 16, 64), (5, 16 * 37, 64 * 9), (8, 12288, 4096), (16, 4096, 4096), (32, 1024, 2048),
          (27, 16 * 301, 64 * 21), (8, 2048, 12288)]


@pytest.mark.parametrize("M,I,K", GATEUP)
def test_gateup_swiglu(qb, M, I, K):
    say("gate/up swiglu", M, I, K)
    xb = synth.activations_bf16(M, K, seed=synth.seed_for(11, 0, M + I % 97))
    r = np.random.Generator(np.random.Philox(synth.seed_for(11, 1, M + I % 97)))
    gb = synth.to_bf16_bits((1.0 + 0.2 * r.standard_normal(K)).astype(np.float32))
    # weights large enough for gate values of a few units, where silu is far from linear
    wg = synth.normal_weights(I, K, seed=synth.seed_for(11, 2, M + I % 97)) * np.float32(2.0)
    wu = synth.normal_weights(I, K, seed=synth.seed_for(11, 3, M + I % 97))
    qg, sg = ref.quantize_weights(wg)
    qu, su = ref.quantize_weights(wu)
    inter = qb.interleave_gate_up(f32_to_dev(wg), f32_to_dev(wu))
    wq, sc = qb.quantize_weights(inter)
    # the interleaved matrix quantises to the interleaved codes (per-row step sizes)
    q_all = qb.unpack_weights(wq, 2 * I, K).cpu().numpy().reshape(I // 16, 2, 16, K)
    assert np.array_equal(q_all[:, 0].reshape(I, K), qg) and np.array_equal(q_all[:, 1].reshape(I, K), qu)
    x = bf16_to_dev(xb)
    for name, dev_kw, ref_kw in (("plain", {}, {}), ("rmsnorm", dict(gamma=bf16_to_dev(gb), eps=1e-6), dict(gamma_bits=gb, eps=1e-6))):
        y = qb.w8_gateup_swiglu(x, wq, sc, I, **dev_kw)
        torch.cuda.synchronize()
        want = lr.gateup_swiglu(xb, qg, sg, qu, su, **ref_kw)
        e = err(y, want)
        say("   ", name, "rel err", e)
        # two more bf16 roundings than a plain linear (silu output, product)
        assert e <= TOL, name
    again = qb.w8_gateup_swiglu(x, wq, sc, I, gamma=bf16_to_dev(gb), eps=1e-6)
    assert np.array_equal(bf16_to_host(again), bf16_to_host(y))             # same bits run to run


def test_fused_linear_in_place_residual_strides_and_repeatability(qb):
    say("fused linear in place")
    M, N, K = 8, 1024, 2048
    xb, rb, gb, q, s, wq, sc = case(qb, M, N, K, 7)
    big_x = bf16_to_dev(np.concatenate([xb, xb[:, :64]], axis=1))          # row stride K + 64
    hidden = torch.zeros((M, N + 32), dtype=torch.bfloat16, device="cuda")
    hidden[:, :N] = bf16_to_dev(rb)
    view = hidden[:, :N]
    qb.w8_linear_fused(big_x[:, :K], wq, sc, N, gamma=bf16_to_dev(gb), residual=view, y=view)   # hidden += W(norm(x))
    torch.cuda.synchronize()
    got = bf16_to_host(hidden)
    assert not got[:, N:].any()
    want = lr.fused_linear(xb, q, s, gamma_bits=gb, residual_bits=rb)
    assert ref.rel_maxabs_err(ref.bf16_bits_to_f64(got[:, :N]), ref.bf16_bits_to_f64(want)) <= TOL_EXPECTED
    again = qb.w8_linear_fused(bf16_to_dev(xb), wq, sc, N, gamma=bf16_to_dev(gb), residual=bf16_to_dev(rb))
    assert np.array_equal(bf16_to_host(again), got[:, :N])                 # same bits for any stride, run to run
    # gate/up output into a strided buffer
    I = 512
    wq2, sc2 = qb.quantize_weights(f32_to_dev(synth.normal_weights(2 * I, K, seed=5)))
    buf = torch.zeros((M, I + 8), dtype=torch.bfloat16, device="cuda")
    qb.w8_gateup_swiglu(bf16_to_dev(xb), wq2, sc2, I, y=buf[:, :I])
    dense = qb.w8_gateup_swiglu(bf16_to_dev(xb), wq2, sc2, I)
    out = bf16_to_host(buf)
    assert not out[:, I:].any() and np.array_equal(out[:, :I], bf16_to_host(dense))


def test_rmsnorm_scale_and_large_activations(qb):
    """Rows of very different magnitude (the normalisation must be per token), a row of zeros
    (eps keeps it finite) and a padded M."""
    say("fused linear rmsnorm rows")
    M, N, K = 6, 512, 1024
    xb, rb, gb, q, s, wq, sc = case(qb, M, N, K, 11)
    x = ref.bf16_bits_to_f64(xb)
    x[0] *= 512.0
    x[1] *= 2.0 ** -9
    x[2] = 0.0
    x[3, 17] = 3000.0
    xb = synth.to_bf16_bits(x.astype(np.float32))
    y = qb.w8_linear_fused(bf16_to_dev(xb), wq, sc, N, gamma=bf16_to_dev(gb), eps=1e-6)
    want = lr.fused_linear(xb, q, s, gamma_bits=gb, eps=1e-6)
    got = ref.bf16_bits_to_f64(bf16_to_host(y))
    assert np.isfinite(got).all() and not got[2].any()
    for m in range(M):
        assert ref.rel_maxabs_err(got[m], ref.bf16_bits_to_f64(want[m])) <= TOL_EXPECTED, m


def test_fused_argument_errors(qb):
    say("fused linear argument errors")
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    wq = torch.zeros(64 * 128, dtype=torch.int8, device="cuda")
    sc = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    g = torch.ones(128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.w8_linear_fused(x, wq, sc, 64, gamma=g, eps=-1.0)
    with pytest.raises(qb.QuasarError):
        qb.w8_linear_fused(x, wq, sc, 64, gamma=torch.ones(129, dtype=torch.bfloat16, device="cuda")[1:])   # misaligned gamma
    with pytest.raises(ValueError):
        qb.w8_linear_fused(x, wq, sc, 64, residual=torch.zeros((4, 32), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(qb.QuasarError):
        qb.w8_gateup_swiglu(x, wq, sc, 24)                                   # I not a multiple of 16
    with pytest.raises(qb.QuasarError):
        qb.w8_gateup_swiglu(x, wq, sc, 32, y=torch.zeros((4, 34), dtype=torch.bfloat16, device="cuda")[:, :32])   # ldy % 4


def test_whole_decoder_block_against_composed_oracle(qb):
    """One decoder block of a small Qwen3-shaped model as the library runs it (six launches):
    RMSNorm -> q/k/v, per-head norm + rotary + cache append, attention over prompt + new positions,
    o_proj + residual, RMSNorm -> gate/up -> SwiGLU, down_proj + residual - against the same chain
    composed from the oracles.  The tolerance is the linear bar: one bf16 unit in the last place of
    an intermediate moves the result by far less."""
    from oracle import quasar_attention_ref as at
    say("whole block")
    M, H, Hq, Hkv, I, L, theta, eps = 8, 1024, 8, 2, 2048, 300, 1.0e6, 1e-6
    D = 128
    r = np.random.Generator(np.random.Philox(91))
    def w_(n, k, seed):
        return synth.normal_weights(n, k, seed=synth.seed_for(12, 0, seed))
    def g_(n):
        return synth.to_bf16_bits((1.0 + 0.1 * r.standard_normal(n)).astype(np.float32))
    w_qkv, w_o, w_g, w_u, w_d = w_((Hq + 2 * Hkv) * D, H, 1), w_(H, Hq * D, 2), w_(I, H, 3) * np.float32(2), w_(I, H, 4), w_(H, I, 5)
    g1, g2, gq, gk = g_(H), g_(H), g_(D), g_(D)
    hid = synth.to_bf16_bits((r.standard_normal((M, H)) * 2).astype(np.float32))
    kp = synth.to_bf16_bits(r.standard_normal((L, Hkv, D)).astype(np.float32))
    vp = synth.to_bf16_bits(r.standard_normal((L, Hkv, D)).astype(np.float32))

    # ---- oracle chain
    q_qkv, s_qkv = ref.quantize_weights(w_qkv)
    q_o, s_o = ref.quantize_weights(w_o)
    q_g, s_g = ref.quantize_weights(w_g)
    q_u, s_u = ref.quantize_weights(w_u)
    q_d, s_d = ref.quantize_weights(w_d)
    qkv = lr.fused_linear(hid, q_qkv, s_qkv, gamma_bits=g1, eps=eps).reshape(M, Hq + 2 * Hkv, D)
    pos = np.arange(L, L + M)
    qh = at.head_norm_rope(qkv[:, :Hq], gq, eps, pos, theta)
    kh = at.head_norm_rope(qkv[:, Hq:Hq + Hkv], gk, eps, pos, theta)
    att = at.verify_attention(qh, np.concatenate([kp, kh]), np.concatenate([vp, qkv[:, Hq + Hkv:]])).reshape(M, Hq * D)
    h1 = lr.fused_linear(att, q_o, s_o, residual_bits=hid)
    act = lr.gateup_swiglu(h1, q_g, s_g, q_u, s_u, gamma_bits=g2, eps=eps)
    want = lr.fused_linear(act, q_d, s_d, residual_bits=h1)

    # ---- the library
    wq_qkv, sc_qkv = qb.quantize_weights(f32_to_dev(w_qkv))
    wq_o, sc_o = qb.quantize_weights(f32_to_dev(w_o))
    wq_gu, sc_gu = qb.quantize_weights(qb.interleave_gate_up(f32_to_dev(w_g), f32_to_dev(w_u)))
    wq_d, sc_d = qb.quantize_weights(f32_to_dev(w_d))
    cache = qb.KvCache(Hkv, L + M)
    cache.buf.fill_(0xFF)
    cache.fill(bf16_to_dev(kp), bf16_to_dev(vp), 0)
    h = bf16_to_dev(hid).clone()
    qkv_d = qb.w8_linear_fused(h, wq_qkv, sc_qkv, (Hq + 2 * Hkv) * D, gamma=bf16_to_dev(g1), eps=eps)
    q_d_ = qb.attn_prepare(qkv_d, Hq, cache, L, bf16_to_dev(gq), bf16_to_dev(gk), eps=eps, rope_theta=theta)
    att_d = qb.verify_attention(q_d_, Hq, cache, L + M)
    qb.w8_linear_fused(att_d, wq_o, sc_o, H, residual=h, y=h)
    act_d = qb.w8_gateup_swiglu(h, wq_gu, sc_gu, I, gamma=bf16_to_dev(g2), eps=eps)
    qb.w8_linear_fused(act_d, wq_d, sc_d, H, residual=h, y=h)
    torch.cuda.synchronize()
    e = err(h, want)
    say("   block rel err", e)
    assert e <= TOL
