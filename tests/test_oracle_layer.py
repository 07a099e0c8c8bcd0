"""Pins for the oracle of the block operations around the linears: closed forms, identities that
fix signs and operand roles, independent formulas (vector norm, tanh form of the sigmoid), and the
composition with the pinned int8 linear.  No GPU."""
import numpy as np
import pytest

from oracle import quasar_layer_ref as lr
from oracle import quasar_ref as ref


def bits(a):
    return ref.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def vals(b):
    return ref.bf16_bits_to_f64(b)


def test_rmsnorm_closed_forms():
    # constant rows: x * r = c / sqrt(c^2 + eps); with eps = 0 exactly +-1 times gamma
    K = 64
    g = bits(np.linspace(0.5, 2.0, K))
    x = bits(np.stack([np.full(K, 3.0), np.full(K, -0.25)]))
    out = vals(lr.rmsnorm(x, g, 0.0))
    assert np.array_equal(out[0], vals(g)) and np.array_equal(out[1], -vals(g))
    # eps matters: c = 1, eps = 3 -> r = 1/2
    out = vals(lr.rmsnorm(bits(np.ones((1, K))), bits(np.ones(K)), 3.0))
    assert np.array_equal(out, np.full((1, K), 0.5))
    # one nonzero entry a among K: mean square a^2/K, so x*r = sign(a) sqrt(K) there, 0 elsewhere
    x = np.zeros((1, 16))
    x[0, 5] = -7.0
    out = vals(lr.rmsnorm(bits(x), bits(np.ones(16)), 0.0))
    assert out[0, 5] == -4.0 and np.count_nonzero(out) == 1
    with pytest.raises(ValueError):
        lr.rmsnorm(bits(x), bits(np.ones(15)), 0.0)


def test_rmsnorm_against_vector_norm_and_invariances():
    r = np.random.Generator(np.random.Philox(61))
    M, K = 5, 256
    xb = bits(r.standard_normal((M, K)) * 3)
    gb = bits(1.0 + 0.1 * r.standard_normal(K))
    x = vals(xb)
    want_inner = x / np.linalg.norm(x, axis=1, keepdims=True) * np.sqrt(K)          # eps = 0
    got = vals(lr.rmsnorm(xb, gb, 0.0))
    # two bf16 roundings, each at most half an ulp = 2^-8 relative
    assert np.all(np.abs(got - want_inner * vals(gb)) <= np.abs(want_inner * vals(gb)) * (2.0 ** -7 + 1e-4))
    # with gamma = 1 the output has unit mean square up to rounding
    one = vals(lr.rmsnorm(xb, bits(np.ones(K)), 0.0))
    assert np.allclose(np.mean(one * one, axis=1), 1.0, atol=2e-3)
    # power-of-two rescaling of x changes nothing when eps = 0; gamma acts per column
    assert np.array_equal(lr.rmsnorm(bits(x * 8.0), gb, 0.0), lr.rmsnorm(xb, gb, 0.0))
    g2 = vals(gb).copy()
    g2[7] *= 2.0
    out2 = vals(lr.rmsnorm(xb, bits(g2), 0.0))
    assert np.array_equal(out2[:, 7], 2.0 * got[:, 7]) and np.array_equal(np.delete(out2, 7, 1), np.delete(got, 7, 1))
    # a larger eps shrinks every entry
    assert np.all(np.abs(vals(lr.rmsnorm(xb, gb, 0.5))) <= np.abs(got))


def test_silu_identities():
    g = np.linspace(-12, 12, 481)
    s = lr.silu(g)
    assert s[240] == 0.0                                             # silu(0) = 0
    assert np.allclose(s - lr.silu(-g), g, rtol=0, atol=1e-12)       # silu(x) - silu(-x) = x
    assert np.allclose(s, g * (1.0 + np.tanh(g / 2.0)) / 2.0, rtol=0, atol=1e-12)
    assert abs(lr.silu(np.array([30.0]))[0] - 30.0) < 1e-10 and abs(lr.silu(np.array([-30.0]))[0]) < 1e-10
    assert abs(lr.silu(np.array([1.0]))[0] - 1.0 / (1.0 + np.exp(-1.0))) < 1e-15
    assert lr.silu(g).min() > -0.2785                                # global minimum of silu is about -0.27846


def test_swiglu_operand_roles_and_roundings():
    gate = bits([[0.0, 2.0, -2.0, 1.0]])
    up = bits([[5.0, 1.0, 1.0, -3.0]])
    out = vals(lr.swiglu(gate, up))
    s2 = vals(bits([2.0 / (1.0 + np.exp(-2.0))]))[0]                 # bf16(silu(2))
    sm2 = vals(bits([-2.0 / (1.0 + np.exp(2.0))]))[0]
    s1 = vals(bits([1.0 / (1.0 + np.exp(-1.0))]))[0]
    assert out[0, 0] == 0.0 and out[0, 1] == s2 and out[0, 2] == sm2
    assert out[0, 3] == vals(bits([s1 * -3.0]))[0]
    # swapping the operands is a different function (the gate goes through silu, up does not)
    assert not np.array_equal(lr.swiglu(up, gate), lr.swiglu(gate, up))
    with pytest.raises(ValueError):
        lr.swiglu(gate, up[:, :3])


def test_fused_linear_and_gateup_are_the_compositions():
    r = np.random.Generator(np.random.Philox(62))
    M, N, K = 4, 32, 128
    w = (r.standard_normal((N, K)) * 0.02).astype(np.float32)
    q, s = ref.quantize_weights(w)
    w2 = (r.standard_normal((N, K)) * 0.02).astype(np.float32)
    q2, s2 = ref.quantize_weights(w2)
    xb = bits(r.standard_normal((M, K)))
    gb = bits(1.0 + 0.1 * r.standard_normal(K))
    rb = bits(r.standard_normal((M, N)))
    plain = lr.fused_linear(xb, q, s)
    assert np.array_equal(plain, ref.f64_to_bf16_bits(ref.w8_linear(xb, q, s)))
    assert np.array_equal(lr.fused_linear(xb, q, s, gamma_bits=gb, eps=1e-6),
                          ref.f64_to_bf16_bits(ref.w8_linear(lr.rmsnorm(xb, gb, 1e-6), q, s)))
    # residual: added after the linear's own rounding; zero weights give the residual back
    res = lr.fused_linear(xb, q, s, residual_bits=rb)
    assert np.array_equal(res, bits(vals(plain) + vals(rb)))
    assert np.array_equal(lr.fused_linear(xb, np.zeros_like(q), s, residual_bits=rb), rb)
    assert np.array_equal(lr.fused_linear(xb, q, s, residual_bits=bits(np.zeros((M, N)))), plain)
    # gate/up: the gate goes through silu, the up projection does not
    a = lr.gateup_swiglu(xb, q, s, q2, s2)
    assert np.array_equal(a, lr.swiglu(plain, lr.fused_linear(xb, q2, s2)))
    assert not np.array_equal(a, lr.gateup_swiglu(xb, q2, s2, q, s))
    an = lr.gateup_swiglu(xb, q, s, q2, s2, gamma_bits=gb, eps=1e-6)
    assert np.array_equal(an, lr.swiglu(lr.fused_linear(xb, q, s, gamma_bits=gb), lr.fused_linear(xb, q2, s2, gamma_bits=gb)))
    # zero up weights give zeros; a zero gate gives zeros as well (silu(0) = 0)
    assert not lr.gateup_swiglu(xb, q, s, np.zeros_like(q2), s2).any()
    assert not lr.gateup_swiglu(xb, np.zeros_like(q), s, q2, s2).any()
