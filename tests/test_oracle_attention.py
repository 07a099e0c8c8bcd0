"""Pins for the attention oracle: the rotary embedding against complex multiplication, its
norm and relative-position properties, per-head normalisation closed forms, and attention
special cases (one visible key, equal keys, a dominant key, causality, head grouping).  No GPU."""
import numpy as np
import pytest

from oracle import quasar_attention_ref as at
from oracle import quasar_ref as ref


def bits(a):
    return ref.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def vals(b):
    return ref.bf16_bits_to_f64(b)


def test_rope_is_complex_rotation_and_identity_at_zero():
    r = np.random.Generator(np.random.Philox(71))
    M, H, d, theta = 3, 2, 16, 10000.0
    x = bits(r.standard_normal((M, H, d)))
    ones = bits(np.ones(d))
    # eps = 0 and gamma = 1: n = x / rms(x), rounded twice; position 0 leaves it unchanged
    n0 = vals(at.head_norm_rope(x, ones, 0.0, np.zeros(M), theta))
    xv = vals(x)
    rms = np.sqrt(np.mean(xv * xv, axis=2, keepdims=True))
    assert np.all(np.abs(n0 - xv / rms) <= np.abs(xv / rms) * 2.0 ** -7 + 1e-12)
    # positions p: pairs (i, i + d/2) rotate like complex numbers by p * theta^(-2i/d)
    pos = np.array([1.0, 5.0, 117.0])
    out = vals(at.head_norm_rope(x, ones, 0.0, pos, theta))
    z = (n0[:, :, :d // 2] + 1j * n0[:, :, d // 2:]) * np.exp(1j * pos[:, None, None] * theta ** (-2.0 * np.arange(d // 2) / d))
    want = np.concatenate([z.real, z.imag], axis=2)
    assert np.all(np.abs(out - want) <= np.abs(want) * 2.0 ** -8 + 1e-12)
    # the first frequency is 1 rad per position, the last theta^(-(d-2)/d)
    a = at.rope_angles([2.0], d, theta)
    assert a[0, 0] == 2.0 and abs(a[0, -1] - 2.0 * theta ** (-(d - 2) / d)) < 1e-15


def test_rope_preserves_norm_and_relative_position():
    r = np.random.Generator(np.random.Philox(72))
    d, theta = 32, 1.0e6
    q = bits(r.standard_normal((1, 1, d)))
    k = bits(r.standard_normal((1, 1, d)))
    ones = bits(np.ones(d))
    def rq(p):
        return vals(at.head_norm_rope(q, ones, 0.0, [p], theta))[0, 0]
    def rk(p):
        return vals(at.head_norm_rope(k, ones, 0.0, [p], theta))[0, 0]
    assert abs(np.linalg.norm(rq(0)) - np.linalg.norm(rq(300))) < 0.02 * np.linalg.norm(rq(0))
    # q(p1).k(p2) depends on p1 - p2 only (up to the bf16 rounding of the rotated vectors)
    base = rq(10) @ rk(3)
    for shift in (1, 50, 1000):
        assert abs(rq(10 + shift) @ rk(3 + shift) - base) < 0.03 * np.linalg.norm(rq(0)) * np.linalg.norm(rk(0))
    assert abs(rq(10) @ rk(3) - rq(10) @ rk(9)) > 1e-3          # and it does depend on the difference


def test_head_norm_closed_forms():
    d = 8
    x = np.zeros((1, 2, d))
    x[0, 0, 3] = -5.0                       # one non-zero entry: x * r = -sqrt(d) there
    x[0, 1, :] = 2.0                        # constant head: x * r = 1 everywhere
    g = np.linspace(0.5, 1.375, d)
    out = vals(at.head_norm_rope(bits(x), bits(g), 0.0, [0.0], 10000.0))
    assert out[0, 0, 3] == vals(bits(-vals(bits(np.sqrt(d))) * g[3])) and np.count_nonzero(out[0, 0]) == 1
    assert np.array_equal(out[0, 1], vals(bits(g)))
    # heads are normalised separately: scaling one head by 64 changes nothing (eps = 0)
    x2 = x.copy()
    x2[0, 1] *= 64.0
    assert np.array_equal(at.head_norm_rope(bits(x2), bits(g), 0.0, [0.0], 10000.0), at.head_norm_rope(bits(x), bits(g), 0.0, [0.0], 10000.0))


def test_attention_special_cases():
    r = np.random.Generator(np.random.Philox(73))
    d, Hq, Hkv = 16, 4, 2
    # one cached position, one query: the output is that value row (head h reads kv head h // 2)
    q = bits(r.standard_normal((1, Hq, d)))
    k = bits(r.standard_normal((1, Hkv, d)))
    v = bits(r.standard_normal((1, Hkv, d)))
    out = at.verify_attention(q, k, v)
    for h in range(Hq):
        assert np.array_equal(out[0, h], v[0, h // 2])
    # equal keys: uniform weights, the mean of the visible values
    L = 7
    k = bits(np.tile(r.standard_normal((1, Hkv, d)), (L, 1, 1)))
    v = bits(r.standard_normal((L, Hkv, d)))
    out = vals(at.verify_attention(q, k, v))
    assert np.all(np.abs(out[0, 3] - vals(v)[:, 1].mean(axis=0)) <= 2.0 ** -8 * np.abs(vals(v)[:, 1].mean(axis=0)) + 1e-9)
    # a dominant key: its value row
    k = np.zeros((L, Hkv, d))
    k[4, 0, :] = vals(q)[0, 0] * 40.0
    out = at.verify_attention(q, bits(k), v)
    assert np.array_equal(out[0, 0], v[4, 0])
    with pytest.raises(ValueError):
        at.verify_attention(q, bits(k), v[:, :1])


def test_attention_is_causal_over_the_new_positions():
    r = np.random.Generator(np.random.Philox(74))
    d, Hq, Hkv, M, L = 16, 2, 1, 4, 9
    q = bits(r.standard_normal((M, Hq, d)))
    k = r.standard_normal((L, Hkv, d))
    v = r.standard_normal((L, Hkv, d))
    base = at.verify_attention(q, bits(k), bits(v))
    # changing the key/value of the last position only changes the last query
    k2, v2 = k.copy(), v.copy()
    k2[-1] += 3.0
    v2[-1] -= 2.0
    out = at.verify_attention(q, bits(k2), bits(v2))
    assert np.array_equal(out[:M - 1], base[:M - 1]) and not np.array_equal(out[M - 1], base[M - 1])
    # query m alone over its visible prefix gives the same row
    for m in range(M):
        n_vis = L - M + m + 1
        one = at.verify_attention(q[m:m + 1], bits(k[:n_vis]), bits(v[:n_vis]))
        assert np.array_equal(one[0], base[m])
    # scaling every query by a positive power of two sharpens the weights but a single visible key
    # still returns its value row
    assert np.array_equal(at.verify_attention(bits(vals(q[:1]) * 8.0), bits(k[:1]), bits(v[:1]))[0, 0], bits(v[:1])[0, 0])


def test_attention_two_keys_closed_form_pins_the_score_scale():
    """Softmax over two scores is the logistic function: with q = a e0, k1 = b e0, k2 = 0 the weights are
    sigma(a b / sqrt(d)) and its complement.  The bit patterns in tests/golden/attention_two_keys.txt were
    worked by hand; a score scaled by 1/d (or not at all) gives other bits."""
    import os
    fx = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "attention_two_keys.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                fx[k] = v
    d, a, b = int(fx["d"]), float(fx["a"]), float(fx["b"])
    q = np.zeros((1, 1, d)); q[0, 0, 0] = a
    k = np.zeros((2, 1, d)); k[0, 0, 0] = b
    v = np.zeros((2, 1, d)); v[0, 0, 0] = 1.0; v[1, 0, 1] = 1.0
    out = at.verify_attention(bits(q), bits(k), bits(v))
    assert int(out[0, 0, 0]) == int(fx["w1_bf16"], 16)
    assert int(out[0, 0, 1]) == int(fx["w2_bf16"], 16)
    assert not out[0, 0, 2:].any()
    # the same through grouped heads and a longer prefix of zero keys: n zero keys share what w1 leaves
    n0 = 3
    k2 = np.zeros((1 + n0, 2, d)); k2[0, :, 0] = b
    v2 = np.zeros((1 + n0, 2, d)); v2[0, :, 0] = 1.0
    q2 = np.zeros((1, 4, d)); q2[0, :, 0] = a
    out2 = vals(at.verify_attention(bits(q2), bits(k2), bits(v2)))
    w = np.exp(2.0) / (np.exp(2.0) + n0)
    assert np.all(np.abs(out2[0, :, 0] - w) <= w * 2.0 ** -8)
    # and the value the wrong scale would give is far from what the oracle returns
    assert abs(vals(out)[0, 0, 0] - float(fx["w1_if_scaled_by_d"])) > 0.2
