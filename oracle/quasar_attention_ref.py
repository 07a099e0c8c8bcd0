"""CPU oracle for the attention of a verification step (TEST INFRASTRUCTURE ONLY).

Plain numpy, fp64 inside.  Nothing in the product path imports this file and this file imports
nothing from the product path.

The paper verifies gamma + 1 positions in one forward pass of the target model (Sec. 3.1); the
attention of that pass is the target model's own (grouped-query attention with a key/value cache,
per-head RMSNorm of queries and keys, rotary position embedding, as in the Qwen3 models the paper
evaluates).  Written out here:

* ``head_norm_rope``  per head: n = bf16( gamma * bf16( x * rsqrt(mean x^2 + eps) ) ), then the rotary
                      embedding at the token's position in the rotate-half convention:
                      out[i] = n[i] cos(a_i) - n[i + d/2] sin(a_i),  out[i + d/2] = n[i + d/2] cos(a_i) + n[i] sin(a_i),
                      a_i = position * theta^(-2 i / d), rounded to bf16 once.
* ``verify_attention``  query m (the m-th of the M new positions, the last M of the L_total cached ones) sees
                      positions 0 .. L_total - M + m; scores q.k / sqrt(d); softmax; weighted sum of the values;
                      query head h reads key/value head h // (Hq / Hkv); output rounded to bf16 once.

bf16 values travel as uint16 bit patterns.
"""
from __future__ import annotations

import numpy as np

from . import quasar_ref as ref
from .quasar_layer_ref import _round_bf16


def rope_angles(positions, d: int, theta: float) -> np.ndarray:
    """angles[m, i] = positions[m] * theta^(-2 i / d), i < d / 2."""
    inv = float(theta) ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)
    return np.asarray(positions, dtype=np.float64)[:, None] * inv[None, :]


def head_norm_rope(x_bits, gamma_bits, eps: float, positions, theta: float) -> np.ndarray:
    """x_bits [M, H, d] -> uint16 bf16 bits [M, H, d]."""
    x = ref.bf16_bits_to_f64(x_bits)
    M, H, d = x.shape
    g = ref.bf16_bits_to_f64(gamma_bits).reshape(d)
    r = 1.0 / np.sqrt(np.mean(x * x, axis=2, keepdims=True) + eps)
    n = ref.bf16_bits_to_f64(_round_bf16(ref.bf16_bits_to_f64(_round_bf16(x * r)) * g[None, None, :]))
    a = rope_angles(positions, d, theta)[:, None, :]              # [M, 1, d/2]
    n1, n2 = n[:, :, :d // 2], n[:, :, d // 2:]
    out = np.concatenate([n1 * np.cos(a) - n2 * np.sin(a), n2 * np.cos(a) + n1 * np.sin(a)], axis=2)
    return _round_bf16(out)


def verify_attention(q_bits, k_bits, v_bits) -> np.ndarray:
    """q_bits [M, Hq, d]; k_bits, v_bits [L_total, Hkv, d] (the M new positions are the last M).
    -> uint16 bf16 bits [M, Hq, d]."""
    q = ref.bf16_bits_to_f64(q_bits)
    k = ref.bf16_bits_to_f64(k_bits)
    v = ref.bf16_bits_to_f64(v_bits)
    M, Hq, d = q.shape
    Lt, Hkv, _ = k.shape
    if Hq % Hkv or M > Lt or v.shape != k.shape:
        raise ValueError("shape mismatch")
    G = Hq // Hkv
    out = np.zeros((M, Hq, d))
    for m in range(M):
        n_vis = Lt - M + m + 1
        for h in range(Hq):
            s = k[:n_vis, h // G, :] @ q[m, h, :] / np.sqrt(d)
            p = np.exp(s - s.max())
            p /= p.sum()
            out[m, h, :] = p @ v[:n_vis, h // G, :]
    return _round_bf16(out)
