"""CPU oracle for the block operations fused around the quantised linears (TEST INFRASTRUCTURE ONLY).

Plain numpy, fp64 inside, bf16 roundings (one step, nearest even) exactly where a bf16
implementation of the decoder block has them.  Nothing in the product path imports this file and
this file imports nothing from the product path.

The paper replaces the linears of the target model by quantised ones (Sec. 3.3) and leaves the
rest of the block as the model defines it; for the Qwen3-style block the paper evaluates, the
operations next to the linears are:

* ``rmsnorm``    x^[m, k] = bf16( gamma[k] * bf16( x[m, k] * r_m ) ),  r_m = 1 / sqrt(mean_k x[m, :]^2 + eps)
* ``swiglu``     a[m, k]  = bf16( bf16( silu(g[m, k]) ) * u[m, k] ),   silu(g) = g / (1 + exp(-g))
* ``residual``   y        = bf16( bf16(linear) + residual )
* ``fused_linear``   the int8 linear (Eq. 8, Eq. 10) on the (optionally normalised) activations, plus
                     the residual.
* ``gateup_swiglu``  the gate and up projections (two int8 linears on the same, optionally normalised,
                     activations, each rounded to bf16 as a separate linear is) combined by ``swiglu``.

bf16 values travel as uint16 bit patterns.
"""
from __future__ import annotations

import numpy as np

from . import quasar_ref as ref


def rmsnorm(x_bits, gamma_bits, eps: float) -> np.ndarray:
    """-> uint16 bf16 bits [M, K]."""
    x = ref.bf16_bits_to_f64(x_bits)
    g = ref.bf16_bits_to_f64(gamma_bits).reshape(-1)
    if x.ndim != 2 or g.size != x.shape[1] or eps < 0:
        raise ValueError("x[M,K], gamma[K], eps >= 0")
    r = 1.0 / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + eps)
    t = ref.bf16_bits_to_f64(_round_bf16(x * r))
    return _round_bf16(t * g[None, :])


def silu(g: np.ndarray) -> np.ndarray:
    return g / (1.0 + np.exp(-g))


def swiglu(gate_bits, up_bits) -> np.ndarray:
    """-> uint16 bf16 bits [M, K]."""
    g = ref.bf16_bits_to_f64(gate_bits)
    u = ref.bf16_bits_to_f64(up_bits)
    if g.shape != u.shape:
        raise ValueError("gate and up must have the same shape")
    a = ref.bf16_bits_to_f64(_round_bf16(silu(g)))
    return _round_bf16(a * u)


def fused_linear(x_bits, q, s_bits, *, gamma_bits=None, eps: float = 1e-6, residual_bits=None):
    """y = [residual +] W8([rmsnorm](x)) -> uint16 bf16 bits [M, N]."""
    a = x_bits if gamma_bits is None else rmsnorm(x_bits, gamma_bits, eps)
    lin = _round_bf16(ref.w8_linear(a, q, s_bits))
    if residual_bits is None:
        return lin
    return _round_bf16(ref.bf16_bits_to_f64(lin) + ref.bf16_bits_to_f64(residual_bits))


def gateup_swiglu(x_bits, q_gate, s_gate, q_up, s_up, *, gamma_bits=None, eps: float = 1e-6):
    """a = swiglu( W8_gate([rmsnorm](x)), W8_up([rmsnorm](x)) ) -> uint16 bf16 bits [M, I]."""
    a = x_bits if gamma_bits is None else rmsnorm(x_bits, gamma_bits, eps)
    gate = _round_bf16(ref.w8_linear(a, q_gate, s_gate))
    up = _round_bf16(ref.w8_linear(a, q_up, s_up))
    return swiglu(gate, up)


def _round_bf16(a) -> np.ndarray:
    """fp64 -> bf16 bits in one rounding; zeros and values below bf16's normal range go to zero."""
    a = np.asarray(a, dtype=np.float64)
    out = np.zeros(a.shape, dtype=np.uint16)
    big = np.abs(a) >= 2.0 ** -126
    if np.any(big):
        out[big] = ref.f64_to_bf16_bits(a[big])
    return out
