"""Build and load the naive-C form of the oracle (quasar_ref.c) through ctypes.

Test infrastructure only.  ``build()`` compiles with the host gcc (no fast-math,
so fp32 division and rounding keep IEEE semantics); ``load()`` builds on demand.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "quasar_ref.c")
_LIB = os.path.join(_HERE, "libquasar_ref_c.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class CRef:
    def __init__(self):
        self.lib = ctypes.CDLL(build())
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        self.lib.qref_quantize.argtypes = [vp, i64, i64, i64, vp, vp]
        self.lib.qref_quantize.restype = None
        self.lib.qref_w8_linear.argtypes = [vp, i64, i64, vp, vp, i64, vp]
        self.lib.qref_w8_linear.restype = None
        self.lib.qref_bf16_linear.argtypes = [vp, i64, i64, vp, i64, vp]
        self.lib.qref_bf16_linear.restype = None
        self.lib.qref_lmhead_verify.argtypes = [vp, i64, i64, vp, vp, i64, vp, i64, vp]
        self.lib.qref_lmhead_verify.restype = ctypes.c_int32
        self.lib.qref_quantize_activations.argtypes = [vp, i64, i64, vp, vp, vp]
        self.lib.qref_quantize_activations.restype = None
        self.lib.qref_w8a8_logits.argtypes = [vp, vp, i64, i64, vp, vp, i64, vp]
        self.lib.qref_w8a8_logits.restype = ctypes.c_int32

    @staticmethod
    def _p(a):
        return a.ctypes.data_as(ctypes.c_void_p)

    def quantize(self, w):
        w = np.ascontiguousarray(w, dtype=np.float32)
        N, K = w.shape
        q = np.empty((N, K), dtype=np.int8)
        s = np.empty(N, dtype=np.uint16)
        self.lib.qref_quantize(self._p(w), N, K, K, self._p(q), self._p(s))
        return q, s

    def w8_linear(self, x_bits, q, s_bits):
        x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
        q = np.ascontiguousarray(q, dtype=np.int8)
        s_bits = np.ascontiguousarray(s_bits, dtype=np.uint16)
        M, K = x_bits.shape
        N = q.shape[0]
        y = np.empty((M, N), dtype=np.float64)
        self.lib.qref_w8_linear(self._p(x_bits), M, K, self._p(q), self._p(s_bits), N, self._p(y))
        return y

    def bf16_linear(self, x_bits, w_bits):
        x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
        w_bits = np.ascontiguousarray(w_bits, dtype=np.uint16)
        M, K = x_bits.shape
        N = w_bits.shape[0]
        y = np.empty((M, N), dtype=np.float64)
        self.lib.qref_bf16_linear(self._p(x_bits), M, K, self._p(w_bits), N, self._p(y))
        return y

    def lmhead_verify(self, h_bits, q, s_bits, draft):
        h_bits = np.ascontiguousarray(h_bits, dtype=np.uint16)
        q = np.ascontiguousarray(q, dtype=np.int8)
        s_bits = np.ascontiguousarray(s_bits, dtype=np.uint16)
        draft = np.ascontiguousarray(draft, dtype=np.int32)
        M, K = h_bits.shape
        V = q.shape[0]
        arg = np.empty(M, dtype=np.int32)
        n = self.lib.qref_lmhead_verify(self._p(h_bits), M, K, self._p(q), self._p(s_bits), V,
                                        self._p(draft), draft.size, self._p(arg))
        return arg, int(n)


    def quantize_activations(self, x_bits, smooth=None):
        x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
        M, K = x_bits.shape
        sp = None
        if smooth is not None:
            smooth = np.ascontiguousarray(smooth, dtype=np.float32)
            sp = self._p(smooth)
        xq = np.empty((M, K), dtype=np.int8)
        dx = np.empty(M, dtype=np.float32)
        self.lib.qref_quantize_activations(self._p(x_bits), M, K, sp, self._p(xq), self._p(dx))
        return xq, dx

    def w8a8_logits(self, xq, dx, q, dw_bits):
        xq = np.ascontiguousarray(xq, dtype=np.int8)
        dx = np.ascontiguousarray(dx, dtype=np.float32)
        q = np.ascontiguousarray(q, dtype=np.int8)
        dw_bits = np.ascontiguousarray(dw_bits, dtype=np.uint16)
        M, K = xq.shape
        N = q.shape[0]
        out = np.empty((M, N), dtype=np.float32)
        ovf = self.lib.qref_w8a8_logits(self._p(xq), self._p(dx), M, K, self._p(q), self._p(dw_bits), N,
                                        self._p(out))
        if ovf:
            raise OverflowError("int32 accumulator overflow")
        return out


_cached = None


def load() -> CRef:
    global _cached
    if _cached is None:
        _cached = CRef()
    return _cached
