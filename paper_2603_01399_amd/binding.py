"""Thin ctypes binding over libquasar.so: argument marshalling only.

Every function takes torch CUDA tensors (used purely as device memory), passes
their device pointers and the current torch stream to the C entry point of the
same name, and raises on a non-zero status.  There is no CPU path: importing
this module without the built library raises.
"""
from __future__ import annotations

import ctypes
import os

import torch  # imported first so that the library binds to the HIP runtime torch loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libquasar.so")

F32, BF16 = 0, 1
PATH_AUTO, PATH_VALU, PATH_MFMA = 0, 1, 2

# every symbol declared in include/quasar.h
EXPORTS = (
    "quasar_status_string", "quasar_version", "quasar_set_path", "quasar_get_path",
    "quasar_set_tuning", "quasar_set_tuning_w4", "quasar_lmhead_verify_static", "quasar_set_sequence_form", "quasar_sequence_stamps_bytes", "quasar_sequence_run_stamped",
    "quasar_packed_bytes", "quasar_packed_bytes_bf16", "quasar_workspace_bytes",
    "quasar_quantize_weights", "quasar_unpack_weights", "quasar_w8_linear", "quasar_lmhead_verify",
    "quasar_pack_bf16_weights", "quasar_bf16_linear", "quasar_bf16_lmhead_verify",
    "quasar_read_stream", "quasar_copy_stream",
    "quasar_sequence_plan_bytes", "quasar_sequence_workspace_bytes", "quasar_sequence_prepare",
    "quasar_sequence_run",
    "quasar_quantize_weights_smoothed", "quasar_quantize_activations", "quasar_w8a8_linear",
    "quasar_w8a8_lmhead_verify", "quasar_sequence_prepare_w8a8",
    "quasar_sample_workspace_bytes", "quasar_lmhead_verify_sample",
    "quasar_w4_packed_bytes", "quasar_quantize_weights_w4", "quasar_unpack_weights_w4", "quasar_w4_linear",
    "quasar_w4_lmhead_verify",
    "quasar_drafter_create", "quasar_drafter_destroy", "quasar_drafter_append", "quasar_drafter_length",
    "quasar_drafter_propose",
    "quasar_w8_linear_fused", "quasar_w8_gateup_swiglu",
    "quasar_kv_cache_bytes", "quasar_kv_cache_fill", "quasar_attn_prepare", "quasar_attention_workspace_bytes",
    "quasar_verify_attention",
)


class LinearDesc(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("ldx", ctypes.c_int64), ("w_packed", ctypes.c_void_p),
                ("scales", ctypes.c_void_p), ("y", ctypes.c_void_p), ("ldy", ctypes.c_int64),
                ("N", ctypes.c_int64), ("K", ctypes.c_int64)]


class VerifyDesc(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_void_p), ("ldh", ctypes.c_int64), ("w_packed", ctypes.c_void_p),
                ("scales", ctypes.c_void_p), ("V", ctypes.c_int64), ("K", ctypes.c_int64),
                ("draft_ids", ctypes.c_void_p), ("n_draft", ctypes.c_int64),
                ("out_argmax", ctypes.c_void_p), ("out_accept_len", ctypes.c_void_p)]


class SequenceHandle(ctypes.Structure):
    _fields_ = [("words", ctypes.c_int32 * 16)]



class QuasarError(RuntimeError):
    def __init__(self, fn: str, status: int, text: str):
        super().__init__(f"{fn} failed: status {status} ({text})")
        self.status = status


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2603_01399_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, sz, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    lib.quasar_status_string.argtypes = [ci]
    lib.quasar_status_string.restype = ctypes.c_char_p
    lib.quasar_version.argtypes = []
    lib.quasar_version.restype = ci
    lib.quasar_set_path.argtypes = [ci]
    lib.quasar_get_path.argtypes = []
    lib.quasar_set_tuning.argtypes = [ci, ci, ci]
    for name in ("quasar_packed_bytes", "quasar_packed_bytes_bf16"):
        getattr(lib, name).argtypes = [i64, i64]
        getattr(lib, name).restype = sz
    lib.quasar_workspace_bytes.argtypes = [i64, i64, i64]
    lib.quasar_workspace_bytes.restype = sz
    lib.quasar_quantize_weights.argtypes = [vp, ci, i64, i64, i64, vp, vp, vp]
    lib.quasar_unpack_weights.argtypes = [vp, i64, i64, vp, vp]
    lib.quasar_w8_linear.argtypes = [vp, i64, i64, i64, vp, vp, i64, vp, i64, vp, sz, vp]
    lib.quasar_lmhead_verify.argtypes = [vp, i64, i64, i64, vp, vp, i64, vp, i64, vp, vp, vp, sz, vp]
    lib.quasar_lmhead_verify_static.argtypes = [vp, i64, i64, i64, vp, vp, i64, vp, i64, vp, vp, vp]
    lib.quasar_pack_bf16_weights.argtypes = [vp, ci, i64, i64, i64, vp, vp]
    lib.quasar_bf16_linear.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, vp, sz, vp]
    lib.quasar_bf16_lmhead_verify.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, vp, vp, vp, sz, vp]
    lib.quasar_read_stream.argtypes = [vp, sz, vp, vp]
    lib.quasar_copy_stream.argtypes = [vp, vp, sz, vp]
    lib.quasar_sequence_plan_bytes.argtypes = [i64]
    lib.quasar_sequence_plan_bytes.restype = sz
    lib.quasar_sequence_workspace_bytes.argtypes = [i64, i64]
    lib.quasar_sequence_workspace_bytes.restype = sz
    lib.quasar_sequence_prepare.argtypes = [vp, i64, vp, i64, vp, sz, vp, sz, vp]
    lib.quasar_sequence_run.argtypes = [vp, vp, vp, sz, vp]
    lib.quasar_sequence_stamps_bytes.argtypes = [vp]
    lib.quasar_sequence_stamps_bytes.restype = sz
    lib.quasar_sequence_run_stamped.argtypes = [vp, vp, vp, sz, vp, sz, vp]
    lib.quasar_sequence_prepare_w8a8.argtypes = [vp, i64, vp, vp, vp, i64, vp, sz, vp, sz, vp]
    lib.quasar_sample_workspace_bytes.argtypes = [i64, i64]
    lib.quasar_sample_workspace_bytes.restype = sz
    lib.quasar_lmhead_verify_sample.argtypes = [vp, i64, i64, i64, vp, vp, i64, vp, i64, ctypes.c_float, vp, vp,
                                                vp, vp, vp, vp, sz, vp]
    lib.quasar_w4_packed_bytes.argtypes = [i64, i64]
    lib.quasar_w4_packed_bytes.restype = sz
    lib.quasar_set_tuning_w4.argtypes = [ci, ci]
    lib.quasar_quantize_weights_w4.argtypes = [vp, ci, i64, i64, i64, vp, vp]
    lib.quasar_unpack_weights_w4.argtypes = [vp, i64, i64, vp, vp, vp]
    lib.quasar_w4_linear.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, vp]
    lib.quasar_w4_lmhead_verify.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, vp, vp, vp, sz, vp]
    lib.quasar_w8_linear_fused.argtypes = [vp, i64, i64, i64, vp, ctypes.c_float, vp, vp, i64, vp, i64, vp, i64, vp]
    lib.quasar_w8_gateup_swiglu.argtypes = [vp, i64, i64, i64, vp, ctypes.c_float, vp, vp, i64, vp, i64, vp]
    lib.quasar_kv_cache_bytes.argtypes = [i64, i64]
    lib.quasar_kv_cache_bytes.restype = sz
    lib.quasar_kv_cache_fill.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp]
    lib.quasar_attn_prepare.argtypes = [vp, i64, i64, i64, i64, i64, vp, vp, ctypes.c_float, ctypes.c_float, vp, i64, vp, i64, vp]
    lib.quasar_attention_workspace_bytes.argtypes = [i64, i64, i64, i64]
    lib.quasar_attention_workspace_bytes.restype = sz
    lib.quasar_verify_attention.argtypes = [vp, i64, i64, i64, i64, vp, i64, i64, vp, i64, vp, sz, vp]
    lib.quasar_drafter_create.argtypes = [ci, ci, i64]
    lib.quasar_drafter_create.restype = vp
    lib.quasar_drafter_destroy.argtypes = [vp]
    lib.quasar_drafter_destroy.restype = None
    lib.quasar_drafter_append.argtypes = [vp, vp, i64]
    lib.quasar_drafter_length.argtypes = [vp]
    lib.quasar_drafter_length.restype = i64
    lib.quasar_drafter_propose.argtypes = [vp, i64, vp, vp, vp]
    lib.quasar_quantize_weights_smoothed.argtypes = [vp, ci, i64, i64, i64, vp, vp, vp, vp]
    lib.quasar_quantize_activations.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp]
    lib.quasar_w8a8_linear.argtypes = [vp, i64, i64, i64, vp, vp, vp, i64, vp, i64, vp, sz, vp]
    lib.quasar_w8a8_lmhead_verify.argtypes = [vp, i64, i64, i64, vp, vp, vp, i64, vp, i64, vp, vp, vp, sz, vp]
    return lib


_lib = _load()


def lib() -> ctypes.CDLL:
    return _lib


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise QuasarError(fn, status, _lib.quasar_status_string(status).decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, name, dtype=None):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return t


def status_string(status: int) -> str:
    return _lib.quasar_status_string(status).decode()


def version() -> int:
    return _lib.quasar_version()


def set_path(path: int) -> None:
    _check("quasar_set_path", _lib.quasar_set_path(path))


def get_path() -> int:
    return _lib.quasar_get_path()


def set_tuning(waves: int, wgs_per_cu: int, depth: int = 8) -> None:
    _check("quasar_set_tuning", _lib.quasar_set_tuning(waves, wgs_per_cu, depth))


def set_sequence_form(workgroups_per_cu: int) -> None:
    _check("quasar_set_sequence_form", _lib.quasar_set_sequence_form(workgroups_per_cu))


def packed_bytes(N: int, K: int) -> int:
    return _lib.quasar_packed_bytes(N, K)


def packed_bytes_bf16(N: int, K: int) -> int:
    return _lib.quasar_packed_bytes_bf16(N, K)


def workspace_bytes(M: int, N: int, K: int) -> int:
    return _lib.quasar_workspace_bytes(M, N, K)


def quantize_weights(w: torch.Tensor, wq_packed: torch.Tensor = None, scales: torch.Tensor = None):
    """w [N, K] fp32 or bf16 (last dim contiguous) -> (packed int8 [N*K], scales bf16 [N])."""
    _dev(w, "w")
    if w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be [N, K] with a contiguous last dimension")
    dt = {torch.float32: F32, torch.bfloat16: BF16}.get(w.dtype)
    if dt is None:
        raise TypeError("w must be float32 or bfloat16")
    N, K = w.shape
    if wq_packed is None:
        wq_packed = torch.empty(max(packed_bytes(N, K), 1), dtype=torch.int8, device=w.device)
    if scales is None:
        scales = torch.empty(N, dtype=torch.bfloat16, device=w.device)
    _check("quasar_quantize_weights",
           _lib.quasar_quantize_weights(_ptr(w), dt, N, K, w.stride(0), _ptr(wq_packed), _ptr(scales), _stream()))
    return wq_packed, scales


def quantize_weights_smoothed(w: torch.Tensor, smooth: torch.Tensor, wq_packed: torch.Tensor = None,
                              scales: torch.Tensor = None):
    """As quantize_weights, applied to W diag(s)^-1 (smooth [K] fp32, or None)."""
    _dev(w, "w")
    if w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be [N, K] with a contiguous last dimension")
    dt = {torch.float32: F32, torch.bfloat16: BF16}.get(w.dtype)
    if dt is None:
        raise TypeError("w must be float32 or bfloat16")
    N, K = w.shape
    if smooth is not None:
        _dev(smooth, "smooth", torch.float32)
        if smooth.numel() != K or not smooth.is_contiguous():
            raise ValueError("smooth must be a contiguous [K] vector")
    if wq_packed is None:
        wq_packed = torch.empty(max(packed_bytes(N, K), 1), dtype=torch.int8, device=w.device)
    if scales is None:
        scales = torch.empty(N, dtype=torch.bfloat16, device=w.device)
    _check("quasar_quantize_weights_smoothed",
           _lib.quasar_quantize_weights_smoothed(_ptr(w), dt, N, K, w.stride(0), _ptr(smooth), _ptr(wq_packed),
                                                 _ptr(scales), _stream()))
    return wq_packed, scales


def _smooth_arg(smooth, K):
    if smooth is None:
        return None
    _dev(smooth, "smooth", torch.float32)
    if smooth.numel() != K or not smooth.is_contiguous():
        raise ValueError("smooth must be a contiguous [K] vector")
    return _ptr(smooth)


def quantize_activations(x: torch.Tensor, smooth: torch.Tensor = None):
    """x [M, K] bf16 -> (codes int8 [M, K], step sizes fp32 [M])."""
    _dev(x, "x", torch.bfloat16)
    M, K = x.shape
    xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    dx = torch.empty(M, dtype=torch.float32, device=x.device)
    _check("quasar_quantize_activations",
           _lib.quasar_quantize_activations(_ptr(x), M, K, x.stride(0), _smooth_arg(smooth, K), _ptr(xq), _ptr(dx),
                                            _stream()))
    return xq, dx


def w8a8_linear(x: torch.Tensor, wq_packed: torch.Tensor, scales: torch.Tensor, N: int,
                smooth: torch.Tensor = None, y: torch.Tensor = None) -> torch.Tensor:
    _dev(x, "x", torch.bfloat16)
    _dev(wq_packed, "wq_packed", torch.int8)
    _dev(scales, "scales", torch.bfloat16)
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _check("quasar_w8a8_linear",
           _lib.quasar_w8a8_linear(_ptr(x), M, K, x.stride(0), _smooth_arg(smooth, K), _ptr(wq_packed), _ptr(scales),
                                   N, _ptr(y), y.stride(0), None, 0, _stream()))
    return y


def w8a8_lmhead_verify(hidden: torch.Tensor, wq_packed: torch.Tensor, scales: torch.Tensor, V: int,
                       draft_ids: torch.Tensor, workspace: torch.Tensor, smooth: torch.Tensor = None,
                       out_argmax: torch.Tensor = None, out_accept: torch.Tensor = None):
    _dev(hidden, "hidden", torch.bfloat16)
    _dev(wq_packed, "wq_packed", torch.int8)
    _dev(scales, "scales", torch.bfloat16)
    M, K = hidden.shape
    n_draft = 0 if draft_ids is None else draft_ids.numel()
    if n_draft:
        _dev(draft_ids, "draft_ids", torch.int32)
    if out_argmax is None:
        out_argmax = torch.empty(M, dtype=torch.int32, device=hidden.device)
    if out_accept is None:
        out_accept = torch.empty(1, dtype=torch.int32, device=hidden.device)
    _check("quasar_w8a8_lmhead_verify",
           _lib.quasar_w8a8_lmhead_verify(_ptr(hidden), M, K, hidden.stride(0), _smooth_arg(smooth, K),
                                          _ptr(wq_packed), _ptr(scales), V,
                                          _ptr(draft_ids) if n_draft else None, n_draft, _ptr(out_argmax),
                                          _ptr(out_accept), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream()))
    return out_argmax, out_accept


def lmhead_verify_sample(hidden: torch.Tensor, wq_packed: torch.Tensor, scales: torch.Tensor, V: int,
                         draft_ids: torch.Tensor, temperature: float, u_accept: torch.Tensor,
                         u_sample: torch.Tensor, workspace: torch.Tensor = None):
    """Stochastic verification at temperature T > 0 against a deterministic drafter.
    Returns (accept_len int32 [1], next_token int32 [1], p_draft fp32 [n_draft])."""
    _dev(hidden, "hidden", torch.bfloat16)
    _dev(wq_packed, "wq_packed", torch.int8)
    _dev(scales, "scales", torch.bfloat16)
    _dev(u_sample, "u_sample", torch.float32)
    M, K = hidden.shape
    n_draft = 0 if draft_ids is None else draft_ids.numel()
    if n_draft:
        _dev(draft_ids, "draft_ids", torch.int32)
        _dev(u_accept, "u_accept", torch.float32)
        if u_accept.numel() < n_draft:
            raise ValueError("u_accept needs one entry per candidate")
    if u_sample.numel() < M:
        raise ValueError("u_sample needs one entry per position")
    if workspace is None:
        workspace = torch.empty(max(_lib.quasar_sample_workspace_bytes(M, V), 16), dtype=torch.uint8,
                                device=hidden.device)
    acc = torch.empty(1, dtype=torch.int32, device=hidden.device)
    tok = torch.empty(1, dtype=torch.int32, device=hidden.device)
    pd = torch.empty(max(n_draft, 1), dtype=torch.float32, device=hidden.device)
    _check("quasar_lmhead_verify_sample",
           _lib.quasar_lmhead_verify_sample(_ptr(hidden), M, K, hidden.stride(0), _ptr(wq_packed), _ptr(scales), V,
                                            _ptr(draft_ids) if n_draft else None, n_draft, float(temperature),
                                            _ptr(u_accept) if n_draft else None, _ptr(u_sample), _ptr(acc), _ptr(tok),
                                            _ptr(pd), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream()))
    return acc, tok, pd[:n_draft]


def unpack_weights(wq_packed: torch.Tensor, N: int, K: int) -> torch.Tensor:
    _dev(wq_packed, "wq_packed", torch.int8)
    q = torch.empty((N, K), dtype=torch.int8, device=wq_packed.device)
    _check("quasar_unpack_weights", _lib.quasar_unpack_weights(_ptr(wq_packed), N, K, _ptr(q), _stream()))
    return q


def w8_linear(x: torch.Tensor, wq_packed: torch.Tensor, scales: torch.Tensor, N: int,
              y: torch.Tensor = None, workspace: torch.Tensor = None) -> torch.Tensor:
    _dev(x, "x", torch.bfloat16)
    _dev(wq_packed, "wq_packed", torch.int8)
    _dev(scales, "scales", torch.bfloat16)
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check("quasar_w8_linear",
           _lib.quasar_w8_linear(_ptr(x), M, K, x.stride(0), _ptr(wq_packed), _ptr(scales), N,
                                 _ptr(y), y.stride(0), _ptr(workspace), ws_bytes, _stream()))
    return y


def w4_packed_bytes(N: int, K: int) -> int:
    return _lib.quasar_w4_packed_bytes(N, K)


def set_tuning_w4(waves: int, depth: int) -> None:
    _check("quasar_set_tuning_w4", _lib.quasar_set_tuning_w4(waves, depth))


def quantize_weights_w4(w: torch.Tensor, w4_packed: torch.Tensor = None) -> torch.Tensor:
    """w [N, K] fp32 or bf16 (last dim contiguous) -> packed 4-bit codes + group step sizes (uint8)."""
    _dev(w, "w")
    if w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be [N, K] with a contiguous last dimension")
    dt = {torch.float32: F32, torch.bfloat16: BF16}.get(w.dtype)
    if dt is None:
        raise TypeError("w must be float32 or bfloat16")
    N, K = w.shape
    if w4_packed is None:
        w4_packed = torch.empty(max(w4_packed_bytes(N, K), 1), dtype=torch.uint8, device=w.device)
    _check("quasar_quantize_weights_w4",
           _lib.quasar_quantize_weights_w4(_ptr(w), dt, N, K, w.stride(0), _ptr(w4_packed), _stream()))
    return w4_packed


def unpack_weights_w4(w4_packed: torch.Tensor, N: int, K: int):
    """-> (codes int8 [N, K], step sizes bf16 [N, K // 128])."""
    _dev(w4_packed, "w4_packed", torch.uint8)
    q = torch.empty((N, K), dtype=torch.int8, device=w4_packed.device)
    sc = torch.empty((N, max(K // 128, 1)), dtype=torch.bfloat16, device=w4_packed.device)
    _check("quasar_unpack_weights_w4", _lib.quasar_unpack_weights_w4(_ptr(w4_packed), N, K, _ptr(q), _ptr(sc), _stream()))
    return q, sc


def w4_linear(x: torch.Tensor, w4_packed: torch.Tensor, N: int, y: torch.Tensor = None) -> torch.Tensor:
    _dev(x, "x", torch.bfloat16)
    _dev(w4_packed, "w4_packed", torch.uint8)
    M, K = x.shape
    if w4_packed.numel() < w4_packed_bytes(N, K):
        raise ValueError("w4_packed is smaller than quasar_w4_packed_bytes(N, K)")
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _check("quasar_w4_linear",
           _lib.quasar_w4_linear(_ptr(x), M, K, x.stride(0), _ptr(w4_packed), N, _ptr(y), y.stride(0), _stream()))
    return y


def w4_lmhead_verify(hidden: torch.Tensor, w4_packed: torch.Tensor, V: int, draft_ids: torch.Tensor,
                     workspace: torch.Tensor, out_argmax: torch.Tensor = None, out_accept: torch.Tensor = None):
    _dev(hidden, "hidden", torch.bfloat16)
    _dev(w4_packed, "w4_packed", torch.uint8)
    M, K = hidden.shape
    if w4_packed.numel() < w4_packed_bytes(V, K):
        raise ValueError("w4_packed is smaller than quasar_w4_packed_bytes(V, K)")
    n_draft = 0 if draft_ids is None else draft_ids.numel()
    if n_draft:
        _dev(draft_ids, "draft_ids", torch.int32)
    if out_argmax is None:
        out_argmax = torch.empty(M, dtype=torch.int32, device=hidden.device)
    if out_accept is None:
        out_accept = torch.empty(1, dtype=torch.int32, device=hidden.device)
    _check("quasar_w4_lmhead_verify",
           _lib.quasar_w4_lmhead_verify(_ptr(hidden), M, K, hidden.stride(0), _ptr(w4_packed), V,
                                        _ptr(draft_ids) if n_draft else None, n_draft, _ptr(out_argmax),
                                        _ptr(out_accept), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream()))
    return out_argmax, out_accept


def _gamma_arg(gamma, K):
    if gamma is None:
        return None
    _dev(gamma, "gamma", torch.bfloat16)
    if gamma.numel() != K or not gamma.is_contiguous():
        raise ValueError("gamma must be a contiguous [K] vector")
    return gamma


def w8_linear_fused(x: torch.Tensor, wq_packed: torch.Tensor, scales: torch.Tensor, N: int, *, gamma: torch.Tensor = None,
                    eps: float = 1e-6, residual: torch.Tensor = None, y: torch.Tensor = None) -> torch.Tensor:
    """y = [residual +] W8([RMSNorm](x)); the normalisation (gamma, eps) and the residual are optional."""
    _dev(x, "x", torch.bfloat16)
    _dev(wq_packed, "wq_packed", torch.int8)
    _dev(scales, "scales", torch.bfloat16)
    M, K = x.shape
    gamma = _gamma_arg(gamma, K)
    if residual is not None:
        _dev(residual, "residual", torch.bfloat16)
        if residual.shape != (M, N) or residual.stride(1) != 1:
            raise ValueError("residual must be [M, N] with a contiguous last dimension")
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _check("quasar_w8_linear_fused",
           _lib.quasar_w8_linear_fused(_ptr(x), M, K, x.stride(0), _ptr(gamma), eps, _ptr(wq_packed), _ptr(scales), N,
                                       _ptr(residual), 0 if residual is None else residual.stride(0),
                                       _ptr(y), y.stride(0), _stream()))
    return y


def interleave_gate_up(gate: torch.Tensor, up: torch.Tensor) -> torch.Tensor:
    """[I, K] gate and up weights -> the [2 I, K] matrix quasar_w8_gateup_swiglu expects (rows alternate in
    blocks of 16: gate rows 16 t .. 16 t + 15, then the up rows of the same indices).  Data movement only."""
    I, K = gate.shape
    if up.shape != gate.shape or I % 16:
        raise ValueError("gate and up must have the same [I, K] shape with I a multiple of 16")
    return torch.stack([gate.reshape(I // 16, 16, K), up.reshape(I // 16, 16, K)], dim=1).reshape(2 * I, K)


def w8_gateup_swiglu(x: torch.Tensor, wq_packed: torch.Tensor, scales: torch.Tensor, I: int, *, gamma: torch.Tensor = None,
                     eps: float = 1e-6, y: torch.Tensor = None) -> torch.Tensor:
    """y[M, I] = silu(gate) * up with both projections taken from the row-interleaved [2 I, K] int8 matrix."""
    _dev(x, "x", torch.bfloat16)
    _dev(wq_packed, "wq_packed", torch.int8)
    _dev(scales, "scales", torch.bfloat16)
    M, K = x.shape
    gamma = _gamma_arg(gamma, K)
    if y is None:
        y = torch.empty((M, I), dtype=torch.bfloat16, device=x.device)
    _check("quasar_w8_gateup_swiglu",
           _lib.quasar_w8_gateup_swiglu(_ptr(x), M, K, x.stride(0), _ptr(gamma), eps, _ptr(wq_packed), _ptr(scales), I,
                                        _ptr(y), y.stride(0), _stream()))
    return y


class KvCache:
    """Key/value cache of one layer in the library's layout (head dimension 128)."""

    def __init__(self, n_kv_heads: int, max_len: int, device="cuda"):
        nbytes = _lib.quasar_kv_cache_bytes(n_kv_heads, max_len)
        if nbytes == 0:
            raise ValueError("invalid cache shape")
        self.n_kv_heads, self.max_len = n_kv_heads, max_len
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)

    def fill(self, k: torch.Tensor, v: torch.Tensor, pos0: int = 0) -> None:
        """k, v: [n, n_kv_heads, 128] bf16 contiguous, already normalised and rotated."""
        _dev(k, "k", torch.bfloat16)
        _dev(v, "v", torch.bfloat16)
        if k.shape != v.shape or k.dim() != 3 or k.shape[1] != self.n_kv_heads or k.shape[2] != 128:
            raise ValueError("k and v must be [n, n_kv_heads, 128]")
        k, v = k.contiguous(), v.contiguous()
        _check("quasar_kv_cache_fill", _lib.quasar_kv_cache_fill(_ptr(k), _ptr(v), k.shape[0], self.n_kv_heads, pos0,
                                                                  _ptr(self.buf), self.max_len, _stream()))


def attn_prepare(qkv: torch.Tensor, n_q_heads: int, cache: KvCache, L: int, q_gamma: torch.Tensor,
                 k_gamma: torch.Tensor, eps: float = 1e-6, rope_theta: float = 1.0e6, q_out: torch.Tensor = None):
    """Normalise and rotate the queries and keys of the M new positions, append keys and values at L .. L+M-1."""
    _dev(qkv, "qkv", torch.bfloat16)
    _dev(q_gamma, "q_gamma", torch.bfloat16)
    _dev(k_gamma, "k_gamma", torch.bfloat16)
    M = qkv.shape[0]
    if qkv.stride(1) != 1 or q_gamma.numel() != 128 or k_gamma.numel() != 128:
        raise ValueError("qkv needs a contiguous last dimension; gammas are [128]")
    if q_out is None:
        q_out = torch.empty((M, n_q_heads * 128), dtype=torch.bfloat16, device=qkv.device)
    _check("quasar_attn_prepare",
           _lib.quasar_attn_prepare(_ptr(qkv), M, qkv.stride(0), n_q_heads, cache.n_kv_heads, L, _ptr(q_gamma),
                                    _ptr(k_gamma), eps, rope_theta, _ptr(q_out), q_out.stride(0), _ptr(cache.buf),
                                    cache.max_len, _stream()))
    return q_out


def attention_workspace(M: int, n_q_heads: int, n_kv_heads: int, L_total: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(_lib.quasar_attention_workspace_bytes(M, n_q_heads, n_kv_heads, L_total), 16),
                       dtype=torch.uint8, device=device)


def verify_attention(q: torch.Tensor, n_q_heads: int, cache: KvCache, L_total: int, workspace: torch.Tensor = None,
                     out: torch.Tensor = None) -> torch.Tensor:
    _dev(q, "q", torch.bfloat16)
    M = q.shape[0]
    if workspace is None:
        workspace = attention_workspace(M, n_q_heads, cache.n_kv_heads, L_total, q.device)
    if out is None:
        out = torch.empty((M, n_q_heads * 128), dtype=torch.bfloat16, device=q.device)
    _check("quasar_verify_attention",
           _lib.quasar_verify_attention(_ptr(q), M, q.stride(0), n_q_heads, cache.n_kv_heads, _ptr(cache.buf),
                                        cache.max_len, L_total, _ptr(out), out.stride(0), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream()))
    return out


class Drafter:
    """Prompt-lookup n-gram drafter (host side): append() tokens as they are accepted, propose() a draft."""

    def __init__(self, k_min: int = 1, k_max: int = 4, capacity_hint: int = 0):
        self._h = _lib.quasar_drafter_create(k_min, k_max, capacity_hint)
        if not self._h:
            raise QuasarError("quasar_drafter_create", -1, "invalid lookup range or out of memory")

    def append(self, tokens) -> None:
        import numpy as np
        a = np.ascontiguousarray(tokens, dtype=np.int32).reshape(-1)
        _check("quasar_drafter_append", _lib.quasar_drafter_append(self._h, a.ctypes.data, a.size))

    def __len__(self) -> int:
        return int(_lib.quasar_drafter_length(self._h))

    def propose(self, gamma: int):
        """-> (draft tokens as a list, lookup length that matched or 0)."""
        buf = (ctypes.c_int32 * max(int(gamma), 1))()
        n = ctypes.c_int64(0)
        k = ctypes.c_int(0)
        _check("quasar_drafter_propose",
               _lib.quasar_drafter_propose(self._h, gamma, buf, ctypes.byref(n), ctypes.byref(k)))
        return list(buf[:n.value]), k.value

    def close(self) -> None:
        if self._h:
            _lib.quasar_drafter_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def make_workspace(M: int, N: int, K: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(workspace_bytes(M, N, K), 16), dtype=torch.uint8, device=device)


def lmhead_verify(hidden: torch.Tensor, wq_packed: torch.Tensor, scales: torch.Tensor, V: int,
                  draft_ids: torch.Tensor, workspace: torch.Tensor,
                  out_argmax: torch.Tensor = None, out_accept: torch.Tensor = None):
    _dev(hidden, "hidden", torch.bfloat16)
    _dev(wq_packed, "wq_packed", torch.int8)
    _dev(scales, "scales", torch.bfloat16)
    M, K = hidden.shape
    n_draft = 0 if draft_ids is None else draft_ids.numel()
    if n_draft:
        _dev(draft_ids, "draft_ids", torch.int32)
    if out_argmax is None:
        out_argmax = torch.empty(M, dtype=torch.int32, device=hidden.device)
    if out_accept is None:
        out_accept = torch.empty(1, dtype=torch.int32, device=hidden.device)
    _check("quasar_lmhead_verify",
           _lib.quasar_lmhead_verify(_ptr(hidden), M, K, hidden.stride(0), _ptr(wq_packed), _ptr(scales), V,
                                     _ptr(draft_ids) if n_draft else None, n_draft, _ptr(out_argmax),
                                     _ptr(out_accept), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream()))
    return out_argmax, out_accept


def lmhead_verify_static(hidden: torch.Tensor, wq_packed: torch.Tensor, scales: torch.Tensor, V: int,
                         draft_ids: torch.Tensor, out_argmax: torch.Tensor, out_accept: torch.Tensor):
    """quasar_lmhead_verify_static: no workspace, and the outputs are the caller's (nothing is allocated)."""
    _dev(hidden, "hidden", torch.bfloat16)
    _dev(wq_packed, "wq_packed", torch.int8)
    _dev(scales, "scales", torch.bfloat16)
    _dev(out_argmax, "out_argmax", torch.int32)
    _dev(out_accept, "out_accept", torch.int32)
    M, K = hidden.shape
    n_draft = 0 if draft_ids is None else draft_ids.numel()
    if n_draft:
        _dev(draft_ids, "draft_ids", torch.int32)
    if out_argmax.numel() < M or out_accept.numel() < 1:
        raise ValueError("out_argmax needs M elements and out_accept one")
    _check("quasar_lmhead_verify_static",
           _lib.quasar_lmhead_verify_static(_ptr(hidden), M, K, hidden.stride(0), _ptr(wq_packed), _ptr(scales), V,
                                            _ptr(draft_ids) if n_draft else None, n_draft, _ptr(out_argmax),
                                            _ptr(out_accept), _stream()))
    return out_argmax, out_accept


def pack_bf16_weights(w: torch.Tensor, w_packed: torch.Tensor = None) -> torch.Tensor:
    _dev(w, "w")
    if w.dim() != 2 or w.stride(1) != 1:
        raise ValueError("w must be [N, K] with a contiguous last dimension")
    dt = {torch.float32: F32, torch.bfloat16: BF16}.get(w.dtype)
    if dt is None:
        raise TypeError("w must be float32 or bfloat16")
    N, K = w.shape
    if w_packed is None:
        w_packed = torch.empty(N * K, dtype=torch.bfloat16, device=w.device)
    _check("quasar_pack_bf16_weights",
           _lib.quasar_pack_bf16_weights(_ptr(w), dt, N, K, w.stride(0), _ptr(w_packed), _stream()))
    return w_packed


def bf16_linear(x: torch.Tensor, w_packed: torch.Tensor, N: int, y: torch.Tensor = None,
                workspace: torch.Tensor = None) -> torch.Tensor:
    _dev(x, "x", torch.bfloat16)
    _dev(w_packed, "w_packed", torch.bfloat16)
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check("quasar_bf16_linear",
           _lib.quasar_bf16_linear(_ptr(x), M, K, x.stride(0), _ptr(w_packed), N, _ptr(y), y.stride(0),
                                   _ptr(workspace), ws_bytes, _stream()))
    return y


def bf16_lmhead_verify(hidden: torch.Tensor, w_packed: torch.Tensor, V: int, draft_ids: torch.Tensor,
                       workspace: torch.Tensor, out_argmax: torch.Tensor = None, out_accept: torch.Tensor = None):
    _dev(hidden, "hidden", torch.bfloat16)
    _dev(w_packed, "w_packed", torch.bfloat16)
    M, K = hidden.shape
    n_draft = 0 if draft_ids is None else draft_ids.numel()
    if out_argmax is None:
        out_argmax = torch.empty(M, dtype=torch.int32, device=hidden.device)
    if out_accept is None:
        out_accept = torch.empty(1, dtype=torch.int32, device=hidden.device)
    _check("quasar_bf16_lmhead_verify",
           _lib.quasar_bf16_lmhead_verify(_ptr(hidden), M, K, hidden.stride(0), _ptr(w_packed), V,
                                          _ptr(draft_ids) if n_draft else None, n_draft, _ptr(out_argmax),
                                          _ptr(out_accept), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream()))
    return out_argmax, out_accept


def read_stream(src: torch.Tensor, sink: torch.Tensor, nbytes: int = None) -> None:
    nbytes = src.numel() * src.element_size() if nbytes is None else nbytes
    _check("quasar_read_stream", _lib.quasar_read_stream(_ptr(src), nbytes, _ptr(sink), _stream()))


def copy_stream(dst: torch.Tensor, src: torch.Tensor, nbytes: int = None) -> None:
    nbytes = src.numel() * src.element_size() if nbytes is None else nbytes
    _check("quasar_copy_stream", _lib.quasar_copy_stream(_ptr(dst), _ptr(src), nbytes, _stream()))


class Sequence:
    """One verification step as a single persistent launch (quasar_sequence_prepare / _run).

    linears: list of (x, w_packed, scales_or_None, N, y) tensor tuples in execution order;
    verify: optional (hidden, w_packed, scales_or_None, V, draft_ids, out_argmax, out_accept).
    w8a8=True runs every phase in the W8A8 form; smooth is then an optional list with one
    [K] fp32 vector (or None) per linear, verify_smooth the one of the vocabulary phase.
    The tensors are only borrowed: the caller keeps them alive.
    """

    def __init__(self, linears, verify=None, M=None, w8a8=False, smooth=None, verify_smooth=None):
        descs = (LinearDesc * max(len(linears), 1))()
        keep = []
        for i, (x, wp, sc, N, y) in enumerate(linears):
            _dev(x, "x", torch.bfloat16)
            _dev(y, "y", torch.bfloat16)
            M = x.shape[0] if M is None else M
            d = descs[i]
            d.x, d.ldx, d.w_packed = x.data_ptr(), x.stride(0), wp.data_ptr()
            d.scales = None if sc is None else sc.data_ptr()
            d.y, d.ldy, d.N, d.K = y.data_ptr(), y.stride(0), N, x.shape[1]
            keep.append((x, wp, sc, y))
        vdesc = None
        if verify is not None:
            h, wp, sc, V, draft, out_argmax, out_accept = verify
            M = h.shape[0] if M is None else M
            vdesc = VerifyDesc()
            vdesc.hidden, vdesc.ldh, vdesc.w_packed = h.data_ptr(), h.stride(0), wp.data_ptr()
            vdesc.scales = None if sc is None else sc.data_ptr()
            vdesc.V, vdesc.K = V, h.shape[1]
            n_draft = 0 if draft is None else draft.numel()
            vdesc.draft_ids = draft.data_ptr() if n_draft else None
            vdesc.n_draft = n_draft
            vdesc.out_argmax, vdesc.out_accept_len = out_argmax.data_ptr(), out_accept.data_ptr()
            keep.append(verify)
        self._keep = keep
        self.M = M
        dev = keep[0][0].device
        self.plan = torch.empty(max(_lib.quasar_sequence_plan_bytes(len(linears)), 16), dtype=torch.uint8, device=dev)
        self.workspace = torch.empty(_lib.quasar_sequence_workspace_bytes(len(linears), M), dtype=torch.uint8,
                                     device=dev)
        self.handle = SequenceHandle()
        vptr = None if vdesc is None else ctypes.cast(ctypes.pointer(vdesc), ctypes.c_void_p)
        hptr = ctypes.cast(ctypes.pointer(self.handle), ctypes.c_void_p)
        if not w8a8:
            if smooth is not None or verify_smooth is not None:
                raise ValueError("smoothing vectors belong to the W8A8 form")
            _check("quasar_sequence_prepare",
                   _lib.quasar_sequence_prepare(ctypes.cast(descs, ctypes.c_void_p), len(linears), vptr,
                                                M, _ptr(self.plan), self.plan.numel(),
                                                _ptr(self.workspace), self.workspace.numel(), hptr))
            return
        sm_arr = None
        if smooth is not None:
            if len(smooth) != len(linears):
                raise ValueError("smooth needs one entry per linear")
            sm_arr = (ctypes.c_void_p * max(len(linears), 1))()
            for i, (sv, lin) in enumerate(zip(smooth, linears)):
                if sv is not None:
                    _smooth_arg(sv, lin[0].shape[1])
                    sm_arr[i] = sv.data_ptr()
            keep.append(list(smooth))
        vsm = None
        if verify_smooth is not None:
            vsm = _smooth_arg(verify_smooth, verify[0].shape[1])
            keep.append(verify_smooth)
        _check("quasar_sequence_prepare_w8a8",
               _lib.quasar_sequence_prepare_w8a8(ctypes.cast(descs, ctypes.c_void_p), len(linears),
                                                 None if sm_arr is None else ctypes.cast(sm_arr, ctypes.c_void_p),
                                                 vptr, vsm, M, _ptr(self.plan), self.plan.numel(),
                                                 _ptr(self.workspace), self.workspace.numel(), hptr))

    @property
    def nphases(self) -> int:
        return self.handle.words[1]

    @property
    def workgroups_per_cu(self) -> int:
        return self.handle.words[14]

    @property
    def n_barriers(self) -> int:
        """Phases that wait at a device-wide barrier (inputs in reused or partially overlapping buffers)."""
        return self.handle.words[12]

    @property
    def n_flag_waits(self) -> int:
        """Phases gated by the completion flags of their producer phases (write-once buffers)."""
        return self.handle.words[13]

    def run(self) -> None:
        _check("quasar_sequence_run",
               _lib.quasar_sequence_run(ctypes.cast(ctypes.pointer(self.handle), ctypes.c_void_p), _ptr(self.plan),
                                        _ptr(self.workspace), self.workspace.numel(), _stream()))

    def run_stamped(self) -> torch.Tensor:
        """One step with per-phase time stamps: int64 tensor [nphases, workgroups, 8] (100 MHz ticks, 0 = no share)."""
        hp = ctypes.cast(ctypes.pointer(self.handle), ctypes.c_void_p)
        n = _lib.quasar_sequence_stamps_bytes(hp)
        stamps = torch.zeros(n // 8, dtype=torch.int64, device=self.plan.device)
        _check("quasar_sequence_run_stamped",
               _lib.quasar_sequence_run_stamped(hp, _ptr(self.plan), _ptr(self.workspace), self.workspace.numel(),
                                                _ptr(stamps), n, _stream()))
        return stamps.view(self.nphases, -1, 8)

    def timed_out(self) -> bool:
        """True if a device-wide barrier of the last finished step gave up (synchronises)."""
        return bool(self.workspace[:8].view(torch.int32)[1].item() != 0)
