"""ctypes binding of libfge.so: the same entry points as include/fge.h, taking torch tensors.

Argument marshalling only - every step of the chain runs in the library's HIP kernels.  torch
supplies device memory and the stream.  There is no fallback: if the library is missing or a
call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from . import inputs as _codes   # only the integer codes of activations / row ops / dtypes
from .inputs import (ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_GELU_ERF, ACT_SILU, ACT_CLAMP,        # noqa: F401
                     NORM_NONE, NORM_SOFTMAX, NORM_LAYERNORM, NORM_RMSNORM, NORM_LOGSUMEXP)      # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfge.so")

ACT = {"none": 0, "relu": 1, "gelu_tanh": 2, "gelu_erf": 3, "silu": 4, "clamp": 5}
NORM = {"none": 0, "softmax": 1, "layernorm": 2, "rmsnorm": 3, "logsumexp": 4}
FLAG_TWO_PASS = 1
FLAG_IEEE_FP32 = 2
FLAG_NO_SPLIT_K = 4
FLAG_NO_TABLE = 8
FLAG_TEST_EXPIRE_WAIT = 0x1000
STATUS_OK = 0


class FgeParams(ctypes.Structure):
    _fields_ = [
        ("M", ctypes.c_int32), ("N", ctypes.c_int32), ("K", ctypes.c_int32), ("batch", ctypes.c_int32),
        ("ldx", ctypes.c_int64), ("ldw", ctypes.c_int64), ("ldo", ctypes.c_int64),
        ("batch_stride_x", ctypes.c_int64), ("batch_stride_o", ctypes.c_int64),
        ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("alpha", ctypes.c_float), ("post_scale", ctypes.c_float),
        ("clamp_lo", ctypes.c_float), ("clamp_hi", ctypes.c_float), ("eps", ctypes.c_float),
        ("flags", ctypes.c_int32),
        ("gamma", ctypes.c_void_p), ("beta", ctypes.c_void_p), ("aux_out", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
    ]


class FgeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().fge_status_string(status).decode()
        if status == 7:
            msg += f" (hipError {lib().fge_last_hip_error()})"
        super().__init__(f"{where}: fge status {status}: {msg}")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; builds it first only if no built library exists."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, pp = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(FgeParams)
        for name in ("fused_gemm_epilogue", "unfused_gemm_epilogue", "fge_fused_tiles", "fused_gemm_epilogue_static"):
            getattr(L, name).argtypes = [vp, vp, vp, ci, ci, pp, vp, vp]
            getattr(L, name).restype = ci
        L.fge_static_scratch_init.argtypes = []
        L.fge_static_scratch_init.restype = ci
        L.fge_static_scratch_bytes.argtypes = []
        L.fge_static_scratch_bytes.restype = ctypes.c_size_t
        L.fge_fused_finish.argtypes = [ci, ci, pp, vp, vp]
        L.fge_fused_finish.restype = ci
        L.fge_fused_needs_finish.argtypes = [ci, ci, pp]
        L.fge_fused_needs_finish.restype = ci
        L.fge_fused_k_slices.argtypes = [ci, ci, pp]
        L.fge_fused_k_slices.restype = ci
        L.fge_gemm_bias.argtypes = [vp, vp, vp, pp, vp, vp]
        L.fge_gemm_bias.restype = ci
        L.fge_activation.argtypes = [vp, ci, pp, vp, vp]
        L.fge_activation.restype = ci
        L.fge_row_op.argtypes = [vp, ci, pp, vp, vp]
        L.fge_row_op.restype = ci
        L.fge_workspace_bytes.argtypes = [ci, ci, ci, pp]
        L.fge_workspace_bytes.restype = ctypes.c_size_t
        L.fge_status_string.argtypes = [ci]
        L.fge_status_string.restype = ctypes.c_char_p
        L.fge_last_hip_error.argtypes = []
        L.fge_last_hip_error.restype = ci
        L.fge_tile_name.argtypes = [ci, ci, ci, pp]
        L.fge_tile_name.restype = ctypes.c_char_p
        for name in ("fused_gated_gemm_epilogue", "unfused_gated_gemm_epilogue"):
            getattr(L, name).argtypes = [vp, vp, vp, vp, vp, ci, ci, pp, vp, vp]
            getattr(L, name).restype = ci
        L.fge_gated_workspace_bytes.argtypes = [ci, ci, ci, pp]
        L.fge_gated_workspace_bytes.restype = ctypes.c_size_t
        L.fge_fault_word_offset.argtypes = [ci, ci, pp]
        L.fge_fault_word_offset.restype = ctypes.c_size_t
        L.fge_gated_tile_name.argtypes = [ci, ci, pp]
        L.fge_gated_tile_name.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _code(table, v) -> int:
    return table[v] if isinstance(v, str) else int(v)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return _codes.F32
    if t.dtype == torch.bfloat16:
        return _codes.BF16
    if t.dtype == torch.float16:
        return _codes.F16
    if t.dtype == torch.float8_e4m3fn:
        return _codes.F8E4M3
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def make_params(X: Optional[torch.Tensor], W: Optional[torch.Tensor], out: torch.Tensor, *,
                alpha: float = 1.0, post_scale: float = 1.0, clamp_lo: float = 0.0,
                clamp_hi: float = 0.0, eps: float = 0.0, flags: int = 0,
                gamma: Optional[torch.Tensor] = None, beta: Optional[torch.Tensor] = None,
                aux_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                K: Optional[int] = None, in_dtype: Optional[int] = None) -> FgeParams:
    """Fill the C struct from tensor shapes and strides.  X is (M, K) or (batch, M, K) with unit
    stride along K; W is (N, K); out is (M, N) or (batch, M, N) with unit stride along N."""
    p = FgeParams()
    if out.dim() == 3:
        p.batch, p.M, p.N = out.shape
        p.batch_stride_o, p.ldo = out.stride(0), out.stride(1)
    else:
        p.batch, (p.M, p.N) = 1, out.shape
        p.batch_stride_o, p.ldo = 0, out.stride(0)
    assert out.stride(-1) == 1
    if X is not None:
        assert X.stride(-1) == 1 and W.stride(-1) == 1 and X.dtype == W.dtype
        p.K = X.shape[-1]
        p.ldx = X.stride(-2)
        p.batch_stride_x = X.stride(0) if X.dim() == 3 else 0
        p.ldw = W.stride(0)
        p.in_dtype = _dt(X)
    else:                       # stage calls that never touch X / W
        p.K = K if K is not None else 16
        p.ldx = p.ldw = p.K
        p.batch_stride_x = p.M * p.K
        p.in_dtype = in_dtype if in_dtype is not None else _dt(out)
    p.out_dtype = _dt(out)
    p.alpha, p.post_scale = alpha, post_scale
    p.clamp_lo, p.clamp_hi, p.eps = clamp_lo, clamp_hi, eps
    p.flags = flags
    p.gamma, p.beta, p.aux_out = _ptr(gamma), _ptr(beta), _ptr(aux_out)
    p.workspace = _ptr(workspace)
    p.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return p


def _check(rc: int, where: str) -> None:
    if rc != STATUS_OK:
        raise FgeError(rc, where)


def fge_workspace_bytes(fused: bool, act, norm, p: FgeParams) -> int:
    n = lib().fge_workspace_bytes(int(bool(fused)), _code(ACT, act), _code(NORM, norm), ctypes.byref(p))
    if n == ctypes.c_size_t(-1).value:
        raise FgeError(4, "fge_workspace_bytes (invalid or unsupported arguments)")
    return n


def fge_tile_name(fused: bool, act, norm, p: FgeParams) -> str:
    s = lib().fge_tile_name(int(bool(fused)), _code(ACT, act), _code(NORM, norm), ctypes.byref(p))
    return "" if s is None else s.decode()


def fused_gemm_epilogue(X, W, b, act, norm, p: FgeParams, out, stream=None) -> None:
    _check(lib().fused_gemm_epilogue(_ptr(X), _ptr(W), _ptr(b), _code(ACT, act), _code(NORM, norm),
                                     ctypes.byref(p), _ptr(out), _stream(stream)), "fused_gemm_epilogue")


def fused_gemm_epilogue_static(X, W, b, act, norm, p: FgeParams, out, stream=None) -> None:
    _check(lib().fused_gemm_epilogue_static(_ptr(X), _ptr(W), _ptr(b), _code(ACT, act), _code(NORM, norm),
                                            ctypes.byref(p), _ptr(out), _stream(stream)), "fused_gemm_epilogue_static")


def fge_static_scratch_init() -> None:
    _check(lib().fge_static_scratch_init(), "fge_static_scratch_init")


def fge_static_scratch_bytes() -> int:
    return lib().fge_static_scratch_bytes()


def unfused_gemm_epilogue(X, W, b, act, norm, p: FgeParams, out, stream=None) -> None:
    _check(lib().unfused_gemm_epilogue(_ptr(X), _ptr(W), _ptr(b), _code(ACT, act), _code(NORM, norm),
                                       ctypes.byref(p), _ptr(out), _stream(stream)), "unfused_gemm_epilogue")


def fge_fused_tiles(X, W, b, act, norm, p: FgeParams, out, stream=None) -> None:
    _check(lib().fge_fused_tiles(_ptr(X), _ptr(W), _ptr(b), _code(ACT, act), _code(NORM, norm),
                                 ctypes.byref(p), _ptr(out), _stream(stream)), "fge_fused_tiles")


def fge_fused_finish(act, norm, p: FgeParams, out, stream=None) -> None:
    _check(lib().fge_fused_finish(_code(ACT, act), _code(NORM, norm), ctypes.byref(p), _ptr(out),
                                  _stream(stream)), "fge_fused_finish")


def fge_fused_k_slices(act, norm, p: FgeParams) -> int:
    rc = lib().fge_fused_k_slices(_code(ACT, act), _code(NORM, norm), ctypes.byref(p))
    if rc < 0:
        raise FgeError(-rc, "fge_fused_k_slices")
    return rc


def fge_fused_needs_finish(act, norm, p: FgeParams) -> bool:
    rc = lib().fge_fused_needs_finish(_code(ACT, act), _code(NORM, norm), ctypes.byref(p))
    if rc < 0:
        raise FgeError(-rc, "fge_fused_needs_finish")
    return bool(rc)


def fge_gemm_bias(X, W, b, p: FgeParams, Y, stream=None) -> None:
    _check(lib().fge_gemm_bias(_ptr(X), _ptr(W), _ptr(b), ctypes.byref(p), _ptr(Y), _stream(stream)),
           "fge_gemm_bias")


def fge_activation(Y, act, p: FgeParams, A, stream=None) -> None:
    _check(lib().fge_activation(_ptr(Y), _code(ACT, act), ctypes.byref(p), _ptr(A), _stream(stream)),
           "fge_activation")


def fge_row_op(A, norm, p: FgeParams, out, stream=None) -> None:
    _check(lib().fge_row_op(_ptr(A), _code(NORM, norm), ctypes.byref(p), _ptr(out), _stream(stream)),
           "fge_row_op")


def fused_gated_gemm_epilogue(X, W1, W2, b1, b2, act, norm, p: FgeParams, out, stream=None) -> None:
    _check(lib().fused_gated_gemm_epilogue(_ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(b2), _code(ACT, act),
                                           _code(NORM, norm), ctypes.byref(p), _ptr(out), _stream(stream)),
           "fused_gated_gemm_epilogue")


def unfused_gated_gemm_epilogue(X, W1, W2, b1, b2, act, norm, p: FgeParams, out, stream=None) -> None:
    _check(lib().unfused_gated_gemm_epilogue(_ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(b2), _code(ACT, act),
                                             _code(NORM, norm), ctypes.byref(p), _ptr(out), _stream(stream)),
           "unfused_gated_gemm_epilogue")


def fge_gated_workspace_bytes(fused: bool, act, norm, p: FgeParams) -> int:
    n = lib().fge_gated_workspace_bytes(int(bool(fused)), _code(ACT, act), _code(NORM, norm), ctypes.byref(p))
    if n == ctypes.c_size_t(-1).value:
        raise FgeError(4, "fge_gated_workspace_bytes (invalid or unsupported arguments)")
    return n


def fge_gated_tile_name(act, norm, p: FgeParams) -> str:
    s = lib().fge_gated_tile_name(_code(ACT, act), _code(NORM, norm), ctypes.byref(p))
    return "" if s is None else s.decode()


def fge_fault_word_offset(act, norm, p: FgeParams) -> Optional[int]:
    """Offset of the fault word in the workspace, or None when the call takes no cooperative form."""
    n = lib().fge_fault_word_offset(_code(ACT, act), _code(NORM, norm), ctypes.byref(p))
    return None if n == ctypes.c_size_t(-1).value else n
