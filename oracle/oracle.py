"""ctypes front of the C float64 oracle (oracle/fge_oracle.c).  TEST INFRASTRUCTURE ONLY.

All arrays are float64 numpy arrays holding the exact values of the stored input bits; the
caller converts fp32 / bf16 storage to float64 before calling."""
import ctypes
from typing import Optional, Tuple

import numpy as np

from . import build as _build

_lib = None
_D = ctypes.POINTER(ctypes.c_double)


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_build.build())
        L.fge_oracle_gemm.argtypes = [_D, _D, ctypes.c_long, ctypes.c_long, ctypes.c_long, _D]
        L.fge_oracle_gemm.restype = None
        L.fge_oracle_scale_bias.argtypes = [_D, _D, ctypes.c_long, ctypes.c_long,
                                            ctypes.c_double, ctypes.c_double]
        L.fge_oracle_scale_bias.restype = None
        L.fge_oracle_act.argtypes = [_D, ctypes.c_long, ctypes.c_int, ctypes.c_double, ctypes.c_double]
        L.fge_oracle_act.restype = None
        L.fge_oracle_rowop.argtypes = [_D, ctypes.c_long, ctypes.c_long, ctypes.c_int,
                                       ctypes.c_double, _D, _D, _D]
        L.fge_oracle_rowop.restype = None
        L.fge_oracle_gate.argtypes = [_D, _D, ctypes.c_long, ctypes.c_int, ctypes.c_double, ctypes.c_double]
        L.fge_oracle_gate.restype = None
        L.fge_oracle_gated_chain.argtypes = [_D] * 7 + [ctypes.c_long] * 3 + [ctypes.c_double] * 2 + [
            ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_int, ctypes.c_double, _D, _D, _D]
        L.fge_oracle_gated_chain.restype = ctypes.c_int
        L.fge_oracle_chain.argtypes = [_D, _D, _D, _D, _D, ctypes.c_long, ctypes.c_long, ctypes.c_long,
                                       ctypes.c_double, ctypes.c_double, ctypes.c_int,
                                       ctypes.c_double, ctypes.c_double, ctypes.c_int,
                                       ctypes.c_double, _D, _D]
        L.fge_oracle_chain.restype = ctypes.c_int
        L.fge_oracle_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_D)


def _c(a: Optional[np.ndarray]) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def threads() -> int:
    return int(lib().fge_oracle_threads())


def gemm(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    X, W = _c(X), _c(W)
    M, K = X.shape
    N, K2 = W.shape
    assert K == K2
    G = np.empty((M, N), dtype=np.float64)
    lib().fge_oracle_gemm(_p(X), _p(W), M, N, K, _p(G))
    return G


def scale_bias(G: np.ndarray, b: Optional[np.ndarray], alpha: float, post_scale: float) -> np.ndarray:
    Y = np.array(G, dtype=np.float64, order="C", copy=True)
    b = _c(b)
    lib().fge_oracle_scale_bias(_p(Y), _p(b), Y.shape[0], Y.shape[1], alpha, post_scale)
    return Y


def act(Y: np.ndarray, kind: int, lo: float = 0.0, hi: float = 0.0) -> np.ndarray:
    A = np.array(Y, dtype=np.float64, order="C", copy=True)
    lib().fge_oracle_act(_p(A), A.size, kind, lo, hi)
    return A


def rowop(A: np.ndarray, norm: int, eps: float = 0.0, gamma=None, beta=None
          ) -> Tuple[np.ndarray, np.ndarray]:
    O = np.array(A, dtype=np.float64, order="C", copy=True)
    M, N = O.shape
    aux = np.full(M, np.nan, dtype=np.float64)
    gamma, beta = _c(gamma), _c(beta)
    lib().fge_oracle_rowop(_p(O), M, N, norm, eps, _p(gamma), _p(beta), _p(aux))
    return O, aux


def chain(X, W, b=None, gamma=None, beta=None, *, alpha=1.0, post_scale=1.0, act=0,
          clamp_lo=0.0, clamp_hi=0.0, norm=0, eps=0.0) -> Tuple[np.ndarray, np.ndarray]:
    """out (M x N float64) and aux (length M; row logsumexp when norm is logsumexp, else NaN)."""
    X, W, b, gamma, beta = _c(X), _c(W), _c(b), _c(gamma), _c(beta)
    M, K = X.shape
    N, K2 = W.shape
    assert K == K2
    out = np.empty((M, N), dtype=np.float64)
    aux = np.full(M, np.nan, dtype=np.float64)
    rc = lib().fge_oracle_chain(_p(X), _p(W), _p(b), _p(gamma), _p(beta), M, N, K,
                                alpha, post_scale, act, clamp_lo, clamp_hi, norm, eps,
                                _p(out), _p(aux))
    if rc != 0:
        raise ValueError("unknown activation or row-op code")
    return out, aux


def gate(G: np.ndarray, U: np.ndarray, kind: int, lo: float = 0.0, hi: float = 0.0) -> np.ndarray:
    """act(G) * U elementwise."""
    A = np.array(G, dtype=np.float64, order="C", copy=True)
    U = _c(U)
    assert A.shape == U.shape
    lib().fge_oracle_gate(_p(A), _p(U), A.size, kind, lo, hi)
    return A


def gated_chain(X, W1, W2, b1=None, b2=None, gamma=None, beta=None, *, alpha=1.0, post_scale=1.0,
                act=0, clamp_lo=0.0, clamp_hi=0.0, norm=0, eps=0.0) -> Tuple[np.ndarray, np.ndarray]:
    """rowop(act(post*(alpha*X.W1^T + b1)) * (post*(alpha*X.W2^T + b2))): out and aux as in chain()."""
    X, W1, W2, b1, b2, gamma, beta = (_c(v) for v in (X, W1, W2, b1, b2, gamma, beta))
    M, K = X.shape
    N = W1.shape[0]
    assert W1.shape == (N, K) and W2.shape == (N, K)
    out = np.empty((M, N), dtype=np.float64)
    work = np.empty((M, N), dtype=np.float64)
    aux = np.full(M, np.nan, dtype=np.float64)
    rc = lib().fge_oracle_gated_chain(_p(X), _p(W1), _p(W2), _p(b1), _p(b2), _p(gamma), _p(beta),
                                      M, N, K, alpha, post_scale, act, clamp_lo, clamp_hi, norm, eps,
                                      _p(out), _p(aux), _p(work))
    if rc != 0:
        raise ValueError("unknown activation or row-op code")
    return out, aux
