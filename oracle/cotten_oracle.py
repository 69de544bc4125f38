"""ctypes front-end of the fp64 CPU oracle in cotten_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg; the product path never touches it.  The wrapper
only converts inputs to contiguous float64 and forwards them; all arithmetic is
in the C file, which states the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cotten_oracle.c")
_LIB = os.path.join(_HERE, "libcotten_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP over slices)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        bp = ctypes.c_void_p
        i, f = ctypes.c_int, ctypes.c_double
        for name in ("cotten_oracle_fwd_quadratic", "cotten_oracle_fwd_linear"):
            fn = getattr(lib, name)
            fn.argtypes = [dp, dp, dp, bp, dp, i, i, i, i, f, f]
            fn.restype = None
        lib.cotten_oracle_bwd.argtypes = [dp, dp, dp, bp, dp, dp, dp, dp, i, i, i, i, f, f]
        lib.cotten_oracle_bwd.restype = None
        lib.cotten_oracle_threads.argtypes = []
        lib.cotten_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().cotten_oracle_threads())


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=np.float64)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _mask_arg(mask, B: int, N: int):
    if mask is None:
        return None, None
    m = np.ascontiguousarray(np.asarray(mask), dtype=np.uint8)
    assert m.shape == (B, N), (m.shape, (B, N))
    return m, ctypes.c_void_p(m.ctypes.data)


def _fwd(fn_name: str, Q, K, V, mask, scale: Optional[float], eps: float) -> np.ndarray:
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    assert Q.ndim == 4 and Q.shape == K.shape == V.shape
    B, H, N, d = Q.shape
    s = 1.0 / N if scale is None else float(scale)
    O = np.empty_like(Q)
    m, mp = _mask_arg(mask, B, N)
    getattr(_load(), fn_name)(_ptr(Q), _ptr(K), _ptr(V), mp, _ptr(O), B, H, N, d, s, float(eps))
    return O


def fwd_quadratic(Q, K, V, mask=None, scale: Optional[float] = None, eps: float = 1e-6):
    """O = scale * (Qhat Khat^T, masked keys removed) V, all N x N cosines formed."""
    return _fwd("cotten_oracle_fwd_quadratic", Q, K, V, mask, scale, eps)


def fwd_linear(Q, K, V, mask=None, scale: Optional[float] = None, eps: float = 1e-6):
    """O = scale * Qhat (Khat^T V): the reordered form with the d x d state."""
    return _fwd("cotten_oracle_fwd_linear", Q, K, V, mask, scale, eps)


def bwd(Q, K, V, dO, mask=None, scale: Optional[float] = None,
        eps: float = 1e-6) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(dQ, dK, dV) of the reordered form for upstream gradient dO."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    assert Q.ndim == 4 and Q.shape == K.shape == V.shape == dO.shape
    B, H, N, d = Q.shape
    s = 1.0 / N if scale is None else float(scale)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    m, mp = _mask_arg(mask, B, N)
    _load().cotten_oracle_bwd(_ptr(Q), _ptr(K), _ptr(V), mp, _ptr(dO), _ptr(dQ), _ptr(dK),
                              _ptr(dV), B, H, N, d, s, float(eps))
    return dQ, dK, dV
