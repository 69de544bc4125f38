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
        lib.cotten_oracle_normaliser.argtypes = [dp, dp, dp, i, i]
        lib.cotten_oracle_normaliser.restype = None
        lib.cotten_oracle_normaliser_bwd.argtypes = [dp, dp, dp, i, i]
        lib.cotten_oracle_normaliser_bwd.restype = None
        lib.cotten_oracle_scaled_fwd.argtypes = [dp, dp, dp, bp, dp, dp, i, i, i, i, f]
        lib.cotten_oracle_scaled_fwd.restype = None
        lib.cotten_oracle_scaled_bwd.argtypes = [dp, dp, dp, bp, dp, dp, dp, dp, dp, dp, i, i, i, i, f]
        lib.cotten_oracle_scaled_bwd.restype = None
        lib.cotten_oracle_causal_fwd.argtypes = [dp, dp, dp, bp, dp, i, i, i, i, f, f]
        lib.cotten_oracle_causal_fwd.restype = None
        lib.cotten_oracle_causal_bwd.argtypes = [dp, dp, dp, bp, dp, dp, dp, dp, i, i, i, i, f, f]
        lib.cotten_oracle_causal_bwd.restype = None
        lib.cotten_oracle_elu_fwd.argtypes = [dp, dp, dp, bp, dp, i, i, i, i, f]
        lib.cotten_oracle_elu_fwd.restype = None
        lib.cotten_oracle_elu_bwd.argtypes = [dp, dp, dp, bp, dp, dp, dp, dp, i, i, i, i, f]
        lib.cotten_oracle_elu_bwd.restype = None
        lib.cotten_oracle_state.argtypes = [dp, dp, bp, dp, i, i, i, i, f]
        lib.cotten_oracle_state.restype = None
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


def state(K, V, mask=None, eps: float = 1e-6) -> np.ndarray:
    """S[b,h] = Khat^T V under the key mask, [B,H,d,d]: the state of the reordered form."""
    K, V = _f64(K), _f64(V)
    assert K.ndim == 4 and K.shape == V.shape
    B, H, N, d = K.shape
    S = np.empty((B, H, d, d), dtype=np.float64)
    m, mp = _mask_arg(mask, B, N)
    _load().cotten_oracle_state(_ptr(K), _ptr(V), mp, _ptr(S), B, H, N, d, float(eps))
    return S


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


def normaliser(m, n) -> np.ndarray:
    """s[b,h] = n_b ** (-m_h): the learnable normaliser 1/n^m, one exponent per head and one
    n per sequence."""
    m, n = _f64(m), _f64(n)
    assert m.ndim == 1 and n.ndim == 1
    s = np.empty((n.shape[0], m.shape[0]), np.float64)
    _load().cotten_oracle_normaliser(_ptr(m), _ptr(n), _ptr(s), n.shape[0], m.shape[0])
    return s


def normaliser_bwd(dlog_s, n) -> np.ndarray:
    """dm[h] = -sum_b ln(n_b) dlog_s[b,h]."""
    g, n = _f64(dlog_s), _f64(n)
    assert g.ndim == 2 and g.shape[0] == n.shape[0]
    dm = np.empty(g.shape[1], np.float64)
    _load().cotten_oracle_normaliser_bwd(_ptr(g), _ptr(n), _ptr(dm), g.shape[0], g.shape[1])
    return dm


def scaled_fwd(Q, K, V, s, mask=None, eps: float = 1e-6) -> np.ndarray:
    """O with one scalar s[b,h] per slice."""
    Q, K, V, s = _f64(Q), _f64(K), _f64(V), _f64(s)
    B, H, N, d = Q.shape
    assert s.shape == (B, H)
    O = np.empty_like(Q)
    m, mp = _mask_arg(mask, B, N)
    _load().cotten_oracle_scaled_fwd(_ptr(Q), _ptr(K), _ptr(V), mp, _ptr(s), _ptr(O), B, H, N, d,
                                     float(eps))
    return O


def scaled_bwd(Q, K, V, dO, s, mask=None, eps: float = 1e-6):
    """(dQ, dK, dV, dlog_s) with one scalar s[b,h] per slice; dlog_s[b,h] = d loss / d log s[b,h]."""
    Q, K, V, dO, s = _f64(Q), _f64(K), _f64(V), _f64(dO), _f64(s)
    B, H, N, d = Q.shape
    assert s.shape == (B, H)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    dlog = np.empty((B, H), np.float64)
    m, mp = _mask_arg(mask, B, N)
    _load().cotten_oracle_scaled_bwd(_ptr(Q), _ptr(K), _ptr(V), mp, _ptr(s), _ptr(dO), _ptr(dQ),
                                     _ptr(dK), _ptr(dV), _ptr(dlog), B, H, N, d, float(eps))
    return dQ, dK, dV, dlog


def causal_fwd(Q, K, V, mask=None, scale: Optional[float] = None, eps: float = 1e-6):
    """Causal variant from its definition: row i attends the valid keys j <= i."""
    return _fwd("cotten_oracle_causal_fwd", Q, K, V, mask, scale, eps)


def causal_bwd(Q, K, V, dO, mask=None, scale: Optional[float] = None, eps: float = 1e-6):
    """(dQ, dK, dV) of the causal variant, through the N x N matrix."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    B, H, N, d = Q.shape
    s = 1.0 / N if scale is None else float(scale)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    m, mp = _mask_arg(mask, B, N)
    _load().cotten_oracle_causal_bwd(_ptr(Q), _ptr(K), _ptr(V), mp, _ptr(dO), _ptr(dQ), _ptr(dK),
                                     _ptr(dV), B, H, N, d, s, float(eps))
    return dQ, dK, dV


def elu_fwd(Q, K, V, mask=None, scale: Optional[float] = None) -> np.ndarray:
    """O_i = scale * sum_j m_j (phi(q_i) . phi(k_j)) v_j with phi = ELU + 1, all N x N scores formed."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    assert Q.ndim == 4 and Q.shape == K.shape == V.shape
    B, H, N, d = Q.shape
    s = 1.0 / N if scale is None else float(scale)
    O = np.empty_like(Q)
    m, mp = _mask_arg(mask, B, N)
    _load().cotten_oracle_elu_fwd(_ptr(Q), _ptr(K), _ptr(V), mp, _ptr(O), B, H, N, d, s)
    return O


def elu_bwd(Q, K, V, dO, mask=None, scale: Optional[float] = None):
    """(dQ, dK, dV) of elu_fwd for upstream gradient dO, through the N x N scores."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    B, H, N, d = Q.shape
    s = 1.0 / N if scale is None else float(scale)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    m, mp = _mask_arg(mask, B, N)
    _load().cotten_oracle_elu_bwd(_ptr(Q), _ptr(K), _ptr(V), mp, _ptr(dO), _ptr(dQ), _ptr(dK),
                                  _ptr(dV), B, H, N, d, s)
    return dQ, dK, dV
