"""Thin ctypes binding of libcotten_attn.so (same names as include/cotten_attn.h).

Argument marshalling only: every arithmetic step runs in the HIP kernels.  torch is
used for device memory (`torch.empty`, `.data_ptr()`) and for the current stream.
There is no CPU fallback: if the library cannot be loaded, or a tensor is not on
the GPU, the call raises.

The library allocates nothing.  Shapes that need a workspace (long sequences cut over
several workgroups) get one from here when the caller passes none: a `torch.empty` buffer
kept per (device, stream), grown when a larger shape arrives; while a stream is being
captured into a graph the buffer is a fresh temporary from the graph's own pool instead.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcotten_attn.so")

COTTEN_F32 = 0
COTTEN_BF16 = 1
COTTEN_F16 = 2
COTTEN_BHND = 0
COTTEN_BNHD = 1
COTTEN_MAP_COSINE = 0
COTTEN_MAP_ELU1 = 1

EXPORTS = (
    "cotten_attn_fwd", "cotten_attn_bwd", "cotten_attn_fwd_ex", "cotten_attn_bwd_ex",
    "cotten_attn_workspace_bytes", "cotten_status_string",
    "cotten_normaliser_fwd", "cotten_normaliser_bwd", "cotten_attn_bwd_static",
    "cotten_attn_workspace_bytes_ex",
)


class CottenParams(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int), ("scale", ctypes.c_float), ("eps", ctypes.c_float),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("slice_scale", ctypes.c_void_p), ("dlog_scale", ctypes.c_void_p),
                ("layout", ctypes.c_int), ("causal", ctypes.c_int),
                ("saved_state", ctypes.c_void_p), ("feature_map", ctypes.c_int)]


class CottenError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"cotten_attn status {status}: {message}")
        self.status = status


_lib = None


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """dlopen the in-tree library; compile it first only when no build exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, ip = ctypes.c_void_p, ctypes.c_int
    lib.cotten_attn_fwd.argtypes = [vp, vp, vp, vp, vp, ip, ip, ip, ip, vp]
    lib.cotten_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, vp]
    lib.cotten_attn_fwd_ex.argtypes = lib.cotten_attn_fwd.argtypes + [ctypes.POINTER(CottenParams)]
    lib.cotten_attn_bwd_ex.argtypes = lib.cotten_attn_bwd.argtypes + [ctypes.POINTER(CottenParams)]
    lib.cotten_attn_bwd_static.argtypes = lib.cotten_attn_bwd_ex.argtypes
    for f in (lib.cotten_attn_fwd, lib.cotten_attn_bwd, lib.cotten_attn_fwd_ex, lib.cotten_attn_bwd_ex,
              lib.cotten_attn_bwd_static):
        f.restype = ctypes.c_int
    lib.cotten_attn_workspace_bytes.argtypes = [ip, ip, ip, ip, ip, ip]
    lib.cotten_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.cotten_attn_workspace_bytes_ex.argtypes = [ip, ip, ip, ip, ip, ctypes.POINTER(CottenParams)]
    lib.cotten_attn_workspace_bytes_ex.restype = ctypes.c_size_t
    lib.cotten_normaliser_fwd.argtypes = [vp, vp, vp, ip, ip, ip, vp]
    lib.cotten_normaliser_bwd.argtypes = [vp, vp, vp, ip, ip, ip, vp]
    lib.cotten_normaliser_fwd.restype = lib.cotten_normaliser_bwd.restype = ctypes.c_int
    lib.cotten_status_string.argtypes = [ip]
    lib.cotten_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def cotten_status_string(status: int) -> str:
    return load_library().cotten_status_string(int(status)).decode()


def cotten_attn_workspace_bytes(B: int, H: int, N: int, d_h: int, dtype: int, is_bwd: bool) -> int:
    return int(load_library().cotten_attn_workspace_bytes(B, H, N, d_h, dtype, int(bool(is_bwd))))


def cotten_attn_workspace_bytes_ex(B: int, H: int, N: int, d_h: int, is_bwd: bool, *, dtype: int,
                                   causal: bool = False) -> int:
    """Workspace bytes of a call with these options (the causal variant has needs of its own)."""
    prm = CottenParams()
    prm.dtype = dtype
    prm.causal = 1 if causal else 0
    return int(load_library().cotten_attn_workspace_bytes_ex(B, H, N, d_h, int(bool(is_bwd)),
                                                             ctypes.byref(prm)))


def _check(status: int) -> None:
    if status != 0:
        raise CottenError(status, cotten_status_string(status))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return COTTEN_F32
    if t.dtype == torch.bfloat16:
        return COTTEN_BF16
    if t.dtype == torch.float16:
        return COTTEN_F16
    raise TypeError(f"unsupported I/O dtype {t.dtype}")


def _prep(name: str, t: torch.Tensor, like: Optional[torch.Tensor] = None) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor (there is no CPU path)")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous [B,H,N,d_h]")
    if like is not None and (t.shape != like.shape or t.dtype != like.dtype or t.device != like.device):
        raise ValueError(f"{name} must match Q in shape, dtype and device")
    return t


def _mask_ptr(mask: Optional[torch.Tensor], B: int, N: int, dev) -> Optional[int]:
    if mask is None:
        return None
    if mask.dtype != torch.uint8 or tuple(mask.shape) != (B, N) or not mask.is_contiguous() or mask.device != dev:
        raise ValueError("mask must be a contiguous uint8 [B,N] tensor on the same device")
    return mask.data_ptr()


def _f32_vector(name: str, t: Optional[torch.Tensor], numel: int, dev) -> Optional[int]:
    if t is None:
        return None
    if t.dtype != torch.float32 or t.numel() != numel or not t.is_contiguous() or t.device != dev:
        raise ValueError(f"{name} must be a contiguous float32 GPU tensor of {numel} elements")
    return t.data_ptr()


def _dims(Q: torch.Tensor, layout: str) -> Tuple[int, int, int, int]:
    """(B, H, N, d_h) of a tensor stored as `layout` ("bhnd" or "bnhd")."""
    if Q.dim() != 4:
        raise ValueError("expected a 4-d tensor")
    if layout == "bhnd":
        B, H, N, d = Q.shape
    elif layout == "bnhd":
        B, N, H, d = Q.shape
    else:
        raise ValueError("layout must be 'bhnd' or 'bnhd'")
    return B, H, N, d


def _params(Q: torch.Tensor, scale, eps, workspace: Optional[torch.Tensor],
            slice_scale: Optional[torch.Tensor] = None,
            dlog_scale: Optional[torch.Tensor] = None, layout: str = "bhnd",
            causal: bool = False, saved_state: Optional[torch.Tensor] = None,
            feature_map: str = "cosine") -> CottenParams:
    p = CottenParams()
    p.causal = int(bool(causal))
    if feature_map not in ("cosine", "elu1"):
        raise ValueError("feature_map must be 'cosine' or 'elu1'")
    p.feature_map = COTTEN_MAP_ELU1 if feature_map == "elu1" else COTTEN_MAP_COSINE
    B, H, _, d = _dims(Q, layout)
    p.saved_state = _f32_vector("saved_state", saved_state, B * H * d * d, Q.device)
    p.layout = COTTEN_BNHD if layout == "bnhd" else COTTEN_BHND
    slices = B * H
    p.slice_scale = _f32_vector("slice_scale", slice_scale, slices, Q.device)
    p.dlog_scale = _f32_vector("dlog_scale", dlog_scale, slices, Q.device)
    p.dtype = _dtype_code(Q)
    p.scale = 0.0 if scale is None else float(scale)
    p.eps = -1.0 if eps is None else float(eps)
    if workspace is not None:
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous GPU tensor")
        p.workspace = workspace.data_ptr()
        p.workspace_bytes = workspace.numel() * workspace.element_size()
    else:
        p.workspace = None
        p.workspace_bytes = 0
    return p


_workspaces = {}    # (device index, stream handle) -> uint8 tensor
_retired = []       # outgrown buffers: work already enqueued may still use them


def _workspace(Q: torch.Tensor, dims, is_bwd: bool, stream_handle: int,
               given: Optional[torch.Tensor], causal: bool = False) -> Optional[torch.Tensor]:
    """The workspace tensor of a call: the caller's, or one of this module's."""
    if given is not None:
        return given
    B, H, N, d = dims
    need = cotten_attn_workspace_bytes_ex(B, H, N, d, is_bwd, dtype=_dtype_code(Q), causal=causal)
    if need == 0:
        return None
    with torch.cuda.device(Q.device):
        if torch.cuda.is_current_stream_capturing():
            return torch.empty(need, dtype=torch.uint8, device=Q.device)
        key = (Q.device.index, stream_handle)
        ws = _workspaces.get(key)
        if ws is None or ws.numel() < need:
            if ws is not None:
                _retired.append(ws)
            ws = torch.empty(max(need, 1 << 20), dtype=torch.uint8, device=Q.device)
            _workspaces[key] = ws
        return ws


def _stream_handle(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def cotten_attn_fwd(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                    mask: Optional[torch.Tensor], O: Optional[torch.Tensor] = None, *,
                    scale: Optional[float] = None, eps: Optional[float] = None,
                    stream=None, workspace: Optional[torch.Tensor] = None,
                    slice_scale: Optional[torch.Tensor] = None,
                    layout: str = "bhnd", causal: bool = False,
                    saved_state: Optional[torch.Tensor] = None,
                    feature_map: str = "cosine") -> torch.Tensor:
    """O = scale * Qhat (Khat^T V) under the key mask; enqueues on the stream and returns O.
    `slice_scale` ([B,H] float32) gives every slice its own scale instead of `scale`;
    `layout` "bnhd" means all tensors are [B,N,H,d_h] instead of [B,H,N,d_h];
    `saved_state` ([B,H,d_h,d_h] float32) receives the state S of every slice for the
    backward call."""
    lib = load_library()
    Q = _prep("Q", Q); K = _prep("K", K, Q); V = _prep("V", V, Q)
    B, H, N, d = _dims(Q, layout)
    if O is None:
        O = torch.empty_like(Q)
    _prep("O", O, Q)
    handle = _stream_handle(stream)
    workspace = _workspace(Q, (B, H, N, d), False, handle, workspace, causal)
    prm = _params(Q, scale, eps, workspace, slice_scale, None, layout, causal, saved_state, feature_map)
    with torch.cuda.device(Q.device):
        _check(lib.cotten_attn_fwd_ex(Q.data_ptr(), K.data_ptr(), V.data_ptr(),
                                      _mask_ptr(mask, B, N, Q.device), O.data_ptr(),
                                      B, H, N, d, handle, ctypes.byref(prm)))
    return O


def cotten_attn_bwd(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                    mask: Optional[torch.Tensor], dO: torch.Tensor,
                    dQ: Optional[torch.Tensor] = None, dK: Optional[torch.Tensor] = None,
                    dV: Optional[torch.Tensor] = None, *, scale: Optional[float] = None,
                    eps: Optional[float] = None, stream=None,
                    workspace: Optional[torch.Tensor] = None,
                    slice_scale: Optional[torch.Tensor] = None,
                    dlog_scale: Optional[torch.Tensor] = None, layout: str = "bhnd",
                    causal: bool = False, static_scratch: bool = False,
                    saved_state: Optional[torch.Tensor] = None, feature_map: str = "cosine"
                    ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """(dQ, dK, dV) for upstream gradient dO; enqueues on the stream and returns the tensors.
    `slice_scale` as in the forward; `dlog_scale` ([B,H] float32), when given, receives
    d loss / d log(scale) of every slice.  With `static_scratch` the call goes to
    cotten_attn_bwd_static: no workspace is passed or allocated, the library's own static
    scratch array serves (the output tensors must then be given, nothing is allocated here).
    `saved_state`: the state the forward call of the same inputs wrote; read instead of being
    rebuilt from K, V."""
    lib = load_library()
    Q = _prep("Q", Q); K = _prep("K", K, Q); V = _prep("V", V, Q); dO = _prep("dO", dO, Q)
    B, H, N, d = _dims(Q, layout)
    dQ = torch.empty_like(Q) if dQ is None else _prep("dQ", dQ, Q)
    dK = torch.empty_like(Q) if dK is None else _prep("dK", dK, Q)
    dV = torch.empty_like(Q) if dV is None else _prep("dV", dV, Q)
    handle = _stream_handle(stream)
    if static_scratch:
        workspace = None
    else:
        workspace = _workspace(Q, (B, H, N, d), True, handle, workspace, causal)
    prm = _params(Q, scale, eps, workspace, slice_scale, dlog_scale, layout, causal, saved_state,
                  feature_map)
    entry = lib.cotten_attn_bwd_static if static_scratch else lib.cotten_attn_bwd_ex
    with torch.cuda.device(Q.device):
        _check(entry(Q.data_ptr(), K.data_ptr(), V.data_ptr(),
                     _mask_ptr(mask, B, N, Q.device), dO.data_ptr(),
                     dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(),
                     B, H, N, d, handle, ctypes.byref(prm)))
    return dQ, dK, dV


def _lengths_ptr(n: Optional[torch.Tensor], B: int, dev) -> Optional[int]:
    if n is None:
        return None
    if n.dtype != torch.int32 or n.numel() != B or not n.is_contiguous() or n.device != dev:
        raise ValueError("n must be a contiguous int32 GPU tensor of B elements")
    return n.data_ptr()


def cotten_normaliser_fwd(m: torch.Tensor, n: Optional[torch.Tensor], B: int, N: int,
                          slice_scale: Optional[torch.Tensor] = None, *, stream=None) -> torch.Tensor:
    """slice_scale[b,h] = n_b ** (-m_h) (n = None: the padded length N for every sequence)."""
    lib = load_library()
    if not m.is_cuda or m.dtype != torch.float32 or not m.is_contiguous() or m.dim() != 1:
        raise ValueError("m must be a contiguous float32 GPU vector [H]")
    H = m.numel()
    if slice_scale is None:
        slice_scale = torch.empty(B, H, device=m.device, dtype=torch.float32)
    with torch.cuda.device(m.device):
        _check(lib.cotten_normaliser_fwd(m.data_ptr(), _lengths_ptr(n, B, m.device),
                                         _f32_vector("slice_scale", slice_scale, B * H, m.device),
                                         B, H, N, _stream_handle(stream)))
    return slice_scale


def cotten_normaliser_bwd(dlog_scale: torch.Tensor, n: Optional[torch.Tensor], N: int,
                          dm: Optional[torch.Tensor] = None, *, stream=None) -> torch.Tensor:
    """dm[h] = -sum_b ln(n_b) * dlog_scale[b,h]."""
    lib = load_library()
    if not dlog_scale.is_cuda or dlog_scale.dim() != 2:
        raise ValueError("dlog_scale must be a GPU tensor [B,H]")
    B, H = dlog_scale.shape
    dev = dlog_scale.device
    if dm is None:
        dm = torch.empty(H, device=dev, dtype=torch.float32)
    with torch.cuda.device(dev):
        _check(lib.cotten_normaliser_bwd(_f32_vector("dlog_scale", dlog_scale, B * H, dev),
                                         _lengths_ptr(n, B, dev), _f32_vector("dm", dm, H, dev),
                                         B, H, N, _stream_handle(stream)))
    return dm
