"""Helpers of the GPU parity tests: move a seeded batch to the GPU, call the library
through its binding (the C ABI), bring results back as float64."""
from __future__ import annotations

import numpy as np
import torch

from paper_2602_06935_amd import binding

FP32_BAR = 1e-5     # relative L2 error allowed for fp32 I/O
BF16_BAR = 2e-2     # relative L2 error allowed for bf16 I/O with fp32 accumulation
F16_BAR = 2.5e-3    # fp16 I/O: the bf16 bar scaled by the ratio of the unit roundoffs (2^-11 / 2^-8)


def rel_l2(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    den = float(np.linalg.norm(ref))
    num = float(np.linalg.norm(got - ref))
    return num / den if den > 0 else num


def bar_for(dtype: str) -> float:
    return {"f32": FP32_BAR, "bf16": BF16_BAR, "f16": F16_BAR}[dtype]


def to_gpu(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    if dtype == "bf16":
        return t.to(torch.bfloat16).contiguous()
    if dtype == "f16":
        return t.to(torch.float16).contiguous()
    return t


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def gpu_fwd(Q, K, V, mask, dtype="f32", scale=None, eps=None, **kw):
    tq, tk, tv = (to_gpu(x, dtype) for x in (Q, K, V))
    tm = None if mask is None else torch.from_numpy(np.ascontiguousarray(mask, dtype=np.uint8)).cuda()
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=scale, eps=eps, **kw)
    torch.cuda.synchronize()
    return to_f64(O)


def gpu_bwd(Q, K, V, dO, mask, dtype="f32", scale=None, eps=None, **kw):
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    tm = None if mask is None else torch.from_numpy(np.ascontiguousarray(mask, dtype=np.uint8)).cuda()
    dQ, dK, dV = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=scale, eps=eps, **kw)
    torch.cuda.synchronize()
    return to_f64(dQ), to_f64(dK), to_f64(dV)
