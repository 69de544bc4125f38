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


# Finer bounds behind the whole-tensor figure, so that a few bad rows or one bad slice cannot
# hide in a large tensor: every slice (b,h) on its own stays within the bar, and every row
# within ROW_FACTOR times the bar.  A row's error is taken relative to its own norm, but not
# to less than ROW_FLOOR times the root-mean-square row norm of its slice, and a slice's
# relative to its own norm, but not to less than SLICE_FLOOR times the root-mean-square slice
# norm of the tensor: results that come out small by cancellation (a gradient nearly parallel
# to its unit row; a one-key slice whose only cosine is near zero) carry the absolute
# rounding error of ordinary ones.
# Sequences of fewer than SHORT_ROWS rows consist of so few cosines that a whole slice can
# cancel (N = 1: O is one cosine times v): their slices are held to the row bound and their
# rows are floored by the root-mean-square row norm of the whole tensor.
ROW_FACTOR = 4.0
ROW_FLOOR = 0.25
SLICE_FLOOR = 0.25
SHORT_ROWS = 8


def check_tensor(name: str, got: np.ndarray, ref: np.ndarray, bar: float,
                 few_terms: bool = False) -> dict:
    """Whole-tensor, per-slice and per-row relative L2 errors of a [B,H,N,d] result against
    the oracle; asserts all three bounds and returns the figures.  `few_terms`: rows and slices
    may consist of a single cosine whatever N is (the causal variant: the first valid row attends
    one key, and a left-padded sequence with one key has one non-zero row) - held as short
    sequences are."""
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape and got.ndim == 4
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    diff2 = ((got - ref) ** 2).sum(axis=-1)          # [B,H,N]
    ref2 = (ref ** 2).sum(axis=-1)
    whole = float(np.sqrt(diff2.sum() / ref2.sum())) if ref2.sum() > 0 else float(np.sqrt(diff2.sum()))
    sl_num, sl_den = np.sqrt(diff2.sum(axis=-1)), np.sqrt(ref2.sum(axis=-1))     # [B,H]
    zero = sl_den == 0
    assert np.all(sl_num[zero] == 0), f"{name}: a slice that must be zero is not"
    sl_floor = SLICE_FLOOR * float(np.sqrt((sl_den ** 2).mean()))
    per_slice = np.where(zero, 0.0, sl_num / np.maximum(np.where(zero, 1.0, sl_den), sl_floor))
    short = few_terms or got.shape[2] < SHORT_ROWS
    if not short:
        rms_row = np.sqrt(ref2.mean(axis=-1, keepdims=True))                      # [B,H,1]
    else:
        rms_row = np.sqrt(ref2.mean())
    den = np.maximum(np.sqrt(ref2), ROW_FLOOR * rms_row)
    per_row = np.where(den > 0, np.sqrt(diff2) / np.where(den > 0, den, 1.0), 0.0)
    out = {"whole": whole, "slice": float(per_slice.max()), "row": float(per_row.max())}
    assert whole <= bar, f"{name}: rel L2 {whole:.3e} above {bar:.0e}"
    worst = np.unravel_index(np.argmax(per_slice), per_slice.shape)
    slice_bar = ROW_FACTOR * bar if short else bar
    assert out["slice"] <= slice_bar, \
        f"{name}: slice {worst} rel L2 {out['slice']:.3e} above {slice_bar:.0e}"
    worst = np.unravel_index(np.argmax(per_row), per_row.shape)
    assert out["row"] <= ROW_FACTOR * bar, \
        f"{name}: row {worst} error {out['row']:.3e} above {ROW_FACTOR * bar:.0e}"
    return out


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
