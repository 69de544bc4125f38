"""Seeded synthetic inputs for the cosine-attention hot path.

This module is shared by the CPU oracle's tests, the GPU parity tests and the
benchmark.  It holds NO arithmetic of the method itself (no normalisation, no
contraction): it only draws random tensors, lengths and masks with the shapes
and value distributions of recommendation batches (padded user histories of
length N in {50, 200, 4096}, d_model 64 = 2x32 and 256 = 4x64, the sweeps of
the paper's Tables 2 and 3), and rounds values to the bf16 grid when a workload
uses 16-bit I/O.  Everything is a pure function of (workload name, seed).

Layout of every tensor: [B, H, N, d_h] row-major; mask: [B, N] uint8, 1 = valid
key.  Padding is on the left: valid positions are N-L_b .. N-1.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "Batch", "make_batch", "round_to_bf16",
    "bf16_bits_from_f32", "f32_from_bf16_bits", "left_pad_mask",
]


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d_h: int
    dtype: str            # "f32" or "bf16" (I/O element type)
    sigma: float          # std-dev of Q, K, V
    lengths: str          # "full" | "uniform" | "geometric"
    len_lo: int
    len_hi: int
    geom_mean: float = 0.0
    tiny_row_frac: float = 0.0   # fraction of Q rows and of K rows scaled by 1e-4
    backward: bool = True
    description: str = ""


# The five configurations of the benchmark contract, in order, and one more shape.
WORKLOADS = {
    "cfg1": Workload("cfg1", 4, 2, 50, 32, "f32", 1.0, "full", 50, 50,
                     backward=False,
                     description="fwd only, fp32, no padding, scale 1/N"),
    "cfg2": Workload("cfg2", 256, 2, 50, 32, "f32", 1.0, "uniform", 3, 50,
                     description="fwd+bwd fp32, lengths U{3..50}, left-padded"),
    "cfg3": Workload("cfg3", 256, 2, 200, 32, "f32", 1.0, "geometric", 5, 200,
                     geom_mean=120.0,
                     description="fwd+bwd fp32, lengths clip(Geom(mean 120),5,200)"),
    "cfg4": Workload("cfg4", 128, 4, 200, 64, "bf16", 0.5, "uniform", 5, 200,
                     tiny_row_frac=0.01,
                     description="fwd+bwd bf16 I/O, lengths U{5..200}, 1% tiny rows"),
    "cfg5": Workload("cfg5", 16, 4, 4096, 64, "bf16", 1.0, "uniform", 1024, 4096,
                     description="long-history stress, bf16 I/O, lengths U{1024..4096}"),
    # Beside the contract: the largest embedding size of the paper's sweep (64, 128, 256) with the
    # two heads of a BERT4Rec layer, i.e. 256-byte rows under 16-bit I/O.
    "emb256": Workload("emb256", 128, 2, 200, 128, "bf16", 0.5, "uniform", 5, 200,
                       description="embedding size 256, two heads: d_h = 128, bf16 I/O, lengths U{5..200}"),
}


@dataclass
class Batch:
    workload: Workload
    seed: int
    Q: np.ndarray              # float32 [B,H,N,d]; on the bf16 grid if dtype == "bf16"
    K: np.ndarray
    V: np.ndarray
    dO: np.ndarray
    mask: Optional[np.ndarray]  # uint8 [B,N] or None (all valid)
    lengths: np.ndarray         # int64 [B]
    scale: float                # scalar normaliser s (1/N)
    eps: float                  # epsilon inside the square root of the row norm

    @property
    def valid_fraction(self) -> float:
        return float(self.lengths.sum()) / float(self.workload.B * self.workload.N)


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of finite float32 values to bf16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array whose every value is exactly representable in bf16 (RNE)."""
    return f32_from_bf16_bits(bf16_bits_from_f32(x)).reshape(np.shape(x))


def round_to_f16(x: np.ndarray) -> np.ndarray:
    """float32 array whose every value is exactly representable in IEEE half (RNE)."""
    return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def left_pad_mask(lengths: np.ndarray, N: int) -> np.ndarray:
    """[B,N] uint8 mask with the last lengths[b] positions of row b set to 1."""
    pos = np.arange(N, dtype=np.int64)[None, :]
    return (pos >= (N - np.asarray(lengths, dtype=np.int64)[:, None])).astype(np.uint8)


def _draw_lengths(w: Workload, rng: np.random.Generator, B: int, N: int) -> np.ndarray:
    lo, hi = min(w.len_lo, N), min(w.len_hi, N)
    if w.lengths == "full":
        return np.full(B, N, dtype=np.int64)
    if w.lengths == "uniform":
        return rng.integers(lo, hi + 1, size=B, dtype=np.int64)
    if w.lengths == "geometric":
        g = rng.geometric(1.0 / w.geom_mean, size=B).astype(np.int64)   # support {1,2,...}
        return np.clip(g, lo, hi)
    raise ValueError(w.lengths)


def make_batch(name: str, seed: int = 0, *, B: Optional[int] = None,
               H: Optional[int] = None, N: Optional[int] = None,
               eps: float = 1e-6) -> Batch:
    """Draw one batch of workload `name`; B/H/N may be overridden for small test cases."""
    w = WORKLOADS[name]
    B = w.B if B is None else B
    H = w.H if H is None else H
    N = w.N if N is None else N
    d = w.d_h
    rng = np.random.default_rng([seed, sum(map(ord, name))])
    shape = (B, H, N, d)
    Q = (rng.standard_normal(shape, dtype=np.float32) * np.float32(w.sigma))
    K = (rng.standard_normal(shape, dtype=np.float32) * np.float32(w.sigma))
    V = (rng.standard_normal(shape, dtype=np.float32) * np.float32(w.sigma))
    dO = rng.standard_normal(shape, dtype=np.float32)
    lengths = _draw_lengths(w, rng, B, N)
    if w.tiny_row_frac > 0.0:
        # independently chosen rows of Q and of K shrunk so the norm epsilon matters
        tq = rng.random((B, H, N)) < w.tiny_row_frac
        tk = rng.random((B, H, N)) < w.tiny_row_frac
        Q[tq] *= np.float32(1e-4)
        K[tk] *= np.float32(1e-4)
    if w.dtype == "bf16":
        Q, K, V, dO = (round_to_bf16(t) for t in (Q, K, V, dO))
    mask = None if w.lengths == "full" else left_pad_mask(lengths, N)
    return Batch(w, seed, Q, K, V, dO, mask, lengths, 1.0 / N, eps)
