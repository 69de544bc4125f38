"""Seeded sweep over the launch plan's decision boundaries: sequence lengths around every tile,
round, kept-tile and residency limit, slice counts around the thresholds at which a sequence is
(not) cut or a backward changes its launch structure, every element type and head dimension,
the cosine and ELU + 1 maps and the causal variant, both layouts, scalar and per-slice scales,
and every kind of mask.  Each case is compared with the fp64 oracle element by element (whole
tensor, per slice, per row) and run twice for a bit-for-bit check."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2602_06935_amd import binding
from tests.gpu_util import bar_for, check_tensor, rel_l2, to_f64, to_gpu

pytestmark = pytest.mark.gpu

LENGTHS = (1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 160, 161, 207, 208, 209, 255, 256, 257, 300,
           511, 512, 513, 1000, 2049)
SLICES = (1, 2, 7, 64, 85, 86, 255, 256, 257, 300, 512)
HEAD_DIMS = {"f32": (16, 32, 64, 128), "bf16": (16, 32, 64, 128), "f16": (16, 32, 64, 128)}
MAX_ROWS = 90_000          # B * H * N of a case (the oracle stays within seconds)
MAX_ROWS_NXN = 400         # N of a case whose oracle forms all N x N scores
N_CASES = 72


def _cases():
    rng = np.random.default_rng(20260227)
    out = []
    while len(out) < N_CASES:
        dtype = ("f32", "bf16", "f16")[int(rng.integers(3))]
        d = int(rng.choice(HEAD_DIMS[dtype]))
        mode = ("cosine", "cosine", "elu1", "causal")[int(rng.integers(4))]
        if mode == "causal" and d == 128:
            continue            # refused
        N = int(rng.choice(LENGTHS))
        BH = int(rng.choice(SLICES))
        if BH * N > MAX_ROWS or (mode != "cosine" and N > MAX_ROWS_NXN):
            continue
        H = int(rng.choice([h for h in (1, 2, 3, 4) if BH % h == 0]))
        out.append(dict(dtype=dtype, d=d, mode=mode, N=N, B=BH // H, H=H,
                        layout=("bhnd", "bnhd")[int(rng.integers(2))],
                        mask=("none", "left", "scattered", "left+empty")[int(rng.integers(4))],
                        per_slice=bool(rng.integers(2)), seed=int(rng.integers(1 << 30))))
    return out


CASES = _cases()


def _id(c):
    return (f"{c['dtype']}-{c['mode']}-B{c['B']}-H{c['H']}-N{c['N']}-d{c['d']}-{c['layout']}-"
            f"{c['mask']}-{'slice' if c['per_slice'] else 'scalar'}")


def _mask(rng, kind, B, N):
    if kind == "none":
        return None
    m = np.zeros((B, N), np.uint8)
    for b in range(B):
        if kind == "scattered":
            m[b] = rng.random(N) < 0.6
            m[b, int(rng.integers(N))] = 1
        else:
            m[b, N - int(rng.integers(1, N + 1)):] = 1
    if kind == "left+empty":
        m[int(rng.integers(B))] = 0
    return m


@pytest.mark.parametrize("c", CASES, ids=_id)
def test_plan_boundaries(oracle, c):
    print(f"[boundaries] {_id(c)} seed={c['seed']}", flush=True)
    dtype, d, B, H, N = c["dtype"], c["d"], c["B"], c["H"], c["N"]
    rng = np.random.default_rng(c["seed"])
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)).astype(np.float32) for _ in range(4))
    if dtype != "f32":
        Q, K, V, dO = (to_gpu(x, dtype).float().cpu().numpy() for x in (Q, K, V, dO))
    mask = _mask(rng, c["mask"], B, N)
    s = rng.uniform(0.01, 0.06, size=(B, H)) if c["per_slice"] else np.full((B, H), 0.04)
    s = s.astype(np.float32)
    kw = dict(layout=c["layout"], eps=1e-6)
    if c["per_slice"]:
        kw["slice_scale"] = torch.from_numpy(s).cuda()
    else:
        kw["scale"] = float(s[0, 0])
    if c["mode"] == "elu1":
        kw["feature_map"] = "elu1"
    if c["mode"] == "causal":
        kw["causal"] = True
    lay = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if c["layout"] == "bnhd" else (lambda t: t)
    tq, tk, tv, tg = (lay(to_gpu(x, dtype)) for x in (Q, K, V, dO))
    tm = None if mask is None else torch.from_numpy(mask).cuda()
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, **kw)
    grads = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, **kw)
    O2 = binding.cotten_attn_fwd(tq, tk, tv, tm, **kw)
    grads2 = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, **kw)
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and all(torch.equal(a, b) for a, b in zip(grads, grads2))

    # the oracle takes one scale per call: slice by slice where the scales differ
    refs = [np.empty(Q.shape) for _ in range(4)]
    groups = [(slice(b, b + 1), slice(h, h + 1)) for b in range(B) for h in range(H)] \
        if c["per_slice"] else [(slice(0, B), slice(0, H))]
    for sl in groups:
        sc = float(s[sl][0, 0])
        mk = None if mask is None else mask[sl[0]]
        q, k, v, g = Q[sl], K[sl], V[sl], dO[sl]
        if c["mode"] == "cosine":
            refs[0][sl] = oracle.fwd_linear(q, k, v, mk, scale=sc, eps=1e-6)
            r = oracle.bwd(q, k, v, g, mk, scale=sc, eps=1e-6)
        elif c["mode"] == "elu1":
            refs[0][sl] = oracle.elu_fwd(q, k, v, mk, scale=sc)
            r = oracle.elu_bwd(q, k, v, g, mk, scale=sc)
        else:
            refs[0][sl] = oracle.causal_fwd(q, k, v, mk, scale=sc, eps=1e-6)
            r = oracle.causal_bwd(q, k, v, g, mk, scale=sc, eps=1e-6)
        for dst, x in zip(refs[1:], r[:3]):
            dst[sl] = x
    bar = bar_for(dtype)
    for n, got, ref in zip(("O", "dQ", "dK", "dV"), (O, *grads), refs):
        e = check_tensor(n, to_f64(lay(got) if c["layout"] == "bnhd" else got), ref, bar,
                         few_terms=c["mode"] == "causal")
        print(f"[boundaries]   {n}: whole {e['whole']:.2e} slice {e['slice']:.2e} row {e['row']:.2e}",
              flush=True)
    if mask is not None:
        dead = np.broadcast_to((mask == 0)[:, None, :, None], Q.shape)
        for got in grads[1:]:
            g64 = to_f64(lay(got) if c["layout"] == "bnhd" else got)
            assert np.all(g64[dead] == 0.0), "masked rows of dK, dV must be exact zeros"
