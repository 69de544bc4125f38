"""256-byte rows on the matrix cores (fp32 d_h = 64; bf16 / fp16 d_h = 128): the state in four
quadrants, the row norm over both halves of a row.  Parity against the fp64 oracle on shapes
that take one workgroup per slice (no reduction of partial states), several workgroups per
slice, ragged tails inside a 64-row round, every kind of mask, both layouts, per-slice scales,
the kept state and d loss / d log(scale)."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2602_06935_amd import binding
from tests.gpu_util import bar_for, check_tensor, rel_l2, to_f64, to_gpu

pytestmark = pytest.mark.gpu

CODE = {"f32": binding.COTTEN_F32, "bf16": binding.COTTEN_BF16, "f16": binding.COTTEN_F16}


def _inputs(seed, dtype, B, H, N, d):
    rng = np.random.default_rng(seed)
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)).astype(np.float32) for _ in range(4))
    Q[0, 0, N // 2] *= 1e-4                     # a tiny row: the epsilon matters
    K[0, 0, N - 1] *= 1e-4
    if dtype != "f32":
        Q, K, V, dO = (to_gpu(x, dtype).float().cpu().numpy() for x in (Q, K, V, dO))
    mask = np.zeros((B, N), np.uint8)
    for b in range(B):
        mask[b, N - int(rng.integers(1, N + 1)):] = 1          # padded at the front
    if B > 1:
        mask[1] = (rng.random(N) < 0.5).astype(np.uint8)        # scattered
        mask[1, 0] = 1
    if B > 2:
        mask[2] = 0                                             # no key at all
    return Q, K, V, dO, mask


@pytest.mark.parametrize("dtype,B,H,N,d", [
    ("bf16", 3, 2, 1, 128), ("bf16", 3, 2, 17, 128), ("bf16", 4, 2, 200, 128),
    ("f16", 3, 2, 130, 128), ("f32", 3, 2, 65, 64), ("f32", 4, 2, 200, 64),
    ("bf16", 300, 2, 70, 128),      # 600 slices: one workgroup per slice, no reduction
    ("f32", 280, 2, 100, 64),
    ("bf16", 2, 2, 3000, 128),      # long sequences cut over many workgroups
    ("f32", 1, 3, 2500, 64),
    ("bf16", 130, 2, 300, 128),     # one launch per direction, tiles streamed (N > 256)
    ("f32", 128, 2, 520, 64),
    ("f16", 100, 1, 200, 128),      # one launch per direction, the backward's tiles kept
    ("bf16", 100, 1, 256, 128),     # the longest sequence the kept backward takes
    ("bf16", 100, 1, 257, 128),     # the shortest it does not
    ("f16", 128, 2, 300, 128),      # one launch, tiles streamed, fp16
    ("f16", 2, 2, 600, 128),        # three launches, workgroups of eight waves, fp16
    ("bf16", 257, 1, 40, 128),      # forward with two slices per workgroup, the last one alone
    ("f32", 129, 3, 90, 64),
    ("bf16", 100, 2, 600, 128),     # three launches, workgroups of four waves (600 of them)
    ("f32", 100, 2, 600, 64),
    ("f16", 100, 2, 600, 128),
])
def test_wide_rows_parity(oracle, dtype, B, H, N, d):
    print(f"[wide rows] {dtype} B={B} H={H} N={N} d={d}", flush=True)
    Q, K, V, dO, mask = _inputs(7300 + N + d + B, dtype, B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.05, eps=1e-6)
    dQ, dK, dV = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=0.05, eps=1e-6)
    O2 = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.05, eps=1e-6)
    g2 = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=0.05, eps=1e-6)
    torch.cuda.synchronize()
    ref_o = oracle.fwd_linear(Q, K, V, mask, scale=0.05, eps=1e-6)
    ref_g = oracle.bwd(Q, K, V, dO, mask, scale=0.05, eps=1e-6)
    bar = bar_for(dtype)
    for n, g, r in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), (ref_o, *ref_g)):
        e = check_tensor(n, to_f64(g), r, bar)
        print(f"[wide rows]   {n}: whole {e['whole']:.2e} slice {e['slice']:.2e} row {e['row']:.2e}", flush=True)
    dead = np.broadcast_to((mask == 0)[:, None, :, None], ref_o.shape)
    assert np.all(to_f64(dK)[dead] == 0.0) and np.all(to_f64(dV)[dead] == 0.0)
    if B > 2:
        assert np.all(to_f64(O)[2] == 0.0)
    assert torch.equal(O, O2) and all(torch.equal(a, c) for a, c in zip((dQ, dK, dV), g2))


@pytest.mark.parametrize("dtype,d,B,H,N", [
    ("bf16", 128, 3, 3, 333), ("f32", 64, 3, 3, 333),    # state, reduction, apply launches
    ("bf16", 128, 45, 2, 120), ("f32", 64, 45, 2, 120),  # one launch, the backward's tiles kept
    ("bf16", 128, 130, 2, 300), ("f32", 64, 130, 2, 300),  # one launch, tiles streamed
])
def test_wide_rows_layout_scales_state_dlog(oracle, dtype, d, B, H, N):
    """[B,N,H,d] layout bit for bit; per-slice scales; the kept state against the oracle's and
    read back by the backward; d loss / d log(scale) = sum_i dO_i . O_i; garbage in masked rows."""
    print(f"[wide rows] layout / scales / state / dlog: {dtype} B={B} H={H} N={N} d={d}", flush=True)
    Q, K, V, dO, mask = _inputs(7999 + d, dtype, B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    ss = torch.rand(B, H, device="cuda") * 0.05 + 0.01
    state = torch.zeros(B, H, d, d, device="cuda")
    dlog = torch.zeros(B, H, device="cuda")
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, slice_scale=ss, saved_state=state)
    grads = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=ss, dlog_scale=dlog)
    grads_kept = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=ss, saved_state=state)
    sw = lambda t: t.permute(0, 2, 1, 3).contiguous()
    O2 = binding.cotten_attn_fwd(sw(tq), sw(tk), sw(tv), tm, slice_scale=ss, layout="bnhd")
    grads2 = binding.cotten_attn_bwd(sw(tq), sw(tk), sw(tv), tm, sw(tg), slice_scale=ss, layout="bnhd")
    # masked rows may hold anything
    tk2, tv2 = tk.clone(), tv.clone()
    deadt = (tm == 0)[:, None, :, None].expand_as(tk2)
    tk2[deadt] = float("nan")
    tv2[deadt] = float("inf")
    O3 = binding.cotten_attn_fwd(tq, tk2, tv2, tm, slice_scale=ss)
    grads3 = binding.cotten_attn_bwd(tq, tk2, tv2, tm, tg, slice_scale=ss)
    torch.cuda.synchronize()
    assert torch.equal(sw(O), O2) and all(torch.equal(sw(a), c) for a, c in zip(grads, grads2))
    assert torch.equal(O, O3) and all(torch.equal(a, c) for a, c in zip(grads, grads3))
    s64 = ss.double().cpu().numpy()
    bar = bar_for(dtype)
    refs = [np.empty(Q.shape) for _ in range(4)]
    ref_dlog = np.empty((B, H))
    for b in range(B):
        for h in range(H):
            sl = (slice(b, b + 1), slice(h, h + 1))
            refs[0][sl] = oracle.fwd_linear(Q[sl], K[sl], V[sl], mask[b:b + 1], scale=s64[b, h])
            for dst, g in zip(refs[1:], oracle.bwd(Q[sl], K[sl], V[sl], dO[sl], mask[b:b + 1], scale=s64[b, h])):
                dst[sl] = g
            ref_dlog[b, h] = float((dO[sl].astype(np.float64) * refs[0][sl]).sum())
    for n, g, r in zip(("O", "dQ", "dK", "dV"), (O, *grads), refs):
        check_tensor(n, to_f64(g), r, bar)
    for n, g, r in zip(("dQ", "dK", "dV"), grads_kept, refs[1:]):
        check_tensor(n + " (kept state)", to_f64(g), r, bar)
    assert rel_l2(dlog.double().cpu().numpy(), ref_dlog) <= 5 * bar
    ref_state = oracle.state(K, V, mask)
    assert rel_l2(state.double().cpu().numpy(), ref_state) <= bar


@pytest.mark.parametrize("dtype,B,H,N,d", [("bf16", 100, 1, 200, 128), ("f32", 128, 2, 300, 64),
                                           ("bf16", 3, 1, 700, 128)])
def test_wide_rows_without_mask(oracle, dtype, B, H, N, d):
    """mask = NULL: every key takes part (kept tiles, streamed tiles, three launches)."""
    print(f"[wide rows] no mask: {dtype} B={B} H={H} N={N} d={d}", flush=True)
    Q, K, V, dO, _ = _inputs(7100 + N + d, dtype, B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    O = binding.cotten_attn_fwd(tq, tk, tv, None, scale=0.03, eps=1e-6)
    grads = binding.cotten_attn_bwd(tq, tk, tv, None, tg, scale=0.03, eps=1e-6)
    torch.cuda.synchronize()
    ref_o = oracle.fwd_linear(Q, K, V, None, scale=0.03, eps=1e-6)
    ref_g = oracle.bwd(Q, K, V, dO, None, scale=0.03, eps=1e-6)
    bar = bar_for(dtype)
    for n, g, r in zip(("O", "dQ", "dK", "dV"), (O, *grads), (ref_o, *ref_g)):
        check_tensor(n, to_f64(g), r, bar)
