"""GPU parity of the causal variant (row i attends the valid keys j <= i) against the fp64
oracle, which states it from the N x N definition (no prefix state)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_06935_amd import binding
from paper_2602_06935_amd.inputs import round_to_bf16, round_to_f16

from gpu_util import bar_for, check_tensor, rel_l2, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def _inputs(seed, dtype, B, H, N, d):
    rng = np.random.default_rng(seed)
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)).astype(np.float32) for _ in range(4))
    if dtype == "bf16":
        Q, K, V, dO = (round_to_bf16(x) for x in (Q, K, V, dO))
    if dtype == "f16":
        Q, K, V, dO = (round_to_f16(x) for x in (Q, K, V, dO))
    mask = (rng.random((B, N)) < 0.7).astype(np.uint8)
    mask[0] = 1
    if B > 1:
        mask[1, : N // 2] = 0           # the first half of the rows sees no key at all
    return Q, K, V, dO, mask


@pytest.mark.parametrize("dtype,d", [("f32", 32), ("f32", 64), ("f32", 16), ("bf16", 64), ("f16", 32)])
@pytest.mark.parametrize("N", [1, 16, 50, 203])
def test_causal_parity(oracle, dtype, d, N):
    B, H = 3, 2
    print(f"[causal] {dtype} d={d} N={N}", flush=True)
    Q, K, V, dO, mask = _inputs(4000 + N + d, dtype, B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.3, causal=True)
    dQ, dK, dV = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=0.3, causal=True)
    torch.cuda.synchronize()
    ref_o = oracle.causal_fwd(Q, K, V, mask, scale=0.3)
    ref_g = oracle.causal_bwd(Q, K, V, dO, mask, scale=0.3)
    bar = bar_for(dtype)
    errs = [rel_l2(to_f64(O), ref_o)] + [rel_l2(to_f64(g), r) for g, r in zip((dQ, dK, dV), ref_g)]
    print("[causal]   " + " ".join(f"{e:.2e}" for e in errs), flush=True)
    assert max(errs) <= bar, errs
    dead = np.broadcast_to((mask == 0)[:, None, :, None], ref_o.shape)
    assert np.all(to_f64(dK)[dead] == 0.0) and np.all(to_f64(dV)[dead] == 0.0)
    if N > 1:
        # rows before the first valid key see nothing
        first = int(np.argmax(mask[1] != 0))
        assert np.all(to_f64(O)[1, :, :first] == 0.0)
    # the last row sees every key: it equals the bidirectional row
    full = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.3)
    torch.cuda.synchronize()
    assert rel_l2(to_f64(O)[:, :, -1], to_f64(full)[:, :, -1]) <= 2 * bar


@pytest.mark.parametrize("dtype,d,N", [("bf16", 64, 300), ("f16", 32, 260), ("bf16", 16, 230),
                                       ("f16", 64, 209), ("f32", 32, 300)])
def test_causal_16bit_beyond_the_resident_limit(oracle, dtype, d, N):
    """Sequences just beyond the 208 rows one workgroup keeps in LDS: two chunks, the second
    short."""
    B, H = 4, 2
    print(f"[causal] long {dtype} d={d} N={N}", flush=True)
    Q, K, V, dO, mask = _inputs(4500 + N + d, dtype, B, H, N, d)
    mask[2] = 0                          # a sequence without any valid key
    mask[3] = 0
    mask[3, N - 37:] = 1                 # left-padded
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.2, causal=True)
    dQ, dK, dV = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=0.2, causal=True)
    O2 = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.2, causal=True)
    g2 = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=0.2, causal=True)
    torch.cuda.synchronize()
    ref_o = oracle.causal_fwd(Q, K, V, mask, scale=0.2)
    ref_g = oracle.causal_bwd(Q, K, V, dO, mask, scale=0.2)
    bar = bar_for(dtype)
    for n, g, r in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), (ref_o, *ref_g)):
        e = check_tensor(n, to_f64(g), r, bar)
        print(f"[causal]   {n}: whole {e['whole']:.2e} slice {e['slice']:.2e} row {e['row']:.2e}", flush=True)
    assert np.all(to_f64(O)[2] == 0.0)
    dead = np.broadcast_to((mask == 0)[:, None, :, None], ref_o.shape)
    assert np.all(to_f64(dK)[dead] == 0.0) and np.all(to_f64(dV)[dead] == 0.0)
    assert torch.equal(O, O2) and all(torch.equal(a, c) for a, c in zip((dQ, dK, dV), g2))


@pytest.mark.parametrize("dtype,B,H,N,d", [
    ("bf16", 3, 2, 417, 64),     # three chunks, the last of one row
    ("bf16", 2, 2, 1000, 64),    # five chunks
    ("f16", 2, 3, 640, 32),      # narrower rows on the same kernels
    ("bf16", 2, 2, 420, 16),
    ("f32", 3, 2, 416, 32),      # two full chunks
    ("f32", 2, 2, 900, 32),
    ("f32", 2, 2, 500, 16),
])
def test_causal_over_several_chunks(oracle, dtype, B, H, N, d):
    """Sequences of more than 208 rows on the matrix cores: 208-row chunks, one workgroup each,
    joined by the states of the chunks before (queries) and after (keys) through the workspace.
    Checked against the N x N oracle, which knows no chunks."""
    print(f"[causal] chunks {dtype} B={B} H={H} N={N} d={d}", flush=True)
    Q, K, V, dO, mask = _inputs(4700 + N + d, dtype, B, H, N, d)
    if B > 2:
        mask[2] = 0
        mask[2, 230:260] = 1             # first chunk without a key, the keys of the second one
        mask[2, N - 3:] = 1              #   seen by every later chunk
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.2, causal=True)
    dQ, dK, dV = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=0.2, causal=True)
    O2 = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.2, causal=True)
    g2 = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=0.2, causal=True)
    torch.cuda.synchronize()
    ref_o = oracle.causal_fwd(Q, K, V, mask, scale=0.2)
    ref_g = oracle.causal_bwd(Q, K, V, dO, mask, scale=0.2)
    bar = bar_for(dtype)
    for n, g, r in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), (ref_o, *ref_g)):
        e = check_tensor(n, to_f64(g), r, bar)
        print(f"[causal]   {n}: whole {e['whole']:.2e} slice {e['slice']:.2e} row {e['row']:.2e}", flush=True)
    dead = np.broadcast_to((mask == 0)[:, None, :, None], ref_o.shape)
    assert np.all(to_f64(dK)[dead] == 0.0) and np.all(to_f64(dV)[dead] == 0.0)
    if B > 2:
        assert np.all(to_f64(O)[2, :, :230] == 0.0)
    assert torch.equal(O, O2) and all(torch.equal(a, c) for a, c in zip((dQ, dK, dV), g2))
    # the last row sees every key: it equals the bidirectional row
    full = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.2)
    torch.cuda.synchronize()
    assert rel_l2(to_f64(O)[:, :, -1], to_f64(full)[:, :, -1]) <= 2 * bar


def test_causal_chunks_layout_scales_workspace(oracle):
    """[B,N,H,d] layout and per-slice scales over several chunks; the caller's own workspace;
    a workspace that is too small is refused."""
    B, H, N, d = 3, 2, 450, 64
    Q, K, V, dO, mask = _inputs(4801, "bf16", B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, "bf16") for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    ss = torch.rand(B, H, device="cuda") * 0.1 + 0.05
    need = binding.cotten_attn_workspace_bytes_ex(B, H, N, d, True, dtype=binding.COTTEN_BF16, causal=True)
    assert need == 2 * B * H * 3 * 64 * 64 * 4
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, slice_scale=ss, causal=True, workspace=ws)
    grads = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=ss, causal=True, workspace=ws)
    sw = lambda t: t.permute(0, 2, 1, 3).contiguous()
    O2 = binding.cotten_attn_fwd(sw(tq), sw(tk), sw(tv), tm, slice_scale=ss, causal=True, layout="bnhd")
    grads2 = binding.cotten_attn_bwd(sw(tq), sw(tk), sw(tv), tm, sw(tg), slice_scale=ss, causal=True,
                                     layout="bnhd")
    torch.cuda.synchronize()
    assert torch.equal(sw(O), O2) and all(torch.equal(sw(a), c) for a, c in zip(grads, grads2))
    s64 = ss.double().cpu().numpy()
    refs = [np.empty(Q.shape) for _ in range(4)]
    for b in range(B):
        for h in range(H):
            sl = (slice(b, b + 1), slice(h, h + 1))
            refs[0][sl] = oracle.causal_fwd(Q[sl], K[sl], V[sl], mask[b:b + 1], scale=s64[b, h])
            for dst, g in zip(refs[1:], oracle.causal_bwd(Q[sl], K[sl], V[sl], dO[sl], mask[b:b + 1],
                                                           scale=s64[b, h])):
                dst[sl] = g
    for n, g, r in zip(("O", "dQ", "dK", "dV"), (O, *grads), refs):
        check_tensor(n, to_f64(g), r, bar_for("bf16"))
    with pytest.raises(binding.CottenError) as e:
        binding.cotten_attn_bwd(tq, tk, tv, tm, tg, causal=True, workspace=ws[: need - 16])
    assert e.value.status == -6
    # the entry point with the static scratch array serves the causal variant as well
    out = [torch.empty_like(tq) for _ in range(3)]
    binding.cotten_attn_bwd(tq, tk, tv, tm, tg, *out, slice_scale=ss, causal=True, static_scratch=True)
    torch.cuda.synchronize()
    assert all(torch.equal(a, c) for a, c in zip(grads, out))


def test_causal_layout_scales_and_errors(oracle):
    B, H, N, d = 4, 2, 70, 32
    Q, K, V, dO, mask = _inputs(4999, "f32", B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, "f32") for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    ss = torch.rand(B, H, device="cuda") + 0.1
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, slice_scale=ss, causal=True)
    grads = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=ss, causal=True)
    sw = lambda t: t.permute(0, 2, 1, 3).contiguous()
    O2 = binding.cotten_attn_fwd(sw(tq), sw(tk), sw(tv), tm, slice_scale=ss, causal=True, layout="bnhd")
    grads2 = binding.cotten_attn_bwd(sw(tq), sw(tk), sw(tv), tm, sw(tg), slice_scale=ss, causal=True,
                                     layout="bnhd")
    torch.cuda.synchronize()
    assert torch.equal(sw(O), O2) and all(torch.equal(sw(a), c) for a, c in zip(grads, grads2))
    # per-slice scales: slice by slice against the oracle with that scale
    s64 = ss.double().cpu().numpy()
    for b, h in ((0, 0), (3, 1)):
        sl = (slice(b, b + 1), slice(h, h + 1))
        ref = oracle.causal_fwd(Q[sl], K[sl], V[sl], mask[b:b + 1], scale=s64[b, h])
        assert rel_l2(to_f64(O)[sl], ref) <= 1e-5
    # what is not available is refused on the host
    with pytest.raises(binding.CottenError) as e:
        binding.cotten_attn_bwd(tq, tk, tv, tm, tg, causal=True, dlog_scale=torch.empty(B, H, device="cuda"))
    assert e.value.status == -7
    big = torch.zeros(1, 1, 8, 128, device="cuda")
    with pytest.raises(binding.CottenError) as e:
        binding.cotten_attn_fwd(big, big, big, None, causal=True)
    assert e.value.status == -3
