"""The state S = Khat^T V handed from the forward call to the backward call
(cotten_params.saved_state): the forward writes it, the backward reads it instead of walking
K, V a first time.  Checked on every kernel family: the written state against the oracle's,
the gradients of the state-reading backward against the oracle and against the rebuilding
backward."""
import numpy as np
import pytest
import torch

from paper_2602_06935_amd import binding
from paper_2602_06935_amd.inputs import round_to_bf16, round_to_f16

from gpu_util import bar_for, check_tensor, rel_l2, to_f64, to_gpu

pytestmark = pytest.mark.gpu

# (dtype, B, H, N, d): which kernels serve the shape
CASES = [
    ("bf16", 9, 4, 200, 64),     # slice kept in LDS, 13 tiles
    ("bf16", 70, 4, 200, 64),    # the same with workgroups that take two slices
    ("bf16", 5, 2, 100, 64),     # 7 tiles
    ("f16", 5, 2, 208, 32),      # narrower state on the same kernels
    ("bf16", 3, 2, 61, 16),
    ("bf16", 64, 4, 180, 64),    # forward on the fused kernel that keeps its tiles, backward in LDS
    ("f32", 6, 2, 200, 32),      # one workgroup per slice, tiles kept in registers
    ("f32", 5, 2, 130, 16),
    ("f32", 130, 2, 300, 32),    # one workgroup per slice, streaming
    ("bf16", 66, 4, 520, 64),
    ("f32", 2, 2, 1030, 32),     # sequence cut over several workgroups
    ("bf16", 3, 2, 3000, 64),
    ("f16", 2, 2, 1030, 32),
    ("f32", 2, 2, 150, 64),      # 256-byte rows: state written, backward rebuilds it
    ("f32", 2, 2, 150, 128),     # 512-byte rows: the same
]


def _inputs(seed, dtype, B, H, N, d):
    rng = np.random.default_rng(seed)
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)).astype(np.float32) for _ in range(4))
    if dtype == "bf16":
        Q, K, V, dO = (round_to_bf16(x) for x in (Q, K, V, dO))
    if dtype == "f16":
        Q, K, V, dO = (round_to_f16(x) for x in (Q, K, V, dO))
    mask = np.zeros((B, N), np.uint8)
    for b in range(B):
        if b % 3 == 0:
            mask[b, N - int(rng.integers(1, N + 1)):] = 1     # left-padded
        elif b % 3 == 1:
            mask[b] = rng.random(N) < 0.5                     # scattered
        else:
            mask[b, : int(rng.integers(1, N + 1))] = 1        # right-padded
    if B > 1:
        mask[1] = 0                                           # no valid key at all
    return Q, K, V, dO, mask


@pytest.mark.parametrize("dtype,B,H,N,d", CASES)
def test_saved_state(oracle, dtype, B, H, N, d):
    print(f"[saved] {dtype} B={B} H={H} N={N} d={d}", flush=True)
    Q, K, V, dO, mask = _inputs(1234 + N + d, dtype, B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    S = torch.full((B, H, d, d), float("nan"), device="cuda")
    scale = 0.5 / N
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=scale, saved_state=S)
    O_plain = binding.cotten_attn_fwd(tq, tk, tv, tm, scale=scale)
    torch.cuda.synchronize()
    # the forward result does not depend on whether the state is kept
    assert torch.equal(O, O_plain)
    # the kept state is the oracle's state, to the rounding of the operands
    S_ref = oracle.state(K, V, mask)
    S_got = S.double().cpu().numpy()
    assert np.isfinite(S_got).all()
    e = rel_l2(S_got, S_ref)
    print(f"[saved]   state rel L2 {e:.2e}", flush=True)
    assert e <= bar_for(dtype)
    if B > 1:
        assert np.all(S_got[1] == 0.0)

    with_state = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=scale, saved_state=S)
    rebuilt = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=scale)
    again = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, scale=scale, saved_state=S)
    torch.cuda.synchronize()
    refs = oracle.bwd(Q, K, V, dO, mask, scale=scale)
    bar = bar_for(dtype)
    for n, g, r, other, rep in zip(("dQ", "dK", "dV"), with_state, refs, rebuilt, again):
        res = check_tensor(n, to_f64(g), r, bar)
        print(f"[saved]   {n}: whole {res['whole']:.2e} slice {res['slice']:.2e} row {res['row']:.2e}"
              f"  vs rebuilding call {rel_l2(to_f64(g), to_f64(other)):.2e}", flush=True)
        assert torch.equal(g, rep), f"{n}: not repeatable bit for bit"
    dead = np.broadcast_to((mask == 0)[:, None, :, None], Q.shape)
    assert np.all(to_f64(with_state[1])[dead] == 0.0) and np.all(to_f64(with_state[2])[dead] == 0.0)


def test_saved_state_with_layout_scales_and_dlog(oracle):
    """[B,N,H,d] layout and per-slice scales through the state-reading backward; a call that also
    wants d loss / d log(scale) still answers correctly (it rebuilds the state)."""
    B, H, N, d = 6, 4, 200, 64
    Q, K, V, dO, mask = _inputs(99, "bf16", B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, "bf16") for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    ss = (torch.rand(B, H, device="cuda") + 0.5) / N
    S = torch.empty(B, H, d, d, device="cuda")
    sw = lambda t: t.permute(0, 2, 1, 3).contiguous()
    binding.cotten_attn_fwd(tq, tk, tv, tm, slice_scale=ss, saved_state=S)
    S2 = torch.empty_like(S)
    binding.cotten_attn_fwd(sw(tq), sw(tk), sw(tv), tm, slice_scale=ss, saved_state=S2, layout="bnhd")
    g1 = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=ss, saved_state=S)
    g2 = binding.cotten_attn_bwd(sw(tq), sw(tk), sw(tv), tm, sw(tg), slice_scale=ss, saved_state=S2,
                                 layout="bnhd")
    dlog = torch.empty(B, H, device="cuda")
    g3 = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=ss, saved_state=S, dlog_scale=dlog)
    dlog_ref = torch.empty(B, H, device="cuda")
    g4 = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=ss, dlog_scale=dlog_ref)
    torch.cuda.synchronize()
    assert torch.equal(S, S2)
    for a, b in zip(g1, g2):
        assert torch.equal(sw(a), b)
    assert torch.equal(dlog, dlog_ref) and all(torch.equal(a, b) for a, b in zip(g3, g4))
    refs = oracle.scaled_bwd(Q, K, V, dO, ss.double().cpu().numpy(), mask)
    for n, g, r in zip(("dQ", "dK", "dV"), g1, refs[:3]):
        check_tensor(n, to_f64(g), r, bar_for("bf16"))
