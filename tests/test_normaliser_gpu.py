"""GPU parity of the learnable normaliser 1/n^m (scaled CosineAttention): per-slice scales in
both directions, d loss / d log(scale) from the backward call, and the exponent gradient,
against the fp64 oracle, on every kernel family (resident, fused, split, wide rows)."""
import numpy as np
import pytest
import torch

from paper_2602_06935_amd import binding
from paper_2602_06935_amd.inputs import round_to_bf16, round_to_f16

from gpu_util import bar_for, rel_l2, to_f64, to_gpu

pytestmark = pytest.mark.gpu

# (label, dtype, B, H, N, d): one shape per kernel family and element format
CASES = [
    ("resident bf16", "bf16", 5, 4, 200, 64),
    ("resident fp16", "f16", 5, 4, 120, 64),
    ("split fp16", "f16", 2, 2, 1030, 64),
    ("fused f32", "f32", 5, 2, 200, 32),
    ("fused bf16 (N above the resident limit)", "bf16", 70, 4, 230, 64),
    ("split bf16", "bf16", 2, 2, 1030, 64),
    ("split f32", "f32", 2, 2, 1030, 32),
    ("half-width rows f32 d=16 (fused)", "f32", 3, 2, 70, 16),
    ("half-width rows bf16 d=32 (resident)", "bf16", 3, 2, 150, 32),
    ("half-width rows bf16 d=32 (split)", "bf16", 2, 2, 1030, 32),
    ("256-byte rows f32 d=64", "f32", 3, 2, 70, 64),
    ("quarter-width rows bf16 d=16 (split)", "bf16", 2, 2, 300, 16),
    ("256-byte rows f32 d=64, several splits", "f32", 2, 2, 300, 64),
    ("512-byte rows f32 d=128", "f32", 3, 2, 70, 128),
    ("256-byte rows bf16 d=128, one launch", "bf16", 45, 2, 100, 128),
]


def _inputs(seed, dtype, B, H, N, d):
    rng = np.random.default_rng(seed)
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)).astype(np.float32) for _ in range(4))
    if dtype == "bf16":
        Q, K, V, dO = (round_to_bf16(x) for x in (Q, K, V, dO))
    if dtype == "f16":
        Q, K, V, dO = (round_to_f16(x) for x in (Q, K, V, dO))
    lengths = rng.integers(1, N + 1, size=B)
    lengths[0] = N
    mask = np.zeros((B, N), np.uint8)
    for b, L in enumerate(lengths):
        mask[b, N - L:] = 1
    m = rng.uniform(0.4, 1.4, size=H).astype(np.float32)
    return Q, K, V, dO, mask, lengths.astype(np.int32), m


@pytest.mark.parametrize("label,dtype,B,H,N,d", CASES)
def test_learnable_normaliser_end_to_end(oracle, label, dtype, B, H, N, d):
    print(f"[normaliser] {label}: {dtype} B={B} H={H} N={N} d={d}", flush=True)
    Q, K, V, dO, mask, lengths, m = _inputs(900 + N + d, dtype, B, H, N, d)
    bar = bar_for(dtype)
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    tn = torch.from_numpy(lengths).cuda()
    tmexp = torch.from_numpy(m).cuda()

    # s[b,h] = n_b^(-m_h) with n = valid length
    s_gpu = binding.cotten_normaliser_fwd(tmexp, tn, B, N)
    s_ref = oracle.normaliser(m.astype(np.float64), lengths.astype(np.float64))
    assert rel_l2(s_gpu.double().cpu().numpy(), s_ref) <= 2e-6
    # n = NULL: the padded length
    s_pad = binding.cotten_normaliser_fwd(tmexp, None, B, N)
    assert rel_l2(s_pad.double().cpu().numpy(),
                  oracle.normaliser(m.astype(np.float64), np.full(B, float(N)))) <= 2e-6

    # both directions with the scales the GPU made (the oracle gets the same fp32 values)
    s_used = s_gpu.double().cpu().numpy()
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, slice_scale=s_gpu)
    dlog = torch.empty(B, H, device="cuda", dtype=torch.float32)
    dQ, dK, dV = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=s_gpu, dlog_scale=dlog)
    torch.cuda.synchronize()
    ref_o = oracle.scaled_fwd(Q, K, V, s_used, mask)
    ref_q, ref_k, ref_v, ref_dlog = oracle.scaled_bwd(Q, K, V, dO, s_used, mask)
    errs = {"O": rel_l2(to_f64(O), ref_o), "dQ": rel_l2(to_f64(dQ), ref_q),
            "dK": rel_l2(to_f64(dK), ref_k), "dV": rel_l2(to_f64(dV), ref_v),
            "dlog": rel_l2(dlog.double().cpu().numpy(), ref_dlog)}
    print("[normaliser]   " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    for k, v in errs.items():
        assert v <= bar, f"{k}: rel L2 {v:.3e} above {bar:.0e}"

    # exponent gradient: dm_h = -sum_b ln(n_b) dlog[b,h]
    dm = binding.cotten_normaliser_bwd(dlog, tn, N)
    torch.cuda.synchronize()
    ref_dm = oracle.normaliser_bwd(ref_dlog, lengths.astype(np.float64))
    e = rel_l2(dm.double().cpu().numpy(), ref_dm)
    print(f"[normaliser]   dm={e:.2e}", flush=True)
    assert e <= 5 * bar          # a sum with cancellation over the batch

    # same bits on a second run; a scalar scale equals a constant slice_scale bit for bit
    dlog2 = torch.empty_like(dlog)
    again = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=s_gpu, dlog_scale=dlog2)
    torch.cuda.synchronize()
    assert torch.equal(dlog, dlog2) and all(torch.equal(a, c) for a, c in zip(again, (dQ, dK, dV)))
    const = torch.full((B, H), 0.25, device="cuda", dtype=torch.float32)
    assert torch.equal(binding.cotten_attn_fwd(tq, tk, tv, tm, scale=0.25),
                       binding.cotten_attn_fwd(tq, tk, tv, tm, slice_scale=const))


def test_normaliser_argument_errors():
    m = torch.ones(2, device="cuda")
    with pytest.raises(ValueError):
        binding.cotten_normaliser_fwd(m, torch.ones(3, device="cuda"), 3, 10)   # n must be int32
    lib = binding.load_library()
    assert lib.cotten_normaliser_fwd(None, None, None, 1, 1, 1, None) == -1
    assert lib.cotten_normaliser_bwd(None, None, None, 1, 1, 1, None) == -1
    assert lib.cotten_normaliser_fwd(m.data_ptr(), None, m.data_ptr(), 0, 1, 1, None) == -2


@pytest.mark.parametrize("label,dtype,B,H,N,d", CASES)
def test_bnhd_layout_equals_bhnd_bit_for_bit(label, dtype, B, H, N, d):
    """[B,N,H,d_h] tensors (the per-head view of a d_model-wide projection): the same kernels
    with other strides, so every output must equal the [B,H,N,d_h] call bit for bit."""
    print(f"[layout] {label}: {dtype} B={B} H={H} N={N} d={d}", flush=True)
    Q, K, V, dO, mask, lengths, m = _inputs(1900 + N + d, dtype, B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, dtype) for x in (Q, K, V, dO))
    tm = torch.from_numpy(mask).cuda()
    ss = torch.rand(B, H, device="cuda") + 0.1
    dlog = torch.empty(B, H, device="cuda")
    O = binding.cotten_attn_fwd(tq, tk, tv, tm, slice_scale=ss)
    grads = binding.cotten_attn_bwd(tq, tk, tv, tm, tg, slice_scale=ss, dlog_scale=dlog)
    sw = lambda t: t.permute(0, 2, 1, 3).contiguous()      # [B,H,N,d] -> [B,N,H,d]
    dlog2 = torch.empty_like(dlog)
    O2 = binding.cotten_attn_fwd(sw(tq), sw(tk), sw(tv), tm, slice_scale=ss, layout="bnhd")
    grads2 = binding.cotten_attn_bwd(sw(tq), sw(tk), sw(tv), tm, sw(tg), slice_scale=ss,
                                     dlog_scale=dlog2, layout="bnhd")
    torch.cuda.synchronize()
    assert O2.shape == (B, N, H, d)
    assert torch.equal(sw(O), O2) and torch.equal(dlog, dlog2)
    for a, c in zip(grads, grads2):
        assert torch.equal(sw(a), c)


def test_layout_argument_errors():
    lib = binding.load_library()
    t = torch.zeros(1, 1, 16, 32, device="cuda")
    prm = binding.CottenParams()
    prm.dtype, prm.scale, prm.eps, prm.layout = 0, 0.0, -1.0, 7
    import ctypes
    rc = lib.cotten_attn_fwd_ex(t.data_ptr(), t.data_ptr(), t.data_ptr(), None, t.data_ptr(),
                                1, 1, 16, 32, None, ctypes.byref(prm))
    assert rc == -2
    with pytest.raises(ValueError):
        binding.cotten_attn_fwd(t, t, t, None, layout="nhbd")


def test_autograd_wrapper(oracle):
    """The autograd plumbing: gradients of sum(O * dO) with respect to Q, K, V and the
    per-slice scales equal what the backward entry point returns and what the oracle says."""
    from paper_2602_06935_amd.autograd import cosine_attention
    B, H, N, d = 4, 2, 120, 32
    Q, K, V, dO, mask, lengths, m = _inputs(77, "f32", B, H, N, d)
    tq, tk, tv, tg = (to_gpu(x, "f32").requires_grad_(i < 3) for i, x in enumerate((Q, K, V, dO)))
    tm = torch.from_numpy(mask).cuda()
    ss = (torch.rand(B, H, device="cuda") + 0.2).requires_grad_(True)
    O = cosine_attention(tq, tk, tv, tm, slice_scale=ss)
    (O * tg).sum().backward()
    torch.cuda.synchronize()
    s64 = ss.detach().double().cpu().numpy()
    ref = oracle.scaled_bwd(Q, K, V, dO, s64, mask)
    for got, want in zip((tq.grad, tk.grad, tv.grad), ref[:3]):
        assert rel_l2(to_f64(got), want) <= 1e-5
    assert rel_l2(ss.grad.double().cpu().numpy(), ref[3] / s64) <= 1e-5
