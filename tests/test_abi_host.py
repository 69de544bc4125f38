"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before any device work."""
import ctypes
import os
import re

import pytest

from paper_2602_06935_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cotten_attn.h")


@pytest.fixture(scope="module")
def lib():
    return binding.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cotten_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    seen = set()
    for code in range(0, -10, -1):
        s = binding.cotten_status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 10
    assert binding.cotten_status_string(-99) == "unknown status"


def _fwd(lib, Q=0x1000, K=0x2000, V=0x3000, mask=None, O=0x4000, B=2, H=2, N=8, d=32, prm=None):
    if prm is None:
        return lib.cotten_attn_fwd(Q, K, V, mask, O, B, H, N, d, None)
    return lib.cotten_attn_fwd_ex(Q, K, V, mask, O, B, H, N, d, None, ctypes.byref(prm))


def _bwd(lib, Q=0x1000, K=0x2000, V=0x3000, dO=0x4000, dQ=0x5000, dK=0x6000, dV=0x7000,
         B=2, H=2, N=8, d=32):
    return lib.cotten_attn_bwd(Q, K, V, None, dO, dQ, dK, dV, B, H, N, d, None)


def test_validation_errors_touch_no_device(lib):
    assert _fwd(lib, Q=None) == -1
    assert _fwd(lib, O=None) == -1
    assert _bwd(lib, dO=None) == -1
    assert _bwd(lib, dK=None) == -1
    assert lib.cotten_attn_fwd_ex(0x1000, 0x2000, 0x3000, None, 0x4000, 1, 1, 8, 32, None, None) == -1
    assert _fwd(lib, B=0) == -2
    assert _fwd(lib, N=-5) == -2
    assert _bwd(lib, H=0) == -2
    assert _fwd(lib, d=48) == -3
    assert _fwd(lib, d=256) == -3
    assert _fwd(lib, d=96) == -3
    assert _bwd(lib, d=0) == -3
    assert _fwd(lib, K=0x2004) == -5
    assert _bwd(lib, dV=0x7008) == -5
    p = binding.CottenParams(7, 0.0, -1.0, None, 0)
    assert _fwd(lib, prm=p) == -4
    p = binding.CottenParams(binding.COTTEN_BF16, float("nan"), -1.0, None, 0)
    assert _fwd(lib, prm=p) == -7
    p = binding.CottenParams(binding.COTTEN_F32, 0.0, float("inf"), None, 0)
    assert _fwd(lib, prm=p) == -7
    # layout must be one of the two enumerators
    p = binding.CottenParams(binding.COTTEN_F32, 0.0, -1.0, None, 0, None, None, 5)
    assert _fwd(lib, prm=p) == -2
    # rows of a slice are addressed with 31-bit byte offsets: 2^24 rows of 128 bytes do not
    # fit, nor do 2^22 rows that lie 8 heads x 128 bytes apart in the [B,N,H,d] layout
    assert _fwd(lib, N=1 << 24) == -2
    p = binding.CottenParams(binding.COTTEN_F32, 0.0, -1.0, None, 0, None, None, binding.COTTEN_BNHD)
    assert _fwd(lib, H=8, N=1 << 22, prm=p) == -2
    # the causal variant: flag must be 0 or 1, d_h at most 64
    p = binding.CottenParams(binding.COTTEN_F32, 0.0, -1.0, None, 0, None, None, 0, 2)
    assert _fwd(lib, prm=p) == -7
    p = binding.CottenParams(binding.COTTEN_F32, 0.0, -1.0, None, 0, None, None, 0, 1)
    assert _fwd(lib, d=128, prm=p) == -3
    # the feature map: one of the two enumerators, not with causal
    # (positional: ..., layout, causal, saved_state, feature_map)
    p = binding.CottenParams(binding.COTTEN_F32, 0.0, -1.0, None, 0, None, None, 0, 0, None, 2)
    assert _fwd(lib, prm=p) == -7
    p = binding.CottenParams(binding.COTTEN_F32, 0.0, -1.0, None, 0, None, None, 0, 1, None, 1)
    assert _fwd(lib, prm=p) == -7
    # a saved state must be 16-byte aligned like every other tensor
    p = binding.CottenParams(binding.COTTEN_F32, 0.0, -1.0, None, 0, None, None, 0, 0, 0x9004, 0)
    assert _fwd(lib, prm=p) == -5
    # the normaliser entry points validate on the host as well
    assert lib.cotten_normaliser_fwd(None, None, 0x1000, 4, 2, 50, None) == -1
    assert lib.cotten_normaliser_fwd(0x1000, None, None, 4, 2, 50, None) == -1
    assert lib.cotten_normaliser_bwd(0x1000, None, None, 4, 2, 50, None) == -1
    assert lib.cotten_normaliser_bwd(0x1000, None, 0x2000, 0, 2, 50, None) == -2


def test_workspace_rules(lib):
    f = binding.cotten_attn_workspace_bytes
    assert f(0, 2, 50, 32, 0, False) == 0 and f(4, 2, 50, 48, 0, False) == 0
    for (B, H, N, d, dt) in [(256, 2, 50, 32, 0), (256, 2, 200, 32, 0), (128, 4, 200, 64, 1),
                             (16, 4, 4096, 64, 1), (1, 1, 1 << 20, 64, 1)]:
        fw, bw = f(B, H, N, d, dt, False), f(B, H, N, d, dt, True)
        assert bw <= 2 * max(fw, 1) + 2 * B * H * d * d * 4
        # only d x d states, a bounded number of them: independent of N once N is long
        assert bw <= 2 * (2 * B * H + 2049) * d * d * 4
    # a caller-provided workspace that is too small is refused on the host
    need = f(16, 4, 4096, 64, 1, True)
    if need > 16:
        p = binding.CottenParams(binding.COTTEN_BF16, 0.0, -1.0, 0x10000, need - 16)
        assert lib.cotten_attn_bwd_ex(0x1000, 0x2000, 0x3000, None, 0x4000, 0x5000, 0x6000, 0x7000,
                                      16, 4, 4096, 64, None, ctypes.byref(p)) == -6
        p = binding.CottenParams(binding.COTTEN_BF16, 0.0, -1.0, 0x10004, need)
        assert lib.cotten_attn_bwd_ex(0x1000, 0x2000, 0x3000, None, 0x4000, 0x5000, 0x6000, 0x7000,
                                      16, 4, 4096, 64, None, ctypes.byref(p)) == -5


def test_causal_workspace_rules(lib):
    """The causal variant passes one d x d state per 208-row chunk and slice through the
    workspace (two in the backward call) once a sequence has more than one chunk; the sizing
    function that looks at the params says so, and a call without it is refused on the host."""
    f = binding.cotten_attn_workspace_bytes_ex
    BF, F32 = binding.COTTEN_BF16, binding.COTTEN_F32
    assert f(4, 2, 208, 64, True, dtype=BF, causal=True) == 0
    assert f(4, 2, 209, 64, False, dtype=BF, causal=True) == 4 * 2 * 2 * 64 * 64 * 4
    assert f(4, 2, 209, 64, True, dtype=BF, causal=True) == 2 * 4 * 2 * 2 * 64 * 64 * 4
    assert f(4, 2, 1000, 16, True, dtype=BF, causal=True) == 2 * 4 * 2 * 5 * 64 * 64 * 4   # padded states
    assert f(3, 2, 4096, 32, False, dtype=F32, causal=True) == 3 * 2 * 20 * 32 * 32 * 4
    assert f(3, 2, 4096, 64, True, dtype=F32, causal=True) == 0          # vector-ALU scan: none
    assert f(3, 2, 4096, 128, True, dtype=F32, causal=True) == 0         # not available at all
    # without the causal flag it is the plain function
    for args in [(16, 4, 4096, 64, BF), (256, 2, 200, 32, F32)]:
        for bwd in (False, True):
            assert f(*args[:4], bwd, dtype=args[4]) == binding.cotten_attn_workspace_bytes(*args, bwd)
    assert lib.cotten_attn_workspace_bytes_ex(4, 2, 300, 64, 1, None) == 0
    ptrs = (0x1000, 0x2000, 0x3000, None, 0x4000, 0x5000, 0x6000, 0x7000)
    need = f(4, 2, 300, 64, True, dtype=BF, causal=True)
    p = binding.CottenParams(BF, 0.0, -1.0, None, 0)
    p.causal = 1
    assert lib.cotten_attn_bwd_ex(*ptrs, 4, 2, 300, 64, None, ctypes.byref(p)) == -6
    assert lib.cotten_attn_fwd_ex(*ptrs[:5], 4, 2, 300, 64, None, ctypes.byref(p)) == -6
    p.workspace, p.workspace_bytes = 0x10000, need - 4
    assert lib.cotten_attn_bwd_ex(*ptrs, 4, 2, 300, 64, None, ctypes.byref(p)) == -6


def test_library_never_allocates_a_workspace(lib):
    """A shape that needs a workspace and comes without one is refused on the host, before any
    device work: with params->workspace NULL, and through the plain entry points, which have
    no way to pass one.  (Runs without a GPU: the pointers are never dereferenced.)"""
    f = binding.cotten_attn_workspace_bytes
    ptrs = (0x1000, 0x2000, 0x3000, None, 0x4000, 0x5000, 0x6000, 0x7000)
    for bwd in (False, True):
        assert f(16, 4, 4096, 64, binding.COTTEN_BF16, bwd) > 0      # cfg5's shape
        p = binding.CottenParams(binding.COTTEN_BF16, 0.0, -1.0, None, 0)
        if bwd:
            assert lib.cotten_attn_bwd_ex(*ptrs, 16, 4, 4096, 64, None, ctypes.byref(p)) == -6
        else:
            assert lib.cotten_attn_fwd_ex(*ptrs[:5], 16, 4, 4096, 64, None, ctypes.byref(p)) == -6
        # the same length in fp32 with d_h = 32 through the plain entry points
        assert f(16, 4, 4096, 32, binding.COTTEN_F32, bwd) > 0
    assert lib.cotten_attn_fwd(*ptrs[:5], 16, 4, 4096, 32, None) == -6
    assert lib.cotten_attn_bwd(*ptrs, 16, 4, 4096, 32, None) == -6


def test_static_scratch_entry_point_checks_on_the_host(lib):
    """cotten_attn_bwd_static validates like cotten_attn_bwd_ex and refuses, before any device
    work, a call whose partial states do not fit its static scratch array."""
    ptrs = (0x1000, 0x2000, 0x3000, None, 0x4000, 0x5000, 0x6000, 0x7000)
    p = binding.CottenParams(binding.COTTEN_BF16, 0.0, -1.0, None, 0)
    assert lib.cotten_attn_bwd_static(*ptrs, 2, 2, 64, 48, None, ctypes.byref(p)) == -3
    assert lib.cotten_attn_bwd_static(*ptrs, 0, 2, 64, 64, None, ctypes.byref(p)) == -2
    assert lib.cotten_attn_bwd_static(*ptrs, 2, 2, 64, 64, None, None) == -1
    assert binding.cotten_attn_workspace_bytes(1, 200, 50000, 64, binding.COTTEN_BF16, True) > (32 << 20)
    assert lib.cotten_attn_bwd_static(*ptrs, 1, 200, 50000, 64, None, ctypes.byref(p)) == -9


def test_sources_hold_no_allocation_or_synchronisation():
    """The boundary's contract: the library never allocates, frees or synchronises."""
    csrc = os.path.join(ROOT, "paper_2602_06935_amd", "csrc")
    banned = re.compile(r"\b(hipMalloc\w*|hipFree\w*|hipDeviceSynchronize|hipStreamSynchronize|"
                        r"hipHostMalloc|hipExtMallocWithFlags)\b")
    for name in sorted(os.listdir(csrc)):
        text = open(os.path.join(csrc, name)).read()
        text = re.sub(r"//.*", "", text)
        assert not banned.search(text), name


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 1, 8, 32)
    with pytest.raises(ValueError):
        binding.cotten_attn_fwd(x, x, x, None)
