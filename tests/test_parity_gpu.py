"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle on the
same seeded inputs.  Bars: relative L2 error per output tensor <= 1e-5 for fp32 I/O and
<= 2e-2 for bf16 I/O with fp32 accumulation."""
import numpy as np
import pytest
import torch

from paper_2602_06935_amd import binding
from paper_2602_06935_amd.inputs import WORKLOADS, make_batch, round_to_bf16, round_to_f16

from gpu_util import FP32_BAR, bar_for, check_tensor, gpu_bwd, gpu_fwd, rel_l2, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _check_batch(oracle, b, fwd=True, bwd=True, label=""):
    w = b.workload
    bar = bar_for(w.dtype)
    errs = {}
    results = []
    if fwd:
        ref = oracle.fwd_linear(b.Q, b.K, b.V, b.mask, scale=b.scale, eps=b.eps)
        got = gpu_fwd(b.Q, b.K, b.V, b.mask, w.dtype, scale=b.scale, eps=b.eps)
        results.append(("O", got, ref))
    if bwd:
        refs = oracle.bwd(b.Q, b.K, b.V, b.dO, b.mask, scale=b.scale, eps=b.eps)
        gots = gpu_bwd(b.Q, b.K, b.V, b.dO, b.mask, w.dtype, scale=b.scale, eps=b.eps)
        for n, g, r in zip(("dQ", "dK", "dV"), gots, refs):
            results.append((n, g, r))
            if b.mask is not None and n in ("dK", "dV"):
                dead = np.broadcast_to((b.mask == 0)[:, None, :, None], g.shape)
                assert np.all(g[dead] == 0.0), f"{n}: masked rows must be exact zeros"
    _say(f"[parity] {label or w.name} seed={b.seed} shape={b.Q.shape} {w.dtype}")
    for n, g, r in results:
        errs[n] = check_tensor(n, g, r, bar)
        _say(f"[parity]   {n}: whole {errs[n]['whole']:.2e}  worst slice {errs[n]['slice']:.2e}"
             f"  worst row {errs[n]['row']:.2e}")
    return errs


# ------------------------------------------------------------- the five workloads

@pytest.mark.parametrize("seed", [0, 42, 123])
def test_cfg1_forward_full_size(oracle, seed):
    b = make_batch("cfg1", seed)
    _check_batch(oracle, b, fwd=True, bwd=False)
    # the plain entry point (fp32, scale 1/N, eps 1e-6) through its own symbol
    lib = binding.load_library()
    tq, tk, tv = (to_gpu(x, "f32") for x in (b.Q, b.K, b.V))
    O = torch.empty_like(tq)
    rc = lib.cotten_attn_fwd(tq.data_ptr(), tk.data_ptr(), tv.data_ptr(), None, O.data_ptr(),
                             4, 2, 50, 32, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert rc == 0
    assert rel_l2(to_f64(O), oracle.fwd_quadratic(b.Q, b.K, b.V, None, scale=1 / 50, eps=1e-6)) <= FP32_BAR


@pytest.mark.parametrize("name,seed", [("cfg2", 0), ("cfg2", 42), ("cfg3", 0), ("cfg3", 123),
                                       ("cfg4", 0), ("cfg4", 42), ("emb256", 0), ("emb256", 42)])
def test_workloads_full_size(oracle, name, seed):
    _check_batch(oracle, make_batch(name, seed))


def test_cfg4_tiny_rows_reported_separately(oracle):
    b = make_batch("cfg4", 7)
    ref = oracle.bwd(b.Q, b.K, b.V, b.dO, b.mask, scale=b.scale, eps=b.eps)
    got = gpu_bwd(b.Q, b.K, b.V, b.dO, b.mask, "bf16", scale=b.scale, eps=b.eps)
    for name, X, g, r in (("dQ", b.Q, got[0], ref[0]), ("dK", b.K, got[1], ref[1])):
        tiny = np.linalg.norm(X, axis=-1) < 1e-2
        e_tiny, e_norm = rel_l2(g[tiny], r[tiny]), rel_l2(g[~tiny], r[~tiny])
        _say(f"[parity] cfg4 {name}: tiny rows {e_tiny:.2e}  normal rows {e_norm:.2e}")
        assert e_tiny <= 2e-2 and e_norm <= 2e-2


def test_cfg5_long_history(oracle):
    b = make_batch("cfg5", 0)
    w = b.workload
    _check_batch(oracle, b)
    # the linear GPU path against the QUADRATIC definition on 2 sampled slices
    got = gpu_fwd(b.Q, b.K, b.V, b.mask, w.dtype, scale=b.scale, eps=b.eps)
    rng = np.random.default_rng(5)
    for _ in range(2):
        bi, hi = int(rng.integers(w.B)), int(rng.integers(w.H))
        sl = (slice(bi, bi + 1), slice(hi, hi + 1))
        ref = oracle.fwd_quadratic(b.Q[sl], b.K[sl], b.V[sl], b.mask[bi:bi + 1], scale=b.scale, eps=b.eps)
        e = rel_l2(got[sl], ref)
        _say(f"[parity] cfg5 slice ({bi},{hi}) vs quadratic form: {e:.2e}")
        assert e <= 2e-2


# ------------------------------------------------------------------- edge cases

def _case(seed, B, H, N, d, dtype="f32", sigma=1.0):
    rng = np.random.default_rng(seed)
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)).astype(np.float32) * np.float32(sigma) for _ in range(4))
    if dtype == "bf16":
        Q, K, V, dO = (round_to_bf16(x) for x in (Q, K, V, dO))
    if dtype == "f16":
        Q, K, V, dO = (round_to_f16(x) for x in (Q, K, V, dO))
    return Q, K, V, dO


def _check_case(oracle, Q, K, V, dO, mask, dtype, scale=None, eps=None, label=""):
    bar = bar_for(dtype)
    oe = 1e-6 if eps is None else eps
    ref_o = oracle.fwd_linear(Q, K, V, mask, scale=scale, eps=oe)
    ref_g = oracle.bwd(Q, K, V, dO, mask, scale=scale, eps=oe)
    got_o = gpu_fwd(Q, K, V, mask, dtype, scale=scale, eps=eps)
    got_g = gpu_bwd(Q, K, V, dO, mask, dtype, scale=scale, eps=eps)
    _say(f"[parity] {label} shape={Q.shape} {dtype}")
    for n, g, r in zip(("O", "dQ", "dK", "dV"), (got_o, *got_g), (ref_o, *ref_g)):
        e = check_tensor(n, g, r, bar)
        _say(f"[parity]   {n}: whole {e['whole']:.2e}  worst slice {e['slice']:.2e}  worst row {e['row']:.2e}")
    return got_o, got_g


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [16, 32, 64])
@pytest.mark.parametrize("N", [1, 7, 33, 200, 515])
def test_ragged_shapes(oracle, dtype, d, N):
    B, H = 3, 2
    Q, K, V, dO = _case(N * 100 + d, B, H, N, d, dtype)
    mask = (np.random.default_rng(N + d).random((B, N)) < 0.7).astype(np.uint8)
    mask[:, -1] = 1
    _check_case(oracle, Q, K, V, dO, mask, dtype, label=f"ragged N={N} d={d}")


@pytest.mark.parametrize("dtype,d", [("f32", 32), ("bf16", 64)])
def test_mask_semantics(oracle, dtype, d):
    B, H, N = 4, 2, 77
    Q, K, V, dO = _case(11, B, H, N, d, dtype)
    mask = np.zeros((B, N), np.uint8)
    mask[0, :] = 1            # full
    mask[1, -1] = 1           # a single valid key
    mask[2, ::3] = 1          # scattered (not contiguous padding)
    # batch row 3: no valid key at all -> O = 0, dK = dV = 0
    got_o, got_g = _check_case(oracle, Q, K, V, dO, mask, dtype, label="mask semantics")
    assert np.all(got_o[3] == 0.0) and np.all(got_g[1][3] == 0.0) and np.all(got_g[2][3] == 0.0)
    # garbage (NaN, Inf, huge) in masked K/V rows changes nothing, bit for bit
    K2, V2 = K.copy(), V.copy()
    dead = np.broadcast_to((mask == 0)[:, None, :, None], K.shape)
    K2[dead] = np.nan
    V2[dead] = np.inf
    o2 = gpu_fwd(Q, K2, V2, mask, dtype)
    g2 = gpu_bwd(Q, K2, V2, dO, mask, dtype)
    assert np.array_equal(o2, got_o)
    for a, c in zip(g2, got_g):
        assert np.array_equal(a, c)
    # mask = NULL equals an all-ones mask, bit for bit
    ones = np.ones((B, N), np.uint8)
    assert np.array_equal(gpu_fwd(Q, K, V, None, dtype), gpu_fwd(Q, K, V, ones, dtype))


@pytest.mark.parametrize("N", [16, 48, 113, 207, 208, 209])
def test_short_bf16_lengths_around_the_resident_limit(oracle, N):
    """bf16 d_h = 64 up to 208 rows is served by the kernels that keep a slice in LDS, 209 rows by
    the streaming kernels: both sides of the limit, full tiles and ragged tails."""
    B, H, d = 3, 2, 64
    Q, K, V, dO = _case(7000 + N, B, H, N, d, "bf16")
    lengths = [N, max(1, N // 3), 1]
    mask = np.zeros((B, N), np.uint8)
    for b, L in enumerate(lengths):
        mask[b, N - L:] = 1
    _check_case(oracle, Q, K, V, dO, mask, "bf16", label=f"short bf16 N={N}")


def test_resident_workgroups_take_several_slices(oracle):
    """More slices than compute units: a persistent workgroup walks three slices and more,
    with its next slice prefetched while the current one is worked on.  The masks mix tiles
    without any valid key at the start, in the middle and at the end of a sequence."""
    B, H, N, d = 175, 4, 200, 64          # 700 slices
    Q, K, V, dO = _case(31, B, H, N, d, "bf16")
    rng = np.random.default_rng(5)
    mask = np.zeros((B, N), np.uint8)
    for b in range(B):
        kind = b % 4
        if kind == 0:                      # left padding
            mask[b, N - int(rng.integers(1, N + 1)):] = 1
        elif kind == 1:                    # right padding
            mask[b, :int(rng.integers(1, N + 1))] = 1
        elif kind == 2:                    # two islands with whole dead tiles between them
            mask[b, 16:40] = 1
            mask[b, 150:171] = 1
        else:                              # scattered
            mask[b] = rng.random(N) < 0.3
    mask[7] = 0                            # no valid key at all
    got_o, got_g = _check_case(oracle, Q, K, V, dO, mask, "bf16", label="700 slices, mixed masks")
    assert np.all(got_o[7] == 0.0) and np.all(got_g[1][7] == 0.0) and np.all(got_g[2][7] == 0.0)
    dead = np.broadcast_to((mask == 0)[:, None, :, None], got_g[1].shape)
    assert np.all(got_g[1][dead] == 0.0) and np.all(got_g[2][dead] == 0.0)
    # run-to-run: bit for bit
    again = gpu_bwd(Q, K, V, dO, mask, "bf16")
    for a, c in zip(again, got_g):
        assert np.array_equal(a, c)


@pytest.mark.parametrize("eps", [1e-12, 1e-6, 1e-3])
def test_eps_and_scale(oracle, eps):
    Q, K, V, dO = _case(21, 2, 2, 90, 32)
    Q[0, 0, :5] *= 1e-4          # rows whose norm is comparable to sqrt(eps)
    K[1, 1, 3:9] *= 1e-4
    mask = np.ones((2, 90), np.uint8); mask[1, :40] = 0
    _check_case(oracle, Q, K, V, dO, mask, "f32", scale=0.37, eps=eps, label=f"eps={eps}")


def test_zero_rows_stay_finite(oracle):
    Q, K, V, dO = _case(22, 2, 1, 40, 32)
    Q[0, 0, 3] = 0.0
    K[1, 0, 5] = 0.0
    _check_case(oracle, Q, K, V, dO, None, "f32", label="zero rows")


def test_deterministic_bits_and_caller_workspace():
    b = make_batch("cfg3", 1, B=32)
    w = b.workload
    o1 = gpu_fwd(b.Q, b.K, b.V, b.mask, w.dtype)
    g1 = gpu_bwd(b.Q, b.K, b.V, b.dO, b.mask, w.dtype)
    need = binding.cotten_attn_workspace_bytes(32, w.H, w.N, w.d_h, binding.COTTEN_F32, True)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        o2 = gpu_fwd(b.Q, b.K, b.V, b.mask, w.dtype, workspace=ws)
        g2 = gpu_bwd(b.Q, b.K, b.V, b.dO, b.mask, w.dtype, workspace=ws, stream=side)
    assert np.array_equal(o1, o2)
    for a, c in zip(g1, g2):
        assert np.array_equal(a, c)


@pytest.mark.parametrize("dtype,d", [("f32", 32), ("bf16", 64)])
def test_long_sequence_split_path(oracle, dtype, d):
    """Few slices, long sequence: the sequence is cut over several workgroups per slice, and
    the partial states travel through the workspace (the library's own or the caller's)."""
    B, H, N = 2, 2, 1030
    Q, K, V, dO = _case(77, B, H, N, d, dtype)
    mask = np.zeros((B, N), np.uint8)
    mask[0, 400:] = 1
    mask[1, ::2] = 1
    got_o, got_g = _check_case(oracle, Q, K, V, dO, mask, dtype, label=f"split path d={d}")
    code = binding.COTTEN_F32 if dtype == "f32" else binding.COTTEN_BF16
    need = binding.cotten_attn_workspace_bytes(B, H, N, d, code, True)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    for _ in range(2):
        assert np.array_equal(gpu_fwd(Q, K, V, mask, dtype), got_o)
        for a, c in zip(gpu_bwd(Q, K, V, dO, mask, dtype), got_g):
            assert np.array_equal(a, c)
    assert np.array_equal(gpu_fwd(Q, K, V, mask, dtype, workspace=ws), got_o)
    for a, c in zip(gpu_bwd(Q, K, V, dO, mask, dtype, workspace=ws), got_g):
        assert np.array_equal(a, c)


@pytest.mark.parametrize("dtype,d", [("f32", 32), ("bf16", 64)])
def test_extreme_shapes(oracle, dtype, d):
    """Very many short slices (persistent workgroups loop 100+ times / tens of thousands of
    workgroups) and one very long ragged sequence (thousands of tiles per slice, 49999 rows)."""
    B, H, N = 4096, 8, 16
    Q, K, V, dO = _case(61, B, H, N, d, dtype)
    mask = (np.random.default_rng(62).random((B, N)) < 0.5).astype(np.uint8)
    mask[::7] = 0
    _check_case(oracle, Q, K, V, dO, mask, dtype, label=f"32768 slices of 16 rows, d={d}")
    B, H, N = 1, 2, 49999
    Q, K, V, dO = _case(63, B, H, N, d, dtype)
    mask = np.zeros((B, N), np.uint8)
    mask[0, 12345:] = 1
    mask[0, 30000:30100] = 0
    _check_case(oracle, Q, K, V, dO, mask, dtype, label=f"one sequence of {N} rows, d={d}")


@pytest.mark.parametrize("B,H,N,d", [(6, 4, 200, 64), (3, 2, 77, 64), (70, 4, 230, 64), (2, 2, 1030, 64),
                                     (3, 2, 70, 32), (2, 2, 300, 16)])
def test_fp16_io(oracle, B, H, N, d):
    """IEEE half I/O (the mixed-precision mode of the paper's training runs) on every kernel
    family: resident (N <= 208), fused and split streamers (d_h = 64), narrower rows (d_h = 32, 16).
    Bar 2.5e-3: unit roundoff 2^-11 against bf16's 2^-8 and its bar of 2e-2."""
    Q, K, V, dO = _case(8000 + N + d, B, H, N, d, "f16")
    rng = np.random.default_rng(N)
    mask = np.zeros((B, N), np.uint8)
    for b in range(B):
        mask[b, N - int(rng.integers(1, N + 1)):] = 1
    got_o, got_g = _check_case(oracle, Q, K, V, dO, mask, "f16", label=f"fp16 N={N} d={d}")
    dead = np.broadcast_to((mask == 0)[:, None, :, None], got_o.shape)
    assert np.all(got_g[1][dead] == 0.0) and np.all(got_g[2][dead] == 0.0)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("N", [33, 200, 700])
def test_head_dim_128(oracle, dtype, N):
    """d_h = 128 (d_model 256 with two heads): the kernels for 256-byte rows (16-bit) and for
    512-byte rows (fp32)."""
    B, H, d = 2, 2, 128
    Q, K, V, dO = _case(9100 + N, B, H, N, d, dtype)
    mask = (np.random.default_rng(N).random((B, N)) < 0.7).astype(np.uint8)
    mask[:, -1] = 1
    got_o, got_g = _check_case(oracle, Q, K, V, dO, mask, dtype, label=f"d=128 N={N}")
    dead = np.broadcast_to((mask == 0)[:, None, :, None], got_o.shape)
    assert np.all(got_g[1][dead] == 0.0) and np.all(got_g[2][dead] == 0.0)


@pytest.mark.parametrize("dtype,d,N", [("f16", 64, 200), ("bf16", 32, 180), ("bf16", 16, 208), ("bf16", 64, 161)])
def test_many_short_slices_16bit(oracle, dtype, d, N):
    """256 slices and more of 16-bit sequences above 160 rows: the forward runs on the fused
    kernel that keeps its tiles in registers, the backward on the resident kernel."""
    B, H = 64, 4
    Q, K, V, dO = _case(9500 + N + d, B, H, N, d, dtype)
    rng = np.random.default_rng(N + d)
    mask = np.zeros((B, N), np.uint8)
    for b in range(B):
        mask[b, N - int(rng.integers(1, N + 1)):] = 1
    mask[5] = 0
    got_o, got_g = _check_case(oracle, Q, K, V, dO, mask, dtype, label=f"256 slices {dtype} d={d} N={N}")
    assert np.all(got_o[5] == 0.0)
    dead = np.broadcast_to((mask == 0)[:, None, :, None], got_o.shape)
    assert np.all(got_g[1][dead] == 0.0) and np.all(got_g[2][dead] == 0.0)


def test_long_sequences_with_many_slices(oracle):
    """256 slices of more than 2048 rows: the backward stays on one workgroup per slice (fused
    streaming kernel), the forward is cut into splits."""
    B, H, N, d = 128, 2, 2100, 32
    Q, K, V, dO = _case(9700, B, H, N, d, "f32")
    rng = np.random.default_rng(3)
    mask = np.zeros((B, N), np.uint8)
    for b in range(B):
        mask[b, N - int(rng.integers(1, N + 1)):] = 1
    _check_case(oracle, Q, K, V, dO, mask, "f32", label="256 slices x 2100 rows")


def _mixed_masks(B, N, seed):
    """Left-padded, right-padded, scattered and island masks in turn; one sequence without any
    valid key and one with a single valid key."""
    rng = np.random.default_rng(seed)
    mask = np.zeros((B, N), np.uint8)
    for b in range(B):
        kind = b % 4
        if kind == 0:
            mask[b, N - int(rng.integers(1, N + 1)):] = 1
        elif kind == 1:
            mask[b, :int(rng.integers(1, N + 1))] = 1
        elif kind == 2:
            mask[b] = rng.random(N) < 0.4
        else:
            mask[b, N // 5:N // 4] = 1
            mask[b, N - 40:N - 3] = 1
    mask[3] = 0
    mask[4] = 0
    mask[4, N // 2] = 1
    return mask


@pytest.mark.parametrize("dtype,B,H,N,d", [("f32", 128, 2, 520, 32), ("bf16", 64, 4, 700, 64),
                                           ("f16", 64, 4, 700, 64), ("f32", 256, 2, 2100, 32),
                                           ("bf16", 128, 4, 2100, 64)])
def test_streaming_forward_with_many_slices(oracle, dtype, B, H, N, d):
    """More than 256 rows with at least 256 slices (512 beyond 2048 rows): forward and backward
    both run on the fused streaming kernels that re-read their tiles (one workgroup per slice,
    tiles not kept in registers, no workspace)."""
    code = {"f32": binding.COTTEN_F32, "bf16": binding.COTTEN_BF16, "f16": binding.COTTEN_F16}[dtype]
    assert binding.cotten_attn_workspace_bytes(B, H, N, d, code, False) == 0
    assert binding.cotten_attn_workspace_bytes(B, H, N, d, code, True) == 0
    Q, K, V, dO = _case(9800 + N + d, B, H, N, d, dtype)
    mask = _mixed_masks(B, N, N + d)
    got_o, got_g = _check_case(oracle, Q, K, V, dO, mask, dtype, label=f"streaming fwd {dtype} {B}x{H}x{N}x{d}")
    assert np.all(got_o[3] == 0.0)
    dead = np.broadcast_to((mask == 0)[:, None, :, None], got_o.shape)
    assert np.all(got_g[1][dead] == 0.0) and np.all(got_g[2][dead] == 0.0)
    # run to run: bit for bit
    assert np.array_equal(gpu_fwd(Q, K, V, mask, dtype), got_o)
    for a, c in zip(gpu_bwd(Q, K, V, dO, mask, dtype), got_g):
        assert np.array_equal(a, c)


def test_binding_reports_library_errors():
    x = torch.zeros(1, 1, 8, 48, device="cuda")
    with pytest.raises(binding.CottenError) as ei:
        binding.cotten_attn_fwd(x, x, x, None)
    assert ei.value.status == -3
