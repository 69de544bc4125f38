"""The library's calls only enqueue kernels: the very first call of a process may already be
recorded into a HIP graph (nothing is allocated, nothing synchronises, the one-time kernel
attributes are set without touching the stream).  Runs in a child process so that the captured
call really is the first one the library sees."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import sys
sys.path.insert(0, %(root)r)
import torch
from paper_2602_06935_amd import binding

torch.cuda.set_device(0)
code = {torch.float32: binding.COTTEN_F32, torch.bfloat16: binding.COTTEN_BF16}
# (dtype, B, H, N, d): sequence cut over several workgroups (needs a workspace), slice kept
# in LDS, one workgroup per slice with tiles in registers, streaming; 256-byte rows with three
# launches in the backward, with one launch per direction (tiles kept, tiles streamed);
# 512-byte rows
shapes = [(torch.bfloat16, 2, 2, 1500, 64), (torch.bfloat16, 5, 2, 200, 64),
          (torch.float32, 6, 2, 200, 32), (torch.float32, 130, 2, 300, 32),
          (torch.float32, 2, 2, 150, 64), (torch.bfloat16, 100, 1, 200, 128),
          (torch.bfloat16, 130, 2, 300, 128), (torch.float32, 2, 2, 100, 128)]
gen = torch.Generator(device="cuda").manual_seed(1)
for dt, B, H, N, d in shapes:
    print("capture case", dt, B, H, N, d, flush=True)
    q, k, v, g = (torch.randn(B, H, N, d, device="cuda", generator=gen).to(dt) for _ in range(4))
    mask = (torch.rand(B, N, device="cuda", generator=gen) < 0.7).to(torch.uint8)
    mask[:, -1] = 1
    need = max(binding.cotten_attn_workspace_bytes(B, H, N, d, code[dt], True),
               binding.cotten_attn_workspace_bytes(B, H, N, d, code[dt], False))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    outs = [torch.zeros_like(q) for _ in range(4)]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.cotten_attn_fwd(q, k, v, mask, outs[0], workspace=ws)
        binding.cotten_attn_bwd(q, k, v, mask, g, outs[1], outs[2], outs[3], workspace=ws)
    eager = None
    for replay in range(3):
        for o in outs:
            o.fill_(7.0)
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        # the program's own eager work between the replays
        e = [torch.empty_like(q) for _ in range(4)]
        binding.cotten_attn_fwd(q, k, v, mask, e[0], workspace=ws)
        binding.cotten_attn_bwd(q, k, v, mask, g, e[1], e[2], e[3], workspace=ws)
        torch.cuda.synchronize()
        eager = e if eager is None else eager
        for a, b, c in zip(got, e, eager):
            assert torch.equal(a, b) and torch.equal(b, c), (dt, B, H, N, d, replay)
        assert all(torch.isfinite(a.float()).all() for a in got)
print("CAPTURE-OK", flush=True)
"""


def test_first_call_of_a_process_inside_stream_capture():
    env = dict(os.environ)
    out = subprocess.run([sys.executable, "-u", "-c", CHILD % {"root": ROOT}], env=env,
                         capture_output=True, text=True, timeout=110)
    print(out.stdout[-3000:], out.stderr[-3000:], flush=True)
    assert out.returncode == 0 and "CAPTURE-OK" in out.stdout
