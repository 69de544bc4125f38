#!/usr/bin/env python3
"""Benchmark of the cosine-attention hot path on one MI355X.

One step = one forward call + one backward call of the library on one synthetic
recommendation-shaped batch that is already resident in HBM.  Prints ONE JSON line:
whole-step tokens/s, the HBM roofline of the dominant (backward) launch measured with
events on the launch stream, and the fp64 CPU oracle timed on the host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--no-cpu]

Successive steps rotate over independent buffer sets whose total size exceeds the
256 MB memory-side cache twice over, so every step streams from HBM.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0, "f16": 2500.0}   # dense, published
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
ROTATE_BYTES = 640 << 20       # rotate over at least this many bytes of tensors


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-others", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--no-graph", action="store_true", help="launch every step from Python instead of replaying a HIP graph")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of 64 MiB (reference for HBM byte counters)")
    ap.add_argument("--warm-cache", action="store_true", help="one buffer set only (cache-resident)")
    return ap.parse_args()


class DeviceBatch:
    """R independent copies of one batch on the GPU (same values, distinct addresses)."""

    def __init__(self, batch, torch, rotate_bytes):
        w = batch.workload
        self.batch = batch
        self.dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        self.esize = 2 if w.dtype == "bf16" else 4
        self.tensor_bytes = batch.Q.size * self.esize
        self.R = max(1, -(-rotate_bytes // (11 * self.tensor_bytes)))
        host = [torch.from_numpy(x).to(self.dt) for x in (batch.Q, batch.K, batch.V, batch.dO)]
        self.mask = None if batch.mask is None else torch.from_numpy(batch.mask).cuda()
        self.sets = []
        for _ in range(self.R):
            q, k, v, g = (h.cuda() for h in host)
            outs = [torch.empty_like(q) for _ in range(4)]     # O, dQ, dK, dV
            self.sets.append((q, k, v, g, *outs))
        # mask-aware algorithmic bytes (masked K/V rows need not be read)
        f = batch.valid_fraction
        self.bytes_fwd = (2 + 2 * f) * self.tensor_bytes
        self.bytes_bwd = (5 + 2 * f) * self.tensor_bytes
        self.bytes_fwd_dense = 4 * self.tensor_bytes
        self.bytes_bwd_dense = 7 * self.tensor_bytes
        self.tokens = w.B * batch.Q.shape[2]
        # algorithmic flops of the backward call per token-head: S (2 d^2, valid keys only), dS
        # and g (2 d^2 each, every row), dV and h (4 d^2, valid keys only)
        rows = w.B * w.H * batch.Q.shape[2]
        self.flops_bwd = rows * w.d_h * w.d_h * (4 + 6 * f)


def run_steps(db, binding, n, first=0, fwd=True, bwd=True):
    b = db.batch
    for i in range(first, first + n):
        q, k, v, g, O, dQ, dK, dV = db.sets[i % db.R]
        if fwd:
            binding.cotten_attn_fwd(q, k, v, db.mask, O, scale=b.scale, eps=b.eps)
        if bwd:
            binding.cotten_attn_bwd(q, k, v, db.mask, g, dQ, dK, dV, scale=b.scale, eps=b.eps)


def event_ms(torch, fn):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1)


def capture(db, binding, torch, n, first=0, fwd=True, bwd=True):
    """Record n steps (their kernel launches, nothing else) into one HIP graph."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_steps(db, binding, n, first=first, fwd=fwd, bwd=bwd)
    return g


def measure(db, binding, torch, steps, warmup, use_graph=True):
    """W untimed steps, then exactly K timed steps between two device synchronisations.
    With use_graph the K steps are replayed from one HIP graph, so the host only pays one
    launch and the GPU sees the kernels back to back (how a launch-bound loop is deployed)."""
    run_steps(db, binding, warmup)
    torch.cuda.synchronize()
    if use_graph:
        g_step = capture(db, binding, torch, steps, first=warmup)
        g_fwd = capture(db, binding, torch, steps, bwd=False)
        g_bwd = capture(db, binding, torch, steps, fwd=False)
        g_step.replay()                      # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        step_fn, fwd_fn, bwd_fn = g_step.replay, g_fwd.replay, g_bwd.replay
    else:
        step_fn = lambda: run_steps(db, binding, steps, first=warmup)
        fwd_fn = lambda: run_steps(db, binding, steps, bwd=False)
        bwd_fn = lambda: run_steps(db, binding, steps, fwd=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_fn()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    # per-launch durations: K back-to-back launches of one direction between two events
    fwd_fn(); bwd_fn()
    torch.cuda.synchronize()
    fwd_ms = event_ms(torch, fwd_fn) / steps
    bwd_ms = event_ms(torch, bwd_fn) / steps
    ms = wall_ms / steps
    return {
        "ms_per_step": ms,
        "tokens_per_s": db.tokens / (ms * 1e-3),
        "fwd_us": fwd_ms * 1e3,
        "bwd_us": bwd_ms * 1e3,
        "fwd_gbs": db.bytes_fwd / (fwd_ms * 1e-3) / 1e9,
        "bwd_gbs": db.bytes_bwd / (bwd_ms * 1e-3) / 1e9,
        "step_gbs": (db.bytes_fwd + db.bytes_bwd) / (ms * 1e-3) / 1e9,
        "step_gbs_dense": (db.bytes_fwd_dense + db.bytes_bwd_dense) / (ms * 1e-3) / 1e9,
    }


def measured_traffic(workload, kernel_tags):
    """HBM bytes per backward call, from the committed rocprofv3 counter summary of this
    workload: FETCH_SIZE + WRITE_SIZE (scaled by the copy kernel's reading) summed over the
    kernels of the call, i.e. those whose name contains one of `kernel_tags`.  None when no
    summary is there."""
    import glob
    paths = sorted(glob.glob(os.path.join(ROOT, "profiles", f"*_path_{workload}.txt")))
    if not paths:
        return None
    total, seen = 0.0, 0
    for line in open(paths[-1]):
        parts = line.strip().split(",")      # kernel names may contain commas themselves
        if len(parts) >= 3 and parts[0] in ("FETCH_SIZE", "WRITE_SIZE") \
                and any(t in ",".join(parts[1:-1]) for t in kernel_tags) \
                and parts[-1].endswith("MB per launch"):
            total += float(parts[-1].split()[0]) * 1e6
            seen += 1
    return int(total) if seen else None


# kernels one backward call launches (resident or fused: one; long sequences: three)
BWD_KERNELS = ("resident_bwd_kernel", "fused_bwd_kernel", "split_state_kernel", "split_q_kernel",
               "split_kv_kernel")


def cpu_baseline(batch, budget_s=12.0):
    """The fp64 oracle (forward + backward, linear form) on the host cores, on a bounded
    sample: the first `nb` batch rows of the same workload, sized for ~budget_s seconds."""
    from oracle import cotten_oracle as orc
    w = batch.workload

    def one(nb):
        sl = slice(0, nb)
        m = None if batch.mask is None else batch.mask[sl]
        t0 = time.perf_counter()
        orc.fwd_linear(batch.Q[sl], batch.K[sl], batch.V[sl], m, scale=batch.scale, eps=batch.eps)
        orc.bwd(batch.Q[sl], batch.K[sl], batch.V[sl], batch.dO[sl], m, scale=batch.scale, eps=batch.eps)
        return time.perf_counter() - t0

    B, N = batch.Q.shape[0], batch.Q.shape[2]
    nb = max(1, min(B, 8))
    t = one(nb)                                   # also warms the library up
    t = one(nb)
    want = nb * budget_s / max(t, 1e-4)           # batch rows worth ~budget_s seconds
    if want <= B:
        nb, reps = int(max(1, want)), 1
    else:
        nb, reps = B, int(min(1000, max(1, round(want / B))))
    t = sum(one(nb) for _ in range(reps))
    return {"value": reps * nb * N / t, "unit": "tokens/s", "cores": orc.threads(), "kind": "oracle",
            "sample": f"{reps} pass(es) over the first {nb} of {B} batch rows of {w.name} "
                      f"(fwd+bwd, fp64, incl. fp32->fp64 widening), {t:.2f} s"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_06935_amd import binding
    from paper_2602_06935_amd.inputs import WORKLOADS, make_batch

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    binding.load_library()

    rot = 0 if args.warm_cache else ROTATE_BYTES
    w = WORKLOADS[args.workload]
    batch = make_batch(args.workload, args.seed)
    db = DeviceBatch(batch, torch, rot)
    res = measure(db, binding, torch, args.steps, args.warmup, not args.no_graph)

    others = {}
    if not args.no_others:
        for name in ("cfg2", "cfg3", "cfg4", "cfg5"):
            if name == args.workload:
                continue
            ob = make_batch(name, args.seed)
            odb = DeviceBatch(ob, torch, rot)
            r = measure(odb, binding, torch, max(20, args.steps // 4), max(5, args.warmup // 4), not args.no_graph)
            others[name] = {
                "tokens_per_s": round(r["tokens_per_s"], 1), "ms_per_step": round(r["ms_per_step"], 5),
                "fwd_us": round(r["fwd_us"], 2), "bwd_us": round(r["bwd_us"], 2),
                "bwd_frac_of_hbm_peak": round(r["bwd_gbs"] / HBM_PEAK_GBS, 4),
                "fwd_frac_of_hbm_peak": round(r["fwd_gbs"] / HBM_PEAK_GBS, 4),
                "step_frac_of_hbm_peak": round(r["step_gbs"] / HBM_PEAK_GBS, 4),
                "valid_fraction": round(ob.valid_fraction, 4), "buffer_sets": odb.R,
            }
            del odb, ob
            torch.cuda.empty_cache()

    if args.copy_calibration:
        # a plain copy of known size: 64 MiB read + 64 MiB written per launch
        src = [torch.empty(16 << 20, dtype=torch.float32, device="cuda").normal_() for _ in range(6)]
        dst = [torch.empty_like(x) for x in src]
        for i in range(24):
            dst[i % 6].copy_(src[i % 6])
        torch.cuda.synchronize()

    cpu = None if args.no_cpu else cpu_baseline(batch)

    out = {
        "metric": "cosine-attn fwd+bwd tokens/sec",
        "value": round(res["tokens_per_s"], 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(res["ms_per_step"], 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "bf16 I/O, f32 accumulate",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: B={w.B} H={w.H} N={w.N} d_h={w.d_h} {w.dtype}, {w.description}",
            "valid_fraction": round(batch.valid_fraction, 4),
            "buffer_sets_rotated": db.R,
            "seed": args.seed,
            "launch": "python per step" if args.no_graph else "one HIP graph of K steps",
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "backward call (cotten_attn_bwd)",
            "achieved": round(res["bwd_gbs"], 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(res["bwd_gbs"] / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic(w.name, BWD_KERNELS),
            "launch_us": round(res["bwd_us"], 2),
            "algorithmic_bytes_per_launch": int(db.bytes_bwd),
            "forward": {"achieved": round(res["fwd_gbs"], 1), "frac": round(res["fwd_gbs"] / HBM_PEAK_GBS, 4),
                        "launch_us": round(res["fwd_us"], 2), "algorithmic_bytes_per_launch": int(db.bytes_fwd)},
            "step": {"achieved": round(res["step_gbs"], 1), "frac": round(res["step_gbs"] / HBM_PEAK_GBS, 4),
                     "achieved_dense_bytes": round(res["step_gbs_dense"], 1)},
            # the contractions run on the matrix cores: how much of their peak the call uses
            "matrix_cores": {"achieved": round(db.flops_bwd / (res["bwd_us"] * 1e-6) / 1e12, 2),
                             "peak": MFMA_PEAK_TFLOPS[w.dtype], "unit": "TFLOP/s",
                             "frac": round(db.flops_bwd / (res["bwd_us"] * 1e-6) / 1e12
                                           / MFMA_PEAK_TFLOPS[w.dtype], 4)},
        },
        "cpu_baseline": cpu,
        "other_workloads": others,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
