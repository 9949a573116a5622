#!/usr/bin/env python3
"""Throughput of the fused attention forward on one MI355X.

A step is one attn_fwd call (the whole hot path: Q load, K/V stream, Q.K^T, online softmax, P.V,
epilogue) on one batch of the synthetic workload, inputs resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5] [--no-cpu] [--cold] [--data zeros]

Timing follows the paper's protocol (Section 3.6 and 5.1: warm up 100 iterations, time 100, take
the mean); `--cold` adds a second figure with the caches flushed between iterations, each launch
under its own event pair, as the paper does for its reward signal.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0}   # MI355X published dense matrix peak, TFLOP/s

# HBM bytes per launch from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch, each
# scaled by what the same counter reads for a plain 1 GiB copy: 2.0 and 1.0), keyed by workload; valid
# only for the kernel source they were taken with (sha256 over the kernel and its configuration header),
# otherwise reported as null.
TRAFFIC = {
    "B2_H32_S4096_D128_bf16_causal": {"fetch_kib": 153292 * 2.0, "write_kib": 132096 * 1.0,
                                      "kernel_sha256": "d03b8df2a2e6efa91ffbe6f1527bc0a82dd29cf65018df34d06c90c1aa238c9a"},
    "B1_H32_S16384_D128_bf16_causal": {"fetch_kib": 747435 * 2.0, "write_kib": 264192 * 1.0,
                                       "kernel_sha256": "d03b8df2a2e6efa91ffbe6f1527bc0a82dd29cf65018df34d06c90c1aa238c9a"},
}


def kernel_source_sha256(csrc):
    import hashlib
    h = hashlib.sha256()
    for f in ("attn_fwd_gfx950.hip", "attn_launch.h"):
        h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()


def measured_traffic(workload_name):
    t = TRAFFIC.get(workload_name)
    if t is None:
        return None
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2501_08071_amd", "csrc")
    try:
        sha = kernel_source_sha256(csrc)
    except OSError:
        return None
    if sha != t["kernel_sha256"]:
        return None   # the kernel changed since the counters were taken
    return (t["fetch_kib"] + t["write_kib"]) * 1024.0


def cpu_baseline(w, q, k, v, budget_s=15.0):
    """The fp64 oracle as it stands, timed on the host cores over a bounded row sample of the workload."""
    import oracle
    from paper_2501_08071_amd import inputs as I  # noqa: F401

    def pairs(rows):
        return w.B * w.H * (int((rows + 1).sum()) if w.causal else len(rows) * w.S)

    rng = np.random.default_rng(0)
    probe = np.sort(rng.choice(w.S, max(1, min(w.S, 16)), replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    oracle.attn_oracle(q, k, v, w.causal, w.scale, w.dtype, rows=probe)
    dt = time.perf_counter() - t0
    rate = pairs(probe) / dt                       # includes the per-head widening of K and V
    n = int(min(w.S, max(len(probe), budget_s * rate / (pairs(np.arange(w.S)) / w.S))))
    rows = np.sort(rng.choice(w.S, n, replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    oracle.attn_oracle(q, k, v, w.causal, w.scale, w.dtype, rows=rows)
    dt = time.perf_counter() - t0
    flops = 4.0 * w.D * pairs(rows)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} of {w.S} query rows (seeded random) of every (b,h), {dt:.1f} s, fp64",
            "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", type=int, default=3,
                    help="1..5; 3 is the headline (S=4096, D=128, causal, bf16); 6, 7: the paper's own attention shape")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--cold", action="store_true", help="also time with caches flushed between launches")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--data", choices=["synthetic", "zeros"], default="synthetic",
                    help="zeros: all-zero q, k, v -- a diagnostic (same instruction stream, far less switching "
                         "power, so the clock is not power-limited); never the headline figure")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run 10 plain device-to-device copies of MIB MiB (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2501_08071_amd as P
    from paper_2501_08071_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.calibrate_copy:
        # a plain copy kernel of known size: what FETCH_SIZE / WRITE_SIZE read for it scales those counters
        n = args.calibrate_copy << 20
        src = torch.ones(n // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n, "copies": 10}))
        return
    w = I.workload(args.workload)
    seed = I.BASE_SEED if args.seed is None else args.seed
    q, k, v = I.gen_inputs(w, seed)
    tdt = torch.float16 if w.dtype == I.F16 else torch.bfloat16
    dq, dk, dv = (torch.from_numpy(t.view(np.int16)).cuda().view(tdt) for t in (q, k, v))
    if args.data == "zeros":
        dq, dk, dv = (torch.zeros_like(t) for t in (dq, dk, dv))
    o = torch.empty((w.B, w.H, w.S, w.D), dtype=torch.float32, device="cuda")
    lse = torch.empty((w.B, w.H, w.S), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        P.attn_fwd(dq, dk, dv, w.causal, w.scale, o=o, lse=lse, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = ev0.elapsed_time(ev1) / args.steps          # mean launch duration on the launch stream

    tflops = w.flops * args.steps / wall / 1e12
    achieved = w.flops / (kern_ms * 1e-3) / 1e12
    peak = PEAK_TFLOPS[w.dtype_name]
    out = {
        "metric": "attention fwd TFLOP/s on 1 MI355X and % of bf16 MFMA peak",
        "value": tflops, "unit": "TFLOP/s", "pct_of_mfma_peak": 100.0 * tflops / peak,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype_name,
        "data": "synthetic" if args.data == "synthetic" else "zeros (diagnostic only, not the metric's workload)",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "S": w.S, "D": w.D, "causal": w.causal,
                   "scale": w.scale, "seed": seed, "flops_per_step": w.flops,
                   "kernel": P.attn_kernel_name(w.S, w.D, w.dtype, w.causal)},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": measured_traffic(w.name), "traffic_unit": "bytes/launch",
                     "algorithmic_bytes": (3 * 2 + 4) * w.B * w.H * w.S * w.D + 4 * w.B * w.H * w.S,
                     "kernel_ms": kern_ms},
    }

    if args.cold:
        flush = torch.empty(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB > L2 + Infinity Cache
        times = []
        for _ in range(args.steps):
            flush.add_(1.0)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            step()
            b.record(stream)
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b))
        cold_ms = float(np.mean(times))
        out["cold_cache"] = {"ms": cold_ms, "tflops": w.flops / (cold_ms * 1e-3) / 1e12, "std_ms": float(np.std(times))}

    if not args.no_cpu and args.data == "synthetic":
        out["cpu_baseline"] = cpu_baseline(w, q, k, v)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
