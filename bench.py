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
    "B2_H32_S4096_D128_bf16_causal": {"fetch_kib": 155902 * 2.0, "write_kib": 132096 * 1.0,
                                      "kernel_sha256": "8588ab871894aae9d781d31635330ff34a3e98d3cf0dd654f8c91f84a62fc9f3"},
    "B1_H32_S16384_D128_bf16_causal": {"fetch_kib": 889285 * 2.0, "write_kib": 264192 * 1.0,
                                       "kernel_sha256": "8588ab871894aae9d781d31635330ff34a3e98d3cf0dd654f8c91f84a62fc9f3"},
}


# the same for the row kernels (workload name as bench_rowop reports it)
ROW_TRAFFIC = {
    "softmax_512x4096_f16 x16 rows": {"fetch_kib": 32803.1 * 2.0, "write_kib": 65536.0 * 1.0,
                                      "kernel_sha256": "efc90703c88cd78fc96c429b78ffe9d0151fd5461670fbd9a3e86f4f176ea240"},
    "rmsnorm_1x32x4096x64_f16 x16 rows": {"fetch_kib": 131108.2 * 2.0, "write_kib": 262144.0 * 1.0,
                                          "kernel_sha256": "efc90703c88cd78fc96c429b78ffe9d0151fd5461670fbd9a3e86f4f176ea240"},
}


# and for the GEMM + LeakyReLU kernels (the paper's shape; the 256 x 256 tile's launches)
GEMM_TRAFFIC = {
    "mmLeakyReLu_1x512x512x2048_f16": {"fetch_kib": 10272.7 * 2.0, "write_kib": 512.0 * 1.0,
                                       "kernel_sha256": "b6afad5d4c268aac16fd22caac707ccbf4ce59cb3d783dfc272c3eabafb2a914"},
    "mmLeakyReLu_1x4096x4096x4096_f16": {"fetch_kib": 147536.0 * 2.0, "write_kib": 32768.0 * 1.0,
                                         "kernel_sha256": "b6afad5d4c268aac16fd22caac707ccbf4ce59cb3d783dfc272c3eabafb2a914"},
    "mmLeakyReLu_1x8192x8192x8192_f16": {"fetch_kib": 786595.4 * 2.0, "write_kib": 131072.0 * 1.0,
                                         "kernel_sha256": "b6afad5d4c268aac16fd22caac707ccbf4ce59cb3d783dfc272c3eabafb2a914"},
}


def kernel_source_sha256(csrc, files=("attn_fwd_gfx950.hip", "attn_launch.h")):
    import hashlib
    h = hashlib.sha256()
    for f in files:
        h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()


def measured_traffic(workload_name):
    t = TRAFFIC.get(workload_name)
    files = ("attn_fwd_gfx950.hip", "attn_launch.h")
    if t is None:
        t = ROW_TRAFFIC.get(workload_name)
        files = ("rowops_gfx950.hip", "rowops_launch.h")
    if t is None:
        t = GEMM_TRAFFIC.get(workload_name)
        files = ("gemm_gfx950.hip", "gemm_launch.h")
    if t is None:
        return None
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2501_08071_amd", "csrc")
    try:
        sha = kernel_source_sha256(csrc, files)
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


def bench_rowop(args):
    """The paper's memory-bound kernels (Table 2): one step = one launch over the whole matrix.  HBM roofline:
    algorithmic bytes = every element read once and written once (plus the weight once)."""
    import torch
    import paper_2501_08071_amd as P
    from paper_2501_08071_amd import inputs as I

    name = {"softmax": "softmax_512x4096_f16", "rmsnorm": "rmsnorm_1x32x4096x64_f16"}[args.op]
    op, n_rows, n, dt = I.ROWOP_SHAPES[name]
    n_rows *= args.rows_mul
    xb = I.gen_rows(n_rows, n, dt, tensor_id=0)
    x = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.float16)
    y = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    if op == "softmax":
        def step():
            P.softmax_rows_fwd(x, y=y, stream=stream)
        nbytes = 2 * 2 * n_rows * n
    else:
        wb = I.gen_rows(1, n, dt, tensor_id=1)[0]
        wt = torch.from_numpy(wb.view(np.int16)).cuda().view(torch.float16)

        def step():
            P.rmsnorm_fwd(x, wt, 1e-6, y=y, stream=stream)
        nbytes = 2 * 2 * n_rows * n + 2 * n
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
    kern_ms = ev0.elapsed_time(ev1) / args.steps
    achieved = nbytes / (kern_ms * 1e-3) / 1e9
    wname = name if args.rows_mul == 1 else f"{name} x{args.rows_mul} rows"
    out = {
        "metric": f"row {op} GB/s of algorithmic bytes (each element read once, written once) on 1 MI355X",
        "value": nbytes * args.steps / wall / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wname, "n_rows": n_rows,
                   "row_len": n, "io_dtype": "f16", "path": P.rowops_path(0 if op == "softmax" else 1, n, dt)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": 8000.0, "unit": "GB/s", "frac": achieved / 8000.0,
                     "traffic": measured_traffic(wname), "traffic_unit": "bytes/launch", "algorithmic_bytes": nbytes,
                     "kernel_ms": kern_ms},
    }
    if not args.no_cpu:
        from oracle import rowops as R
        m = min(n_rows, 4096 if op == "softmax" else 1 << 17)
        t0 = time.perf_counter()
        if op == "softmax":
            R.softmax_rows(xb[:m], dt)
        else:
            R.rmsnorm_rows(xb[:m], wb, 1e-6, dt)
        dtm = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2 * 2 * m * n / dtm / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"the first {m} of {n_rows} rows, {dtm:.1f} s, fp64 numpy", "seconds": dtm}
    print(json.dumps(out))


def blas_threads():
    """Threads the numpy matmul of the oracle runs on: the thread pool's own count where it can be asked,
    else the environment's limit, else the processors of this process."""
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads") for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return int(max(n))
    except Exception:
        pass
    for var in ("OPENBLAS_NUM_THREADS", "OMP_NUM_THREADS"):
        if os.environ.get(var, "").isdigit():
            return int(os.environ[var])
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count()


def bench_gemm(args):
    """The paper's fused GEMM + LeakyReLU (Table 2: B, M, N, K = 1, 512, 512, 2048, float16), or a square one of
    --gemm-size.  MFMA roofline: 2 M N K flops per launch."""
    import torch
    import paper_2501_08071_amd as P
    from paper_2501_08071_amd import inputs as I

    if args.gemm_size:
        name = f"mmLeakyReLu_1x{args.gemm_size}x{args.gemm_size}x{args.gemm_size}_f16"
        batch, M, N, K, dt = 1, args.gemm_size, args.gemm_size, args.gemm_size, I.F16
    else:
        name = "mmLeakyReLu_1x512x512x2048_f16"
        batch, M, N, K, dt = I.GEMM_SHAPES[name]
    ab, bb = I.gen_gemm(batch, M, N, K, dt)
    a = torch.from_numpy(ab.view(np.int16)).cuda().view(torch.float16)
    b = torch.from_numpy(bb.view(np.int16)).cuda().view(torch.float16)
    c = torch.empty((batch, M, N), dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        P.gemm_leakyrelu_fwd(a, b, 0.01, c=c, stream=stream)

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
    kern_ms = ev0.elapsed_time(ev1) / args.steps
    flops = 2.0 * batch * M * N * K
    achieved = flops / (kern_ms * 1e-3) / 1e12
    out = {
        "metric": "fused GEMM + LeakyReLU TFLOP/s (2 M N K flops) on 1 MI355X",
        "value": flops * args.steps / wall / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": name, "batch": batch, "M": M, "N": N, "K": K, "slope": 0.01,
                   "path": P.gemm_path(batch, M, N, K, dt)},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS["f16"], "unit": "TFLOP/s",
                     "frac": achieved / PEAK_TFLOPS["f16"], "traffic": measured_traffic(name), "traffic_unit": "bytes/launch",
                     "algorithmic_bytes": 2 * batch * (M * K + K * N + M * N), "kernel_ms": kern_ms},
    }
    if not args.no_cpu:
        from oracle import gemm as G
        m = min(M, 256)
        t0 = time.perf_counter()
        G.gemm_leakyrelu(ab[:, :m], bb, 0.01, dt)
        dtm = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * batch * m * N * K / dtm / 1e12, "unit": "TFLOP/s", "cores": blas_threads(),
                               "kind": "oracle", "sample": f"the first {m} of {M} rows of a, {dtm:.2f} s, fp64 numpy matmul",
                               "seconds": dtm}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--op", choices=["attn", "softmax", "rmsnorm", "gemm"], default="attn",
                    help="attn: the hot path (default); softmax, rmsnorm, gemm: the paper's memory-bound kernels and its "
                         "fused GEMM + LeakyReLU at Table 2's shapes")
    ap.add_argument("--gemm-size", type=int, default=0, help="gemm: a square problem M = N = K of this size instead of Table 2's")
    ap.add_argument("--rows-mul", type=int, default=1,
                    help="softmax, rmsnorm: multiply the number of rows of the paper's shape (its own shape is a few MB)")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", type=int, default=3,
                    help="1..5; 3 is the headline (S=4096, D=128, causal, bf16); 6, 7: the paper's own attention shape")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--cold", action="store_true", help="also time with caches flushed between launches")
    ap.add_argument("--no-probe", action="store_true", help="skip the matrix-instruction-only probe (roofline.mfma_only_measured)")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--data", choices=["synthetic", "zeros"], default="synthetic",
                    help="zeros: all-zero q, k, v -- a diagnostic (same instruction stream, far less switching "
                         "power, so the clock is not power-limited); never the headline figure")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run 10 plain device-to-device copies of MIB MiB (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2501_08071_amd as P
    from paper_2501_08071_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.op == "gemm":
        bench_gemm(args)
        return
    if args.op != "attn":
        bench_rowop(args)
        return
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

    kernel_name = P.attn_kernel_name(w.S, w.D, w.dtype, w.causal)
    rows = P.attn_launch_rows(w.B, w.H, w.S, w.D, w.dtype, w.causal)
    if rows != P.attn_tile_rows(w.D, w.dtype, w.causal):       # a small problem: the same kernel with half the wavefronts
        kernel_name = kernel_name.rsplit(",", 1)[0] + f", {rows // 32}>"
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
                   "kernel": kernel_name},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": measured_traffic(w.name), "traffic_unit": "bytes/launch",
                     "algorithmic_bytes": (3 * 2 + 4) * w.B * w.H * w.S * w.D + 4 * w.B * w.H * w.S,
                     "kernel_ms": kern_ms},
    }

    # second denominator: what nothing but matrix instructions of this type sustain on this chip, on random and
    # on constant operands (the clock under matrix load depends on the operand bits that switch)
    if not args.no_probe:
        rnd = P.attn_mfma_probe(dtype=w.dtype, random_operands=True)
        const = P.attn_mfma_probe(dtype=w.dtype, random_operands=False)
        out["roofline"]["mfma_only_measured"] = {"random_operands": rnd, "constant_operands": const, "unit": "TFLOP/s",
                                                  "frac_of_random": achieved / rnd}

    if args.cold:
        # the paper's protocol (Sections 3.6, 5.1) with cold caches: every launch under its own event pair, a 1 GiB
        # buffer (more than L2 + Infinity Cache) rewritten before it, outside the pair; mean of `steps` launches,
        # repeated 5 times: mean and standard deviation of the 5 means
        flush = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        means = []
        for _ in range(5):
            times = []
            for _ in range(args.steps):
                flush.add_(1.0)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                step()
                b.record(stream)
                torch.cuda.synchronize()
                times.append(a.elapsed_time(b))
            means.append(float(np.mean(times)))
        cold_ms = float(np.mean(means))
        out["cold_cache"] = {"ms": cold_ms, "tflops": w.flops / (cold_ms * 1e-3) / 1e12, "std_ms_of_5_runs": float(np.std(means)),
                             "runs": 5, "launches_per_run": args.steps}

    if not args.no_cpu and args.data == "synthetic":
        out["cpu_baseline"] = cpu_baseline(w, q, k, v)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
