#!/usr/bin/env python3
"""Throughput of the fused attention forward on one MI355X.

A step is one attn_fwd call (the whole hot path: Q load, K/V stream, Q.K^T, online softmax, P.V,
epilogue) on one batch of the synthetic workload, inputs resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..7] [--no-cpu] [--brief] [--cold] [--data zeros]

Timing follows the paper's protocol (Sections 3.6 and 5.1: warm-up iterations, then timed ones, the mean;
differences of about 1 % count as noise).  Before the W warm-up steps the harness launches the kernel back
to back until the launch time has settled: the first launches of a process run up to 20 % slower, for some
tens of milliseconds, until the chip's clock and power management have found their level under the new load,
so a short warm-up would time the transient, not the kernel (`settle` in the output says how long it took).
The full line (and `--cold`) also carries the figure with the caches flushed between launches, each launch
under its own event pair, five runs, as the paper does for its reward signal (`cold_cache`).

Next to the headline the same line carries short runs of the other workloads (`workloads`), the paper's
memory-bound pair and its fused GEMM at Table 2's shapes and at one streaming size (`also`), and the
secondary bounds of every attention configuration (`roofline.bounds`); `--brief` leaves these out (used
under the profiler, where only the headline kernel is wanted).
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np

PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0}   # MI355X published dense matrix peak, TFLOP/s
PEAK_HBM_GBS = 8000.0                           # MI355X published HBM bandwidth, GB/s
ROOT = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(ROOT, "paper_2501_08071_amd", "csrc")

# HBM bytes per launch from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch, each
# scaled by what the same counter reads for a plain 1 GiB copy: 2.0 and 1.0), keyed by workload, with the
# summary under profiles/ that holds the counter values; valid only for the kernel source they were taken
# with (sha256 over the kernel's sources), otherwise reported as null.
ATTN_FILES = ("attn_fwd_gfx950.hip", "attn_fwd_rows64_gfx950.hip", "attn_launch.h", "attn_device.h", "gfx950_common.h")
ROW_FILES = ("rowops_gfx950.hip", "rowops_launch.h")
GEMM_FILES = ("gemm_gfx950.hip", "gemm_launch.h", "gfx950_common.h")
TRAFFIC = {
    "B2_H32_S4096_D128_bf16_causal": {"fetch_kib": 147418 * 2.0, "write_kib": 132096 * 1.0, "files": ATTN_FILES,
                                      "kernel_sha256": "90cf59d9fbf8f596177c62da2977753833bbabfe9f23af8e242831a8f3448e93",
                                      "source": "profiles/attn_fwd_kernel_S4096_D128_bf16_causal.md"},
    "B1_H32_S16384_D128_bf16_causal": {"fetch_kib": 920443 * 2.0, "write_kib": 264192 * 1.0, "files": ATTN_FILES,
                                       "kernel_sha256": "90cf59d9fbf8f596177c62da2977753833bbabfe9f23af8e242831a8f3448e93",
                                       "source": "profiles/attn_fwd_kernel_all_workloads.md"},
    "B16_H16_S2048_D64_f16_peaky": {"fetch_kib": 98509.6 * 2.0, "write_kib": 133120 * 1.0, "files": ATTN_FILES,
                                    "kernel_sha256": "90cf59d9fbf8f596177c62da2977753833bbabfe9f23af8e242831a8f3448e93",
                                    "source": "profiles/attn_fwd_kernel_S2048_D64_f16.md"},
    "B4_H16_S1024_D64_f16": {"fetch_kib": 12472.7 * 2.0, "write_kib": 16640 * 1.0, "files": ATTN_FILES,
                             "kernel_sha256": "90cf59d9fbf8f596177c62da2977753833bbabfe9f23af8e242831a8f3448e93",
                             "source": "profiles/attn_fwd_kernel_S2048_D64_f16.md"},
    # the row kernels (workload name as rowop_run reports it)
    "softmax_512x4096_f16 x16 rows": {"fetch_kib": 32802.5 * 2.0, "write_kib": 65536.0 * 1.0, "files": ROW_FILES,
                                      "kernel_sha256": "efc90703c88cd78fc96c429b78ffe9d0151fd5461670fbd9a3e86f4f176ea240",
                                      "source": "profiles/rowop_reg_kernel_softmax_rmsnorm.md"},
    "rmsnorm_1x32x4096x64_f16 x16 rows": {"fetch_kib": 131108.0 * 2.0, "write_kib": 262144.0 * 1.0, "files": ROW_FILES,
                                          "kernel_sha256": "efc90703c88cd78fc96c429b78ffe9d0151fd5461670fbd9a3e86f4f176ea240",
                                          "source": "profiles/rowop_reg_kernel_softmax_rmsnorm.md"},
    # the GEMM + LeakyReLU kernels (the paper's shape; the 256 x 256 tile's launches)
    "mmLeakyReLu_1x512x512x2048_f16": {"fetch_kib": 10272.5 * 2.0, "write_kib": 512.0 * 1.0, "files": GEMM_FILES,
                                       "kernel_sha256": "4621da25a85d63d48a6b552e285a1a26e4d75c798cc8b9d9c8efe85953557683",
                                       "source": "profiles/gemm_lrelu_kernel_mmLeakyReLu.md"},
    "mmLeakyReLu_1x4096x4096x4096_f16": {"fetch_kib": 147536.0 * 2.0, "write_kib": 32768.0 * 1.0, "files": GEMM_FILES,
                                         "kernel_sha256": "4621da25a85d63d48a6b552e285a1a26e4d75c798cc8b9d9c8efe85953557683",
                                         "source": "profiles/gemm_lrelu_kernel_mmLeakyReLu.md"},
}


def kernel_source_sha256(files):
    import hashlib
    h = hashlib.sha256()
    for f in files:
        h.update(open(os.path.join(CSRC, f), "rb").read())
    return h.hexdigest()


def measured_traffic(workload_name):
    """(bytes per launch, profile it came from), or (None, None) when there are no counters for this workload or
    the kernel has changed since they were taken."""
    t = TRAFFIC.get(workload_name)
    if t is None:
        return None, None
    try:
        sha = kernel_source_sha256(t["files"])
    except OSError:
        return None, None
    if sha != t["kernel_sha256"]:
        return None, None
    return (t["fetch_kib"] + t["write_kib"]) * 1024.0, t["source"]


# ---- timing ---------------------------------------------------------------------------------------

def settle(step, stream, torch, max_s=1.5, min_s=0.05):
    """Launch back to back until the launch time has settled: windows of launches, each under one event pair;
    done when at least `min_s` seconds of load have passed and the means of the last two windows agree within
    1 %, or after `max_s` seconds.  Returns what happened."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    step()
    e1.record(stream)
    torch.cuda.synchronize()
    first_ms = e0.elapsed_time(e1)
    per_window = int(min(200, max(10, math.ceil(4.0 / max(first_ms, 1e-3)))))   # about 4 ms of launches, 10 to 200
    windows, launches, t_start = [], 1, time.perf_counter()
    while True:
        e0.record(stream)
        for _ in range(per_window):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        windows.append(e0.elapsed_time(e1) / per_window)
        launches += per_window
        elapsed = time.perf_counter() - t_start
        agree = len(windows) >= 2 and abs(windows[-1] - windows[-2]) <= 0.01 * windows[-1]
        if (elapsed >= min_s and len(windows) >= 3 and agree) or elapsed >= max_s:
            return {"launches": launches, "seconds": elapsed, "settled": bool(agree), "first_launch_ms": first_ms,
                    "first_window_ms": windows[0], "slowest_window_ms": max(windows), "last_window_ms": windows[-1],
                    "launches_per_window": per_window}


def measure(step, stream, torch, warmup, steps, do_settle=True):
    """The timing protocol of every mode: settle, `warmup` untimed steps, then exactly `steps` steps between
    synchronisations (wall clock for `value`, one event pair on the launch stream for the kernel time), then the
    same number of steps once more with every launch under its own event pair (minimum, median, maximum)."""
    st = settle(step, stream, torch) if do_settle else None
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = ev0.elapsed_time(ev1) / steps          # mean launch duration on the launch stream
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    evs[0].record(stream)
    for i in range(steps):
        step()
        evs[i + 1].record(stream)
    torch.cuda.synchronize()
    each = np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(steps)])
    return {"wall_s": wall, "kernel_ms": kern_ms, "settle": st,
            "per_launch_ms": {"n": steps, "min": float(each.min()), "median": float(np.median(each)), "max": float(each.max()),
                              "mean": float(each.mean())}}


# ---- attention ------------------------------------------------------------------------------------

def attn_device_inputs(w, torch, seed, zeros=False):
    from paper_2501_08071_amd import inputs as I
    q, k, v = I.gen_inputs(w, seed)
    tdt = torch.float16 if w.dtype == I.F16 else torch.bfloat16
    dq, dk, dv = (torch.from_numpy(t.view(np.int16)).cuda().view(tdt) for t in (q, k, v))
    if zeros:
        dq, dk, dv = (torch.zeros_like(t) for t in (dq, dk, dv))
    return (q, k, v), (dq, dk, dv)


def attn_step(P, torch, w, dev):
    dq, dk, dv = dev
    o = torch.empty((w.B, w.H, w.S, w.D), dtype=torch.float32, device="cuda")
    lse = torch.empty((w.B, w.H, w.S), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        P.attn_fwd(dq, dk, dv, w.causal, w.scale, o=o, lse=lse, stream=stream)
    step.outputs = (o, lse)
    return step, stream


def attn_algorithmic_bytes(w):
    return (3 * 2 + 4) * w.B * w.H * w.S * w.D + 4 * w.B * w.H * w.S


def attn_bounds(P, w, probes):
    """The other bounds of one attention configuration, in ms per launch, next to the matrix-core bound:
    hbm          the bytes the method must move (q, k, v once, o, lse) at the published HBM bandwidth
    softmax_valu the vector work of the softmax (per score: multiply-add, exp2, row-sum addition, half a
                 conversion) at the rate the vector pipes sustain when they do nothing else (measured in this run)
    l2           the K and V bytes the workgroups stream from L2 into LDS (every workgroup its own copy of the
                 keys it sees) at the L2 read bandwidth measured in this run
    issue_port   the vector work of the softmax plus what the matrix instructions take from the issue of the other
                 wavefront on their SIMD (two wavefronts per SIMD, one port), at 2.4 GHz
    launch_floor what a kernel that does nothing costs per launch, back to back"""
    rows = P.attn_launch_rows(w.B, w.H, w.S, w.D, w.dtype, w.causal)
    nqt = (w.S + rows - 1) // rows
    scores = w.B * w.H * (w.S * (w.S + 1) // 2 if w.causal else w.S * w.S)
    if w.causal:
        keys_streamed = sum(min(w.S, (t + 1) * rows) for t in range(nqt))
    else:
        keys_streamed = nqt * w.S
    l2_bytes = w.B * w.H * keys_streamed * w.D * 2 * 2
    out = {"mfma_ms": w.flops / (PEAK_TFLOPS[w.dtype_name] * 1e12) * 1e3,
           "hbm_ms": attn_algorithmic_bytes(w) / (PEAK_HBM_GBS * 1e9) * 1e3,
           "scores": scores, "l2_to_lds_bytes": l2_bytes}
    if probes:
        # one issue port per SIMD for vector and matrix instructions (1024 SIMDs at the nominal 2.4 GHz): the vector work
        # of 64 scores and what a matrix instruction takes from the wavefront next to it, both measured in this run
        t = "bf16" if w.dtype_name == "bf16" else "f16"
        cycles = scores / 64.0 * probes["issue"][f"valu_cycles_per_64_scores_{t}"] + w.flops / 32768.0 * probes["issue"]["mfma_issue_cycles"]
        out["issue_port_ms"] = cycles / (1024 * 2.4e9) * 1e3
        out["softmax_valu_ms"] = scores / probes["softmax_valu_scores_per_s"] * 1e3
        out["l2_ms"] = l2_bytes / probes["l2_read_bytes_per_s"] * 1e3
        out["launch_floor_us"] = probes["launch_floor_us"]
    return out


def run_probes(P, dtype):
    return {"mfma_random_tflops": P.probe_mfma(dtype=dtype, random_operands=True),
            "mfma_constant_tflops": P.probe_mfma(dtype=dtype, random_operands=False),
            "softmax_valu_scores_per_s": P.probe_softmax_valu(full=True),
            "exp2_fma_per_s": P.probe_softmax_valu(full=False),
            "l2_read_bytes_per_s": P.probe_l2_read(),
            "launch_floor_us": P.probe_launch_floor_us(),
            "issue": P.probe_issue_share()}


def cpu_baseline(w, q, k, v, budget_s=15.0, got=None):
    """The fp64 oracle as it stands, timed on the host cores over a bounded row sample of the workload.  With `got`
    (the o and lse tensors the timed launches wrote) the sampled rows are also compared: `parity`."""
    import oracle

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
    o_ref, l_ref = oracle.attn_oracle(q, k, v, w.causal, w.scale, w.dtype, rows=rows)
    dt = time.perf_counter() - t0
    flops = 4.0 * w.D * pairs(rows)
    out = {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
           "sample": f"{n} of {w.S} query rows (seeded random) of every (b,h), {dt:.1f} s, fp64",
           "seconds": dt}
    if got is not None:
        # the timed configuration's own output against the oracle, on the sampled rows (the bar of the test-suite)
        o, lse = got
        idx = rows.astype(np.int64)
        d = np.abs(o[:, :, idx].cpu().numpy().astype(np.float64) - o_ref)
        dl = np.abs(lse[:, :, idx].cpu().numpy().astype(np.float64) - l_ref) / np.maximum(1.0, np.abs(l_ref))
        out["parity"] = {"rows": int(n), "max_abs": float(d.max()), "mean_abs": float(d.mean()), "lse_rel": float(dl.max()),
                         "within_bar": bool(d.max() <= 2e-2 and d.mean() <= 2e-3 and dl.max() <= 1e-3)}
    return out


def cpu_whole_problem(w, q, k, v):
    """The oracle on a whole (small) workload: with all host threads and with one."""
    import oracle
    out = {}
    n_all = oracle.num_threads()
    for key, n in (("all_threads", n_all), ("one_thread", 1)):
        oracle.set_num_threads(n)
        t0 = time.perf_counter()
        oracle.attn_oracle(q, k, v, w.causal, w.scale, w.dtype)
        dt = time.perf_counter() - t0
        out[key] = {"value": w.flops / dt / 1e12, "unit": "TFLOP/s", "cores": n, "kind": "oracle", "sample": "the whole workload, fp64",
                    "seconds": dt}
    oracle.set_num_threads(n_all)
    return out


def attn_short_run(P, torch, wid, seed, probes, steps=20, with_cpu=False):
    """One of the other workloads, briefly: settle, 5 warm-up and `steps` timed launches."""
    from paper_2501_08071_amd import inputs as I
    w = I.workload(wid)
    host, dev = attn_device_inputs(w, torch, seed)
    cpu = cpu_whole_problem(w, *host) if with_cpu and wid in (1, 2) else None   # the two the oracle finishes in a second or two
    step, stream = attn_step(P, torch, w, dev)
    m = measure(step, stream, torch, 5, steps)
    peak = PEAK_TFLOPS[w.dtype_name]
    tf = w.flops / (m["kernel_ms"] * 1e-3) / 1e12
    traffic, source = measured_traffic(w.name)
    return {"workload": w.name, "id": wid, "ms": m["kernel_ms"], "tflops": tf, "frac": tf / peak,
            "kernel": P.attn_kernel_name(w.B, w.H, w.S, w.D, w.dtype, w.causal), "steps": steps,
            "per_launch_ms": m["per_launch_ms"], "settle_launches": m["settle"]["launches"],
            "traffic": traffic, "traffic_source": source, "algorithmic_bytes": attn_algorithmic_bytes(w),
            "bounds": attn_bounds(P, w, probes), "cpu_baseline": cpu}


# ---- the paper's memory-bound pair ------------------------------------------------------------------

def rowop_run(P, torch, op, rows_mul, warmup, steps, with_cpu, floor_us=None):
    """Row softmax or rmsnorm at Table 2's shape (times rows_mul rows): one step = one launch over the whole
    matrix.  HBM roofline: algorithmic bytes = every element read once and written once (plus the weight once)."""
    from paper_2501_08071_amd import inputs as I
    name = {"softmax": "softmax_512x4096_f16", "rmsnorm": "rmsnorm_1x32x4096x64_f16"}[op]
    _, n_rows, n, dt = I.ROWOP_SHAPES[name]
    n_rows *= rows_mul
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
    m = measure(step, stream, torch, warmup, steps)
    achieved = nbytes / (m["kernel_ms"] * 1e-3) / 1e9
    wname = name if rows_mul == 1 else f"{name} x{rows_mul} rows"
    traffic, source = measured_traffic(wname)
    out = {
        "metric": f"row {op} GB/s of algorithmic bytes (each element read once, written once) on 1 MI355X",
        "value": nbytes * steps / m["wall_s"] / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": m["wall_s"] * 1e3 / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wname, "n_rows": n_rows, "row_len": n, "io_dtype": "f16",
                   "path": P.rowops_path(0 if op == "softmax" else 1, n, dt)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                     "traffic": traffic, "traffic_unit": "bytes/launch", "traffic_source": source,
                     "algorithmic_bytes": nbytes, "kernel_ms": m["kernel_ms"], "per_launch_ms": m["per_launch_ms"],
                     "launch_floor_us": floor_us, "hbm_bound_us": nbytes / (PEAK_HBM_GBS * 1e9) * 1e6},
        "settle": m["settle"],
    }
    if with_cpu:
        from oracle import rowops as R
        mrows = min(n_rows, 4096 if op == "softmax" else 1 << 17)
        t0 = time.perf_counter()
        if op == "softmax":
            R.softmax_rows(xb[:mrows], dt)
        else:
            R.rmsnorm_rows(xb[:mrows], wb, 1e-6, dt)
        dtm = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2 * 2 * mrows * n / dtm / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"the first {mrows} of {n_rows} rows, {dtm:.1f} s, fp64 numpy", "seconds": dtm}
    return out


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


def gemm_run(P, torch, size, warmup, steps, with_cpu, floor_us=None, bmm=False):
    """The paper's fused GEMM + LeakyReLU (Table 2: B, M, N, K = 1, 512, 512, 2048, float16), a square one of
    `size`, or (`bmm`) Table 2's batch matrix multiplication, B, M, N, K = 4, 512, 512, 2048: the same kernel with
    slope 1, which makes the activation the identity.  MFMA roofline: 2 B M N K flops per launch."""
    from paper_2501_08071_amd import inputs as I
    slope = 1.0 if bmm else 0.01
    if bmm:
        name = "bmm_4x512x512x2048_f16"
        batch, M, N, K, dt = I.GEMM_SHAPES[name]
    elif size:
        name = f"mmLeakyReLu_1x{size}x{size}x{size}_f16"
        batch, M, N, K, dt = 1, size, size, size, I.F16
    else:
        name = "mmLeakyReLu_1x512x512x2048_f16"
        batch, M, N, K, dt = I.GEMM_SHAPES[name]
    ab, bb = I.gen_gemm(batch, M, N, K, dt)
    a = torch.from_numpy(ab.view(np.int16)).cuda().view(torch.float16)
    b = torch.from_numpy(bb.view(np.int16)).cuda().view(torch.float16)
    c = torch.empty((batch, M, N), dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        P.gemm_leakyrelu_fwd(a, b, slope, c=c, stream=stream)

    m = measure(step, stream, torch, warmup, steps)
    flops = 2.0 * batch * M * N * K
    achieved = flops / (m["kernel_ms"] * 1e-3) / 1e12
    nbytes = 2 * batch * (M * K + K * N + M * N)
    traffic, source = measured_traffic(name)
    out = {
        "metric": "fused GEMM + LeakyReLU TFLOP/s (2 M N K flops) on 1 MI355X",
        "value": flops * steps / m["wall_s"] / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": m["wall_s"] * 1e3 / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": name, "batch": batch, "M": M, "N": N, "K": K, "slope": slope,
                   "path": P.gemm_path(batch, M, N, K, dt)},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS["f16"], "unit": "TFLOP/s",
                     "frac": achieved / PEAK_TFLOPS["f16"], "traffic": traffic, "traffic_unit": "bytes/launch",
                     "traffic_source": source, "algorithmic_bytes": nbytes, "kernel_ms": m["kernel_ms"],
                     "per_launch_ms": m["per_launch_ms"], "launch_floor_us": floor_us,
                     "mfma_bound_us": flops / (PEAK_TFLOPS["f16"] * 1e12) * 1e6, "hbm_bound_us": nbytes / (PEAK_HBM_GBS * 1e9) * 1e6},
        "settle": m["settle"],
    }
    if with_cpu:
        from oracle import gemm as G
        mm = min(M, 256)
        t0 = time.perf_counter()
        G.gemm_leakyrelu(ab[:, :mm], bb, slope, dt)
        dtm = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * batch * mm * N * K / dtm / 1e12, "unit": "TFLOP/s", "cores": blas_threads(),
                               "kind": "oracle", "sample": f"the first {mm} of {M} rows of a, {dtm:.2f} s, fp64 numpy matmul",
                               "seconds": dtm}
    return out


def brief(o):
    """What an `also` entry keeps of a full mode's line."""
    r = o["roofline"]
    return {"workload": o["config"]["workload"], "value": o["value"], "unit": o["unit"], "ms": r["kernel_ms"],
            "roofline": r, "cpu_baseline": o.get("cpu_baseline"), "settle_launches": o["settle"]["launches"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--op", choices=["attn", "softmax", "rmsnorm", "gemm", "bmm"], default="attn",
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
    ap.add_argument("--brief", action="store_true",
                    help="the headline workload only: no other workloads, no other kernels, no probes, no oracle timing")
    ap.add_argument("--no-settle", action="store_true", help="skip the settling launches (shows the power transient)")
    ap.add_argument("--cold", action="store_true", help="also time with caches flushed between launches (the full line does anyway; this adds it to --brief)")
    ap.add_argument("--no-probe", action="store_true", help="skip the probes (measured denominators and bounds)")
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
    if args.brief:
        args.no_cpu = args.no_probe = True

    import torch
    import paper_2501_08071_amd as P
    from paper_2501_08071_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.op in ("gemm", "bmm"):
        floor = None if args.no_probe else P.probe_launch_floor_us()
        print(json.dumps(gemm_run(P, torch, args.gemm_size, args.warmup, args.steps, not args.no_cpu, floor, bmm=args.op == "bmm")))
        return
    if args.op != "attn":
        floor = None if args.no_probe else P.probe_launch_floor_us()
        print(json.dumps(rowop_run(P, torch, args.op, args.rows_mul, args.warmup, args.steps, not args.no_cpu, floor)))
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

    t_begin = time.perf_counter()
    w = I.workload(args.workload)
    seed = I.BASE_SEED if args.seed is None else args.seed
    (q, k, v), dev = attn_device_inputs(w, torch, seed, zeros=args.data == "zeros")
    step, stream = attn_step(P, torch, w, dev)
    m = measure(step, stream, torch, args.warmup, args.steps, do_settle=not args.no_settle)
    wall, kern_ms = m["wall_s"], m["kernel_ms"]

    tflops = w.flops * args.steps / wall / 1e12
    achieved = w.flops / (kern_ms * 1e-3) / 1e12
    peak = PEAK_TFLOPS[w.dtype_name]
    traffic, source = measured_traffic(w.name)
    out = {
        "metric": "attention fwd TFLOP/s on 1 MI355X and % of bf16 MFMA peak",
        "value": tflops, "unit": "TFLOP/s", "pct_of_mfma_peak": 100.0 * tflops / peak,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype_name,
        "data": "synthetic" if args.data == "synthetic" else "zeros (diagnostic only, not the metric's workload)",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "S": w.S, "D": w.D, "causal": w.causal,
                   "scale": w.scale, "seed": seed, "flops_per_step": w.flops,
                   "kernel": P.attn_kernel_name(w.B, w.H, w.S, w.D, w.dtype, w.causal)},
        "settle": m["settle"],
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": traffic, "traffic_unit": "bytes/launch", "traffic_source": source,
                     "algorithmic_bytes": attn_algorithmic_bytes(w),
                     "kernel_ms": kern_ms, "per_launch_ms": m["per_launch_ms"]},
    }

    # measured denominators: what nothing but matrix instructions of this type sustain on this chip, on random and
    # on constant operands (the clock under matrix load depends on the operand bits that switch); the vector rate of
    # the softmax's work; the L2 read bandwidth; the cost of an empty launch
    probes = None
    if not args.no_probe:
        probes = run_probes(P, w.dtype)
        out["roofline"]["mfma_only_measured"] = {"random_operands": probes["mfma_random_tflops"],
                                                  "constant_operands": probes["mfma_constant_tflops"], "unit": "TFLOP/s",
                                                  "frac_of_random": achieved / probes["mfma_random_tflops"]}
        out["roofline"]["probes"] = probes
    out["roofline"]["bounds"] = attn_bounds(P, w, probes)

    if args.cold or (not args.brief and args.data == "synthetic"):
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
        del flush

    if not args.no_cpu and args.data == "synthetic":
        out["cpu_baseline"] = cpu_baseline(w, q, k, v, got=step.outputs)

    if not args.brief and args.data == "synthetic":
        del dev, step
        torch.cuda.empty_cache()
        # the other workloads, briefly (1, 2, 4, 5 and the paper's own attention shape, workload 6), whichever is not the headline
        out["workloads"] = [attn_short_run(P, torch, wid, seed, probes, with_cpu=not args.no_cpu) for wid in (1, 2, 4, 5, 6) if wid != args.workload]
        # the paper's other kernels: Table 2's shapes, and one size that streams from HBM
        floor = probes["launch_floor_us"] if probes else None
        cpu = not args.no_cpu
        out["also"] = {
            "softmax": [brief(rowop_run(P, torch, "softmax", mul, 20, 50, cpu and mul == 1, floor)) for mul in (1, 16)],
            "rmsnorm": [brief(rowop_run(P, torch, "rmsnorm", mul, 20, 50, cpu and mul == 1, floor)) for mul in (1, 16)],
            "gemm": [brief(gemm_run(P, torch, size, 20, 50, cpu and size == 0, floor)) for size in (0, 4096)],
            "bmm": [brief(gemm_run(P, torch, 0, 20, 50, cpu, floor, bmm=True))],
        }
    out["bench_seconds"] = time.perf_counter() - t_begin
    print(json.dumps(out))


if __name__ == "__main__":
    main()
