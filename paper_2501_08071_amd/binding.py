"""Thin Python binding of the C-ABI library (include/attn.h): argument marshalling only.

PyTorch supplies device memory and the stream; every step of the attention path runs inside
the HIP kernel.  There is no CPU or PyTorch fallback: if the shared library is missing the
import fails loudly.
"""
from __future__ import annotations

import ctypes
import os

# torch first: it carries its own copy of the HIP runtime (same soname as the system one), and the
# process must end up with ONE runtime that owns both torch's streams and this library's kernels
import torch

from . import build as _build

F16 = 0
BF16 = 1


class AttnError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"attn_fwd failed with status {status}: {msg}")
        self.status = status


def _load() -> ctypes.CDLL:
    if not os.path.exists(_build.LIB):
        try:
            _build.build_lib()
        except Exception as e:  # no compiler, or the build failed: there is nothing to fall back to
            raise ImportError(f"{_build.LIB} is missing and could not be built: {e}") from e
    lib = ctypes.CDLL(_build.LIB)
    vp = ctypes.c_void_p
    lib.attn_fwd.argtypes = [vp, vp, vp, vp, vp] + [ctypes.c_int] * 5 + [ctypes.c_float, ctypes.c_int, vp]
    lib.attn_fwd.restype = ctypes.c_int
    lib.attn_fwd_o16.argtypes = lib.attn_fwd.argtypes
    lib.attn_fwd_o16.restype = ctypes.c_int
    lib.attn_supported.argtypes = [ctypes.c_int] * 4
    lib.attn_supported.restype = ctypes.c_int
    lib.attn_status_str.argtypes = [ctypes.c_int]
    lib.attn_status_str.restype = ctypes.c_char_p
    lib.attn_kernel_name.argtypes = [ctypes.c_int] * 6
    lib.attn_kernel_name.restype = ctypes.c_char_p
    for f in (lib.attn_tile_rows, lib.attn_tile_keys):
        f.argtypes = [ctypes.c_int] * 3
        f.restype = ctypes.c_int
    lib.attn_launch_rows.argtypes = [ctypes.c_int] * 6
    lib.attn_launch_rows.restype = ctypes.c_int
    # include/probe.h
    lib.probe_mfma.argtypes = [vp] + [ctypes.c_int] * 4 + [vp]
    lib.probe_mfma.restype = ctypes.c_longlong
    lib.probe_softmax_valu.argtypes = [vp] + [ctypes.c_int] * 3 + [vp]
    lib.probe_softmax_valu.restype = ctypes.c_longlong
    lib.probe_l2_read.argtypes = [vp, vp] + [ctypes.c_int] * 3 + [vp]
    lib.probe_l2_read.restype = ctypes.c_longlong
    lib.probe_empty.argtypes = [ctypes.c_int, ctypes.c_int, vp]
    lib.probe_empty.restype = ctypes.c_int
    lib.probe_issue_share.argtypes = [vp] + [ctypes.c_int] * 4 + [vp]
    lib.probe_issue_share.restype = ctypes.c_int
    # include/rowops.h
    lib.softmax_rows_fwd.argtypes = [vp, vp, ctypes.c_longlong, ctypes.c_int, ctypes.c_int, vp]
    lib.softmax_rows_fwd.restype = ctypes.c_int
    lib.rmsnorm_fwd.argtypes = [vp, vp, vp, ctypes.c_longlong, ctypes.c_int, ctypes.c_float, ctypes.c_int, vp]
    lib.rmsnorm_fwd.restype = ctypes.c_int
    lib.rowops_path.argtypes = [ctypes.c_int] * 3
    lib.rowops_path.restype = ctypes.c_int
    lib.rowops_status_str.argtypes = [ctypes.c_int]
    lib.rowops_status_str.restype = ctypes.c_char_p
    # include/gemm.h
    lib.gemm_leakyrelu_fwd.argtypes = [vp, vp, vp] + [ctypes.c_int] * 4 + [ctypes.c_float, ctypes.c_int, vp]
    lib.gemm_leakyrelu_fwd.restype = ctypes.c_int
    lib.gemm_path.argtypes = [ctypes.c_int] * 5
    lib.gemm_path.restype = ctypes.c_int
    lib.gemm_status_str.argtypes = [ctypes.c_int]
    lib.gemm_status_str.restype = ctypes.c_char_p
    return lib


lib = _load()


def attn_status_str(status: int) -> str:
    return lib.attn_status_str(int(status)).decode()


def attn_supported(S: int, D: int, dtype: int, causal: bool) -> bool:
    return bool(lib.attn_supported(int(S), int(D), int(dtype), int(bool(causal))))


def attn_kernel_name(B: int, H: int, S: int, D: int, dtype: int, causal: bool):
    n = lib.attn_kernel_name(int(B), int(H), int(S), int(D), int(dtype), int(bool(causal)))
    return n.decode() if n else None


def attn_tile_rows(D: int, dtype: int, causal: bool) -> int:
    return int(lib.attn_tile_rows(int(D), int(dtype), int(bool(causal))))


def attn_tile_keys(D: int, dtype: int, causal: bool) -> int:
    return int(lib.attn_tile_keys(int(D), int(dtype), int(bool(causal))))


def attn_launch_rows(B: int, H: int, S: int, D: int, dtype: int, causal: bool) -> int:
    return int(lib.attn_launch_rows(int(B), int(H), int(S), int(D), int(dtype), int(bool(causal))))


# ---- include/probe.h: measuring aids (no product path calls them) -------------------------------

def _timed_probe(launch, repeats: int) -> float:
    """Best rate (units of the launch's return value per second) of `repeats` launches after one warm-up."""
    st = torch.cuda.current_stream()
    best = 0.0
    for i in range(repeats + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        n = int(launch(st.cuda_stream))
        e1.record(st)
        torch.cuda.synchronize()
        if n < 0:
            raise RuntimeError("probe: bad argument or refused launch")
        if i:
            best = max(best, n / (e0.elapsed_time(e1) * 1e-3))
    return best


def probe_mfma(iters: int = 2000, dtype: int = BF16, random_operands: bool = True, workgroups: int = 2048,
               repeats: int = 5) -> float:
    """TFLOP/s that nothing but matrix instructions sustain (best of `repeats` launches, HIP events)."""
    out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    return _timed_probe(lambda st: lib.probe_mfma(out.data_ptr(), workgroups, iters, int(dtype), int(bool(random_operands)), st),
                        repeats) / 1e12


def probe_softmax_valu(iters: int = 4000, full: bool = True, workgroups: int = 2048, repeats: int = 3) -> float:
    """Scores per second whose softmax vector work (multiply-add, exp2; with `full` also the row-sum addition and the
    conversion to bfloat16) the vector pipes sustain when they do nothing else."""
    out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    return _timed_probe(lambda st: lib.probe_softmax_valu(out.data_ptr(), workgroups, iters, int(bool(full)), st), repeats)


def probe_l2_read(region_kib: int = 1024, iters: int = 64, workgroups: int = 2048, repeats: int = 3) -> float:
    """Bytes per second the compute units read from regions that stay in their XCD's L2."""
    buf = torch.zeros(8 * region_kib * 256, dtype=torch.int32, device="cuda")
    out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    return _timed_probe(lambda st: lib.probe_l2_read(buf.data_ptr(), out.data_ptr(), region_kib, workgroups, iters, st), repeats)


def probe_launch_floor_us(workgroups: int = 256, threads: int = 256, launches: int = 200) -> float:
    """Microseconds per launch of a kernel that does nothing, back to back on the current stream (mean)."""
    st = torch.cuda.current_stream()
    for _ in range(20):
        lib.probe_empty(workgroups, threads, st.cuda_stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(launches):
        if lib.probe_empty(workgroups, threads, st.cuda_stream) != 0:
            raise RuntimeError("probe_empty: bad argument or refused launch")
    e1.record(st)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / launches


def probe_issue_share(iters: int = 400, workgroups: int = 256) -> dict:
    """What the two wavefronts of a SIMD cost each other, in shader-clock cycles (medians over all wavefronts):
    mfma_cycles_alone                       per 32x32x16 matrix instruction, its wavefront alone on the SIMD
    valu_cycles_per_64_scores_{bf16,f16}    the softmax's vector work of one score in each of the 64 lanes (the
                                            bfloat16 kernel's mix, or the binary16 one with its dot instructions),
                                            the wavefront alone on the SIMD
    ..._next_to_mfma                        the same while the other wavefront streams matrix instructions
    mfma_cycles_next_to_{bf16,f16}          per matrix instruction of that other wavefront meanwhile
    mfma_issue_cycles                       what one matrix instruction adds to the time of a vector wavefront without
                                            dot instructions (the bfloat16 mix)"""
    out = torch.zeros(workgroups * 16, dtype=torch.int64, device="cuda")
    st = torch.cuda.current_stream()

    def run(matrix_on, vmode):
        for _ in range(2):   # the second launch counts
            if lib.probe_issue_share(out.data_ptr(), workgroups, iters, matrix_on, vmode, st.cuda_stream) != 0:
                raise RuntimeError("probe_issue_share: bad argument or refused launch")
        torch.cuda.synchronize()
        r = out.cpu().reshape(workgroups, 8, 2).to(torch.float64)
        return r[:, :4].reshape(-1, 2), r[:, 4:].reshape(-1, 2)     # matrix wavefronts, vector wavefronts: (cycles, iterations)

    def med(t):
        return float(t.median())

    res = {}
    m, _ = run(1, 0)
    res["mfma_cycles_alone"] = med(m[:, 0] / (32.0 * m[:, 1]))
    for vmode, name in ((1, "bf16"), (2, "f16")):
        _, v0 = run(0, vmode)
        alone = med(v0[:, 0] / (32.0 * v0[:, 1]))
        m, v = run(1, vmode)
        together = med(v[:, 0] / (32.0 * v[:, 1]))
        mfma_per_cycle = med(32.0 * m[:, 1] / m[:, 0])
        res[f"valu_cycles_per_64_scores_{name}"] = alone
        res[f"valu_cycles_per_64_scores_{name}_next_to_mfma"] = together
        res[f"mfma_cycles_next_to_{name}"] = 1.0 / mfma_per_cycle
        if vmode == 1:
            res["mfma_issue_cycles"] = (together - alone) / (together * mfma_per_cycle)
    return res


def attn_fwd_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S, D, causal, scale, dtype, stream) -> int:
    """The C entry point as is: device addresses as ints (0 = NULL), returns the status."""
    return int(lib.attn_fwd(q_ptr or None, k_ptr or None, v_ptr or None, o_ptr or None, lse_ptr or None,
                            int(B), int(H), int(S), int(D), int(causal), float(scale), int(dtype),
                            stream or None))


def attn_fwd_o16_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S, D, causal, scale, dtype, stream) -> int:
    """attn_fwd_o16 as is: device addresses as ints (0 = NULL), returns the status."""
    return int(lib.attn_fwd_o16(q_ptr or None, k_ptr or None, v_ptr or None, o_ptr or None, lse_ptr or None,
                                int(B), int(H), int(S), int(D), int(causal), float(scale), int(dtype),
                                stream or None))


def attn_fwd_o16(q, k, v, causal: bool, scale: float, o=None, lse=None, stream=None, want_lse: bool = True):
    """attn_fwd_o16 on torch device tensors: as attn_fwd, with o in the dtype of q, k, v."""
    return attn_fwd(q, k, v, causal, scale, o=o, lse=lse, stream=stream, want_lse=want_lse, _o16=True)


def attn_fwd(q, k, v, causal: bool, scale: float, o=None, lse=None, stream=None, want_lse: bool = True,
             _o16: bool = False):
    """attn_fwd on torch device tensors.

    q, k, v : [B,H,S,D] contiguous torch.float16 or torch.bfloat16 tensors on the GPU.
    o, lse  : optional preallocated fp32 outputs ([B,H,S,D], [B,H,S]); allocated if None.
    stream  : a torch.cuda.Stream (default: the current stream).
    Returns (o, lse).  Asynchronous, like the C call.
    """
    if q.dtype == torch.float16:
        dtype = F16
    elif q.dtype == torch.bfloat16:
        dtype = BF16
    else:
        raise TypeError("q, k, v must be float16 or bfloat16")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share one dtype")
    if q.dim() != 4 or k.shape != q.shape or v.shape != q.shape:
        raise ValueError("q, k, v must be [B,H,S,D] of one shape")
    for t in (q, k, v):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("q, k, v must be contiguous device tensors")
    B, H, S, D = q.shape
    odt = q.dtype if _o16 else torch.float32
    if o is None:
        o = torch.empty((B, H, S, D), dtype=odt, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty((B, H, S), dtype=torch.float32, device=q.device)
    for t, shp, dt in ((o, (B, H, S, D), odt), (lse, (B, H, S), torch.float32)):
        if t is not None and (t.dtype != dt or tuple(t.shape) != shp or not t.is_contiguous() or not t.is_cuda):
            raise ValueError("o / lse must be contiguous device tensors of shape [B,H,S,D] / [B,H,S] (lse fp32; o fp32, "
                             "or the input dtype for attn_fwd_o16)")
    st = (stream or torch.cuda.current_stream(q.device)).cuda_stream
    rc = (attn_fwd_o16_raw if _o16 else attn_fwd_raw)(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                                      lse.data_ptr() if lse is not None else 0, B, H, S, D, causal, scale,
                                                      dtype, st)
    if rc != 0:
        raise AttnError(rc, attn_status_str(rc))
    return o, lse


# ---- include/rowops.h ------------------------------------------------------------------------

class RowopsError(RuntimeError):
    def __init__(self, what: str, status: int, msg: str):
        super().__init__(f"{what} failed with status {status}: {msg}")
        self.status = status


def rowops_status_str(status: int) -> str:
    return lib.rowops_status_str(int(status)).decode()


def rowops_path(op: int, row_len: int, dtype: int) -> int:
    return int(lib.rowops_path(int(op), int(row_len), int(dtype)))


def softmax_rows_fwd_raw(x_ptr, y_ptr, n_rows, n_cols, dtype, stream) -> int:
    """The C entry point as is: device addresses as ints (0 = NULL), returns the status."""
    return int(lib.softmax_rows_fwd(x_ptr or None, y_ptr or None, int(n_rows), int(n_cols), int(dtype), stream or None))


def rmsnorm_fwd_raw(x_ptr, w_ptr, y_ptr, n_rows, d, eps, dtype, stream) -> int:
    """The C entry point as is: device addresses as ints (0 = NULL), returns the status."""
    return int(lib.rmsnorm_fwd(x_ptr or None, w_ptr or None, y_ptr or None, int(n_rows), int(d), float(eps), int(dtype),
                               stream or None))


def _row_args(x, y):
    if x.dtype == torch.float16:
        dtype = F16
    elif x.dtype == torch.bfloat16:
        dtype = BF16
    else:
        raise TypeError("x must be float16 or bfloat16")
    if x.dim() < 1 or not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous device tensor with the rows along the last dimension")
    if y is None:
        y = torch.empty_like(x)
    elif y.dtype != x.dtype or y.shape != x.shape or not y.is_cuda or not y.is_contiguous():
        raise ValueError("y must be a contiguous device tensor of the shape and dtype of x")
    n = x.shape[-1]
    return dtype, y, (x.numel() // n if n else 0), n


def softmax_rows_fwd(x, y=None, stream=None):
    """softmax_rows_fwd on a torch device tensor: softmax over the last dimension, result in x's dtype."""
    dtype, y, n_rows, n = _row_args(x, y)
    st = (stream or torch.cuda.current_stream(x.device)).cuda_stream
    rc = softmax_rows_fwd_raw(x.data_ptr(), y.data_ptr(), n_rows, n, dtype, st)
    if rc != 0:
        raise RowopsError("softmax_rows_fwd", rc, rowops_status_str(rc))
    return y


def rmsnorm_fwd(x, w, eps: float, y=None, stream=None):
    """rmsnorm_fwd on torch device tensors: x [..., d], w [d] of one dtype; result in x's dtype."""
    dtype, y, n_rows, n = _row_args(x, y)
    if w.dtype != x.dtype or tuple(w.shape) != (n,) or not w.is_cuda or not w.is_contiguous():
        raise ValueError("w must be a contiguous device tensor [d] of x's dtype")
    st = (stream or torch.cuda.current_stream(x.device)).cuda_stream
    rc = rmsnorm_fwd_raw(x.data_ptr(), w.data_ptr(), y.data_ptr(), n_rows, n, eps, dtype, st)
    if rc != 0:
        raise RowopsError("rmsnorm_fwd", rc, rowops_status_str(rc))
    return y


# ---- include/gemm.h --------------------------------------------------------------------------

class GemmError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"gemm_leakyrelu_fwd failed with status {status}: {msg}")
        self.status = status


def gemm_status_str(status: int) -> str:
    return lib.gemm_status_str(int(status)).decode()


def gemm_path(batch: int, M: int, N: int, K: int, dtype: int) -> int:
    return int(lib.gemm_path(int(batch), int(M), int(N), int(K), int(dtype)))


def gemm_leakyrelu_fwd_raw(a_ptr, b_ptr, c_ptr, batch, M, N, K, slope, dtype, stream) -> int:
    """The C entry point as is: device addresses as ints (0 = NULL), returns the status."""
    return int(lib.gemm_leakyrelu_fwd(a_ptr or None, b_ptr or None, c_ptr or None, int(batch), int(M), int(N), int(K),
                                      float(slope), int(dtype), stream or None))


def gemm_leakyrelu_fwd(a, b, slope: float = 0.01, c=None, stream=None):
    """gemm_leakyrelu_fwd on torch device tensors: a [batch, M, K] (or [M, K]), b [batch, K, N] (or [K, N])
    of one 16-bit dtype; returns c [batch, M, N] (or [M, N]) in that dtype."""
    if a.dtype == torch.float16:
        dtype = F16
    elif a.dtype == torch.bfloat16:
        dtype = BF16
    else:
        raise TypeError("a and b must be float16 or bfloat16")
    if b.dtype != a.dtype or a.dim() != b.dim() or a.dim() not in (2, 3):
        raise TypeError("a and b must share one dtype and be both [M,K],[K,N] or both [batch,M,K],[batch,K,N]")
    a3, b3 = (a, b) if a.dim() == 3 else (a[None], b[None])
    if a3.shape[0] != b3.shape[0] or a3.shape[2] != b3.shape[1]:
        raise ValueError("a must be [batch, M, K] and b [batch, K, N]")
    for t in (a, b):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("a and b must be contiguous device tensors")
    batch, M, K = a3.shape
    N = b3.shape[2]
    shape = (batch, M, N) if a.dim() == 3 else (M, N)
    if c is None:
        c = torch.empty(shape, dtype=a.dtype, device=a.device)
    elif c.dtype != a.dtype or tuple(c.shape) != shape or not c.is_cuda or not c.is_contiguous():
        raise ValueError("c must be a contiguous device tensor [batch, M, N] of the dtype of a")
    st = (stream or torch.cuda.current_stream(a.device)).cuda_stream
    rc = gemm_leakyrelu_fwd_raw(a.data_ptr(), b.data_ptr(), c.data_ptr(), batch, M, N, K, slope, dtype, st)
    if rc != 0:
        raise GemmError(rc, gemm_status_str(rc))
    return c
