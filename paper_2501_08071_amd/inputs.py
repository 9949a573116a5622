"""Seeded synthetic inputs for the attention-forward workloads.

This module serves both the CPU oracle's tests and the HIP path, and therefore
holds none of the method's arithmetic: it only draws reproducible random
numbers and rounds them to 16 bits.

Generator: a counter-based SplitMix64 stream (Steele, Lea, Flood 2014: the
state after n steps is seed + n*0x9E3779B97F4A7C15, passed through the
published 64-bit finaliser).  Element n of a tensor uses counters 2n and 2n+1:
two uniforms in (0,1) -> one standard normal by Box-Muller in fp64, cast to
fp32, scaled in fp32, then rounded to nearest-even binary16 / bfloat16.
Uniform tensors use counter 2n only.  Each tensor has its own stream, keyed by
(base seed, workload id, tensor id), so values do not depend on any library's
RNG or version.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

F16 = 0
BF16 = 1
BASE_SEED = 20250108

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1


@dataclass(frozen=True)
class Workload:
    """One synthetic attention-forward workload (shape, dtype, distributions)."""
    id: int
    name: str
    B: int
    H: int
    S: int
    D: int
    dtype: int            # F16 / BF16 : the type of q, k, v
    causal: bool
    qk_dist: str          # "normal"
    qk_mul: float         # multiplier applied in fp32 before rounding
    v_dist: str           # "normal" | "uniform_pm1"

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def flops(self) -> float:
        """Counted FLOPs: 4*B*H*S^2*D, halved under the causal mask."""
        f = 4.0 * self.B * self.H * self.S * self.S * self.D
        return f / 2 if self.causal else f

    @property
    def dtype_name(self) -> str:
        return "f16" if self.dtype == F16 else "bf16"


# The five workloads: ids follow the order of the benchmark configuration list.
WORKLOADS = (
    Workload(1, "B1_H1_S128_D64_f16", 1, 1, 128, 64, F16, False, "normal", 1.0, "normal"),
    Workload(2, "B4_H16_S1024_D64_f16", 4, 16, 1024, 64, F16, False, "normal", 1.0, "normal"),
    Workload(3, "B2_H32_S4096_D128_bf16_causal", 2, 32, 4096, 128, BF16, True, "normal", 1.0, "normal"),
    Workload(4, "B1_H32_S16384_D128_bf16_causal", 1, 32, 16384, 128, BF16, True, "normal", 1.0, "normal"),
    Workload(5, "B16_H16_S2048_D64_f16_peaky", 16, 16, 2048, 64, F16, False, "normal", 4.0, "uniform_pm1"),
)
# Not one of the five: the shape the paper runs its flash-attention kernel on (Table 2: B, n_head, seq_len,
# d_head = 1, 4, 4096, 32, fp16); the paper does not say whether it is causal, both are kept.
EXTRA_WORKLOADS = (
    Workload(6, "B1_H4_S4096_D32_f16_paper", 1, 4, 4096, 32, F16, False, "normal", 1.0, "normal"),
    Workload(7, "B1_H4_S4096_D32_f16_paper_causal", 1, 4, 4096, 32, F16, True, "normal", 1.0, "normal"),
)


def workload(wid: int) -> Workload:
    return (WORKLOADS + EXTRA_WORKLOADS)[wid - 1]


# ---- SplitMix64 -------------------------------------------------------------------------

def _mix_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def splitmix64_scalar(seed: int, n: int) -> int:
    """Output number n (0-based) of the SplitMix64 stream started at `seed`."""
    return _mix_int(seed + (n + 1) * 0x9E3779B97F4A7C15)


def splitmix64(seed: int, counters: np.ndarray) -> np.ndarray:
    """Vectorised: output number counters[i] of the stream started at `seed`."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed & _MASK64) + (counters.astype(np.uint64) + np.uint64(1)) * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def tensor_seed(base_seed: int, workload_id: int, tensor_id: int) -> int:
    """Independent stream key for one tensor (tensor_id: 0=q, 1=k, 2=v)."""
    return _mix_int(_mix_int(_mix_int(base_seed) + workload_id) + tensor_id)


def _uniform01(seed: int, counters: np.ndarray) -> np.ndarray:
    """Uniform in the open interval (0,1): (top 53 bits + 0.5) / 2^53."""
    return ((splitmix64(seed, counters) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


# ---- rounding to 16 bits ----------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bfloat16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> IEEE binary16 bit patterns."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    return f32_to_f16_bits(x) if dtype == F16 else f32_to_bf16_bits(x)


def bits_to_f64(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of 16-bit patterns (used by tests to build expectations)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


# ---- tensors ----------------------------------------------------------------------------

_CHUNK = 1 << 21


def _fill(seed: int, n: int, dist: str, mul: float, dtype: int) -> np.ndarray:
    out = np.empty(n, np.uint16)

    def work(start: int) -> None:
        stop = min(n, start + _CHUNK)
        idx = np.arange(start, stop, dtype=np.uint64)
        if dist == "normal":
            u1 = _uniform01(seed, idx * np.uint64(2))
            u2 = _uniform01(seed, idx * np.uint64(2) + np.uint64(1))
            z = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * np.pi) * u2)
        elif dist == "uniform_pm1":
            z = 2.0 * _uniform01(seed, idx * np.uint64(2)) - 1.0
        else:
            raise ValueError(dist)
        x = z.astype(np.float32) * np.float32(mul)
        out[start:stop] = to_bits(x, dtype)

    starts = range(0, n, _CHUNK)
    if n <= _CHUNK:
        work(0)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(work, starts))
    return out


def gen_tensors(B: int, H: int, S: int, D: int, dtype: int, *, workload_id: int = 0,
                seed: int = BASE_SEED, qk_mul: float = 1.0, v_dist: str = "normal"):
    """q, k, v as uint16 bit patterns, each [B,H,S,D] contiguous."""
    n = B * H * S * D
    shape = (B, H, S, D)
    q = _fill(tensor_seed(seed, workload_id, 0), n, "normal", qk_mul, dtype).reshape(shape)
    k = _fill(tensor_seed(seed, workload_id, 1), n, "normal", qk_mul, dtype).reshape(shape)
    v = _fill(tensor_seed(seed, workload_id, 2), n, v_dist, 1.0, dtype).reshape(shape)
    return q, k, v


def gen_inputs(w: Workload, seed: int = BASE_SEED):
    """The three input tensors of a named workload."""
    return gen_tensors(w.B, w.H, w.S, w.D, w.dtype, workload_id=w.id, seed=seed,
                       qk_mul=w.qk_mul, v_dist=w.v_dist)


# ---- row operations (the paper's memory-bound kernels, Table 2) ---------------------------

ROWOP_SHAPES = {
    "softmax_512x4096_f16": ("softmax", 512, 4096, F16),            # n_rows, n_cols (Table 2)
    "rmsnorm_1x32x4096x64_f16": ("rmsnorm", 1 * 32 * 4096, 64, F16),   # B * n_head * seq_len rows of d_head (Table 2)
}


def gen_rows(n_rows: int, n_cols: int, dtype: int, *, tensor_id: int = 0, seed: int = BASE_SEED,
             dist: str = "normal", mul: float = 1.0) -> np.ndarray:
    """A seeded [n_rows, n_cols] matrix of 16-bit patterns (tensor_id separates x from the weight)."""
    return _fill(tensor_seed(seed, 100, tensor_id), n_rows * n_cols, dist, mul, dtype).reshape(n_rows, n_cols)


GEMM_SHAPES = {
    "mmLeakyReLu_1x512x512x2048_f16": (1, 512, 512, 2048, F16),      # B, M, N, K (Table 2)
    "bmm_4x512x512x2048_f16": (4, 512, 512, 2048, F16),              # Table 2's batch matrix multiplication: the same kernel with slope 1
}


def gen_gemm(batch: int, M: int, N: int, K: int, dtype: int, *, seed: int = BASE_SEED):
    """Seeded a [batch, M, K] and b [batch, K, N] as 16-bit patterns, entries N(0,1)."""
    a = _fill(tensor_seed(seed, 200, 0), batch * M * K, "normal", 1.0, dtype).reshape(batch, M, K)
    b = _fill(tensor_seed(seed, 200, 1), batch * K * N, "normal", 1.0, dtype).reshape(batch, K, N)
    return a, b
