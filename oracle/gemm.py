"""fp64 CPU oracle for the fused GEMM + LeakyReLU -- TEST INFRASTRUCTURE ONLY.

The paper's second compute-bound kernel (Table 2: mmLeakyReLu, B, M, N, K = 1, 512, 512, 2048, float16;
Section 5.1 describes it as a matrix product with the activation fused into its epilogue; Section 5.4 studies
its schedule).  No formula is
given; the plain definition is

    c[b, m, n] = f( sum_k a[b, m, k] * b[b, k, n] ),      f(t) = t if t >= 0 else slope * t

on the already rounded 16-bit inputs, in float64.  The matrix product is numpy's (a library primitive as
one step); `gemm_leakyrelu_loops` is a second routine that writes the triple loop out.

Only the tests, the smoke check and the bench's cpu_baseline leg may import this module; the product
path never does, and this module imports nothing from the HIP side.
"""
from __future__ import annotations

import numpy as np

F16 = 0
BF16 = 1


def widen(bits, dtype: int) -> np.ndarray:
    """16-bit patterns (uint16) -> float64, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == F16:
        return b.view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"dtype {dtype}")


def leaky_relu_f64(t: np.ndarray, slope: float) -> np.ndarray:
    t = np.asarray(t, dtype=np.float64)
    return np.where(t >= 0.0, t, slope * t)


def gemm_leakyrelu_f64(a: np.ndarray, b: np.ndarray, slope: float) -> np.ndarray:
    """a [batch, M, K], b [batch, K, N] (float64) -> [batch, M, N]."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if a.ndim != 3 or b.ndim != 3 or a.shape[0] != b.shape[0] or a.shape[2] != b.shape[1]:
        raise ValueError("a must be [batch, M, K] and b [batch, K, N]")
    return leaky_relu_f64(np.matmul(a, b), float(slope))


def gemm_leakyrelu_loops(a: np.ndarray, b: np.ndarray, slope: float) -> np.ndarray:
    """The same by three written-out loops (tiny shapes only)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    nb, M, K = a.shape
    N = b.shape[2]
    c = np.zeros((nb, M, N))
    for i in range(nb):
        for m in range(M):
            for n in range(N):
                t = 0.0
                for k in range(K):
                    t += a[i, m, k] * b[i, k, n]
                c[i, m, n] = t if t >= 0.0 else slope * t
    return c


def gemm_leakyrelu(a_bits, b_bits, slope: float, dtype: int) -> np.ndarray:
    """16-bit inputs a [batch, M, K], b [batch, K, N] (uint16 patterns); float64 result."""
    return gemm_leakyrelu_f64(widen(a_bits, dtype), widen(b_bits, dtype), slope)


def abs_product(a_bits, b_bits, dtype: int) -> np.ndarray:
    """sum_k |a[m,k]| |b[k,n]|: the scale of the rounding error of any summation order (for tolerances)."""
    return np.matmul(np.abs(widen(a_bits, dtype)), np.abs(widen(b_bits, dtype)))
