"""fp64 CPU oracle for the two memory-bound row operations -- TEST INFRASTRUCTURE ONLY.

The paper evaluates two memory-bound kernels next to the compute-bound ones (Table 2: softmax over
n_rows x n_cols = 512 x 4096, rmsnorm over B, n_head, seq_len, d_head = 1, 32, 4096, 64, both float16)
and names them without a formula (Section 5.1); both have a plain textbook definition, which is what
is written out here, in numpy float64, on the already rounded 16-bit inputs:

  softmax   y[i, j] = exp(x[i, j] - m_i) / sum_j' exp(x[i, j'] - m_i),   m_i = max_j x[i, j]
  rmsnorm   y[i, j] = x[i, j] / sqrt(mean_j' x[i, j']^2 + eps) * w[j]

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
    if dtype == BF16:   # bfloat16 is the upper half of a binary32
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"dtype {dtype}")


def softmax_f64(x: np.ndarray) -> np.ndarray:
    """Row softmax of a float64 matrix [n_rows, n_cols], two passes per row, as defined above."""
    x = np.asarray(x, dtype=np.float64)
    if x.ndim != 2 or x.shape[1] < 1:
        raise ValueError("x must be [n_rows, n_cols >= 1]")
    y = np.empty_like(x)
    for i in range(x.shape[0]):
        m = x[i].max()
        e = np.exp(x[i] - m)
        y[i] = e / e.sum()
    return y


def rmsnorm_f64(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """Row RMS normalisation of a float64 matrix [n_rows, d] with weight [d], as defined above."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    if x.ndim != 2 or x.shape[1] < 1 or w.shape != (x.shape[1],):
        raise ValueError("x must be [n_rows, d >= 1] and w [d]")
    y = np.empty_like(x)
    for i in range(x.shape[0]):
        ms = (x[i] * x[i]).sum() / x.shape[1]
        y[i] = x[i] / np.sqrt(ms + eps) * w
    return y


def softmax_rows(x_bits, dtype: int) -> np.ndarray:
    """Row softmax of 16-bit inputs [n_rows, n_cols] (uint16 patterns); float64 result."""
    return softmax_f64(widen(x_bits, dtype))


def rmsnorm_rows(x_bits, w_bits, eps: float, dtype: int) -> np.ndarray:
    """RMS normalisation of 16-bit inputs x [n_rows, d], w [d] (uint16 patterns); float64 result."""
    return rmsnorm_f64(widen(x_bits, dtype), widen(w_bits, dtype), float(eps))
