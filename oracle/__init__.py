"""fp64 CPU oracle for fused attention forward -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``attn_oracle.c`` (the plain two-pass definition of
``O = softmax(Q K^T * scale [+ causal mask]) V`` and its logsumexp).  Only the
tests, the smoke check and the bench's ``cpu_baseline`` leg may import this
package; the product path never does, and this package imports nothing from
the HIP side.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F16 = 0
BF16 = 1


def build(force: bool = False) -> str:
    """Compile attn_oracle.c with gcc (no fast-math: fp64 sums stay in written order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int)
        common = [u16p, u16p, u16p] + [ctypes.c_int] * 5 + [ctypes.c_double, ctypes.c_int]
        lib.attn_oracle_rows.argtypes = common + [i32p, ctypes.c_int, f64p, f64p]
        lib.attn_oracle_rows.restype = ctypes.c_int
        lib.attn_oracle.argtypes = common + [f64p, f64p]
        lib.attn_oracle.restype = ctypes.c_int
        lib.attn_bruteforce.argtypes = common + [f64p, f64p, f64p]
        lib.attn_bruteforce.restype = ctypes.c_int
        lib.oracle_widen.argtypes = [ctypes.c_uint, ctypes.c_int]
        lib.oracle_widen.restype = ctypes.c_double
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _bits(a, shape):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("oracle inputs are uint16 bit patterns (binary16 or bfloat16)")
    if a.shape != shape:
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def attn_oracle(q, k, v, causal: bool, scale: float, dtype: int, rows=None):
    """Attention forward in fp64.

    q, k, v : uint16 arrays [B,H,S,D] holding binary16 (dtype=F16) or bfloat16
              (dtype=BF16) bit patterns.
    rows    : optional 1-D int array of query rows; the same subset is
              evaluated for every (b,h).  Rows are independent, so the subset
              result is exact for the rows it covers.
    returns : (O [B,H,R,D] float64, lse [B,H,R] float64) with R = len(rows) or S.
    """
    lib = _load()
    B, H, S, D = q.shape
    q, k, v = (_bits(x, (B, H, S, D)) for x in (q, k, v))
    if rows is None:
        o = np.empty((B, H, S, D), np.float64)
        lse = np.empty((B, H, S), np.float64)
        rc = lib.attn_oracle(_p(q, ctypes.c_uint16), _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16),
                             B, H, S, D, int(bool(causal)), float(scale), int(dtype),
                             _p(o, ctypes.c_double), _p(lse, ctypes.c_double))
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        R = rows.shape[0]
        o = np.empty((B, H, R, D), np.float64)
        lse = np.empty((B, H, R), np.float64)
        rc = lib.attn_oracle_rows(_p(q, ctypes.c_uint16), _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16),
                                  B, H, S, D, int(bool(causal)), float(scale), int(dtype),
                                  _p(rows, ctypes.c_int), R,
                                  _p(o, ctypes.c_double), _p(lse, ctypes.c_double))
    if rc != 0:
        raise ValueError("attn_oracle: bad argument")
    return o, lse


def attn_bruteforce(q, k, v, causal: bool, scale: float, dtype: int):
    """Long-double, full-matrix, no-max-subtraction twin (tiny shapes, small logits).

    returns (O [B,H,S,D], lse [B,H,S], P [B,H,S,S]) as float64.
    """
    lib = _load()
    B, H, S, D = q.shape
    q, k, v = (_bits(x, (B, H, S, D)) for x in (q, k, v))
    o = np.empty((B, H, S, D), np.float64)
    lse = np.empty((B, H, S), np.float64)
    p = np.empty((B, H, S, S), np.float64)
    rc = lib.attn_bruteforce(_p(q, ctypes.c_uint16), _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16),
                             B, H, S, D, int(bool(causal)), float(scale), int(dtype),
                             _p(o, ctypes.c_double), _p(lse, ctypes.c_double), _p(p, ctypes.c_double))
    if rc != 0:
        raise ValueError("attn_bruteforce: bad argument")
    return o, lse, p


def widen(bits16: int, dtype: int) -> float:
    """The oracle's own 16-bit -> fp64 decoder, exposed so tests can pin it."""
    return float(_load().oracle_widen(int(bits16), int(dtype)))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))
