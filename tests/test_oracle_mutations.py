"""Planted mistakes (in a copy of the oracle, on the CPU) must be caught by the pins.

Each mutation rewrites one expression of oracle/attn_oracle.c into a plausible slip,
compiles the copy, and runs three pins against it: the zero-query closed form, the
causal-first-row identity and the library fp64 softmax.  A mutation that survives
all three would mean the pins are too weak.
"""
import ctypes
import math
import os
import subprocess

import numpy as np
import pytest
import torch

from paper_2501_08071_amd import inputs as I

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "attn_oracle.c")

MUTATIONS = {
    "none": None,
    "scale_dropped": ("s[j] = scale * dot;", "s[j] = dot;"),
    "mask_excludes_diagonal": ("const int nj = causal ? i + 1 : S;", "const int nj = causal ? (i > 0 ? i : 1) : S;"),
    "mask_off_by_one_wide": ("const int nj = causal ? i + 1 : S;", "const int nj = causal ? (i + 2 < S ? i + 2 : S) : S;"),
    "no_normalisation": ("for (int d = 0; d < D; ++d) orow[d] /= l;", ""),
    "lse_log2": ("= m + log(l);", "= m + log2(l);"),
    "lse_without_max": ("= m + log(l);", "= log(l);"),
    "k_transposed_index": ("dot += qd[d] * kd[(size_t)j * D + d];", "dot += qd[d] * kd[((size_t)d * S + j) % ((size_t)S * D)];"),
    "v_row_shifted": ("orow[d] += s[j] * vd[(size_t)j * D + d];", "orow[d] += s[j] * vd[(size_t)(j ? j - 1 : 0) * D + d];"),
    "sign_flipped": ("s[j] = exp(s[j] - m);", "s[j] = exp(m - s[j]);"),
    "bf16_shift_wrong": ("uint32_t bits = ((uint32_t)h) << 16;", "uint32_t bits = ((uint32_t)h) << 15;"),
    "f16_bias_wrong": ("expo - 25);", "expo - 24);"),
}


def _compile(tmp_path, name, mut):
    src = open(SRC).read()
    if mut is not None:
        assert src.count(mut[0]) == 1, f"mutation anchor for {name} not unique"
        src = src.replace(mut[0], mut[1])
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(src)
    subprocess.run(["gcc", "-O1", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    u16p, f64p = ctypes.POINTER(ctypes.c_uint16), ctypes.POINTER(ctypes.c_double)
    lib.attn_oracle.argtypes = [u16p] * 3 + [ctypes.c_int] * 5 + [ctypes.c_double, ctypes.c_int, f64p, f64p]
    return lib


def _run(lib, q, k, v, causal, scale, dtype):
    B, H, S, D = q.shape
    o, lse = np.empty((B, H, S, D)), np.empty((B, H, S))
    ptr = lambda a, t: a.ctypes.data_as(ctypes.POINTER(t))
    rc = lib.attn_oracle(ptr(q, ctypes.c_uint16), ptr(k, ctypes.c_uint16), ptr(v, ctypes.c_uint16),
                         B, H, S, D, int(causal), scale, dtype, ptr(o, ctypes.c_double), ptr(lse, ctypes.c_double))
    assert rc == 0
    return o, lse


def _pins_hold(lib) -> bool:
    ok = True
    for dtype in (I.F16, I.BF16):
        S, D, scale = 24, 8, 0.4
        q, k, v = I.gen_tensors(1, 2, S, D, dtype, workload_id=90)
        Q, K, V = (I.bits_to_f64(t, dtype) for t in (q, k, v))
        # zero-query closed form (causal): running mean of V, lse = ln(i+1)
        o, lse = _run(lib, np.zeros_like(q), k, v, True, scale, dtype)
        ok &= np.abs(o - np.cumsum(V, 2) / np.arange(1, S + 1)[None, None, :, None]).max() < 1e-12
        ok &= np.abs(lse - np.log(np.arange(1, S + 1))).max() < 1e-12
        # causal first row
        o, lse = _run(lib, q, k, v, True, scale, dtype)
        ok &= np.abs(o[:, :, 0] - V[:, :, 0]).max() < 1e-12
        ok &= np.abs(lse[:, :, 0] - scale * (Q[:, :, 0] * K[:, :, 0]).sum(-1)).max() < 1e-12
        # library softmax, both mask settings
        for causal in (False, True):
            o, lse = _run(lib, q, k, v, causal, scale, dtype)
            s = torch.from_numpy(Q) @ torch.from_numpy(K).transpose(-1, -2) * scale
            if causal:
                s = s.masked_fill(torch.ones(S, S, dtype=torch.bool).triu(1), float("-inf"))
            ok &= np.abs(o - (torch.softmax(s, -1) @ torch.from_numpy(V)).numpy()).max() < 1e-12
            ok &= np.abs(lse - torch.logsumexp(s, -1).numpy()).max() < 1e-12
    return bool(ok)


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_mutation_is_caught(tmp_path, name):
    lib = _compile(tmp_path, name, MUTATIONS[name])
    if name == "none":
        assert _pins_hold(lib)
    else:
        assert not _pins_hold(lib), f"planted mistake '{name}' survived the pins"
