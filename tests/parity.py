"""Shared helpers of the GPU parity tests: run the HIP path on bit patterns, compare with the oracle."""
import numpy as np
import torch

import oracle
import paper_2501_08071_amd as P
from paper_2501_08071_amd import inputs as I

# the bar for fp16/bf16 inputs: max-abs 2e-2 and mean-abs 2e-3 on O; logsumexp within 1e-3 relative,
# read as |d| <= 1e-3 * max(1, |lse_ref|) because a pure relative error is undefined at lse = 0
MAX_ABS = 2e-2
MEAN_ABS = 2e-3
LSE_REL = 1e-3


def to_device(bits: np.ndarray, dtype: int) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.float16 if dtype == I.F16 else torch.bfloat16)


def run_gpu(q, k, v, dtype, causal, scale, want_lse=True):
    dq, dk, dv = (to_device(t, dtype) for t in (q, k, v))
    o, lse = P.attn_fwd(dq, dk, dv, causal, scale, want_lse=want_lse)
    torch.cuda.synchronize()
    return o.cpu().numpy(), (lse.cpu().numpy() if lse is not None else None)


def errors(o_gpu, lse_gpu, o_ref, lse_ref):
    d = np.abs(o_gpu.astype(np.float64) - o_ref)
    dl = np.abs(lse_gpu.astype(np.float64) - lse_ref) / np.maximum(1.0, np.abs(lse_ref))
    return float(d.max()), float(d.mean()), float(dl.max())


def assert_parity(o_gpu, lse_gpu, o_ref, lse_ref, what=""):
    assert np.isfinite(o_gpu).all() and np.isfinite(lse_gpu).all(), f"{what}: non-finite output"
    mx, mean, lrel = errors(o_gpu, lse_gpu, o_ref, lse_ref)
    assert mx <= MAX_ABS, f"{what}: max-abs {mx:.3e} > {MAX_ABS}"
    assert mean <= MEAN_ABS, f"{what}: mean-abs {mean:.3e} > {MEAN_ABS}"
    assert lrel <= LSE_REL, f"{what}: lse rel {lrel:.3e} > {LSE_REL}"
    return mx, mean, lrel


def check_full(q, k, v, dtype, causal, scale, what=""):
    o, lse = run_gpu(q, k, v, dtype, causal, scale)
    o_ref, lse_ref = oracle.attn_oracle(q, k, v, causal, scale, dtype)
    return assert_parity(o, lse, o_ref, lse_ref, what)


def edge_rows(S: int, br: int, bc: int, extra: int, seed: int) -> np.ndarray:
    """First/last rows, every query-tile and key-tile edge +-1, plus `extra` seeded random rows."""
    rows = {0, 1, S - 2, S - 1}
    for step in (br, bc, 32):
        for e in range(step, S, step):
            rows.update((e - 1, e, e + 1))
    rows = {r for r in rows if 0 <= r < S}
    rng = np.random.default_rng(seed)
    rows.update(int(r) for r in rng.integers(0, S, extra))
    return np.array(sorted(rows), np.int32)
