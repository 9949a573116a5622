"""Every schedule variant the tuner can visit must compute attention: parity against the oracle."""
import ctypes
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2501_08071_amd import inputs as I
from paper_2501_08071_amd import tune
from parity import assert_parity, to_device

pytestmark = pytest.mark.gpu
BUILT = [s for s in tune.all_states() if os.path.exists(tune.variant_path(s))]


# Small problems take the instances with four wavefronts per workgroup; the wide one has more than 128 tiles and takes the
# eight-wavefront instance (or, in its state, the kernel with 64 query rows per wavefront), which is what the tuner times
# on the benchmark workloads; the D = 32 shape runs the interleaved loop (barrier period, operand read-ahead).
SHAPES = [(1, 2, 300, 128, I.BF16, True), (1, 2, 517, 64, I.F16, False), (1, 1, 640, 128, I.F16, False),
          (3, 43, 300, 128, I.BF16, True), (3, 43, 257, 64, I.F16, True), (1, 2, 300, 32, I.F16, True)]


@pytest.mark.skipif(not BUILT, reason="schedule variants not built (python -m paper_2501_08071_amd.tune build)")
@pytest.mark.parametrize("state", BUILT, ids=tune.state_name)
def test_variant_parity(state):
    lib = ctypes.CDLL(tune.variant_path(state))
    vp = ctypes.c_void_p
    lib.attn_fwd.argtypes = [vp] * 5 + [ctypes.c_int] * 5 + [ctypes.c_float, ctypes.c_int, vp]
    lib.attn_launch_rows.argtypes = [ctypes.c_int] * 6
    lib.attn_kernel_name.argtypes = [ctypes.c_int] * 6
    lib.attn_kernel_name.restype = ctypes.c_char_p
    for (B, H, S, D, dtype, causal) in SHAPES:
        wide = B * H > 128
        assert lib.attn_launch_rows(B, H, S, D, dtype, int(causal)) == (256 if wide else 128)
        name = lib.attn_kernel_name(B, H, S, D, dtype, int(causal)).decode()
        assert ("rows64" in name) == (wide and D == 128 and dict(zip(tune.KNOBS, state))["rows64"] == 1)
        q, k, v = I.gen_tensors(B, H, S, D, dtype, workload_id=300 + D)
        dq, dk, dv = (to_device(t, dtype) for t in (q, k, v))
        o = torch.empty((B, H, S, D), dtype=torch.float32, device="cuda")
        lse = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
        scale = 1.0 / np.sqrt(D)
        rc = lib.attn_fwd(dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, S, D, int(causal),
                          scale, dtype, None)
        assert rc == 0
        torch.cuda.synchronize()
        o_ref, l_ref = oracle.attn_oracle(q, k, v, causal, scale, dtype)
        assert_parity(o.cpu().numpy(), lse.cpu().numpy(), o_ref, l_ref, f"{tune.state_name(state)} B={B} H={H} S={S} D={D}")


# Longer runs for the race detector: several wraps of the LDS buffer ring, causal (wavefronts that finish early keep
# issuing loads), ragged last blocks, both launch modes, all three head dimensions.
POISON_SHAPES = SHAPES + [(1, 2, 1100, 128, I.BF16, True), (2, 70, 700, 128, I.F16, False), (1, 3, 1500, 64, I.F16, True),
                          (2, 70, 900, 64, I.BF16, True), (1, 2, 1100, 32, I.F16, True), (2, 70, 500, 32, I.BF16, False)]


@pytest.mark.skipif(not os.path.exists(tune.POISON_LIB), reason="debug build not there (python -m paper_2501_08071_amd.tune build)")
def test_poisoned_buffers_parity():
    """The shipped schedule built with every LDS buffer filled with NaN patterns right before the load that overwrites
    it: a read of a buffer that was already given away (a load issued too early, a missing barrier) would put a NaN
    into the output.  Everything finite and within the bar means no such read happened on these shapes."""
    lib = ctypes.CDLL(tune.POISON_LIB)
    vp = ctypes.c_void_p
    lib.attn_fwd.argtypes = [vp] * 5 + [ctypes.c_int] * 5 + [ctypes.c_float, ctypes.c_int, vp]
    for (B, H, S, D, dtype, causal) in POISON_SHAPES:
        q, k, v = I.gen_tensors(B, H, S, D, dtype, workload_id=500 + D)
        dq, dk, dv = (to_device(t, dtype) for t in (q, k, v))
        o = torch.empty((B, H, S, D), dtype=torch.float32, device="cuda")
        lse = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
        scale = 1.0 / np.sqrt(D)
        for _ in range(3):   # timing differs from launch to launch
            o.zero_()
            rc = lib.attn_fwd(dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, S, D, int(causal),
                              scale, dtype, None)
            assert rc == 0
            torch.cuda.synchronize()
            assert bool(torch.isfinite(o).all()) and bool(torch.isfinite(lse).all()), f"poison reached the output: B={B} H={H} S={S} D={D}"
        o_ref, l_ref = oracle.attn_oracle(q, k, v, causal, scale, dtype)
        assert_parity(o.cpu().numpy(), lse.cpu().numpy(), o_ref, l_ref, f"debug_poison B={B} H={H} S={S} D={D}")
