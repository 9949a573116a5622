"""Parity of the HIP row kernels (softmax, rmsnorm; include/rowops.h) against the float64 oracle.

Tolerance.  Both kernels compute in fp32 and round once, to nearest even, into the 16-bit output type.  The
fp32 part is within 3e-5 relative of the exact value (the exponent's argument (x - m) log2(e) is rounded to
fp32 at magnitudes up to a few hundred: 2^-24 * 300 * ln 2 = 1.3e-5; sums of up to 16384 fp32 terms of
one sign; one-ulp exp2, sqrt and division), the final rounding adds half an ulp of the output: 2^-11
relative for binary16, 2^-8 for bfloat16; below the smallest normal binary16 value the spacing is the
absolute 2^-24.  So |y - ref| <= (2^-p + 3e-5) |ref| + floor, p = 11 / 8, floor = 2^-25 (binary16: half a
subnormal step) or 1e-37 (bfloat16: its smallest normal values; fp32 flushes nothing above that).
"""
import numpy as np
import pytest
import torch

from oracle import rowops as R
from paper_2501_08071_amd import inputs as I

pytestmark = pytest.mark.gpu

REL = {I.F16: 2.0 ** -11 + 3e-5, I.BF16: 2.0 ** -8 + 3e-5}
FLOOR = {I.F16: 2.0 ** -25, I.BF16: 1e-37}
TDT = {I.F16: torch.float16, I.BF16: torch.bfloat16}


@pytest.fixture(scope="module")
def P():
    import paper_2501_08071_amd as pkg
    assert torch.cuda.is_available()
    pkg.lib
    return pkg


def dev(bits, dtype):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(TDT[dtype])


def host_bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def check(y_bits, ref, dtype, what):
    got = R.widen(y_bits, dtype).reshape(ref.shape)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - ref)
    tol = REL[dtype] * np.abs(ref) + FLOOR[dtype]
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), f"{what}: |{got[worst]} - {ref[worst]}| = {err[worst]:.3e} > {tol[worst]:.3e} at {worst}"


# row lengths: every registers-path instance (8 .. 64 lanes per row, a workgroup per row with 1, 2, 4, 8
# chunks per thread), lengths that leave lanes and chunks idle, and general-path lengths (odd, 1, > 16384)
LENGTHS = [8, 16, 24, 64, 72, 128, 200, 256, 264, 512, 520, 1000, 2048, 2056, 4096, 4104, 8192, 8200, 16384,
           1, 2, 7, 9, 63, 1001, 4095, 16392, 20001]


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("n", LENGTHS)
def test_softmax_small(P, n, dtype):
    n_rows = 37 if n <= 4104 else 5          # several workgroups and a ragged last one
    xb = I.gen_rows(n_rows, n, dtype, mul=3.0)
    assert P.rowops_path(0, n, dtype) == (1 if n % 8 == 0 and n <= 16384 else 2)
    y = P.softmax_rows_fwd(dev(xb, dtype))
    torch.cuda.synchronize()
    check(host_bits(y), R.softmax_rows(xb, dtype), dtype, f"softmax n={n}")


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("n", LENGTHS)
def test_rmsnorm_small(P, n, dtype):
    n_rows = 37 if n <= 4104 else 5
    xb = I.gen_rows(n_rows, n, dtype, tensor_id=0)
    wb = I.gen_rows(1, n, dtype, tensor_id=1)[0]
    y = P.rmsnorm_fwd(dev(xb, dtype), dev(wb, dtype), 1e-6)
    torch.cuda.synchronize()
    check(host_bits(y), R.rmsnorm_rows(xb, wb, 1e-6, dtype), dtype, f"rmsnorm d={n}")


def test_softmax_paper_shape_every_element(P):
    """Table 2: softmax over n_rows x n_cols = 512 x 4096, float16."""
    _, n_rows, n, dt = I.ROWOP_SHAPES["softmax_512x4096_f16"]
    xb = I.gen_rows(n_rows, n, dt)
    y = P.softmax_rows_fwd(dev(xb, dt))
    torch.cuda.synchronize()
    check(host_bits(y), R.softmax_rows(xb, dt), dt, "softmax 512x4096")


def test_rmsnorm_paper_shape_every_element(P):
    """Table 2: rmsnorm over B, n_head, seq_len, d_head = 1, 32, 4096, 64, float16 (131072 rows of 64)."""
    _, n_rows, n, dt = I.ROWOP_SHAPES["rmsnorm_1x32x4096x64_f16"]
    xb = I.gen_rows(n_rows, n, dt, tensor_id=0)
    wb = I.gen_rows(1, n, dt, tensor_id=1)[0]
    x = dev(xb, dt).view(1, 32, 4096, 64)
    y = P.rmsnorm_fwd(x, dev(wb, dt), 1e-6)
    torch.cuda.synchronize()
    assert y.shape == x.shape
    check(host_bits(y).reshape(n_rows, n), R.rmsnorm_rows(xb, wb, 1e-6, dt), dt, "rmsnorm 1x32x4096x64")


def test_many_rows_stride_over_the_grid(P):
    """More row groups than the grid has workgroups: the kernels stride."""
    dt = I.F16
    xb = I.gen_rows(8192 * 32 + 77, 8, dt)             # 8 lanes per row, 32 rows per workgroup, > 8192 groups
    wb = I.gen_rows(1, 8, dt, tensor_id=1)[0]
    check(host_bits(P.rmsnorm_fwd(dev(xb, dt), dev(wb, dt), 1e-5)), R.rmsnorm_rows(xb, wb, 1e-5, dt), dt, "rmsnorm many rows")
    check(host_bits(P.softmax_rows_fwd(dev(xb, dt))), R.softmax_rows(xb, dt), dt, "softmax many rows")
    xb = I.gen_rows(8192 + 5, 9, dt)                   # general path, one workgroup per row, > 8192 rows
    check(host_bits(P.softmax_rows_fwd(dev(xb, dt))), R.softmax_rows(xb, dt), dt, "softmax many rows, general path")


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_degenerate_rows(P, dtype):
    # constant rows -> 1/n; one dominant entry -> (1, 0, ...); the largest finite inputs; a row of zeros for rmsnorm
    big = 65504.0 if dtype == I.F16 else 3.0e38
    rows = np.zeros((6, 64), np.float32)
    rows[0, :] = 2.5
    rows[1, 3] = 40.0
    rows[2, :] = -big
    rows[2, 5] = big
    rows[3, :] = big
    rows[4, ::2] = -1.0
    xb = I.to_bits(rows, dtype)
    y = P.softmax_rows_fwd(dev(xb, dtype))
    check(host_bits(y), R.softmax_rows(xb, dtype), dtype, "softmax degenerate")
    got = R.widen(host_bits(y), dtype)
    assert np.all(got[0] == R.widen(I.to_bits(np.float32([1 / 64]), dtype), dtype)[0])
    assert got[2, 5] == 1.0 and got[2].sum() == 1.0
    x2 = rows.copy()
    x2[2, :] = 0.0
    x2[3, :] = 100.0
    xb2 = I.to_bits(x2, dtype)
    wb = I.to_bits(np.linspace(-2, 2, 64, dtype=np.float32), dtype)
    for eps in (0.0, 1e-6, 1.0):
        if eps == 0.0:
            xb_e = np.delete(xb2, [2, 5], axis=0)     # 0/0 is left out: inputs are assumed to make sense
        else:
            xb_e = xb2
        y = P.rmsnorm_fwd(dev(xb_e, dtype), dev(wb, dtype), eps)
        check(host_bits(y), R.rmsnorm_rows(xb_e, wb, eps, dtype), dtype, f"rmsnorm degenerate eps={eps}")


def test_in_place_and_preallocated(P):
    dt = I.BF16
    for n in (64, 4096, 1001):
        xb = I.gen_rows(19, n, dt, mul=2.0)
        x = dev(xb, dt)
        ref = R.softmax_rows(xb, dt)
        out = torch.full_like(x, 7.0)
        assert P.softmax_rows_fwd(x, y=out) is out
        check(host_bits(out), ref, dt, "softmax preallocated")
        P.softmax_rows_fwd(x, y=x)
        check(host_bits(x), ref, dt, "softmax in place")
        wb = I.gen_rows(1, n, dt, tensor_id=1)[0]
        x = dev(xb, dt)
        P.rmsnorm_fwd(x, dev(wb, dt), 1e-6, y=x)
        check(host_bits(x), R.rmsnorm_rows(xb, wb, 1e-6, dt), dt, "rmsnorm in place")


def test_empty_input_and_errors(P):
    x = torch.empty((0, 64), dtype=torch.float16, device="cuda")
    assert P.softmax_rows_fwd(x).shape == (0, 64)
    assert P.rmsnorm_fwd(x, torch.ones(64, dtype=torch.float16, device="cuda"), 1e-6).shape == (0, 64)
    x = torch.ones((4, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(P.RowopsError) as e:
        P.rmsnorm_fwd(x, torch.ones(64, dtype=torch.float16, device="cuda"), -1.0)
    assert e.value.status == -4
    with pytest.raises(TypeError):
        P.softmax_rows_fwd(x.float())
    with pytest.raises(ValueError):
        P.rmsnorm_fwd(x, torch.ones(32, dtype=torch.float16, device="cuda"), 1e-6)
    with pytest.raises(ValueError):
        P.softmax_rows_fwd(x.t())


def test_side_stream_and_repeatability(P):
    dt = I.F16
    xb = I.gen_rows(512, 4096, dt)
    x = dev(xb, dt)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        a = P.softmax_rows_fwd(x, stream=s)
    s.synchronize()
    b = P.softmax_rows_fwd(x)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    check(host_bits(a), R.softmax_rows(xb, dt), dt, "softmax side stream")
