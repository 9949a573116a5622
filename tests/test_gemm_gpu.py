"""Parity of the HIP fused GEMM + LeakyReLU (include/gemm.h) against the float64 oracle.

Tolerance.  Products of two 16-bit values are exact in fp32; the K-term sum is accumulated in fp32 in some
order (the matrix cores' own), whose error is at most about K 2^-24 sum_k |a||b| and in practice a small
multiple of 2^-24 sum_k |a||b|; the activation multiplies by the slope (one more fp32 rounding) and the
result is rounded once into the 16-bit output type (half an ulp: 2^-11 relative for binary16, 2^-8 for
bfloat16; below binary16's smallest normal the spacing is 2^-24).  So
    |c - ref| <= 2^-p |ref| + 2^-20 max(1, |slope|) sum_k |a||b| + floor,   p = 11 / 8, floor = 2^-25 / 1e-37.
2^-20 is 16 times the unit roundoff of fp32: room for sums of a few thousand terms.
"""
import numpy as np
import pytest
import torch

from oracle import gemm as G
from paper_2501_08071_amd import inputs as I

pytestmark = pytest.mark.gpu

P_BITS = {I.F16: 11, I.BF16: 8}
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


def check(c_bits, a, b, slope, dtype, what):
    ref = G.gemm_leakyrelu(a, b, slope, dtype)
    got = G.widen(c_bits, dtype).reshape(ref.shape)
    assert np.all(np.isfinite(got)), what
    tol = 2.0 ** -P_BITS[dtype] * np.abs(ref) + 2.0 ** -20 * max(1.0, abs(slope)) * G.abs_product(a, b, dtype) + FLOOR[dtype]
    err = np.abs(got - ref)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), f"{what}: |{got[worst]} - {ref[worst]}| = {err[worst]:.3e} > {tol[worst]:.3e} at {worst}"


def run(P, batch, M, N, K, dtype, slope=0.01):
    a, b = I.gen_gemm(batch, M, N, K, dtype)
    c = P.gemm_leakyrelu_fwd(dev(a, dtype), dev(b, dtype), slope)
    torch.cuda.synchronize()
    assert c.shape == (batch, M, N)
    check(host_bits(c), a, b, slope, dtype, f"gemm {batch}x{M}x{N}x{K} path {P.gemm_path(batch, M, N, K, dtype)}")


# (batch, M, N, K): 64 x 64 tiles (path 3) with whole and ragged tiles in M and N, one and several k blocks
SMALL_TILES = [(1, 64, 64, 32), (1, 64, 64, 64), (1, 128, 128, 224), (1, 65, 72, 96), (1, 1, 8, 32), (1, 200, 136, 160),
               (3, 70, 64, 128), (1, 576, 520, 256), (2, 127, 120, 32)]
# 32 x 32 tiles with K split over the four wavefronts (path 5): at most 256 tiles, K >= 256; whole and ragged tiles,
# numbers of k blocks that leave wavefronts with unequal shares (9, 11) or fewer blocks than stages, batches
SPLITK_TILES = [(1, 128, 128, 256), (1, 33, 8, 2048), (1, 320, 264, 288), (3, 200, 136, 352), (1, 1, 8, 256),
                (1, 512, 480, 1024), (2, 97, 72, 4096)]
# 128 x 128 tiles (path 2): at least 192 of them, but fewer than 192 tiles of 256 x 256
BIG_TILES = [(1, 1792, 1792, 64), (1, 2048, 1536, 96), (2, 1300, 1288, 128), (1, 1793, 1800, 32)]
# 256 x 256 tiles (path 1): at least 192 of them; whole and ragged tiles, one and several k blocks, batches
HUGE_TILES = [(1, 3584, 3584, 64), (1, 3585, 3592, 32), (3, 2100, 2056, 96), (1, 4096, 3072, 160)]
# the plain kernel (path 4): K not a multiple of 32, N not a multiple of 8, K = 0
PLAIN = [(1, 5, 7, 3), (2, 33, 9, 31), (1, 64, 64, 40), (1, 16, 12, 64), (1, 3, 8, 0), (1, 1, 1, 1)]


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("shape", SMALL_TILES)
def test_small_tiles(P, shape, dtype):
    assert P.gemm_path(*shape, dtype) == 3
    run(P, *shape, dtype)


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("shape", SPLITK_TILES)
def test_split_k_tiles(P, shape, dtype):
    assert P.gemm_path(*shape, dtype) == 5
    run(P, *shape, dtype)


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("shape", BIG_TILES)
def test_big_tiles(P, shape, dtype):
    assert P.gemm_path(*shape, dtype) == 2
    run(P, *shape, dtype)


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("shape", HUGE_TILES)
def test_huge_tiles(P, shape, dtype):
    assert P.gemm_path(*shape, dtype) == 1
    run(P, *shape, dtype)


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("shape", PLAIN)
def test_plain_kernel(P, shape, dtype):
    assert P.gemm_path(*shape, dtype) == 4
    run(P, *shape, dtype)


def test_paper_shape_every_element(P):
    """Table 2: mmLeakyReLu, B, M, N, K = 1, 512, 512, 2048, float16."""
    batch, M, N, K, dt = I.GEMM_SHAPES["mmLeakyReLu_1x512x512x2048_f16"]
    run(P, batch, M, N, K, dt, slope=0.01)


def test_paper_bmm_shape_every_element(P):
    """Table 2: bmm, B, M, N, K = 4, 512, 512, 2048, float16: slope 1 makes the activation the identity."""
    batch, M, N, K, dt = I.GEMM_SHAPES["bmm_4x512x512x2048_f16"]
    run(P, batch, M, N, K, dt, slope=1.0)


@pytest.mark.parametrize("slope", [0.0, 1.0, -0.5, 0.2])
def test_slopes(P, slope):
    run(P, 1, 96, 80, 64, I.F16, slope=slope)
    run(P, 1, 9, 5, 7, I.BF16, slope=slope)


def test_structured_operands_catch_a_wrong_index(P):
    """a = a one-hot selection of rows of b: c[m, :] = f(b[sel[m], :]) exactly; any mix-up of m, n or k shows."""
    dt = I.F16
    M, N, K = 96, 72, 64
    rng = np.random.default_rng(3)
    sel = rng.integers(0, K, M)
    a = np.zeros((1, M, K), np.float32)
    a[0, np.arange(M), sel] = 1.0
    bb = I.gen_rows(K, N, dt).reshape(1, K, N)
    ab = I.to_bits(a, dt).reshape(1, M, K)
    c = P.gemm_leakyrelu_fwd(dev(ab, dt), dev(bb, dt), 0.5)
    got = G.widen(host_bits(c), dt)[0]
    rows = G.widen(bb, dt)[0][sel]
    exp = np.where(rows >= 0, rows, 0.5 * rows)
    assert np.array_equal(got, G.widen(I.to_bits(exp.astype(np.float32), dt), dt))


def test_two_dimensional_call_preallocated_and_side_stream(P):
    dt = I.BF16
    a, b = I.gen_gemm(1, 130, 64, 64, dt)
    c = torch.full((130, 64), 3.0, dtype=torch.bfloat16, device="cuda")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        out = P.gemm_leakyrelu_fwd(dev(a, dt)[0], dev(b, dt)[0], 0.01, c=c, stream=s)
    s.synchronize()
    assert out is c
    check(host_bits(c), a, b, 0.01, dt, "2-d call")
    c2 = P.gemm_leakyrelu_fwd(dev(a, dt), dev(b, dt), 0.01)
    torch.cuda.synchronize()
    assert torch.equal(c2[0].view(torch.int16), c.view(torch.int16))     # run to run bit-identical


def test_empty_and_errors(P):
    z = torch.empty((0, 64), dtype=torch.float16, device="cuda")
    b = torch.ones((64, 8), dtype=torch.float16, device="cuda")
    assert P.gemm_leakyrelu_fwd(z, b).shape == (0, 8)
    a = torch.ones((4, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(P.GemmError) as e:
        P.gemm_leakyrelu_fwd(a, b, float("nan"))
    assert e.value.status == -4
    with pytest.raises(ValueError):
        P.gemm_leakyrelu_fwd(a, torch.ones((32, 8), dtype=torch.float16, device="cuda"))
    with pytest.raises(TypeError):
        P.gemm_leakyrelu_fwd(a.float(), b.float())
