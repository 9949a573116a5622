"""The seeded generator: published SplitMix64 vectors, rounding bit patterns, distributions."""
import numpy as np
import pytest

from paper_2501_08071_amd import inputs as I


def test_splitmix64_published_vectors():
    # first outputs of the reference splitmix64 with seed 1234567 (widely reproduced test vector)
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    got = [I.splitmix64_scalar(1234567, n) for n in range(5)]
    assert got == want
    vec = I.splitmix64(1234567, np.arange(5, dtype=np.uint64))
    assert [int(x) for x in vec] == want
    assert I.splitmix64_scalar(0, 0) == 0xE220A8397B1DCDAF


def test_counter_based_chunks_agree():
    a = I._fill(99, 3 * I._CHUNK + 17, "normal", 1.0, I.BF16)
    old = I._CHUNK
    try:
        I._CHUNK = 4096 * 7
        b = I._fill(99, 3 * old + 17, "normal", 1.0, I.BF16)
    finally:
        I._CHUNK = old
    assert np.array_equal(a, b)


@pytest.mark.parametrize("x,bits", [
    (1.0, 0x3F80), (-2.0, 0xC000), (0.0, 0x0000), (-0.0, 0x8000),
    (1.00390625, 0x3F80),          # 1 + 2^-8: tie, rounds to even (down)
    (1.01171875, 0x3F82),          # 1 + 3*2^-8: tie, rounds to even (up)
    (1.00390637, 0x3F81),          # just above the tie
    (3.140625, 0x4049), (3.1415927, 0x4049), (65280.0, 0x477F),
    (3.3895314e38, 0x7F7F),        # largest finite bfloat16
])
def test_bf16_rne_bit_patterns(x, bits):
    assert int(I.f32_to_bf16_bits(np.array([x], np.float32))[0]) == bits


@pytest.mark.parametrize("x,bits", [
    (1.0, 0x3C00), (-2.0, 0xC000), (0.0, 0x0000), (-0.0, 0x8000),
    (1.00048828125, 0x3C00),       # 1 + 2^-11: tie to even (down)
    (1.00146484375, 0x3C02),       # 1 + 3*2^-11: tie to even (up)
    (65504.0, 0x7BFF), (5.9604645e-08, 0x0001), (2.9802322e-08, 0x0000),  # subnormal, tie->0
    (6.1035156e-05, 0x0400), (0.333251953125, 0x3555),
])
def test_f16_rne_bit_patterns(x, bits):
    assert int(I.f32_to_f16_bits(np.array([x], np.float32))[0]) == bits


def test_widening_is_exact_inverse():
    allbits = np.arange(0, 0x7C00, dtype=np.uint16)       # all finite non-negative binary16
    back = I.f32_to_f16_bits(I.bits_to_f64(allbits, I.F16).astype(np.float32))
    assert np.array_equal(back, allbits)
    allbits = np.arange(0, 0x7F80, dtype=np.uint16)       # all finite non-negative bfloat16
    back = I.f32_to_bf16_bits(I.bits_to_f64(allbits, I.BF16).astype(np.float32))
    assert np.array_equal(back, allbits)


def test_distributions_and_stream_independence():
    q, k, v = I.gen_tensors(2, 4, 256, 64, I.F16, workload_id=7)
    for t in (q, k, v):
        x = I.bits_to_f64(t, I.F16)
        assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert not np.array_equal(q, k) and not np.array_equal(k, v)
    xq, xk = I.bits_to_f64(q, I.F16).ravel(), I.bits_to_f64(k, I.F16).ravel()
    assert abs(np.corrcoef(xq, xk)[0, 1]) < 0.01
    # 4th moment of a standard normal is 3
    assert abs((xq ** 4).mean() - 3.0) < 0.15
    q2, _, _ = I.gen_tensors(2, 4, 256, 64, I.F16, workload_id=7)
    assert np.array_equal(q, q2)
    q3, _, _ = I.gen_tensors(2, 4, 256, 64, I.F16, workload_id=7, seed=1)
    assert not np.array_equal(q, q3)


def test_peaky_workload_recipe():
    w = I.workload(5)
    q, k, v = I.gen_tensors(1, 2, 512, w.D, w.dtype, workload_id=w.id, qk_mul=w.qk_mul, v_dist=w.v_dist)
    xq, xv = I.bits_to_f64(q, w.dtype), I.bits_to_f64(v, w.dtype)
    assert abs(xq.std() - 4.0) < 0.05
    assert xv.min() >= -1.0 and xv.max() <= 1.0 and abs(xv.mean()) < 0.02
    assert abs(xv.var() - 1.0 / 3.0) < 0.01


def test_workload_table():
    assert [w.id for w in I.WORKLOADS] == [1, 2, 3, 4, 5]
    w3 = I.workload(3)
    assert (w3.B, w3.H, w3.S, w3.D, w3.dtype, w3.causal) == (2, 32, 4096, 128, I.BF16, True)
    assert abs(w3.flops - 274.877906944e9) < 1
    assert abs(I.workload(5).flops - 274.877906944e9) < 1
    assert abs(I.workload(4).flops - 2199.023255552e9) < 1
    assert I.workload(1).flops == 4 * 128 * 128 * 64
