"""Pins of the row-operation oracle (softmax, rmsnorm) to closed forms, invariants and library routines.

The paper names both kernels without a formula (Table 2, Section 5.1) and prints no worked example, so none
of these are the paper's values: they are what the textbook definitions fix.
"""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import rowops as R
from paper_2501_08071_amd import inputs as I


def _rand_bits(n_rows, n_cols, dtype, tid=0, mul=1.0):
    return I.gen_rows(n_rows, n_cols, dtype, tensor_id=tid, mul=mul)


# ---------------------------------------------------------------- widening

def test_widen_exact_values():
    assert R.widen(np.array([0x3C00, 0xC000, 0x0001, 0x7BFF], np.uint16), R.F16).tolist() == [1.0, -2.0, 2.0 ** -24, 65504.0]
    assert R.widen(np.array([0x3F80, 0xC000, 0x4049], np.uint16), R.BF16).tolist() == [1.0, -2.0, 3.140625]
    with pytest.raises(ValueError):
        R.widen(np.zeros(1, np.uint16), 2)


# ---------------------------------------------------------------- softmax

def test_softmax_rows_sum_to_one_and_nonnegative():
    for dt in (R.F16, R.BF16):
        y = R.softmax_rows(_rand_bits(7, 333, dt, mul=3.0), dt)
        assert np.all(y >= 0.0)
        np.testing.assert_allclose(y.sum(axis=1), 1.0, rtol=0, atol=1e-14)


def test_softmax_constant_row_is_uniform():
    for n in (1, 2, 5, 4096):
        y = R.softmax_f64(np.full((2, n), -7.25))
        assert np.array_equal(y, np.full((2, n), 1.0 / n))


def test_softmax_two_columns_is_the_logistic_function():
    a = np.array([0.0, 1.5, -3.0, 20.0])
    b = np.array([0.0, -0.5, 4.0, -20.0])
    y = R.softmax_f64(np.stack([a, b], axis=1))
    np.testing.assert_allclose(y[:, 0], 1.0 / (1.0 + np.exp(b - a)), rtol=1e-15)
    np.testing.assert_allclose(y[:, 1], 1.0 / (1.0 + np.exp(a - b)), rtol=1e-15)


def test_softmax_hand_worked_row():
    # exp of ln 1, ln 2, ln 3 is 1, 2, 3: weights 1/6, 1/3, 1/2 (the order matters: a transposed or reversed
    # result fails)
    y = R.softmax_f64(np.log(np.array([[1.0, 2.0, 3.0]])))
    np.testing.assert_allclose(y, [[1 / 6, 1 / 3, 1 / 2]], rtol=4e-16)


def test_softmax_shift_invariance_and_no_overflow():
    x = R.widen(_rand_bits(3, 50, R.F16, mul=2.0), R.F16)
    np.testing.assert_allclose(R.softmax_f64(x + 1000.0), R.softmax_f64(x), rtol=1e-12)
    big = R.softmax_f64(np.array([[65504.0, 65503.0, -65504.0]]))   # the largest binary16 values
    assert np.all(np.isfinite(big)) and big[0, 2] == 0.0
    np.testing.assert_allclose(big[0, :2], [1 / (1 + np.exp(-1.0)), 1 / (1 + np.exp(1.0))], rtol=1e-15)


def test_softmax_rows_are_independent_and_ordered():
    x = R.widen(_rand_bits(4, 17, R.BF16), R.BF16)
    y = R.softmax_f64(x)
    for i in range(4):
        np.testing.assert_array_equal(R.softmax_f64(x[i:i + 1])[0], y[i])
    j = np.argsort(x[0])
    assert np.all(np.diff(y[0][j]) >= 0)          # monotone in the logit
    assert y[0].argmax() == x[0].argmax()


def test_softmax_against_library_routine():
    for dt in (R.F16, R.BF16):
        bits = _rand_bits(9, 257, dt, mul=4.0)
        np.testing.assert_allclose(R.softmax_rows(bits, dt), scipy.special.softmax(R.widen(bits, dt), axis=1),
                                   rtol=1e-13, atol=1e-300)


# ---------------------------------------------------------------- rmsnorm

def test_rmsnorm_three_four():
    # mean of squares of (3, 4) is 12.5
    y = R.rmsnorm_f64(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0)
    np.testing.assert_allclose(y, [[3 / np.sqrt(12.5), 8 / np.sqrt(12.5)]], rtol=1e-15)
    # eps goes under the root, next to the mean (not to the sum, not outside the root)
    y = R.rmsnorm_f64(np.array([[3.0, 4.0]]), np.array([1.0, 1.0]), 3.5)
    np.testing.assert_allclose(y, [[0.75, 1.0]], rtol=1e-15)


def test_rmsnorm_ones_returns_the_weight():
    w = np.array([0.5, -2.0, 3.0, 7.0])
    assert np.array_equal(R.rmsnorm_f64(np.ones((2, 4)), w, 0.0), np.stack([w, w]))
    assert np.array_equal(R.rmsnorm_f64(-np.ones((1, 4)), w, 0.0), -w[None])


def test_rmsnorm_scale_invariance_and_unit_mean_square():
    x = R.widen(_rand_bits(5, 64, R.F16), R.F16)
    w = np.ones(64)
    y = R.rmsnorm_f64(x, w, 0.0)
    np.testing.assert_allclose(R.rmsnorm_f64(4.0 * x, w, 0.0), y, rtol=1e-15)      # a power of two: exact scaling
    np.testing.assert_allclose((y * y).mean(axis=1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(R.rmsnorm_f64(x, 3.0 * w, 0.0), 3.0 * y, rtol=1e-15)


def test_rmsnorm_zero_row_and_eps():
    y = R.rmsnorm_f64(np.zeros((1, 8)), np.ones(8), 1e-6)
    assert np.array_equal(y, np.zeros((1, 8)))
    x = np.array([[1e-4, -1e-4]])
    np.testing.assert_allclose(R.rmsnorm_f64(x, np.ones(2), 1e-6), x / np.sqrt(1e-8 + 1e-6), rtol=1e-15)


def test_rmsnorm_against_library_routine():
    for dt in (R.F16, R.BF16):
        xb, wb = _rand_bits(11, 64, dt, 0), _rand_bits(1, 64, dt, 1)[0]
        ref = torch.nn.functional.rms_norm(torch.from_numpy(R.widen(xb, dt)), (64,), torch.from_numpy(R.widen(wb, dt)), eps=1e-6)
        np.testing.assert_allclose(R.rmsnorm_rows(xb, wb, 1e-6, dt), ref.numpy(), rtol=1e-13)


def test_rmsnorm_rows_are_independent():
    x = R.widen(_rand_bits(3, 24, R.BF16), R.BF16)
    w = R.widen(_rand_bits(1, 24, R.BF16, 1)[0], R.BF16)
    y = R.rmsnorm_f64(x, w, 1e-5)
    for i in range(3):
        np.testing.assert_array_equal(R.rmsnorm_f64(x[i:i + 1], w, 1e-5)[0], y[i])


def test_shape_errors():
    with pytest.raises(ValueError):
        R.softmax_f64(np.zeros((2, 0)))
    with pytest.raises(ValueError):
        R.rmsnorm_f64(np.zeros((2, 4)), np.zeros(3), 0.0)


def test_generator_shapes_of_the_papers_table():
    assert I.ROWOP_SHAPES["softmax_512x4096_f16"][1:3] == (512, 4096)
    assert I.ROWOP_SHAPES["rmsnorm_1x32x4096x64_f16"][1:3] == (131072, 64)
    a = I.gen_rows(4, 16, I.F16)
    assert a.shape == (4, 16) and a.dtype == np.uint16
    assert np.array_equal(a, I.gen_rows(4, 16, I.F16)) and not np.array_equal(a, I.gen_rows(4, 16, I.F16, tensor_id=1))
