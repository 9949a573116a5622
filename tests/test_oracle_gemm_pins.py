"""Pins of the GEMM + LeakyReLU oracle: hand values, brute force, algebraic identities, library routines.
The paper names the kernel (Table 2, Section 5.1) without a formula and prints no worked example."""
import numpy as np
import pytest
import torch

from oracle import gemm as G
from paper_2501_08071_amd import inputs as I


def test_hand_worked_two_by_two():
    a = np.array([[[1.0, 2.0], [3.0, -4.0]]])
    b = np.array([[[5.0, -6.0], [-7.0, 8.0]]])
    # a @ b = [[-9, 10], [43, -50]]; negative entries times the slope (rows of a times columns of b: the
    # transposed product b @ a would give [[-13, 34], [17, -46]])
    c = G.gemm_leakyrelu_f64(a, b, 0.5)
    assert np.array_equal(c, [[[-4.5, 10.0], [43.0, -25.0]]])
    assert np.array_equal(G.gemm_leakyrelu_loops(a, b, 0.5), c)


def test_leaky_relu_cases():
    t = np.array([-2.0, -0.0, 0.0, 3.0])
    assert np.array_equal(G.leaky_relu_f64(t, 0.01), [-0.02, 0.0, 0.0, 3.0])
    assert np.array_equal(G.leaky_relu_f64(t, 0.0), [0.0, 0.0, 0.0, 3.0])      # slope 0 is the plain ReLU
    assert np.array_equal(G.leaky_relu_f64(t, 1.0), t)                          # slope 1 is the identity


def test_brute_force_on_small_shapes():
    for dt in (G.F16, G.BF16):
        a = I.gen_rows(2 * 5, 7, dt, tensor_id=0).reshape(2, 5, 7)
        b = I.gen_rows(2 * 7, 3, dt, tensor_id=1).reshape(2, 7, 3)
        np.testing.assert_allclose(G.gemm_leakyrelu(a, b, 0.01, dt),
                                   G.gemm_leakyrelu_loops(G.widen(a, dt), G.widen(b, dt), 0.01), rtol=1e-14, atol=1e-14)


def test_identity_and_batches_are_independent():
    x = G.widen(I.gen_rows(2 * 6, 6, G.F16).reshape(2, 6, 6), G.F16)
    eye = np.stack([np.eye(6), np.eye(6)])
    assert np.array_equal(G.gemm_leakyrelu_f64(x, eye, 0.25), np.where(x >= 0, x, 0.25 * x))
    assert np.array_equal(G.gemm_leakyrelu_f64(eye, x, 0.25), np.where(x >= 0, x, 0.25 * x))
    y = G.gemm_leakyrelu_f64(x, x, 0.01)
    assert np.array_equal(y[1], G.gemm_leakyrelu_f64(x[1:], x[1:], 0.01)[0])


def test_positive_homogeneity_and_sign_flip():
    a = G.widen(I.gen_rows(9, 16, G.BF16, tensor_id=0).reshape(1, 9, 16), G.BF16)
    b = G.widen(I.gen_rows(16, 5, G.BF16, tensor_id=1).reshape(1, 16, 5), G.BF16)
    c = G.gemm_leakyrelu_f64(a, b, 0.125)
    np.testing.assert_array_equal(G.gemm_leakyrelu_f64(4.0 * a, b, 0.125), 4.0 * c)
    # f(-t) relates to f(t): where c > 0 the flipped product is -slope * c, where c < 0 it is -c / slope
    d = G.gemm_leakyrelu_f64(-a, b, 0.125)
    np.testing.assert_allclose(d, np.where(c > 0, -0.125 * c, -c / 0.125), rtol=1e-15)
    # transposition: (a b)^T = b^T a^T, and the activation is elementwise
    ct = G.gemm_leakyrelu_f64(b.transpose(0, 2, 1), a.transpose(0, 2, 1), 0.125)
    np.testing.assert_allclose(ct, c.transpose(0, 2, 1), rtol=1e-14, atol=1e-14)


def test_against_library_routines():
    for dt in (G.F16, G.BF16):
        a = I.gen_rows(33, 40, dt, tensor_id=0).reshape(1, 33, 40)
        b = I.gen_rows(40, 17, dt, tensor_id=1).reshape(1, 40, 17)
        ta, tb = torch.from_numpy(G.widen(a, dt)), torch.from_numpy(G.widen(b, dt))
        ref = torch.nn.functional.leaky_relu(torch.bmm(ta, tb), negative_slope=0.01).numpy()
        np.testing.assert_allclose(G.gemm_leakyrelu(a, b, 0.01, dt), ref, rtol=1e-13, atol=1e-13)


def test_abs_product_bounds_the_result():
    a = I.gen_rows(8, 32, G.F16, tensor_id=0).reshape(1, 8, 32)
    b = I.gen_rows(32, 8, G.F16, tensor_id=1).reshape(1, 32, 8)
    assert np.all(np.abs(G.gemm_leakyrelu(a, b, 1.0, G.F16)) <= G.abs_product(a, b, G.F16) + 1e-12)


def test_shape_errors():
    with pytest.raises(ValueError):
        G.gemm_leakyrelu_f64(np.zeros((1, 2, 3)), np.zeros((1, 4, 2)), 0.01)
    with pytest.raises(ValueError):
        G.gemm_leakyrelu_f64(np.zeros((2, 3)), np.zeros((3, 2)), 0.01)
    with pytest.raises(ValueError):
        G.widen(np.zeros(1, np.uint16), 3)
