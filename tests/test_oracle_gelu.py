"""Pins of the bias-GeLU oracle (exact GeLU(z) = z Phi(z); Section 4.1 names the MLP's non-linearity only)."""
import numpy as np

import oracle


def test_gelu_textbook_values_and_symmetry():
    z = np.array([[0.0, 1.0, -1.0, 2.0, -2.0, 10.0, -10.0]])
    y = oracle.bias_gelu_fwd(z)[0]
    # standard normal CDF from the tables: Phi(1) = 0.8413447460685429, Phi(2) = 0.9772498680518208
    assert abs(y[0]) == 0.0
    assert abs(y[1] - 0.8413447460685429) < 1e-15 and abs(y[2] + (1 - 0.8413447460685429)) < 1e-15
    assert abs(y[3] - 2 * 0.9772498680518208) < 1e-15 and abs(y[4] + 2 * (1 - 0.9772498680518208)) < 1e-14
    assert abs(y[5] - 10.0) < 1e-20 + 1e-15 and abs(y[6]) < 1e-20
    # Phi(z) + Phi(-z) = 1  =>  GeLU(z) - GeLU(-z) = z, for any z
    rng = np.random.default_rng(0)
    w = rng.normal(size=(7, 33)) * 3
    assert np.max(np.abs(oracle.bias_gelu_fwd(w) - oracle.bias_gelu_fwd(-w) - w)) < 1e-15


def test_gelu_matches_the_normal_cdf_of_a_library():
    """z Phi(z) with Phi from scipy's normal distribution (a different routine from the erf the oracle calls)."""
    from scipy.stats import norm
    rng = np.random.default_rng(1)
    x, bias = rng.normal(size=(19, 40)) * 2, rng.normal(size=40)
    z = x + bias
    assert np.max(np.abs(oracle.bias_gelu_fwd(x, bias) - z * norm.cdf(z))) < 1e-14
    # bias is per column and optional
    assert np.array_equal(oracle.bias_gelu_fwd(x, np.zeros(40)), oracle.bias_gelu_fwd(x))
    assert not np.array_equal(oracle.bias_gelu_fwd(x, bias), oracle.bias_gelu_fwd(x))


def test_gelu_backward_is_the_derivative_of_the_forward():
    rng = np.random.default_rng(2)
    rows, h = 11, 24
    x, bias, dy = rng.normal(size=(rows, h)) * 1.5, rng.normal(size=h) * 0.3, rng.normal(size=(rows, h))
    g = oracle.bias_gelu_bwd(dy, x, bias)
    eps = 1e-6
    fd = (oracle.bias_gelu_fwd(x + eps, bias) - oracle.bias_gelu_fwd(x - eps, bias)) / (2 * eps)   # elementwise map: dy/dx is diagonal
    assert np.max(np.abs(g["dx"] - dy * fd)) < 1e-8
    # dbias: the loss sum(dy * y) differentiated with respect to one bias entry at a time
    for c in (0, 7, h - 1):
        bp, bm = bias.copy(), bias.copy()
        bp[c] += eps
        bm[c] -= eps
        fdc = (np.sum(dy * oracle.bias_gelu_fwd(x, bp)) - np.sum(dy * oracle.bias_gelu_fwd(x, bm))) / (2 * eps)
        assert abs(g["dbias"][c] - fdc) < 1e-7
    assert np.max(np.abs(g["dbias"] - g["dx"].sum(axis=0))) < 1e-13
    # GeLU'(0) = Phi(0) = 1/2; GeLU' -> 1 and 0 at +-infinity
    d0 = oracle.bias_gelu_bwd(np.ones((1, 3)), np.array([[0.0, 12.0, -12.0]]))["dx"][0]
    assert abs(d0[0] - 0.5) < 1e-16 and abs(d0[1] - 1.0) < 1e-15 and abs(d0[2]) < 1e-15
