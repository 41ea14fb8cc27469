"""Pins of the interference-model oracle (paper Sec. 4.4) against closed forms
and the defining property of least squares."""

import numpy as np
import pytest

from oracle import interference as I
from paper_2109_01611_amd import inputs


def samples(seed, n, c, noise=0.0):
    f = inputs.uniform(seed, "intf/features", 4 * n).reshape(n, 4)
    y = f @ np.array(c[:4]) + c[4] + noise * inputs.normal(seed, "intf/noise", n)
    return f, y


def test_noiseless_samples_give_back_the_coefficients():
    c = [0.31, -0.07, 0.52, 0.11, 1.02]
    f, y = samples(1, 40, c)
    assert np.allclose(I.fit(f, y), c, rtol=0, atol=1e-12)
    assert np.allclose(I.predict(c, f), y, rtol=0, atol=1e-12)
    assert I.relative_errors(c, f, y).max() < 1e-12


def test_residual_is_orthogonal_to_every_column():
    f, y = samples(2, 300, [0.2, 0.1, 0.4, 0.3, 1.0], noise=0.05)
    c = I.fit(f, y)
    r = y - I.predict(c, f)
    X = I.design_matrix(f)
    assert np.abs(X.T @ r).max() < 1e-10          # the normal equations
    # and no other coefficient vector does better
    for k in range(5):
        d = np.zeros(5)
        d[k] = 1e-3
        assert np.sum((y - I.predict(c + d, f)) ** 2) > np.sum(r ** 2)


def test_single_active_feature_reduces_to_simple_regression():
    n = 200
    f = np.zeros((n, 4))
    x = inputs.uniform(3, "intf/x", n)
    # the other three columns must not be collinear with the constant: give them independent values with no effect
    f[:, 0] = x
    f[:, 1:] = inputs.uniform(3, "intf/rest", 3 * n).reshape(n, 3)
    y = 1.5 * x + 0.7 + 0.01 * inputs.normal(3, "intf/n", n)
    c = I.fit(f, y)
    # compare with the textbook slope of y regressed on all columns via the partial-out identity
    # (Frisch-Waugh): regress x and y on the other columns, then the slope of the residuals
    Z = np.concatenate([f[:, 1:], np.ones((n, 1))], axis=1)
    proj = Z @ np.linalg.solve(Z.T @ Z, Z.T)
    rx, ry = x - proj @ x, y - proj @ y
    assert c[0] == pytest.approx(float(rx @ ry / (rx @ rx)), rel=1e-10)


def test_scaling_a_feature_scales_its_coefficient():
    f, y = samples(4, 120, [0.3, 0.2, 0.1, 0.4, 1.0], noise=0.02)
    c = I.fit(f, y)
    g = f.copy()
    g[:, 2] *= 8.0
    d = I.fit(g, y)
    assert d[2] == pytest.approx(c[2] / 8.0, rel=1e-10)
    assert np.allclose(np.delete(d, 2), np.delete(c, 2), rtol=1e-9)


def test_degenerate_samples_are_refused():
    f = np.ones((10, 4))
    with pytest.raises(ValueError):
        I.fit(f, np.ones(10))


def test_relative_error_and_percentile():
    c = [0, 0, 0, 0, 2.0]
    f = np.zeros((4, 4))
    assert np.allclose(I.relative_errors(c, f, [1.0, 2.0, 4.0, 2.5]), [1.0, 0.0, 0.5, 0.2])
    v = [0.5, 0.1, 0.4, 0.2, 0.3, 0.6, 0.7, 0.8, 0.9, 1.0]
    assert I.percentile(v, 90) == 0.9 and I.percentile(v, 95) == 1.0 and I.percentile(v, 10) == 0.1
    assert I.percentile(v, 50) == 0.5 and I.percentile([3.0], 90) == 3.0
