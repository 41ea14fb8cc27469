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


def test_utilisation_closed_forms():
    # a run that issues exactly the peak request rate and moves exactly the peak bandwidth for its whole
    # latency is 100 % utilised; half the traffic, or twice the time, is 50 %
    l2_peak, mem_peak = 3.0e11, 8.0e12
    ms = 2.5
    l2, mem = I.utilisation(l2_peak * ms * 1e-3, 0.75 * mem_peak * ms * 1e-3, 0.25 * mem_peak * ms * 1e-3, ms,
                            l2_peak, mem_peak)
    assert l2 == pytest.approx(1.0, rel=1e-14) and mem == pytest.approx(1.0, rel=1e-14)
    l2h, memh = I.utilisation(l2_peak * ms * 1e-3, 0.75 * mem_peak * ms * 1e-3, 0.25 * mem_peak * ms * 1e-3, 2 * ms,
                              l2_peak, mem_peak)
    assert l2h == pytest.approx(0.5, rel=1e-14) and memh == pytest.approx(0.5, rel=1e-14)
    # reads and writes both count, the L2 figure does not depend on the bytes and vice versa
    a = I.utilisation(1e6, 4e6, 0.0, 1.0, l2_peak, mem_peak)
    b = I.utilisation(1e6, 0.0, 4e6, 1.0, l2_peak, mem_peak)
    c = I.utilisation(2e6, 1e6, 3e6, 1.0, l2_peak, mem_peak)
    assert a == b and c[1] == a[1] and c[0] == pytest.approx(2 * a[0], rel=1e-14)
    # hand numbers: 1.2e6 requests in 0.5 ms against 3e11/s; 3 MB + 1 MB in 0.5 ms against 8 TB/s
    l2, mem = I.utilisation(1.2e6, 3e6, 1e6, 0.5, l2_peak, mem_peak)
    assert l2 == pytest.approx(0.008, rel=1e-12) and mem == pytest.approx(0.001, rel=1e-12)


def test_factor_is_corun_over_solo():
    assert I.factors([3.0, 1.0, 2.2], [2.0, 1.0, 2.0]) == pytest.approx([1.5, 1.0, 1.1], rel=1e-15)


def test_split_has_the_papers_counts_and_is_a_partition():
    # Sec. 4.4: 2,500 samples, 1,750 for training and 750 for validation
    keys = list(inputs.uniform(9, "intf/split", 2500))
    tr, va = I.split(keys)
    assert (len(tr), len(va)) == (1750, 750)
    assert sorted(tr + va) == list(range(2500))
    assert max(keys[i] for i in tr) <= min(keys[i] for i in va)       # by key order
    assert I.split(keys) == (tr, va)                                    # deterministic
    for n, want in ((10, 7), (3, 2), (1, 0), (19, 13)):
        assert len(I.split(list(range(n)))[0]) == want                  # floor(0.7 n)
    # equal keys keep their index order
    assert I.split([0.5, 0.1, 0.5, 0.1, 0.5, 0.1, 0.5, 0.1, 0.5, 0.1]) == ([1, 3, 5, 7, 9, 0, 2], [4, 6, 8])


def test_worst_slowdown_and_overhead_by_hand():
    c = [1.0, 0.0, 0.0, 2.0, 0.9]
    f = [[0.1, 0.9, 0.9, 0.0], [0.3, 0.0, 0.0, 0.05], [0.0, 0.0, 0.0, 0.1]]       # factors 1.0, 1.3, 1.1
    assert I.worst_slowdown(c, f) == pytest.approx(0.3, rel=1e-12)
    assert I.worst_slowdown(c, [[0.0, 0.5, 0.5, 0.0]]) == 0.0                       # a predicted speed-up is no slowdown
    fac = [1.0 + 0.01 * k for k in range(1, 11)]                                     # overheads 1 % .. 10 %
    at, share = I.overhead(fac, (50.0, 90.0, 95.0, 100.0), 0.055)
    assert at == pytest.approx([0.05, 0.09, 0.10, 0.10], abs=1e-12)                # nearest rank: ranks 5, 9, 10, 10
    assert share == 0.5
    assert I.overhead([1.25, 1.125], (100.0,), 0.25)[1] == 0.5                       # strictly below (exact in binary)
