"""Library interference model (include/gpulet_sched.h) against the numpy oracle:
coefficients, predictions and error percentiles to 1e-9 (both fp64; the library
solves by Householder QR, the oracle by SVD).  Host-only code."""

import numpy as np
import pytest

from oracle import interference as I
from paper_2109_01611_amd import gpulet, inputs, sched


def samples(seed, n, c, noise):
    f = inputs.uniform(seed, "intf/features", 4 * n).reshape(n, 4)
    f[:, 2:] *= 0.3                                   # memory utilisation lives on a smaller range
    y = f @ np.array(c[:4]) + c[4] + noise * inputs.normal(seed, "intf/noise", n)
    return f, y


@pytest.mark.parametrize("seed,n,noise", [(1, 5, 0.0), (2, 40, 0.0), (3, 1500, 0.05), (4, 750, 0.2), (5, 64, 1e-6)])
def test_fit_predict_and_error_match(seed, n, noise):
    c_true = [0.31, -0.07, 0.52, 0.11, 1.02]
    f, y = samples(seed, n, c_true, noise)
    want = I.fit(f, y)
    got = np.array(sched.interference_fit(f.tolist(), y.tolist()))
    assert np.abs(got - want).max() <= 1e-9 * max(1.0, np.abs(want).max())
    if noise == 0.0:
        assert np.abs(got - c_true).max() <= 1e-9
    pred = np.array(sched.interference_predict(got.tolist(), f.tolist()))
    assert np.abs(pred - I.predict(want, f)).max() <= 1e-9
    y_pos = np.abs(y) + 0.5
    qs = (10.0, 50.0, 90.0, 95.0, 100.0)
    e = sched.interference_error(want.tolist(), f.tolist(), y_pos.tolist(), qs)
    errs = I.relative_errors(want, f, y_pos)
    assert e == pytest.approx([I.percentile(errs, q) for q in qs], rel=1e-9)


def test_train_validate_split_as_in_the_paper():
    # 2,500 samples, 1,750 for training and 750 for validation (Sec. 4.4), the split drawn from a seeded stream
    f, y = samples(6, 2500, [0.25, 0.15, 0.6, 0.35, 1.0], 0.03)
    order = np.argsort(inputs.uniform(6, "intf/split", 2500), kind="stable")
    tr, va = order[:1750], order[1750:]
    c_lib = sched.interference_fit(f[tr].tolist(), y[tr].tolist())
    c_ref = I.fit(f[tr], y[tr])
    assert np.abs(np.array(c_lib) - c_ref).max() <= 1e-9
    e_lib = sched.interference_error(c_lib, f[va].tolist(), y[va].tolist(), (90.0, 95.0))
    errs = I.relative_errors(c_ref, f[va], y[va])
    assert e_lib == pytest.approx([I.percentile(errs, 90), I.percentile(errs, 95)], rel=1e-7)
    assert e_lib[1] < 0.1


def test_argument_errors():
    f, y = samples(7, 10, [0.1, 0.2, 0.3, 0.4, 1.0], 0.0)
    with pytest.raises(gpulet.GpuletError):
        sched.interference_fit(f[:4].tolist(), y[:4].tolist())              # fewer samples than coefficients
    with pytest.raises(gpulet.GpuletError):
        sched.interference_fit(np.ones((10, 4)).tolist(), y.tolist())       # columns equal to the constant
    g = f.copy()
    g[:, 3] = 2.0 * g[:, 0] - g[:, 1]
    with pytest.raises(gpulet.GpuletError):
        sched.interference_fit(g.tolist(), y.tolist())                      # a dependent column
    g = f.copy()
    g[0, 0] = float("nan")
    with pytest.raises(gpulet.GpuletError):
        sched.interference_fit(g.tolist(), y.tolist())
    with pytest.raises(gpulet.GpuletError):
        sched.interference_error([0, 0, 0, 0, 1.0], f.tolist(), (-np.abs(y)).tolist(), (90.0,))
    with pytest.raises(gpulet.GpuletError):
        sched.interference_error([0, 0, 0, 0, 1.0], f.tolist(), np.abs(y).tolist(), (0.0,))
