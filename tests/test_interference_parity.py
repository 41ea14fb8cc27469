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


def test_features_factor_split_slowdown_and_overhead_match():
    n = 600
    cnt = inputs.uniform(8, "intf/counters", 4 * n).reshape(n, 4)
    l2_peak, mem_peak = sched.L2_PEAK_REQ_PER_S, sched.HBM_PEAK_BYTES_PER_S
    feats = []
    for r in cnt:
        args = (r[0] * 3e8, r[1] * 2e9, r[2] * 1e9, 0.05 + 3.0 * r[3])
        got = sched.interference_utilisation(*args)
        want = I.utilisation(*args, l2_peak, mem_peak)
        assert got == pytest.approx(want, rel=1e-13)
        feats.append(got)
    corun = (1.0 + cnt[:, 0]).tolist()
    solo = (0.5 + cnt[:, 1]).tolist()
    fac = sched.interference_factor(corun, solo)
    assert fac == pytest.approx(I.factors(corun, solo), rel=1e-15)
    keys = list(inputs.uniform(8, "intf/keys", n))
    keys[17] = keys[3]                                    # a tie
    assert sched.interference_split(keys) == I.split(keys)
    assert sched.interference_split(list(inputs.uniform(8, "intf/keys2500", 2500))) == \
        I.split(list(inputs.uniform(8, "intf/keys2500", 2500)))
    c = [0.31, -0.07, 0.52, 0.11, 0.95]
    rows = [[a[0], b[0], a[1], b[1]] for a, b in zip(feats[::2], feats[1::2])]
    assert sched.interference_worst_slowdown(c, rows) == pytest.approx(I.worst_slowdown(c, rows), rel=1e-12)
    assert sched.interference_worst_slowdown([0, 0, 0, 0, 0.5], rows) == 0.0
    qs = (1.0, 50.0, 90.0, 99.0, 100.0)
    at, share = sched.interference_overhead(fac, qs, 0.18)
    want_at, want_share = I.overhead(fac, qs, 0.18)
    assert at == pytest.approx(want_at, rel=1e-13, abs=1e-15) and share == want_share


def test_new_entry_points_refuse_bad_arguments():
    with pytest.raises(gpulet.GpuletError):
        sched.interference_utilisation(1.0, 1.0, 1.0, 0.0)               # no latency
    with pytest.raises(gpulet.GpuletError):
        sched.interference_utilisation(-1.0, 1.0, 1.0, 1.0)
    with pytest.raises(gpulet.GpuletError):
        sched.interference_factor([1.0, 2.0], [1.0, 0.0])
    with pytest.raises(gpulet.GpuletError):
        sched.interference_split([0.1, float("nan")])
    with pytest.raises(gpulet.GpuletError):
        sched.interference_overhead([1.1, 1.2], (0.0,), 0.18)
    with pytest.raises(gpulet.GpuletError):
        sched.interference_worst_slowdown([0, 0, 0, 0, float("inf")], [[0, 0, 0, 0]])
