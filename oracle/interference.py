"""Oracle of the interference model (paper Sec. 4.4): plain numpy, fp64.

Test infrastructure only; shares no code with the library's fit.

The model predicts how much slower a model runs on its gpu-let when another
model occupies the rest of the GPU:

    factor = c1*l2_1 + c2*l2_2 + c3*mem_1 + c4*mem_2 + c5

with l2 and mem the L2 and memory-bandwidth utilisation of the victim (1) and
the aggressor (2) measured in their *solo* runs, and c1..c5 found by linear
regression on measured (features, factor) samples.  The paper does not print
its coefficients or samples, so the fit is the textbook definition: ordinary
least squares, here through numpy's SVD-based ``lstsq``.

Readings: ``factor`` is co-run latency over solo latency of the victim on the
same gpu-let (>= 1 means slower); the prediction error is relative,
|predicted - measured| / measured, as in Fig. 9; percentiles are nearest rank.
"""

import math

import numpy as np


def design_matrix(features):
    """features: (n, 4) rows (l2_1, l2_2, mem_1, mem_2) -> (n, 5) with the constant column."""
    f = np.asarray(features, dtype=np.float64).reshape(-1, 4)
    return np.concatenate([f, np.ones((f.shape[0], 1))], axis=1)


def fit(features, factors):
    """Least-squares coefficients (c1..c5)."""
    X = design_matrix(features)
    y = np.asarray(factors, dtype=np.float64)
    c, _, rank, _ = np.linalg.lstsq(X, y, rcond=None)
    if rank < 5:
        raise ValueError("samples do not determine five coefficients")
    return c


def predict(c, features):
    return design_matrix(features) @ np.asarray(c, dtype=np.float64)


def relative_errors(c, features, factors):
    y = np.asarray(factors, dtype=np.float64)
    return np.abs(predict(c, features) - y) / y


def percentile(values, q):
    """Nearest-rank percentile (q in (0, 100])."""
    v = sorted(float(e) for e in values)
    return v[max(0, int(math.ceil(q / 100.0 * len(v))) - 1)]
