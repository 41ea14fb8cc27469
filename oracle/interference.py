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


def utilisation(l2_requests, fetch_bytes, write_bytes, solo_ms, l2_peak_requests_per_s, mem_peak_bytes_per_s):
    """The two features of one solo run (Sec. 4.4): counter totals of the run over its latency,
    relative to the whole GPU's L2 request rate and memory bandwidth -> (l2, mem)."""
    seconds = solo_ms / 1000.0
    l2_rate = l2_requests / seconds
    mem_rate = (fetch_bytes + write_bytes) / seconds
    return l2_rate / l2_peak_requests_per_s, mem_rate / mem_peak_bytes_per_s


def factors(corun_ms, solo_ms):
    """Co-run latency over solo latency of the victim, per sample."""
    return [c / s for c, s in zip(corun_ms, solo_ms)]


def split(keys):
    """70 / 30 split (Sec. 4.4: 1,750 of 2,500 samples train, 750 validate): samples in the order
    of their keys (ties by index), the first floor(0.7 n) train -> (train indices, validation indices)."""
    order = sorted(range(len(keys)), key=lambda i: (keys[i], i))
    n_train = (7 * len(keys)) // 10
    return order[:n_train], order[n_train:]


def worst_slowdown(c, features):
    """Largest predicted factor over the rows, minus one, not below zero."""
    return max(0.0, max(float(v) for v in predict(c, features)) - 1.0)


def overhead(factor_values, qs, threshold):
    """Overhead factor - 1 at the percentiles qs (nearest rank) and the share strictly below threshold."""
    over = [f - 1.0 for f in factor_values]
    return [percentile(over, q) for q in qs], sum(1 for o in over if o < threshold) / len(over)
