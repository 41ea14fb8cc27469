"""The element-wise parity bound of the GPU tests, tested on the CPU: it accepts
what bf16 storage of an fp32-accumulated result produces and rejects single
wrong elements that the normwise figure lets through."""

import numpy as np
import pytest

import oracle
from paper_2109_01611_amd import inputs

from parity_bounds import HALF_ULP_BF16, assert_elementwise, violations


def _layer(seed=5, N=2, C=24, H=9, W=9, K=16):
    x = inputs.tensor(seed, "pb/x", (N, C, H, W), "normal")
    w = inputs.he_normal(seed, "pb/w", (K, C, 3, 3))
    b = inputs.bias(seed, "pb/b", K)
    ref = oracle.conv2d(x, w, b, 1, 1, True)
    mag = oracle.conv2d(np.abs(x), np.abs(w), np.abs(b), 1, 1, False)
    return x, w, b, ref, mag


def test_bf16_rounding_of_the_exact_result_is_inside_the_bound():
    _, _, _, ref, mag = _layer()
    stored = inputs.bf16_round(ref)
    assert not violations(stored, ref, mag).any()
    # ... also after an fp32 accumulation in another order
    x, w, b, ref, mag = _layer(seed=6)
    acc = np.zeros(ref.shape, dtype=np.float32)
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1))).astype(np.float32)
    for c in reversed(range(x.shape[1])):
        for r in range(3):
            for s in range(3):
                acc += xp[:, c, None, r:r + 9, s:s + 9] * w[None, :, c, r, s, None, None].astype(np.float32)
    acc += b[None, :, None, None].astype(np.float32)
    got = inputs.bf16_round(np.maximum(acc, 0))
    assert not violations(got, ref, mag).any()
    assert_elementwise(got, ref, mag)


def test_half_ulp_is_the_right_constant():
    # the worst case of round-to-nearest: a value halfway between two bf16 numbers just above a power of two
    v = np.array([1.0 + 2.0 ** -8 * (1 - 1e-9)])
    r = inputs.bf16_round(v)
    assert abs(r[0] - v[0]) <= HALF_ULP_BF16 * abs(v[0])
    assert abs(r[0] - v[0]) > 0.99 * HALF_ULP_BF16 * abs(v[0])      # the bound is tight, not generous


def test_one_wrong_element_is_caught_although_the_norm_hardly_moves():
    _, _, _, ref, mag = _layer(N=4, C=32, H=14, W=14, K=32)
    got = inputs.bf16_round(ref)
    base = oracle.rel_err(got, ref)[1]
    # a border pixel that missed one of its taps: off by a typical term of its sum
    n, k, p, q = 3, 7, 0, 13
    got_bad = got.copy()
    got_bad[n, k, p, q] = inputs.bf16_round(np.array([ref[n, k, p, q] + mag[n, k, p, q] / (32 * 6)]))[0]
    assert oracle.rel_err(got_bad, ref)[1] <= 4e-3 and oracle.rel_err(got_bad, ref)[1] < base + 2e-3
    bad = violations(got_bad, ref, mag)
    assert bad.sum() == 1 and bad[n, k, p, q]
    with pytest.raises(AssertionError, match=r"1 of \d+ elements"):
        assert_elementwise(got_bad, ref, mag)
    # an element that stayed at its fill value, a NaN, an element of the wrong sign
    for wrong in (-512.0, np.nan, -ref[n, k, p, q] - 1.0):
        g = got.copy()
        g[n, k, p, q] = wrong
        assert violations(g, ref, mag)[n, k, p, q]


def test_shapes_and_sign_of_the_magnitude_are_checked():
    with pytest.raises(ValueError):
        violations(np.zeros((2, 3)), np.zeros((3, 2)), np.zeros((3, 2)))
    with pytest.raises(ValueError):
        violations(np.zeros(3), np.zeros(3), -np.ones(3))
