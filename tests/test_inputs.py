"""Seeded input generator: determinism, chunk independence, moments, and
bfloat16 rounding (round to nearest even) checked against torch's cast."""

import numpy as np
import torch

from paper_2109_01611_amd import inputs, workloads


def test_streams_are_pure_functions_of_seed_name_index():
    a = inputs.normal(0, "t", 1000)
    assert np.array_equal(a, inputs.normal(0, "t", 1000))
    assert np.array_equal(a[:10], inputs.normal(0, "t", 10))
    assert not np.array_equal(a, inputs.normal(1, "t", 1000))
    assert not np.array_equal(a, inputs.normal(0, "u", 1000))
    w = inputs.words(5, "k", 0, 64)
    assert np.array_equal(w[7:20], inputs.words(5, "k", 7, 13))


def test_chunking_does_not_change_values():
    n = inputs._CHUNK + 1234
    u = inputs.uniform(3, "big", n)
    assert np.array_equal(u[inputs._CHUNK:], inputs._unit(inputs.words(3, "big", inputs._CHUNK, 1234)))


def test_moments():
    n = 400000
    u = inputs.uniform(0, "m", n)
    assert 0.0 < u.min() and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 3e-3 and abs(u.var() - 1 / 12) < 1e-3
    z = inputs.normal(0, "m", n)
    assert abs(z.mean()) < 6e-3 and abs(z.var() - 1.0) < 1e-2
    assert abs(np.mean(z ** 4) - 3.0) < 0.1
    w = inputs.he_normal(0, "w", (64, 32, 3, 3))
    assert abs(w.var() / (2.0 / (32 * 9)) - 1.0) < 0.05


def test_bf16_rounding_matches_torch_and_is_exact_roundtrip():
    v = np.concatenate([inputs.normal(2, "r", 50000).astype(np.float32),
                        np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e38, 1e-30],
                                 dtype=np.float32)])
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float32).numpy()
    got = inputs.bf16_round(v)
    assert np.array_equal(got, want)
    bits = inputs.bf16_bits(got)
    assert np.array_equal(inputs.bf16_to_f32(bits), got)
    # ties go to even: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7
    assert inputs.bf16_round(np.float32(1.00390625)) == np.float32(1.0)
    assert inputs.bf16_round(np.float32(1.01171875)) == np.float32(1.015625)


def test_model_tensors_are_bf16_exact_and_seeded():
    m = workloads.lenet5()
    P = workloads.parameters(m, seed=0)
    x = workloads.batch_input(m, 4, seed=0)
    assert x.shape == (4, 1, 28, 28) and x.dtype == np.float32
    assert np.array_equal(inputs.bf16_round(x), x)
    w, b = P["conv2"]
    assert w.shape == (16, 6, 5, 5) and b.shape == (16,)
    assert np.array_equal(inputs.bf16_round(w), w)
    assert np.array_equal(workloads.parameters(m, seed=0)["fc1"][0], P["fc1"][0])
    assert not np.array_equal(workloads.parameters(m, seed=1)["fc1"][0], P["fc1"][0])
    # batch n is a prefix of batch n+1: images do not depend on the batch size
    assert np.array_equal(workloads.batch_input(m, 2, seed=0), x[:2])
