"""Pins of the fp64 CPU oracle against things other than itself: a worked
example computed by hand, brute force in pure Python, delta-kernel and
linearity invariants, closed forms, reductions to library routines, and an
independent float64 PyTorch evaluation.  All CPU only."""

import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2109_01611_amd import workloads

RNG = np.random.default_rng(20210901)


def _read_golden(path):
    blocks, name = {}, None
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line[0].isalpha():
                name = line
                blocks[name] = []
            else:
                blocks[name].append([float(v) for v in line.split()])
    return {k: np.array(v) for k, v in blocks.items()}


# ---------------------------------------------------------------- worked example

def test_worked_3x3_example(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "conv3x3_worked_example.txt"))
    x = g["x"].reshape(1, 1, 3, 3)
    w = g["w"].reshape(1, 1, 3, 3)
    b = g["b"].reshape(1)
    y = oracle.conv2d(x, w, b, stride=1, pad=1)
    assert np.array_equal(y[0, 0], g["y_stride1_pad1"])
    assert not np.array_equal(y[0, 0], g["y_flipped_wrong"])
    assert np.array_equal(oracle.conv2d(x, w, b, 1, 1, relu=True)[0, 0], g["y_stride1_pad1_relu"])
    assert np.array_equal(oracle.conv2d(x, w, b, 2, 1)[0, 0], g["y_stride2_pad1"])


# ---------------------------------------------------------------- brute force

def _brute_conv(x, w, b, stride, pad, relu, residual):
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    y = [[[[0.0] * Q for _ in range(P)] for _ in range(K)] for _ in range(N)]
    for n in range(N):
        for k in range(K):
            for p in range(P):
                for q in range(Q):
                    acc = float(b[k])
                    for c in range(C):
                        for r in range(R):
                            for s in range(S):
                                h = p * stride + r - pad
                                v = q * stride + s - pad
                                if 0 <= h < H and 0 <= v < W:
                                    acc += float(x[n, c, h, v]) * float(w[k, c, r, s])
                    if residual is not None:
                        acc += float(residual[n, k, p, q])
                    if relu:
                        acc = max(acc, 0.0)
                    y[n][k][p][q] = acc
    return np.array(y)


@pytest.mark.parametrize("R,stride,pad", [(1, 1, 0), (1, 2, 0), (3, 1, 0), (3, 1, 1), (3, 2, 1),
                                          (5, 1, 2), (5, 2, 0), (3, 2, 2), (5, 1, 1)])
def test_conv_brute_force(R, stride, pad):
    N, C, K, H, W = 2, 3, 2, 6, 5
    x = RNG.standard_normal((N, C, H, W))
    w = RNG.standard_normal((K, C, R, R))
    b = RNG.standard_normal(K)
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    res = RNG.standard_normal((N, K, P, Q))
    for relu, use_res in itertools.product((False, True), (False, True)):
        got = oracle.conv2d(x, w, b, stride, pad, relu, res if use_res else None)
        want = _brute_conv(x, w, b, stride, pad, relu, res if use_res else None)
        assert got.shape == want.shape
        assert np.max(np.abs(got - want)) < 1e-12


def test_conv_brute_force_nonsquare_kernel():
    x = RNG.standard_normal((1, 2, 5, 7))
    w = RNG.standard_normal((3, 2, 3, 3))
    w[:, :, :, 2] = 0.0  # effectively a 3x2 kernel, exercises r/s not being swapped
    b = np.zeros(3)
    assert np.max(np.abs(oracle.conv2d(x, w, b, 1, 1) - _brute_conv(x, w, b, 1, 1, False, None))) < 1e-12


def test_pool_and_fc_brute_force():
    x = RNG.standard_normal((2, 3, 7, 6))
    for k, stride, pad in [(2, 2, 0), (3, 2, 1), (3, 1, 1), (3, 3, 0), (2, 1, 1)]:
        P = (7 + 2 * pad - k) // stride + 1
        Q = (6 + 2 * pad - k) // stride + 1
        mx = np.empty((2, 3, P, Q))
        av = np.empty((2, 3, P, Q))
        for n, c, p, q in itertools.product(range(2), range(3), range(P), range(Q)):
            vals = [x[n, c, p * stride + r - pad, q * stride + s - pad]
                    for r in range(k) for s in range(k)
                    if 0 <= p * stride + r - pad < 7 and 0 <= q * stride + s - pad < 6]
            mx[n, c, p, q] = max(vals)
            av[n, c, p, q] = sum(vals) / (k * k)
        assert np.array_equal(oracle.maxpool(x, k, stride, pad), mx)
        assert np.max(np.abs(oracle.avgpool(x, k, stride, pad) - av)) < 1e-14
    xf = RNG.standard_normal((3, 5))
    wf = RNG.standard_normal((4, 5))
    bf = RNG.standard_normal(4)
    want = np.array([[bf[o] + sum(xf[n, i] * wf[o, i] for i in range(5)) for o in range(4)]
                     for n in range(3)])
    assert np.max(np.abs(oracle.fc(xf, wf, bf) - want)) < 1e-13
    assert np.max(np.abs(oracle.fc(xf, wf, bf, relu=True) - np.maximum(want, 0))) < 1e-13


# ---------------------------------------------------------------- delta kernels

def test_identity_kernel_returns_input_plus_bias():
    C, R = 3, 5
    x = RNG.standard_normal((2, C, 6, 7))
    w = np.zeros((C, C, R, R))
    for c in range(C):
        w[c, c, R // 2, R // 2] = 1.0
    b = np.array([0.5, -1.0, 2.0])
    y = oracle.conv2d(x, w, b, 1, R // 2)
    assert np.array_equal(y, x + b[None, :, None, None])


@pytest.mark.parametrize("r0,s0", [(0, 0), (0, 2), (2, 1), (1, 0)])
def test_shifted_delta_shifts_the_image(r0, s0):
    x = RNG.standard_normal((1, 1, 5, 6))
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, r0, s0] = 1.0
    y = oracle.conv2d(x, w, None, 1, 1)
    want = np.zeros_like(x)
    dh, dw = r0 - 1, s0 - 1          # y[p,q] = x[p+dh, q+dw], zero outside
    for p in range(5):
        for q in range(6):
            if 0 <= p + dh < 5 and 0 <= q + dw < 6:
                want[0, 0, p, q] = x[0, 0, p + dh, q + dw]
    assert np.array_equal(y, want)


def test_1x1_delta_stride2_subsamples():
    x = RNG.standard_normal((2, 2, 7, 8))
    w = np.eye(2).reshape(2, 2, 1, 1)
    assert np.array_equal(oracle.conv2d(x, w, None, 2, 0), x[:, :, ::2, ::2])


def test_channel_routing_is_not_transposed():
    # w[k=1, c=0] = 1 sends input channel 0 to output channel 1 only.
    x = RNG.standard_normal((1, 2, 4, 4))
    w = np.zeros((3, 2, 1, 1))
    w[1, 0, 0, 0] = 1.0
    y = oracle.conv2d(x, w, None)
    assert np.array_equal(y[:, 1], x[:, 0])
    assert not y[:, 0].any() and not y[:, 2].any()


# ---------------------------------------------------------------- linearity

def test_linearity_in_input_and_weights():
    x1, x2 = RNG.standard_normal((2, 2, 3, 6, 6))
    w1, w2 = RNG.standard_normal((2, 4, 3, 3, 3))
    b = RNG.standard_normal(4)
    a, c = 0.75, -2.5
    f = lambda x, w, bias=None: oracle.conv2d(x, w, bias, 2, 1)
    assert np.max(np.abs(f(a * x1 + c * x2, w1) - (a * f(x1, w1) + c * f(x2, w1)))) < 1e-12
    assert np.max(np.abs(f(x1, a * w1 + c * w2) - (a * f(x1, w1) + c * f(x1, w2)))) < 1e-12
    zero = np.zeros_like(x1)
    lin = lambda x: f(x, w1, b) - f(zero, w1, b)
    assert np.max(np.abs(lin(a * x1 + c * x2) - (a * lin(x1) + c * lin(x2)))) < 1e-12
    # the bias alone is what an all-zero input gives
    assert np.array_equal(f(zero, w1, b), np.broadcast_to(b[None, :, None, None], f(zero, w1, b).shape))


# ---------------------------------------------------------------- closed forms

def test_all_ones_counts_in_bounds_taps():
    C, R, H, W = 3, 3, 5, 4
    x = np.ones((1, C, H, W))
    w = np.ones((2, C, R, R))
    b = np.array([0.25, -0.5])
    y0 = oracle.conv2d(x, w, b, 1, 0)
    assert np.array_equal(y0, np.broadcast_to((C * R * R + b)[None, :, None, None], y0.shape))
    y1 = oracle.conv2d(x, w, b, 1, 1)
    for p in range(H):
        for q in range(W):
            taps = (min(p + 1, H - 1) - max(p - 1, 0) + 1) * (min(q + 1, W - 1) - max(q - 1, 0) + 1)
            assert y1[0, 0, p, q] == taps * C + b[0]
            assert y1[0, 1, p, q] == taps * C + b[1]


@pytest.mark.parametrize("n,k,stride,pad,want", [(224, 7, 2, 3, 112), (112, 3, 2, 1, 56), (28, 5, 1, 2, 28),
                                                 (14, 5, 1, 0, 10), (224, 2, 2, 0, 112), (7, 3, 2, 1, 4),
                                                 (56, 1, 2, 0, 28), (2, 3, 1, 0, 0)])
def test_output_size_rule(n, k, stride, pad, want):
    assert oracle.out_dim(n, k, stride, pad) == want


# ---------------------------------------------------------------- reductions to library routines

def test_1x1_conv_is_a_matmul():
    x = RNG.standard_normal((2, 5, 4, 3))
    w = RNG.standard_normal((7, 5, 1, 1))
    b = RNG.standard_normal(7)
    y = oracle.conv2d(x, w, b)
    want = (x.transpose(0, 2, 3, 1).reshape(-1, 5) @ w.reshape(7, 5).T + b).reshape(2, 4, 3, 7)
    assert np.max(np.abs(y - want.transpose(0, 3, 1, 2))) < 1e-12


def test_full_window_conv_is_fc_and_fc_is_matmul():
    x = RNG.standard_normal((3, 4, 5, 6))
    w = RNG.standard_normal((8, 4, 5, 6))
    b = RNG.standard_normal(8)
    yc = oracle.conv2d(x, w, b)
    yf = oracle.fc(x.reshape(3, -1), w.reshape(8, -1), b)
    assert yc.shape == (3, 8, 1, 1)
    assert np.max(np.abs(yc.reshape(3, 8) - yf)) < 1e-12
    assert np.max(np.abs(yf - (x.reshape(3, -1) @ w.reshape(8, -1).T + b))) < 1e-12


def test_pools_reduce_to_numpy():
    x = RNG.standard_normal((2, 3, 6, 8))
    assert np.max(np.abs(oracle.global_avgpool(x) - x.mean(axis=(2, 3)))) < 1e-15
    want = x.reshape(2, 3, 3, 2, 4, 2).max(axis=(3, 5))
    assert np.array_equal(oracle.maxpool(x, 2, 2), want)
    assert np.max(np.abs(oracle.avgpool(x, 2, 2) - x.reshape(2, 3, 3, 2, 4, 2).mean(axis=(3, 5)))) < 1e-15


def test_stride2_is_subsampled_stride1_and_shift_equivariance():
    x = RNG.standard_normal((1, 2, 9, 9))
    w = RNG.standard_normal((3, 2, 3, 3))
    b = RNG.standard_normal(3)
    assert np.array_equal(oracle.conv2d(x, w, b, 2, 1), oracle.conv2d(x, w, b, 1, 1)[:, :, ::2, ::2])
    xs = np.zeros((1, 2, 12, 12))
    xs[:, :, 4:7, 4:7] = RNG.standard_normal((1, 2, 3, 3))
    y = oracle.conv2d(xs, w, None, 1, 1)
    ys = oracle.conv2d(np.roll(xs, (1, 2), axis=(2, 3)), w, None, 1, 1)
    assert np.array_equal(np.roll(y, (1, 2), axis=(2, 3)), ys)


@pytest.mark.parametrize("C,K,R,stride,pad", [(3, 4, 7, 2, 3), (6, 16, 5, 1, 0), (8, 8, 3, 1, 1),
                                              (5, 3, 3, 2, 1), (4, 6, 1, 2, 0), (2, 2, 5, 1, 2)])
def test_conv_matches_torch_float64(C, K, R, stride, pad):
    x = RNG.standard_normal((2, C, 11, 9))
    w = RNG.standard_normal((K, C, R, R))
    b = RNG.standard_normal(K)
    want = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), stride, pad).numpy()
    got = oracle.conv2d(x, w, b, stride, pad)
    assert got.shape == want.shape
    assert np.max(np.abs(got - want)) < 1e-11


def test_pool_fc_match_torch_float64():
    x = RNG.standard_normal((2, 5, 13, 10))
    xt = torch.from_numpy(x)
    for k, s, p in [(3, 2, 1), (2, 2, 0), (3, 1, 1)]:
        assert np.array_equal(oracle.maxpool(x, k, s, p), F.max_pool2d(xt, k, s, p).numpy())
        assert np.max(np.abs(oracle.avgpool(x, k, s, p) - F.avg_pool2d(xt, k, s, p).numpy())) < 1e-14
    xf, wf, bf = RNG.standard_normal((4, 9)), RNG.standard_normal((6, 9)), RNG.standard_normal(6)
    want = F.linear(torch.from_numpy(xf), torch.from_numpy(wf), torch.from_numpy(bf)).numpy()
    assert np.max(np.abs(oracle.fc(xf, wf, bf) - want)) < 1e-13


# ---------------------------------------------------------------- model tables

def test_model_totals_match_published_counts():
    # LeNet-5: 61,706 parameters with 16*5*5 = 400 flattened features.
    assert oracle.model_params(workloads.lenet5()) == 61706
    # VGG-16: 138,357,544 parameters, 15.47 G multiply-adds per 224x224 image.
    vgg = workloads.vgg16()
    assert oracle.model_params(vgg) == 138357544
    conv, fcf = oracle.model_flops(vgg)
    assert abs((conv + fcf) / 2 / 1e9 - 15.47) < 0.01
    # ResNet-50 (stride on the 3x3): 25,557,032 parameters counting two batch-norm
    # vectors per convolution and no convolution bias; folded, each convolution
    # keeps one bias vector.  4.09 G multiply-adds per image.
    res = workloads.resnet50()
    n_conv_bias = sum(nd.attr["K"] for nd in res.nodes if nd.op == "conv")
    assert n_conv_bias == 26560
    assert oracle.model_params(res) + n_conv_bias == 25557032
    conv, fcf = oracle.model_flops(res)
    assert sum(1 for nd in res.nodes if nd.op == "conv") == 53
    assert abs((conv + fcf) / 2 / 1e9 - 4.09) < 0.01
    # GoogLeNet without auxiliary heads: 57 convolutions, 1024 features into the FC.
    goo = workloads.googlenet()
    assert sum(1 for nd in goo.nodes if nd.op == "conv") == 57
    conv, fcf = oracle.model_flops(goo)
    assert fcf == 2 * 1024 * 1000
    assert abs((conv + fcf) / 1e9 - 3.165) < 0.005
    # single 3x3 layer at batch 32: 2*32*14*14*256*256*9
    conv, _ = oracle.model_flops(workloads.single_conv())
    assert conv * 32 == 7398752256


def _torch_bottleneck_net(x, P):
    """ResNet-shaped wiring written by hand (not from the table)."""
    def cv(t, name, stride=1, pad=0):
        w, b = P[name]
        return F.conv2d(t, torch.from_numpy(w).double(), torch.from_numpy(b).double(), stride, pad)
    t = F.relu(cv(x, "stem", 2, 3))
    t = F.max_pool2d(t, 3, 2, 1)
    for s, reps in enumerate((1, 2), 1):
        for b in range(reps):
            p = "l%d_%d" % (s, b)
            stride = 2 if (s > 1 and b == 0) else 1
            u = F.relu(cv(t, p + "_a"))
            u = F.relu(cv(u, p + "_b", stride, 1))
            u = cv(u, p + "_c")
            sc = cv(t, p + "_proj", stride) if b == 0 else t
            t = F.relu(u + sc)
    t = t.mean(dim=(2, 3))
    w, b = P["fc"]
    return F.linear(t, torch.from_numpy(w).double(), torch.from_numpy(b).double())


def test_resnet_wiring_against_handwritten_torch():
    m = workloads.resnet50(width_div=8, in_hw=32, n_class=10, blocks=(1, 2))
    P = workloads.parameters(m, seed=3)
    x = workloads.batch_input(m, 2, seed=3)
    got = oracle.run_model(m, P, x)
    want = _torch_bottleneck_net(torch.from_numpy(x).double(), P).numpy()
    assert got.shape == (2, 10)
    assert np.max(np.abs(got - want)) < 1e-10 * max(1.0, np.abs(want).max())


def test_inception_wiring_against_handwritten_torch():
    m = workloads.googlenet(width_div=4, in_hw=32, n_class=10, n_blocks=1)
    P = workloads.parameters(m, seed=4)
    x = workloads.batch_input(m, 2, seed=4)

    def cv(t, name, stride=1, pad=0):
        w, b = P[name]
        return F.relu(F.conv2d(t, torch.from_numpy(w).double(), torch.from_numpy(b).double(), stride, pad))
    t = torch.from_numpy(x).double()
    t = F.max_pool2d(cv(t, "stem1", 2, 3), 3, 2, 1)
    t = F.max_pool2d(cv(cv(t, "stem2"), "stem3", 1, 1), 3, 2, 1)
    b1 = cv(t, "i3a_1x1")
    b2 = cv(cv(t, "i3a_3x3r"), "i3a_3x3", 1, 1)
    b3 = cv(cv(t, "i3a_5x5r"), "i3a_5x5", 1, 2)
    b4 = cv(F.max_pool2d(t, 3, 1, 1), "i3a_poolproj")
    t = torch.cat([b1, b2, b3, b4], dim=1).mean(dim=(2, 3))
    w, b = P["fc"]
    want = F.linear(t, torch.from_numpy(w).double(), torch.from_numpy(b).double()).numpy()
    got = oracle.run_model(m, P, x)
    assert np.max(np.abs(got - want)) < 1e-10 * max(1.0, np.abs(want).max())


def test_lenet_and_vgg_wiring_against_handwritten_torch():
    m = workloads.lenet5()
    P = workloads.parameters(m, seed=0)
    x = workloads.batch_input(m, 3, seed=0)
    tp = {k: (torch.from_numpy(w).double(), torch.from_numpy(b).double()) for k, (w, b) in P.items()}
    t = torch.from_numpy(x).double()
    t = F.max_pool2d(F.relu(F.conv2d(t, *tp["conv1"], 1, 2)), 2, 2)
    t = F.max_pool2d(F.relu(F.conv2d(t, *tp["conv2"], 1, 0)), 2, 2)
    t = t.flatten(1)
    assert t.shape[1] == 400
    t = F.relu(F.linear(t, *tp["fc1"]))
    t = F.relu(F.linear(t, *tp["fc2"]))
    want = F.linear(t, *tp["fc3"]).numpy()
    got = oracle.run_model(m, P, x)
    assert got.shape == (3, 10)
    assert np.max(np.abs(got - want)) < 1e-11 * max(1.0, np.abs(want).max())

    m = workloads.vgg16(width_div=16, in_hw=32, n_class=10)
    P = workloads.parameters(m, seed=1)
    x = workloads.batch_input(m, 2, seed=1)
    tp = {k: (torch.from_numpy(w).double(), torch.from_numpy(b).double()) for k, (w, b) in P.items()}
    t = torch.from_numpy(x).double()
    for g, reps in enumerate((2, 2, 3, 3, 3), 1):
        for i in range(1, reps + 1):
            t = F.relu(F.conv2d(t, *tp["conv%d_%d" % (g, i)], 1, 1))
        t = F.max_pool2d(t, 2, 2)
    t = t.flatten(1)
    t = F.relu(F.linear(t, *tp["fc6"]))
    t = F.relu(F.linear(t, *tp["fc7"]))
    want = F.linear(t, *tp["fc8"]).numpy()
    got = oracle.run_model(m, P, x)
    assert np.max(np.abs(got - want)) < 1e-11 * max(1.0, np.abs(want).max())


# ---------------------------------------------------------------- depthwise convolution (SSD-MobileNet shape)

@pytest.mark.parametrize("R,stride,pad", [(3, 1, 1), (3, 2, 1), (3, 1, 0), (5, 2, 2), (1, 1, 0)])
def test_depthwise_brute_force_and_block_diagonal_full_conv(R, stride, pad):
    N, C, H, W = 2, 5, 7, 6
    x = RNG.standard_normal((N, C, H, W))
    w = RNG.standard_normal((C, 1, R, R))
    b = RNG.standard_normal(C)
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    for relu in (False, True):
        got = oracle.depthwise_conv2d(x, w, b, stride, pad, relu)
        want = np.zeros((N, C, P, Q))
        for n, c, p, q in itertools.product(range(N), range(C), range(P), range(Q)):
            acc = float(b[c])
            for r, s in itertools.product(range(R), range(R)):
                h, v = p * stride + r - pad, q * stride + s - pad
                if 0 <= h < H and 0 <= v < W:
                    acc += float(x[n, c, h, v]) * float(w[c, 0, r, s])
            want[n, c, p, q] = max(acc, 0.0) if relu else acc
        assert np.max(np.abs(got - want)) < 1e-12
        # a depthwise convolution is a full convolution whose filter bank is diagonal in (k, c)
        full = np.zeros((C, C, R, R))
        for c in range(C):
            full[c, c] = w[c, 0]
        assert np.max(np.abs(got - oracle.conv2d(x, full, b, stride, pad, relu))) < 1e-12
        t = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), stride, pad, groups=C)
        t = F.relu(t) if relu else t
        assert np.max(np.abs(got - t.numpy())) < 1e-12


def test_depthwise_channels_do_not_mix_and_taps_are_not_transposed():
    x = RNG.standard_normal((1, 3, 6, 6))
    w = np.zeros((3, 1, 3, 3))
    w[0, 0, 1, 1] = 1.0          # channel 0: identity
    w[1, 0, 0, 1] = 1.0          # channel 1: reads the pixel above
    w[2, 0, 1, 2] = 2.0          # channel 2: twice the pixel to the right
    y = oracle.depthwise_conv2d(x, w, None, 1, 1)
    assert np.array_equal(y[0, 0], x[0, 0])
    assert np.array_equal(y[0, 1, 1:], x[0, 1, :-1]) and np.all(y[0, 1, 0] == 0)
    assert np.array_equal(y[0, 2, :, :-1], 2 * x[0, 2, :, 1:]) and np.all(y[0, 2, :, -1] == 0)


def test_ssd_mobilenet_totals_match_published_counts():
    # MobileNets paper (Howard et al. 2017), COCO detection table: SSD 300 with MobileNet,
    # 1.2 billion mult-adds and 6.8 million parameters.
    m = workloads.ssd_mobilenet()
    conv, fcf = oracle.model_flops(m)
    assert fcf == 0
    assert abs(conv / 2 / 1e9 - 1.2) < 0.05
    assert abs(oracle.model_params(m) / 1e6 - 6.8) < 0.05
    assert sum(1 for nd in m.nodes if nd.op == "dwconv") == 13
    # the backbone at 224x224 is MobileNet-v1 without its classifier: that paper gives 569 M mult-adds and
    # 4.2 M parameters including the 1024 -> 1000 fully connected layer
    m224 = workloads.ssd_mobilenet(in_hw=224)
    back = [nd for nd in m224.nodes if nd.name == "stem" or nd.name.startswith(("dw", "pw"))]
    sub = workloads.Model("b", m224.in_shape, m224.in_dist, back, back[-1].dst)
    assert abs((oracle.model_flops(sub)[0] / 2 + 1024 * 1000) / 1e6 - 569) < 1.0
    assert abs((oracle.model_params(sub) + 1024 * 1000 + 1000) / 1e6 - 4.2) < 0.05


def test_ssd_wiring_against_handwritten_torch():
    m = workloads.ssd_mobilenet(width_div=8, in_hw=64, n_class=3)
    P = workloads.parameters(m, seed=5)
    x = workloads.batch_input(m, 2, seed=5)
    T = oracle.run_model(m, P, x, keep=True)

    def cv(t, name, stride=1, pad=0, groups=1):
        w, b = P[name]
        return F.conv2d(t, torch.from_numpy(w).double(), torch.from_numpy(b).double(), stride, pad, groups=groups)
    t = F.relu(cv(torch.from_numpy(x).double(), "stem", 2, 1))
    strides = [1, 2, 1, 2, 1, 2, 1, 1, 1, 1, 1, 2, 1]
    feats = []
    for i, st in enumerate(strides, 1):
        t = F.relu(cv(t, "dw%d" % i, st, 1, groups=t.shape[1]))
        t = F.relu(cv(t, "pw%d" % i))
        if i in (11, 13):
            feats.append(t)
    for j in range(1, 5):
        t = F.relu(cv(t, "extra%d_a" % j))
        t = F.relu(cv(t, "extra%d_b" % j, 2, 1))
        feats.append(t)
    assert len(feats) == 6
    for k, f in enumerate(feats, 1):
        head = torch.cat([cv(f, "box%d" % k), cv(f, "cls%d" % k)], dim=1).numpy()
        name = "y" if k == 6 else "head%d" % k
        assert head.shape == T[name].shape
        assert head.shape[1] == (3 if k == 1 else 6) * (4 + 3)
        assert np.max(np.abs(head - T[name])) < 1e-9 * max(1.0, np.abs(head).max())


def test_run_model_storage_hook_sees_every_computing_layer_once():
    # The hook models an implementation's tensor format; the layers' arithmetic must not change.
    m = workloads.resnet50(width_div=8, in_hw=32, n_class=10, blocks=(1, 2))
    P = workloads.parameters(m, seed=3)
    x = workloads.batch_input(m, 2, seed=3)
    plain = oracle.run_model(m, P, x)
    seen = []

    def ident(a):
        seen.append(a.shape)
        return a

    assert np.array_equal(oracle.run_model(m, P, x, storage=ident), plain)
    assert len(seen) == sum(nd.op in ("conv", "dwconv", "fc", "gavgpool") for nd in m.nodes)
    # a hook that halves every stored tensor scales a bias-free ReLU chain by 2^-depth: checked on
    # the stem alone (one conv, then max-pool, which stores nothing new)
    T = oracle.run_model(m, P, x, keep=True, storage=lambda a: 0.5 * a)
    T0 = oracle.run_model(m, P, x, keep=True)
    first = m.nodes[0]
    assert first.op == "conv"
    assert np.array_equal(T[first.dst], 0.5 * T0[first.dst])


# ---------------------------------------------------------------- the error metric itself

def test_rel_err_hand_computed_values():
    # ||d||_2 / ||ref||_2 on vectors whose norms are known by hand (3-4-5 triangles)
    ref = np.array([[3.0, 4.0]])
    got = np.array([[3.0, 4.5]])
    whole, per = oracle.rel_err(got, ref)
    assert whole == pytest.approx(0.1, abs=1e-15) and per == pytest.approx(0.1, abs=1e-15)
    # the 2-norm, not the 1-norm (1/4) and not the max-norm (1)
    whole, per = oracle.rel_err(np.array([[2.0, 1.0, 1.0, 1.0]]), np.ones((1, 4)))
    assert whole == pytest.approx(0.5, abs=1e-15) and per == pytest.approx(0.5, abs=1e-15)
    # divided by the norm of the reference, not of the result (that would give 1/2)
    whole, per = oracle.rel_err(2.0 * ref, ref)
    assert whole == pytest.approx(1.0, abs=1e-15) and per == pytest.approx(1.0, abs=1e-15)


def test_rel_err_reports_the_worst_image_not_the_mean():
    # two images, only the second is off by one unit: whole tensor 1/sqrt(125), images 0 and 1/10
    ref = np.array([[3.0, 4.0], [6.0, 8.0]])
    got = np.array([[3.0, 4.0], [6.0, 9.0]])
    whole, per = oracle.rel_err(got, ref)
    assert whole == pytest.approx(1.0 / np.sqrt(125.0), abs=1e-15)
    assert per == pytest.approx(0.1, abs=1e-15)          # the mean over images would be 0.05
    # one bad image among many good ones cannot hide in the whole-tensor figure
    ref = np.tile(np.array([[3.0, 4.0]]), (100, 1))
    got = ref.copy()
    got[37] = [3.0, 9.0]
    whole, per = oracle.rel_err(got, ref)
    assert per == pytest.approx(1.0, abs=1e-15) and whole == pytest.approx(0.1, abs=1e-15)
    # a small image that is entirely wrong next to a large one that is right
    ref = np.array([[1e-3, 0.0], [30.0, 40.0]])
    got = np.array([[0.0, 0.0], [30.0, 40.0]])
    whole, per = oracle.rel_err(got, ref)
    assert per == pytest.approx(1.0, abs=1e-12) and whole < 1e-4


def test_rel_err_invariants():
    ref = RNG.standard_normal((3, 4, 5, 6))
    got = ref + 1e-3 * RNG.standard_normal(ref.shape)
    assert oracle.rel_err(ref, ref) == (0.0, 0.0)
    a = oracle.rel_err(got, ref)
    for scale in (1e-6, 7.0, 1e9):                        # both tensors scaled alike: unchanged
        b = oracle.rel_err(scale * got, scale * ref)
        assert b[0] == pytest.approx(a[0], rel=1e-12) and b[1] == pytest.approx(a[1], rel=1e-12)
    # an image is everything behind axis 0, whatever the shape: same figures on the flattened tensor
    assert oracle.rel_err(got.reshape(3, -1), ref.reshape(3, -1)) == a
    # the per-image figure is the largest of the images' own figures, each against its own norm
    each = [np.linalg.norm(got[i] - ref[i]) / np.linalg.norm(ref[i]) for i in range(3)]
    assert a[1] == pytest.approx(max(each), rel=1e-12)
    assert a[0] == pytest.approx(np.linalg.norm(got - ref) / np.linalg.norm(ref), rel=1e-12)
    # permuting the images changes neither figure; the per-image figure is at least the whole one
    b = oracle.rel_err(got[::-1], ref[::-1])
    assert b[0] == pytest.approx(a[0], rel=1e-12) and b[1] == pytest.approx(a[1], rel=1e-12)
    # an all-zero reference raises nothing (the quotient is merely huge)
    z = oracle.rel_err(np.ones((2, 3)), np.zeros((2, 3)))
    assert z[0] > 1e100 and z[1] > 1e100
