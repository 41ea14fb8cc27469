"""The benchmark's layer (ResNet-50-style 3x3 convolution, N=32, C=K=256, 14x14,
bias + ReLU) at full size, on the whole GPU and on gpu-lets of several sizes,
against the fp64 oracle."""

import pytest

import oracle
from paper_2109_01611_amd import gpulet

from gpu_util import LAYER_TOL, assert_close, assert_conv_close, conv_mag, conv_tensors, gpu_conv

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("pct,which", [(100, 0), (20, 0), (80, 1), (50, 1)])
def test_benchmark_layer_full_size_on_gpulets(pct, which):
    # ResNet-50-style 3x3 layer at batch 32: N=32, C=K=256, 14x14, stride 1, pad 1, bias + ReLU
    x, w, b = conv_tensors(0, 32, 256, 14, 14, 256, 3)
    ref = oracle.conv2d(x, w, b, 1, 1, True)
    with gpulet.Partition(0, pct, which) as p:
        got, _ = gpu_conv(p, x, w, b, 1, 1, True)
    assert_close(got, ref, conv_mag(x, w, b, 1, 1), what=(pct, which))


@pytest.mark.parametrize("pct,which", [(20, 0), (60, 1)])
def test_streaming_1x1_kernel_on_small_gpulets(pct, which):
    # few CUs: every workgroup of the streaming kernel walks over many pixel tiles
    x, w, b = conv_tensors(19, 6, 64, 40, 40, 128, 1)
    ref, mag = oracle.conv2d(x, w, b, 1, 0, True), conv_mag(x, w, b, 1, 0)
    with gpulet.Partition(0, pct, which) as small:
        got, _ = gpu_conv(small, x, w, b, 1, 0, True)
        assert_close(got, ref, mag)
        got, _ = gpu_conv(small, x, w, b, 1, 0, True, tile=8)
        assert_close(got, ref, mag)


@pytest.mark.parametrize("pct,which", [(20, 0), (60, 1)])
def test_walking_kernels_on_small_gpulets(pct, which):
    # the kernels whose workgroups walk over many tiles size their grids from the gpu-let's CU
    # count: 64 and 160 CUs here, with one and three filter tiles (a grid that is and is not a
    # multiple of the eight dies)
    import numpy as np
    import torch
    from paper_2109_01611_amd import inputs, lowering
    with gpulet.Partition(0, pct, which) as small:
        for K in (64, 136):
            x, w, b = conv_tensors(23, 3, 64, 40, 24, K, 3)            # weights in registers (tile 10)
            got, raw = gpu_conv(small, x, w, b, 1, 1, True, tile=10)
            assert_conv_close(got, x, w, b, 1, 1, True)
            _, gathered = gpu_conv(small, x, w, b, 1, 1, True, tile=1)
            assert torch.equal(raw, gathered)
        x, w, b = conv_tensors(23, 3, 3, 70, 50, 64, 7)                 # stem kernel (tile 9)
        got, _ = gpu_conv(small, x, w, b, 2, 3, True, tile=9)
        assert_conv_close(got, x, w, b, 2, 3, True)
        N, In, Out = 20, 8192, 200                                      # long-row FC: depth split sized from the CU count
        xf = inputs.tensor(23, "sfx", (N, In), "uniform")
        wf = inputs.he_normal(23, "sfw", (Out, In))
        bf = inputs.bias(23, "sfb", Out)
        xd, wd = lowering.to_device_bf16(xf, "cuda:0"), lowering.to_device_bf16(wf, "cuda:0")
        yd = torch.full((N, Out), -512.0, dtype=torch.float32, device="cuda:0")
        torch.cuda.synchronize()
        gpulet.fc(xd, wd, torch.from_numpy(bf).to("cuda:0"), yd, N, In, Out, True, True, small.stream)
        small.sync()
        assert oracle.rel_err(yd.cpu().numpy().astype(np.float64), oracle.fc(xf, wf, bf, True))[1] <= 1e-4
