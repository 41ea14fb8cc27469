"""The benchmark's layer (ResNet-50-style 3x3 convolution, N=32, C=K=256, 14x14,
bias + ReLU) at full size, on the whole GPU and on gpu-lets of several sizes,
against the fp64 oracle."""

import pytest

import oracle
from paper_2109_01611_amd import gpulet

from gpu_util import LAYER_TOL, conv_tensors, gpu_conv

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("pct,which", [(100, 0), (20, 0), (80, 1), (50, 1)])
def test_benchmark_layer_full_size_on_gpulets(pct, which):
    # ResNet-50-style 3x3 layer at batch 32: N=32, C=K=256, 14x14, stride 1, pad 1, bias + ReLU
    x, w, b = conv_tensors(0, 32, 256, 14, 14, 256, 3)
    ref = oracle.conv2d(x, w, b, 1, 1, True)
    with gpulet.Partition(0, pct, which) as p:
        got, _ = gpu_conv(p, x, w, b, 1, 1, True)
    whole, per_img = oracle.rel_err(got, ref)
    assert max(whole, per_img) <= LAYER_TOL, (whole, per_img)


@pytest.mark.parametrize("pct,which", [(20, 0), (60, 1)])
def test_streaming_1x1_kernel_on_small_gpulets(pct, which):
    # few CUs: every workgroup of the streaming kernel walks over many pixel tiles
    x, w, b = conv_tensors(19, 6, 64, 40, 40, 128, 1)
    ref = oracle.conv2d(x, w, b, 1, 0, True)
    with gpulet.Partition(0, pct, which) as small:
        got, _ = gpu_conv(small, x, w, b, 1, 0, True)
        assert oracle.rel_err(got, ref)[1] <= LAYER_TOL
        got, _ = gpu_conv(small, x, w, b, 1, 0, True, tile=8)
        assert oracle.rel_err(got, ref)[1] <= LAYER_TOL
