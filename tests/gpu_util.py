"""Helpers shared by the GPU parity tests: move seeded host tensors to the
device in the library's layouts, call the C ABI through the binding, and bring
results back as float64 in the oracle's layout."""

import numpy as np
import torch

import oracle
from paper_2109_01611_amd import gpulet, inputs, lowering

from parity_bounds import SLACK, assert_elementwise

DEV = "cuda:0"

# Normwise relative error bounds (bf16 inputs, fp32 accumulation).  One layer
# adds a single bf16 rounding of the output: relative error at most 2^-9 per
# element, about 2^-9 / sqrt(3) = 1.1e-3 normwise, plus fp32 accumulation
# noise that is orders of magnitude smaller; 4e-3 leaves room for cancellation
# heavy outputs.  Whole models compound one such rounding per layer and must
# stay within 1e-2.
LAYER_TOL = 4e-3
MODEL_TOL = 1e-2


def assert_close(got, ref, mag, tol=LAYER_TOL, slack=SLACK, rel=2.0 ** -8, what=""):
    """Both parity bounds of a layer: the normwise one (whole tensor and worst image) and the
    element-wise one of ``parity_bounds`` against the oracle's sum of absolute terms ``mag``."""
    whole, per_img = oracle.rel_err(got, ref)
    assert max(whole, per_img) <= tol, (what, whole, per_img)
    assert_elementwise(got, ref, mag, slack=slack, rel=rel, what=str(what))


def conv_mag(x, w, b, stride, pad, residual=None):
    """The convolution of the operands' absolute values: per output element the sum of the
    absolute values of its terms (oracle arithmetic only)."""
    return oracle.conv2d(np.abs(x), np.abs(w), None if b is None else np.abs(b), stride, pad, False,
                         None if residual is None else np.abs(residual))


def assert_conv_close(got, x, w, b, stride, pad, relu, residual=None, ref=None, mag=None, tol=LAYER_TOL, what=""):
    """``got`` (float64 NCHW) against the oracle's convolution of the same operands."""
    if ref is None:
        ref = oracle.conv2d(x, w, b, stride, pad, relu, residual)
    if mag is None:
        mag = conv_mag(x, w, b, stride, pad, residual)
    assert_close(got, ref, mag, tol=tol, what=what)


def conv_tensors(seed, N, C, H, W, K, R, S=None):
    S = R if S is None else S
    tag = "%d_%d_%d_%d_%d_%d_%d" % (N, C, H, W, K, R, S)
    x = inputs.tensor(seed, "x" + tag, (N, C, H, W), "normal")
    w = inputs.he_normal(seed, "w" + tag, (K, C, R, S))
    b = inputs.bias(seed, "b" + tag, K)
    return x, w, b


def gpu_conv(part, x, w, b, stride, pad, relu, residual=None, ch_total=0, ch_offset=0, tile=-1):
    """Runs gpulet_conv2d_fwd(_ex) on NCHW/KCRS host tensors -> float64 NCHW and the
    raw bf16 device output."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    xd = lowering.nchw_to_nhwc(x, DEV)
    wd = lowering.kcrs_to_krsc(w, DEV)
    bd = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(DEV) if b is not None else None
    ct = ch_total if ch_total else K
    yd = torch.full((N, P, Q, ct), -512.0, dtype=torch.bfloat16, device=DEV)
    rd = lowering.nchw_to_nhwc(residual, DEV) if residual is not None else None
    torch.cuda.synchronize()
    gpulet.set_conv_tile(tile)
    try:
        if residual is None and not ch_total:
            gpulet.conv2d_fwd(xd, wd, bd, yd, N, C, H, W, K, R, S, stride, pad, relu, part.stream)
        else:
            gpulet.conv2d_fwd_ex(xd, wd, bd, yd, N, C, H, W, K, R, S, stride, pad, relu, rd, ch_total,
                                 ch_offset, part.stream)
        part.sync()
    finally:
        gpulet.set_conv_tile(-1)
    return lowering.nhwc_to_nchw(yd), yd
