"""Parity of the single-layer HIP entry points against the fp64 oracle on the same
seeded tensors, normwise (whole tensor and worst image) and element by element
(|got - ref| <= 2^-8 |ref| + 1e-5 * the oracle's sum of absolute terms): tiny and ragged shapes, every tile,
strides, paddings, residual and channel-slice stores, plus the benchmark's
layer at full size on several gpu-let sizes."""

import numpy as np
import pytest
import torch

import oracle
from paper_2109_01611_amd import gpulet, inputs, lowering

from gpu_util import DEV, LAYER_TOL, assert_close, assert_conv_close, conv_mag, conv_tensors, gpu_conv

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def part():
    p = gpulet.Partition(0, 100, 0)
    yield p
    p.destroy()


# N, C, H, W, K, R, stride, pad
CONV_CASES = [
    (1, 3, 7, 7, 5, 3, 1, 1),          # everything smaller than a tile, C not a multiple of 8
    (2, 1, 28, 28, 6, 5, 1, 2),        # LeNet conv1
    (2, 6, 14, 14, 16, 5, 1, 0),       # LeNet conv2
    (2, 3, 33, 31, 64, 7, 2, 3),       # stem-like, odd image
    (3, 8, 9, 9, 8, 1, 1, 0),
    (2, 16, 10, 10, 24, 1, 2, 0),      # strided 1x1 (projection shortcut)
    (2, 24, 13, 13, 40, 3, 2, 1),
    (1, 48, 7, 7, 128, 5, 1, 2),       # inception 5x5
    (1, 136, 5, 5, 72, 3, 1, 1),       # depth 1224: ragged last slice, K not a multiple of 32
    (1, 8, 4, 4, 8, 3, 1, 3),          # padding wider than the kernel reach
    (2, 64, 56, 56, 64, 3, 1, 1),      # several tiles, M = 6272
    (1, 512, 7, 7, 520, 1, 1, 0),      # M = 49, ragged K
    (5, 32, 12, 11, 96, 3, 1, 1),      # M = 660: ragged last pixel tile
    (2, 20, 9, 9, 12, 3, 1, 1),        # C multiple of 4 only
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv_parity_every_tile(part, case):
    N, C, H, W, K, R, stride, pad = case
    x, w, b = conv_tensors(11, N, C, H, W, K, R)
    ref = oracle.conv2d(x, w, b, stride, pad, relu=True)
    mag = conv_mag(x, w, b, stride, pad)
    first = None
    for tile in range(-1, gpulet.CONV_TILES):
        got, raw = gpu_conv(part, x, w, b, stride, pad, True, tile=tile)
        assert_close(got, ref, mag, what=tile)
        if tile < 0 or (tile == 9 and C <= 4):
            continue      # automatic selection and the stem kernel regroup the fp32 sum
        if first is None:
            first = raw.clone()
        else:  # without a split the accumulation order does not depend on the tile
            assert torch.equal(raw, first), tile


# N, C, H, W, K: 3x3, stride 1, pad 1, C a multiple of 64 -> the kernel that keeps input patches in LDS
PATCH_CASES = [
    (3, 64, 14, 14, 64),       # whole rows per block; tiles cross rows and images (M = 588: ragged last tile)
    (9, 128, 7, 7, 72),        # 7-pixel rows: a tile spans three images; K ragged
    (2, 64, 56, 56, 64),       # 14-pixel column blocks, four per row
    (1, 64, 32, 32, 32),       # 16-pixel column blocks: tiles are 8 x 16 rectangles
    (2, 64, 20, 20, 40),       # 16-pixel blocks with a ragged second block (4 of 16 columns)
    (2, 192, 9, 33, 136),      # odd sizes, three channel blocks, three channel tiles
    (1, 64, 5, 3, 8),          # smaller than one tile
    (2, 256, 16, 16, 64),      # block width = row width = 16, four channel blocks
]


@pytest.mark.parametrize("case", PATCH_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv_patch_kernel_parity(part, case):
    N, C, H, W, K = case
    x, w, b = conv_tensors(17, N, C, H, W, K, 3)
    res = inputs.tensor(17, "res_patch", (N, K, H, W), "normal")
    got, raw = gpu_conv(part, x, w, b, 1, 1, True, residual=res, tile=7)
    assert_conv_close(got, x, w, b, 1, 1, True, residual=res)
    _, gathered = gpu_conv(part, x, w, b, 1, 1, True, residual=res, tile=1)
    assert torch.equal(raw, gathered)          # same summation order as the gathering kernel
    ct = K + 16
    got, _ = gpu_conv(part, x, w, b, 1, 1, False, ch_total=ct, ch_offset=8, tile=7)
    assert_conv_close(got[:, 8:8 + K], x, w, b, 1, 1, False)
    assert np.all(got[:, :8] == -512.0) and np.all(got[:, 8 + K:] == -512.0)


# N, C, H, W, K: 3x3, stride 1, pad 1, C a multiple of 64 -> the tall tile (a pixel rectangle of one image
# with its input patch in LDS, weights streamed tap by tap; tile 11)
TALL_CASES = [
    (2, 64, 56, 56, 128),      # 8 x 28 rectangles, one channel block
    (1, 128, 28, 28, 136),     # 28-pixel rows do not divide into 8: ragged last rectangle; ragged second filter tile
    (3, 64, 14, 14, 64),       # the whole image is one tile (196 of 224 rows)
    (2, 192, 9, 33, 72),       # odd sizes, three channel blocks
    (1, 64, 5, 3, 8),          # smaller than anything
    (2, 256, 16, 16, 64),      # four channel blocks
    (1, 64, 112, 112, 128),    # 56 rectangles per image
    (2, 128, 30, 60, 264),     # rectangles ragged in both directions, three filter tiles
    (5, 320, 7, 7, 40),        # five channel blocks, tiny maps: most rows of a tile are not pixels
]


@pytest.mark.parametrize("case", TALL_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv_tall_tile_kernel_parity(part, case):
    N, C, H, W, K = case
    x, w, b = conv_tensors(27, N, C, H, W, K, 3)
    res = inputs.tensor(27, "res_tall", (N, K, H, W), "normal")
    got, raw = gpu_conv(part, x, w, b, 1, 1, True, residual=res, tile=11)
    assert_conv_close(got, x, w, b, 1, 1, True, residual=res)
    _, gathered = gpu_conv(part, x, w, b, 1, 1, True, residual=res, tile=1)
    assert torch.equal(raw, gathered)          # same summation order as the gathering kernel
    _, again = gpu_conv(part, x, w, b, 1, 1, True, residual=res, tile=11)
    assert torch.equal(raw, again)
    ct = K + 16
    got, _ = gpu_conv(part, x, w, None, 1, 1, False, ch_total=ct, ch_offset=8, tile=11)
    assert_conv_close(got[:, 8:8 + K], x, w, None, 1, 1, False)
    assert np.all(got[:, :8] == -512.0) and np.all(got[:, 8 + K:] == -512.0)


# N, C, H, W, K: max pool 3x3 / stride 1 / pad 1 fused into a 1x1 convolution (inception pooling branch)
POOLED_CASES = [
    (2, 192, 28, 28, 32),      # inception 3a
    (3, 480, 14, 14, 64),      # 4a: M = 588, ragged last pixel tile; 7.5 depth slices
    (2, 832, 7, 7, 128),       # 5a: two filter tiles
    (1, 8, 5, 3, 8),           # smaller than a tile, one chunk of depth
    (2, 72, 9, 11, 40),        # ragged depth slice and filter tile
    (1, 64, 1, 1, 16),         # a single pixel: every tap is the pixel itself
    (2, 256, 1, 9, 24),        # one row: vertical taps all clamp
]


@pytest.mark.parametrize("case", POOLED_CASES, ids=lambda c: "x".join(map(str, c)))
def test_maxpool_fused_into_1x1_conv_parity(part, case):
    N, C, H, W, K = case
    x = inputs.tensor(22, "pc/x%d_%d_%d_%d" % (N, C, H, W), (N, C, H, W), "normal")     # negative values too
    w = inputs.he_normal(22, "pc/w%d_%d" % (K, C), (K, C, 1, 1))
    b = inputs.bias(22, "pc/b%d" % K, K)
    xd = lowering.nchw_to_nhwc(x, DEV)
    wd = lowering.kcrs_to_krsc(w, DEV)
    bd = torch.from_numpy(b).to(DEV)
    ct, off = K + 24, 16
    yd = torch.full((N, H, W, ct), -512.0, dtype=torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    gpulet.maxpool3_conv1x1_fwd(xd, wd, bd, yd, N, C, H, W, K, True, ct, off, part.stream)
    part.sync()
    got = lowering.nhwc_to_nchw(yd)
    assert_conv_close(got[:, off:off + K], oracle.maxpool(x, 3, 1, 1), w, b, 1, 0, True)
    assert np.all(got[:, :off] == -512.0) and np.all(got[:, off + K:] == -512.0)
    # the same bits as the pool kernel followed by the convolution kernel
    pooled = torch.empty((N, H, W, C), dtype=torch.bfloat16, device=DEV)
    y2 = torch.full((N, H, W, ct), -512.0, dtype=torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    gpulet.pool(xd, pooled, N, C, H, W, gpulet.POOL_MAX, 3, 1, 1, part.stream)
    gpulet.conv2d_fwd_ex(pooled, wd, bd, y2, N, C, H, W, K, 1, 1, 1, 0, True, None, ct, off, part.stream)
    part.sync()
    assert torch.equal(yd, y2)
    assert np.array_equal(lowering.nhwc_to_nchw(pooled), oracle.maxpool(x, 3, 1, 1))   # max pooling is exact


def test_maxpool_fused_conv_rejects_what_it_cannot_run(part):
    x = torch.zeros((1, 4, 4, 12), dtype=torch.bfloat16, device=DEV)
    w = torch.zeros((8, 1, 1, 12), dtype=torch.bfloat16, device=DEV)
    y = torch.zeros((1, 4, 4, 8), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(gpulet.GpuletError) as e:      # C not a multiple of 8
        gpulet.maxpool3_conv1x1_fwd(x, w, None, y, 1, 12, 4, 4, 8, True, 0, 0, part.stream)
    assert e.value.status == gpulet.EINVAL


# N, channels per stored pixel, first channel read, C, H, W, K, R, stride, pad
SLICE_CASES = [
    (3, 112, 0, 96, 28, 28, 128, 3, 1, 1),     # inception 3a: 3x3 over the first 96 of 112 channels
    (3, 112, 96, 16, 28, 28, 32, 5, 1, 2),     # ... and the 5x5 over the last 16: four taps per depth slice
    (2, 224, 64, 128, 14, 14, 200, 3, 1, 1),   # C a multiple of 64: taps innermost
    (2, 160, 32, 64, 9, 11, 72, 1, 1, 0),      # 1x1 filter
    (2, 40, 8, 24, 13, 13, 40, 3, 2, 1),       # stride 2, three taps per slice
    (2, 21, 5, 9, 10, 10, 20, 3, 1, 1),        # nothing aligned: element-wise gather
    (1, 64, 24, 40, 7, 7, 16, 5, 1, 2),        # a tap straddles depth slices
]


@pytest.mark.parametrize("case", SLICE_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv_reading_a_channel_slice(part, case):
    N, ldx, off, C, H, W, K, R, stride, pad = case
    tag = "sl/" + "_".join(map(str, case))
    wide = inputs.tensor(31, tag + "x", (N, ldx, H, W), "normal")
    w = inputs.he_normal(31, tag + "w", (K, C, R, R))
    b = inputs.bias(31, tag + "b", K)
    x = np.ascontiguousarray(wide[:, off:off + C])
    ref = oracle.conv2d(x, w, b, stride, pad, True)
    mag = conv_mag(x, w, b, stride, pad)
    _, dense = gpu_conv(part, x, w, b, stride, pad, True)
    P, Q = ref.shape[2], ref.shape[3]
    xd = lowering.nchw_to_nhwc(wide, DEV)
    wd = lowering.kcrs_to_krsc(w, DEV)
    bd = torch.from_numpy(b).to(DEV)
    ct, co = K + 16, 8
    for tile in range(-1, gpulet.CONV_TILES):
        yd = torch.full((N, P, Q, ct), -512.0, dtype=torch.bfloat16, device=DEV)
        torch.cuda.synchronize()
        gpulet.set_conv_tile(tile)
        try:
            gpulet.conv2d_fwd_slices(xd, wd, bd, yd, N, C, H, W, K, R, R, stride, pad, True, None, ldx, off, ct, co,
                                     part.stream)
            part.sync()
        finally:
            gpulet.set_conv_tile(-1)
        got = lowering.nhwc_to_nchw(yd[..., co:co + K])
        assert_close(got, ref, mag, what=tile)
        # the bits of the same layer on a dense copy of the slice, and nothing written outside the slice
        assert torch.equal(yd[..., co:co + K], dense), tile
        assert bool((yd[..., :co] == -512.0).all()) and bool((yd[..., co + K:] == -512.0).all()), tile


def test_conv_slice_arguments_are_checked(part):
    x = torch.zeros((1, 4, 4, 32), dtype=torch.bfloat16, device=DEV)
    w = torch.zeros((8, 1, 1, 16), dtype=torch.bfloat16, device=DEV)
    y = torch.zeros((1, 4, 4, 8), dtype=torch.bfloat16, device=DEV)
    for stride_, off in ((32, 24), (32, -8), (8, 0)):
        with pytest.raises(gpulet.GpuletError) as e:
            gpulet.conv2d_fwd_slices(x, w, None, y, 1, 16, 4, 4, 8, 1, 1, 1, 0, True, None, stride_, off, 0, 0,
                                     part.stream)
        assert e.value.status == gpulet.EINVAL


# N, C, H, W, K, k2, stride, (channels per stored input pixel, first channel read),
# (y pixel width, y offset), (y2 pixel width, y2 offset); 0 width = dense
TWO_OUTPUT_CASES = [
    (3, 192, 28, 28, 176, 64, 1, (0, 0), (256, 0), (0, 0)),        # inception 3a: 1x1 branch + both reduce layers
    (2, 480, 14, 14, 304, 192, 1, (0, 0), (512, 0), (0, 0)),       # 4a: ragged pixel tile
    (2, 64, 9, 11, 72, 40, 1, (96, 32), (48, 8), (64, 16)),        # slices on all three tensors
    (2, 40, 13, 13, 56, 8, 2, (0, 0), (0, 0), (0, 0)),             # stride 2, everything dense
    (1, 24, 6, 5, 21, 8, 1, (0, 0), (16, 8), (13, 0)),             # second part cannot take 16-byte stores
    (1, 16, 4, 4, 30, 12, 1, (0, 0), (0, 0), (0, 0)),              # the boundary falls inside an 8-channel group
    (2, 128, 33, 17, 520, 264, 1, (0, 0), (0, 0), (0, 0)),         # several filter tiles on both sides
]


@pytest.mark.parametrize("case", TWO_OUTPUT_CASES, ids=lambda c: "x".join(map(str, c[:7])))
def test_1x1_conv_with_two_outputs(part, case):
    N, C, H, W, K, k2, stride, (ldx, xo), (ldy, yo), (ldy2, yo2) = case
    tag = "two/" + "_".join(map(str, case[:7]))
    wide = inputs.tensor(33, tag + "x", (N, ldx or C, H, W), "normal")
    w = inputs.he_normal(33, tag + "w", (K, C, 1, 1))
    b = inputs.bias(33, tag + "b", K)
    x = np.ascontiguousarray(wide[:, xo:xo + C])
    ref = oracle.conv2d(x, w, b, stride, 0, True)
    mag = conv_mag(x, w, b, stride, 0)
    _, dense = gpu_conv(part, x, w, b, stride, 0, True)         # all K filters to one dense tensor
    P, Q = ref.shape[2], ref.shape[3]
    xd = lowering.nchw_to_nhwc(wide, DEV)
    wd = lowering.kcrs_to_krsc(w, DEV)
    bd = torch.from_numpy(b).to(DEV)
    for tile in range(-1, gpulet.CONV_TILES):
        y1 = torch.full((N, P, Q, ldy or k2), -512.0, dtype=torch.bfloat16, device=DEV)
        y2 = torch.full((N, P, Q, ldy2 or K - k2), -512.0, dtype=torch.bfloat16, device=DEV)
        torch.cuda.synchronize()
        gpulet.set_conv_tile(tile)
        try:
            gpulet.conv1x1_fwd_two_outputs(xd, wd, bd, y1, y2, N, C, H, W, K, k2, stride, True, ldx, xo, ldy, yo,
                                           ldy2, yo2, part.stream)
            part.sync()
        finally:
            gpulet.set_conv_tile(-1)
        a, c = y1[..., yo:yo + k2], y2[..., yo2:yo2 + K - k2]
        got = torch.cat([a, c], dim=3)
        assert_close(lowering.nhwc_to_nchw(got), ref, mag, what=tile)
        assert torch.equal(got, dense), tile                       # the bits of the plain layer
        for t, lo, hi in ((y1, yo, yo + k2), (y2, yo2, yo2 + K - k2)):
            assert bool((t[..., :lo] == -512.0).all()) and bool((t[..., hi:] == -512.0).all()), tile


def test_two_output_arguments_are_checked(part):
    x = torch.zeros((1, 4, 4, 16), dtype=torch.bfloat16, device=DEV)
    w = torch.zeros((24, 1, 1, 16), dtype=torch.bfloat16, device=DEV)
    y = torch.zeros((1, 4, 4, 24), dtype=torch.bfloat16, device=DEV)
    ok = dict(N=1, C=16, H=4, W=4, K=24, k2=8, stride=1, relu=True, stream=part.stream)
    for kw in (dict(ok, k2=0), dict(ok, k2=24), dict(ok, y_ch_stride=4), dict(ok, y2_ch_stride=8),
               dict(ok, y2_ch_stride=24, y2_ch_offset=16), dict(ok, C=12)):
        with pytest.raises(gpulet.GpuletError) as e:
            gpulet.conv1x1_fwd_two_outputs(x, w, None, y, y, **kw)
        assert e.value.status == gpulet.EINVAL, kw
    with pytest.raises(gpulet.GpuletError) as e:
        gpulet.conv1x1_fwd_two_outputs(x, w, None, y, None, **ok)
    assert e.value.status == gpulet.EINVAL


# N, C, H, W, K, k2 (0 = one output)
SIDE_POOL_CASES = [
    (3, 192, 28, 28, 176, 64),      # inception 3a: 1x1 branch, reduce layers and the pool in one launch
    (2, 480, 14, 14, 304, 192),     # 4a
    (2, 832, 7, 7, 96, 0),          # one output; more pool work than convolution tiles
    (1, 8, 5, 3, 8, 0),             # smaller than anything
    (2, 72, 9, 11, 40, 16),         # ragged tiles
    (4, 64, 1, 9, 24, 0),           # one row: vertical taps clamp
]


@pytest.mark.parametrize("case", SIDE_POOL_CASES, ids=lambda c: "x".join(map(str, c)))
def test_1x1_conv_carrying_the_max_pool_of_its_input(part, case):
    N, C, H, W, K, k2 = case
    tag = "sp/" + "_".join(map(str, case))
    x = inputs.tensor(34, tag + "x", (N, C, H, W), "normal")
    w = inputs.he_normal(34, tag + "w", (K, C, 1, 1))
    b = inputs.bias(34, tag + "b", K)
    _, dense = gpu_conv(part, x, w, b, 1, 0, True)
    pooled_ref = oracle.maxpool(x, 3, 1, 1)
    xd = lowering.nchw_to_nhwc(x, DEV)
    wd = lowering.kcrs_to_krsc(w, DEV)
    bd = torch.from_numpy(b).to(DEV)
    for tile in range(-1, gpulet.CONV_TILES):
        y1 = torch.full((N, H, W, k2 or K), -512.0, dtype=torch.bfloat16, device=DEV)
        y2 = torch.full((N, H, W, K - k2), -512.0, dtype=torch.bfloat16, device=DEV) if k2 else None
        pool = torch.full((N, H, W, C), -512.0, dtype=torch.bfloat16, device=DEV)
        torch.cuda.synchronize()
        gpulet.set_conv_tile(tile)
        try:
            gpulet.conv1x1_maxpool3_fwd(xd, wd, bd, y1, y2, pool, N, C, H, W, K, k2, True, stream=part.stream)
            part.sync()
        finally:
            gpulet.set_conv_tile(-1)
        got = torch.cat([y1, y2], dim=3) if k2 else y1
        assert torch.equal(got, dense), tile                                  # the plain layer's bits
        assert np.array_equal(lowering.nhwc_to_nchw(pool), pooled_ref), tile  # a max pool is exact


def test_side_pool_arguments_are_checked(part):
    x = torch.zeros((1, 4, 4, 16), dtype=torch.bfloat16, device=DEV)
    w = torch.zeros((24, 1, 1, 16), dtype=torch.bfloat16, device=DEV)
    y = torch.zeros((1, 4, 4, 24), dtype=torch.bfloat16, device=DEV)
    pool = torch.zeros((1, 4, 4, 16), dtype=torch.bfloat16, device=DEV)
    ok = dict(N=1, C=16, H=4, W=4, K=24, k2=0, relu=True, stream=part.stream)
    with pytest.raises(gpulet.GpuletError) as e:
        gpulet.conv1x1_maxpool3_fwd(x, w, None, y, None, None, **ok)
    assert e.value.status == gpulet.EINVAL
    with pytest.raises(gpulet.GpuletError) as e:
        gpulet.conv1x1_maxpool3_fwd(x, w, None, y, None, pool, **dict(ok, C=12))
    assert e.value.status == gpulet.EINVAL
    with pytest.raises(gpulet.GpuletError) as e:
        gpulet.conv1x1_maxpool3_fwd(x, w, None, y, y, pool, **dict(ok, k2=24))
    assert e.value.status == gpulet.EINVAL
    with pytest.raises(gpulet.GpuletError) as e:       # misaligned destination for the pooled tensor
        gpulet.conv1x1_maxpool3_fwd(x, w, None, y, None, pool.data_ptr() + 2, **ok)
    assert e.value.status == gpulet.EINVAL


def _group_members(seed, N, H, W, specs, wide_c):
    """Members reading channel slices of one wide tensor and writing slices of one concatenated tensor.
    specs: (first input channel, C, K, R, stride, pad, relu)."""
    wide = inputs.tensor(seed, "grp/x%d_%d_%d_%d" % (N, wide_c, H, W), (N, wide_c, H, W), "normal")
    out = []
    for j, (xo, C, K, R, stride, pad, relu) in enumerate(specs):
        w = inputs.he_normal(seed, "grp/w%d_%d_%d_%d" % (j, K, C, R), (K, C, R, R))
        b = inputs.bias(seed, "grp/b%d_%d" % (j, K), K)
        out.append((xo, C, K, R, stride, pad, relu, w, b))
    return wide, out


GROUP_CASES = [
    # inception 3a after the 1x1 layers: 3x3 over channels 0..95, 5x5 over 96..111, 1x1 over another tensor's worth
    (3, 28, 28, 112, [(0, 96, 128, 3, 1, 1, True), (96, 16, 32, 5, 1, 2, True), (0, 112, 32, 1, 1, 0, True)]),
    # a residual block's first layer next to its strided projection (different output sizes: no shared tensor)
    (2, 28, 28, 256, [(0, 256, 128, 1, 1, 0, True), (0, 256, 512, 1, 2, 0, False)]),
    # four members, ragged everything
    (2, 9, 11, 72, [(0, 72, 40, 3, 1, 1, True), (8, 24, 16, 1, 1, 0, False), (32, 40, 72, 5, 1, 2, True),
                    (0, 8, 8, 3, 1, 1, True)]),
    # a member with an odd filter count takes the element-wise epilogue
    (1, 7, 7, 64, [(0, 64, 21, 3, 1, 1, True), (0, 64, 64, 1, 1, 0, True)]),
]


@pytest.mark.parametrize("case", GROUP_CASES, ids=lambda c: "x".join(map(str, c[:4])))
def test_independent_convs_in_one_launch(part, case):
    N, H, W, wide_c, specs = case
    wide, members = _group_members(35, N, H, W, specs, wide_c)
    xd = lowering.nchw_to_nhwc(wide, DEV)
    same_size = len({(H + 2 * m[5] - m[3]) // m[4] + 1 for m in members}) == 1
    total = sum(m[2] for m in members) + 8
    refs, mags, alone, descs, outs = [], [], [], [], []
    off = 8
    for (xo, C, K, R, stride, pad, relu, w, b) in members:
        x = np.ascontiguousarray(wide[:, xo:xo + C])
        refs.append(oracle.conv2d(x, w, b, stride, pad, relu))
        mags.append(conv_mag(x, w, b, stride, pad))
        alone.append(gpu_conv(part, x, w, b, stride, pad, relu)[1])
        P, Q = refs[-1].shape[2], refs[-1].shape[3]
        wd, bd = lowering.kcrs_to_krsc(w, DEV), torch.from_numpy(b).to(DEV)
        descs.append(dict(x=xd, w=wd, b=bd, N=N, C=C, H=H, W=W, K=K, R=R, S=R, stride=stride, pad=pad, relu=relu,
                          x_ch_stride=wide_c, x_ch_offset=xo))
        outs.append((P, Q, K, off))
        off += K
    for tile in range(-1, gpulet.CONV_TILES):
        if same_size:       # slices of one concatenated tensor
            cat = torch.full((N, outs[0][0], outs[0][1], total), -512.0, dtype=torch.bfloat16, device=DEV)
            ys = [cat] * len(members)
            for d, (P, Q, K, o) in zip(descs, outs):
                d.update(y=cat, y_ch_stride=total, y_ch_offset=o)
        else:
            ys = [torch.full((N, P, Q, K), -512.0, dtype=torch.bfloat16, device=DEV) for (P, Q, K, o) in outs]
            for d, y in zip(descs, ys):
                d.update(y=y, y_ch_stride=0, y_ch_offset=0)
        torch.cuda.synchronize()
        gpulet.set_conv_tile(tile)
        try:
            gpulet.conv2d_group_fwd(descs, part.stream)
            part.sync()
        finally:
            gpulet.set_conv_tile(-1)
        for j, (P, Q, K, o) in enumerate(outs):
            got = ys[j][..., o:o + K] if same_size else ys[j]
            assert torch.equal(got, alone[j]), (tile, j)                 # the bits of the member's own launch
            assert_close(lowering.nhwc_to_nchw(got), refs[j], mags[j], what=(tile, j))
        if same_size:
            assert bool((cat[..., :8] == -512.0).all())


# N, H, W, K: 3x3, stride 1, pad 1, exactly 64 input channels -> weights resident in registers (tile 10)
C64_CASES = [
    (3, 14, 14, 64),        # whole rows per block; M = 588: ragged last tile, fewer tiles than workgroups
    (2, 56, 56, 64),        # 14-pixel column blocks
    (1, 32, 32, 32),        # 16-pixel blocks; one filter half empty
    (2, 20, 20, 40),        # ragged second column block, ragged filter tile
    (2, 9, 33, 136),        # odd sizes, three filter tiles (last one 8 wide)
    (1, 5, 3, 8),           # smaller than one tile
    (16, 56, 56, 128),      # several tiles per workgroup, two filter tiles
    (9, 7, 7, 72),          # a tile spans three images
]


@pytest.mark.parametrize("case", C64_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv_3x3_c64_resident_weights_kernel_parity(part, case):
    N, H, W, K = case
    x, w, b = conv_tensors(21, N, 64, H, W, K, 3)
    got, raw = gpu_conv(part, x, w, b, 1, 1, True, tile=10)
    assert_conv_close(got, x, w, b, 1, 1, True)
    _, gathered = gpu_conv(part, x, w, b, 1, 1, True, tile=1)
    assert torch.equal(raw, gathered)          # same summation order as the gathering kernel
    _, again = gpu_conv(part, x, w, b, 1, 1, True, tile=10)
    assert torch.equal(raw, again)
    got, _ = gpu_conv(part, x, w, None, 1, 1, False, ch_total=K + 24, ch_offset=16, tile=10)
    assert_conv_close(got[:, 16:16 + K], x, w, None, 1, 1, False)
    assert np.all(got[:, :16] == -512.0) and np.all(got[:, 16 + K:] == -512.0)


# N, C, H, W, K, stride: 1x1 filters with at most 128 input channels -> the streaming kernel (tile 8)
STREAM_CASES = [
    (1, 64, 5, 5, 24, 1),          # a single ragged tile
    (2, 64, 19, 17, 136, 1),       # M = 646: eleven tiles, last one ragged; two channel tiles, second ragged
    (3, 128, 16, 16, 64, 1),       # two depth slices
    (2, 128, 21, 21, 264, 2),      # strided 1x1 (projection shortcut), three channel tiles
    (8, 64, 56, 56, 256, 1),       # many tiles per workgroup
    (4, 128, 28, 28, 512, 1),
    (3, 32, 30, 30, 64, 1),        # half a depth slice (MobileNet's first pointwise layer)
    (2, 96, 13, 13, 40, 1),        # one and a half slices
    (2, 8, 9, 9, 16, 1),           # a single 16-byte chunk of depth
]


@pytest.mark.parametrize("case", STREAM_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv_streaming_1x1_kernel_parity(part, case):
    N, C, H, W, K, stride = case
    x, w, b = conv_tensors(18, N, C, H, W, K, 1)
    P, Q = (H - 1) // stride + 1, (W - 1) // stride + 1
    res = inputs.tensor(18, "res_stream", (N, K, P, Q), "normal")
    got, raw = gpu_conv(part, x, w, b, stride, 0, True, residual=res, tile=8)
    assert_conv_close(got, x, w, b, stride, 0, True, residual=res)
    _, one_tile_each = gpu_conv(part, x, w, b, stride, 0, True, residual=res, tile=2)
    assert torch.equal(raw, one_tile_each)      # same depth order as the other kernels
    _, again = gpu_conv(part, x, w, b, stride, 0, True, residual=res, tile=8)
    assert torch.equal(raw, again)
    got, _ = gpu_conv(part, x, w, None, stride, 0, False, ch_total=K + 24, ch_offset=16, tile=8)
    assert_conv_close(got[:, 16:16 + K], x, w, None, stride, 0, False)
    assert np.all(got[:, :16] == -512.0) and np.all(got[:, 16 + K:] == -512.0)


# N, C, H, W, K, R, stride, pad: at most four input channels -> the stem kernel (tile 9)
STEM_CASES = [
    (2, 3, 64, 64, 64, 7, 2, 3),       # ImageNet stem: P = Q = 32, one column tile
    (2, 3, 33, 31, 64, 7, 2, 3),       # odd image, ragged row and column tiles
    (3, 3, 40, 70, 64, 3, 1, 1),       # VGG's first layer: three column tiles, last one ragged
    (2, 3, 41, 45, 32, 3, 2, 1),       # MobileNet's first layer: one 32-filter tile
    (2, 1, 28, 28, 6, 5, 1, 2),        # LeNet conv1: one plane, six filters (scalar stores)
    (1, 4, 20, 20, 72, 5, 1, 0),       # four channels, two filter tiles, second ragged; no padding
    (5, 2, 9, 130, 40, 7, 1, 3),       # wide and flat: five column tiles
    (1, 3, 5, 5, 8, 3, 1, 1),          # smaller than one tile
]


@pytest.mark.parametrize("case", STEM_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv_stem_kernel_parity(part, case):
    N, C, H, W, K, R, stride, pad = case
    x, w, b = conv_tensors(19, N, C, H, W, K, R)
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    got, raw = gpu_conv(part, x, w, b, stride, pad, True, tile=9)
    assert_conv_close(got, x, w, b, stride, pad, True)
    _, auto = gpu_conv(part, x, w, b, stride, pad, True)
    assert torch.equal(raw, auto)               # chosen automatically wherever it applies
    got1, _ = gpu_conv(part, x[:1], w, b, stride, pad, True)
    assert np.array_equal(got1, got[:1])        # an image's bits do not depend on the batch
    got, _ = gpu_conv(part, x, w, None, stride, pad, False, tile=9)    # no bias, no ReLU
    assert_conv_close(got, x, w, None, stride, pad, False)
    # with a residual operand the layer stays with the gathering kernel
    res = inputs.tensor(19, "res_stem", (N, K, P, Q), "normal")
    got, raw = gpu_conv(part, x, w, b, stride, pad, True, residual=res, tile=9)
    assert_conv_close(got, x, w, b, stride, pad, True, residual=res)
    _, gathered = gpu_conv(part, x, w, b, stride, pad, True, residual=res, tile=1)
    assert torch.equal(raw, gathered)
    ct = K + 24
    got, _ = gpu_conv(part, x, w, None, stride, pad, False, ch_total=ct, ch_offset=16, tile=9)
    assert_conv_close(got[:, 16:16 + K], x, w, None, stride, pad, False)
    assert np.all(got[:, :16] == -512.0) and np.all(got[:, 16 + K:] == -512.0)


def test_conv_stem_kernel_keeps_a_non_finite_pixel_inside_its_windows(part):
    # the kernel pads filter rows to 8 pixels with zero weights: a neighbour outside the 7-wide
    # window must not leak in as 0 * inf
    N, C, H, W, K, R, stride, pad = 1, 3, 40, 40, 64, 7, 2, 3
    x, w, b = conv_tensors(20, N, C, H, W, K, R)
    x = x.copy()
    x[0, 1, 17, 22] = np.inf
    ref = oracle.conv2d(x, w, b, stride, pad, False)
    got, _ = gpu_conv(part, x, w, b, stride, pad, False, tile=9)
    touched = ~np.isfinite(ref)
    assert touched.any() and not touched.all()
    assert np.array_equal(~np.isfinite(got), touched)
    assert np.array_equal(np.sign(got[touched]), np.sign(ref[touched]))
    clean = np.where(touched, 0.0, got), np.where(touched, 0.0, ref)
    assert oracle.rel_err(*clean)[0] <= LAYER_TOL


@pytest.mark.parametrize("case", [(32, 256, 14, 14, 256, 3, 1, 1), (2, 512, 7, 7, 512, 3, 1, 1),
                                  (4, 1024, 14, 14, 256, 1, 1, 0), (3, 512, 7, 7, 2048, 1, 1, 0),
                                  (1, 64, 9, 9, 40, 5, 1, 2)], ids=lambda c: "x".join(map(str, c)))
def test_conv_split_depth_parity_and_reproducibility(part, case):
    # few output tiles and a long depth: the launcher may let several workgroups share a tile
    N, C, H, W, K, R, stride, pad = case
    x, w, b = conv_tensors(16, N, C, H, W, K, R)
    res = inputs.tensor(16, "res_split", (N, K, (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1), "normal")
    ref = oracle.conv2d(x, w, b, stride, pad, True, residual=res)
    mag = conv_mag(x, w, b, stride, pad, residual=res)
    runs = []
    for max_split in (4, 4, 8, 1):
        gpulet.set_conv_split_k(max_split)
        try:
            got, raw = gpu_conv(part, x, w, b, stride, pad, True, residual=res)
        finally:
            gpulet.set_conv_split_k(1)
        assert_close(got, ref, mag, what=max_split)
        runs.append(raw.clone())
    assert torch.equal(runs[0], runs[1])       # same split, same bits, whoever arrives last
    diff = (runs[0].float() - runs[3].float()).abs().max().item()
    assert diff <= 2.0 ** -6 * max(1.0, runs[3].float().abs().max().item())


def test_conv_is_deterministic(part):
    x, w, b = conv_tensors(12, 4, 64, 28, 28, 96, 3)
    _, r0 = gpu_conv(part, x, w, b, 1, 1, True)
    for _ in range(3):
        _, r = gpu_conv(part, x, w, b, 1, 1, True)
        assert torch.equal(r, r0)


def test_conv_no_bias_no_relu_and_zero_input(part):
    x, w, b = conv_tensors(13, 2, 16, 8, 8, 32, 3)
    got, _ = gpu_conv(part, x, w, None, 1, 1, False)
    assert_conv_close(got, x, w, None, 1, 1, False)
    assert (got < 0).any()
    got, _ = gpu_conv(part, np.zeros_like(x), w, b, 1, 1, False)
    want = inputs.bf16_round(b)[None, :, None, None] * np.ones_like(got)
    assert np.array_equal(got, want)


def test_conv_delta_kernel_copies_input_exactly(part):
    C = 16
    x = inputs.tensor(14, "delta", (2, C, 9, 9), "normal")
    w = np.zeros((C, C, 3, 3), dtype=np.float32)
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    got, _ = gpu_conv(part, x, w, None, 1, 1, False)
    assert np.array_equal(got, x.astype(np.float64))


@pytest.mark.parametrize("tile", [-1, 0, 3, 4, 6, 7])
def test_conv_residual_and_channel_slice(part, tile):
    N, C, H, W, K, R = 2, 32, 10, 10, 40, 3
    x, w, b = conv_tensors(15, N, C, H, W, K, R)
    res = inputs.tensor(15, "res", (N, K, H, W), "normal")
    ref = oracle.conv2d(x, w, b, 1, 1, True, residual=res)
    mag = conv_mag(x, w, b, 1, 1, residual=res)
    got, _ = gpu_conv(part, x, w, b, 1, 1, True, residual=res, tile=tile)
    assert_close(got, ref, mag)
    # store into channels 24..63 of an 72-channel tensor; the rest stays untouched
    got, raw = gpu_conv(part, x, w, b, 1, 1, True, residual=res, ch_total=72, ch_offset=24, tile=tile)
    assert_close(got[:, 24:64], ref, mag)
    assert np.all(got[:, :24] == -512.0) and np.all(got[:, 64:] == -512.0)


# N, C, H, W, k, stride, pad
DW_CASES = [
    (2, 32, 19, 19, 3, 1, 1),       # Q = 19: ragged group of four pixels per thread
    (2, 64, 20, 20, 3, 2, 1),       # MobileNet's stride-2 blocks
    (1, 8, 5, 7, 3, 1, 1),
    (3, 24, 9, 9, 3, 2, 0),
    (1, 16, 11, 11, 5, 1, 2),
    (2, 40, 6, 6, 5, 2, 2),
    (2, 12, 7, 7, 3, 1, 1),         # C not a multiple of 8: scalar path
    (1, 3, 10, 10, 3, 2, 1),
    (1, 512, 10, 10, 3, 1, 1),
    (2, 16, 4, 4, 1, 1, 0),         # 1x1 depthwise = per-channel scale
    (2, 64, 21, 23, 3, 2, 1),       # stride 2, odd sizes: Q = 12, P = 11
    (3, 24, 9, 10, 3, 2, 1),        # stride 2, Q = 5: ragged pair of pixels per thread
    (1, 128, 38, 38, 3, 1, 1),
    (2, 8, 3, 3, 3, 1, 1),          # every window touches the padding
]


@pytest.mark.parametrize("case", DW_CASES, ids=lambda c: "x".join(map(str, c)))
def test_depthwise_conv_parity(part, case):
    N, C, H, W, k, stride, pad = case
    x = inputs.tensor(21, "dw/x", (N, C, H, W), "normal")
    w = inputs.he_normal(21, "dw/w", (C, 1, k, k))
    b = inputs.bias(21, "dw/b", C)
    P, Q = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    xd = lowering.nchw_to_nhwc(x, DEV)
    wd = lowering.to_device_bf16(np.transpose(w[:, 0], (1, 2, 0)), DEV)
    bd = torch.from_numpy(b).to(DEV)
    for relu, bias in ((True, bd), (False, None)):
        yd = torch.full((N, P, Q, C), -512.0, dtype=torch.bfloat16, device=DEV)
        torch.cuda.synchronize()
        gpulet.depthwise_conv2d_fwd(xd, wd, bias, yd, N, C, H, W, k, k, stride, pad, relu, part.stream)
        part.sync()
        got = lowering.nhwc_to_nchw(yd)
        ref = oracle.depthwise_conv2d(x, w, b if bias is not None else None, stride, pad, relu)
        mag = oracle.depthwise_conv2d(np.abs(x), np.abs(w), np.abs(b) if bias is not None else None, stride, pad, False)
        assert_close(got, ref, mag)
        assert not np.any(got == -512.0)


def test_depthwise_argument_errors(part):
    t = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    for bad in [dict(N=0), dict(C=0), dict(k=0), dict(stride=0), dict(pad=-1), dict(H=2, k=5)]:
        a = dict(N=1, C=8, H=4, W=4, k=3, stride=1, pad=1)
        a.update(bad)
        with pytest.raises(gpulet.GpuletError):
            gpulet.depthwise_conv2d_fwd(t, t, None, t, a["N"], a["C"], a["H"], a["W"], a["k"], a["k"], a["stride"],
                                        a["pad"], True, part.stream)
    with pytest.raises(gpulet.GpuletError):
        gpulet.depthwise_conv2d_fwd(None, t, None, t, 1, 8, 4, 4, 3, 3, 1, 1, True, part.stream)


# N, C, H, W, mode, k, stride, pad
POOL_CASES = [
    (2, 6, 28, 28, gpulet.POOL_MAX, 2, 2, 0), (2, 16, 10, 10, gpulet.POOL_MAX, 2, 2, 0),
    (2, 64, 17, 15, gpulet.POOL_MAX, 3, 2, 1), (1, 24, 9, 9, gpulet.POOL_MAX, 3, 1, 1),
    (3, 5, 7, 7, gpulet.POOL_MAX, 3, 2, 1), (2, 40, 8, 8, gpulet.POOL_AVG, 2, 2, 0),
    (2, 7, 9, 9, gpulet.POOL_AVG, 3, 2, 1), (4, 2048, 7, 7, gpulet.POOL_GLOBAL_AVG, 1, 1, 0),
    (3, 1000, 5, 3, gpulet.POOL_GLOBAL_AVG, 1, 1, 0), (2, 13, 6, 6, gpulet.POOL_GLOBAL_AVG, 1, 1, 0),
    (1, 8, 1, 1, gpulet.POOL_GLOBAL_AVG, 1, 1, 0), (1, 1024, 7, 7, gpulet.POOL_GLOBAL_AVG, 1, 1, 0),
    (2, 8, 5, 7, gpulet.POOL_MAX, 3, 1, 1), (1, 64, 12, 12, gpulet.POOL_MAX, 3, 2, 1),
    (2, 40, 7, 9, gpulet.POOL_MAX, 2, 2, 0), (1, 8, 3, 3, gpulet.POOL_MAX, 3, 2, 1),
    (2, 16, 6, 6, gpulet.POOL_MAX, 3, 3, 1), (1, 8, 2, 2, gpulet.POOL_MAX, 3, 1, 2),
    (1, 16, 1, 1, gpulet.POOL_MAX, 3, 1, 1), (2, 48, 9, 4, gpulet.POOL_MAX, 2, 1, 1),
    (1, 16, 9, 9, gpulet.POOL_MAX, 5, 2, 2),
]


@pytest.mark.parametrize("case", POOL_CASES, ids=lambda c: "x".join(map(str, c)))
def test_pool_parity(part, case):
    N, C, H, W, mode, k, stride, pad = case
    x = inputs.tensor(21, "pool%d_%d_%d" % (C, H, mode), (N, C, H, W), "normal")
    if mode == gpulet.POOL_GLOBAL_AVG:
        ref = oracle.global_avgpool(x).reshape(N, C, 1, 1)
    elif mode == gpulet.POOL_MAX:
        ref = oracle.maxpool(x, k, stride, pad)
    else:
        ref = oracle.avgpool(x, k, stride, pad)
    P, Q = ref.shape[2:]
    xd = lowering.nchw_to_nhwc(x, DEV)
    yd = torch.full((N, P, Q, C), -512.0, dtype=torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    gpulet.pool(xd, yd, N, C, H, W, mode, k, stride, pad, part.stream)
    part.sync()
    got = lowering.nhwc_to_nchw(yd)
    if mode == gpulet.POOL_MAX:
        assert np.array_equal(got, ref)            # a max of bf16 values is exact
    else:
        assert np.max(np.abs(got - ref)) <= 2.0 ** -8 * np.max(np.abs(ref)) + 1e-30
        assert oracle.rel_err(got, ref)[1] <= LAYER_TOL


# N, C, H, W, K, destination channels (0: K), first channel written
POOLED_CONV_CASES = [
    (2, 128, 56, 56, 128, 0, 0),      # VGG conv2_2-like: 8 x 28 tiles, two per row
    (3, 64, 28, 28, 192, 0, 0),       # one channel block, ragged filter tile, tile rows 8+8+8+4
    (1, 256, 14, 14, 256, 0, 0),      # whole map in one tile
    (2, 128, 12, 20, 64, 0, 0),       # 10 x 20 + 2 x 20 tiles, half a filter tile
    (2, 192, 6, 34, 136, 0, 0),       # one 6 x 34 tile per image, K a multiple of 8 only (second filter tile: 8 filters)
    (1, 128, 10, 58, 64, 0, 0),       # column tiles of 20, 20 and 18 pixels
    (1, 64, 2, 2, 8, 0, 0),           # one window
    # 64 input channels and column blocks of a power of two: the resident-weight kernel's pooled epilogue
    (2, 64, 32, 32, 64, 0, 0),        # 8 x 16 tiles, two column blocks
    (1, 64, 64, 48, 128, 0, 0),       # two filter tiles, three column blocks
    (3, 64, 8, 8, 72, 0, 0),          # 8-pixel rows: tiles span two images; ragged filter tile
    (2, 64, 10, 58, 64, 96, 32),      # ragged last column block, rows of two images in one tile, channel slice
    (2, 128, 16, 16, 72, 200, 64),    # stored as a channel slice of wider pixels
]


@pytest.mark.parametrize("case", POOLED_CONV_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv3x3_maxpool2_fused_parity(part, case):
    N, C, H, W, K, ct, co = case
    x, w, b = conv_tensors(23, N, C, H, W, K, 3)
    full = oracle.conv2d(x, w, b, 1, 1, relu=True)
    ref = oracle.maxpool(full, 2, 2, 0)
    mag = oracle.maxpool(conv_mag(x, w, b, 1, 1), 2, 2, 0)       # the largest bound of a window covers its maximum
    xd, wd = lowering.nchw_to_nhwc(x, DEV), lowering.kcrs_to_krsc(w, DEV)
    bd = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(DEV)
    ctot = ct if ct else K
    yd = torch.full((N, H // 2, W // 2, ctot), -512.0, dtype=torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    gpulet.conv3x3_maxpool2_fwd(xd, wd, bd, yd, N, C, H, W, K, ct, co, part.stream)
    part.sync()
    got = lowering.nhwc_to_nchw(yd[..., co:co + K])
    assert_close(got, ref, mag, what=case)
    if ct:                                                        # channels outside the slice are untouched
        rest = torch.cat([yd[..., :co], yd[..., co + K:]], dim=-1)
        assert bool((rest == -512.0).all())
    # the same bits as the layer followed by the pool kernel, whatever tile runs the layer
    for tile in (-1, 11, 1):
        _, raw = gpu_conv(part, x, w, b, 1, 1, True, tile=tile)
        pd = torch.empty((N, H // 2, W // 2, K), dtype=torch.bfloat16, device=DEV)
        gpulet.pool(raw, pd, N, K, H, W, gpulet.POOL_MAX, 2, 2, 0, part.stream)
        part.sync()
        assert torch.equal(pd, yd[..., co:co + K]), tile


def test_conv3x3_maxpool2_argument_errors(part):
    def call(N, C, H, W, K, ct=0, co=0, shift=0):
        x = torch.zeros(N * H * W * C + 8, dtype=torch.bfloat16, device=DEV)[shift:]
        w = torch.zeros(K * 9 * C, dtype=torch.bfloat16, device=DEV)
        b = torch.zeros(K, device=DEV)
        y = torch.zeros(N * (H // 2) * (W // 2) * (ct if ct else K) + 8, dtype=torch.bfloat16, device=DEV)
        return gpulet.lib.gpulet_conv3x3_maxpool2_fwd(gpulet.ptr(x), gpulet.ptr(w), gpulet.ptr(b), gpulet.ptr(y), N, C, H, W,
                                                      K, ct, co, part.stream)
    assert call(1, 64, 8, 8, 64) == gpulet.OK
    assert call(1, 64, 7, 8, 64) == gpulet.EINVAL        # odd height: windows would hang over the edge
    assert call(1, 64, 8, 9, 64) == gpulet.EINVAL
    assert call(1, 96, 8, 8, 64) == gpulet.EINVAL        # not whole 64-channel blocks
    assert call(1, 64, 8, 8, 60) == gpulet.EINVAL        # 16-byte stores need K % 8 == 0
    assert call(1, 64, 8, 8, 64, 100, 0) == gpulet.EINVAL
    assert call(1, 64, 8, 8, 64, 128, 4) == gpulet.EINVAL
    assert call(1, 64, 8, 8, 64, 96, 40) == gpulet.EINVAL  # slice past the pixel
    assert call(1, 64, 8, 8, 64, shift=4) == gpulet.EINVAL # misaligned x
    part.sync()


def test_conv_timeline_records_ordered_stamps_for_the_patch_and_tall_kernels(part):
    def run(N, C, H, W, K, R, pad, tile):
        x = torch.zeros((N, H, W, C), dtype=torch.bfloat16, device=DEV)
        w = torch.zeros((K, R, R, C), dtype=torch.bfloat16, device=DEV)
        b = torch.zeros(K, device=DEV)
        y = torch.full((N, H, W, K), 3.0, dtype=torch.bfloat16, device=DEV)
        torch.cuda.synchronize()
        gpulet.set_conv_tile(tile)
        try:
            rows = gpulet.conv2d_timeline(x, w, b, y, N, C, H, W, K, R, R, 1, pad, True, stream=part.stream, warmup=3)
        finally:
            gpulet.set_conv_tile(-1)
        assert bool((y == 0).all())                 # the stamped launch is a full launch of the layer
        return rows
    for tile, shape in ((7, (32, 256, 14, 14, 256, 3, 1)), (11, (4, 128, 56, 56, 128, 3, 1))):
        rows = run(*shape, tile)
        assert len(rows) == 8, tile
        for r in rows:
            assert r[7] == 0 and all(0 < a <= b for a, b in zip(r[:6], r[1:7])), (tile, r)   # points in program order
            assert r[6] - r[0] < 20000, (tile, r)                                        # within 200 us (10 ns units)
        starts = [r[0] for r in rows]
        assert max(starts) - min(starts) < 1000          # the first workgroups of a launch start within 10 us of one another
    rows = run(16, 64, 112, 112, 64, 3, 1, 10)            # weights in registers: six pixel tiles per workgroup at least
    assert len(rows) == 8
    for r in rows:
        assert all(0 < a <= b for a, b in zip(r[:6], r[1:7])) and r[2] < r[7] < r[2] + 2000, r
    assert run(2, 64, 8, 8, 64, 1, 0, -1) == []           # a 1x1 layer runs a kernel that records nothing


# N, In, Out
FC_CASES = [(32, 400, 120), (32, 120, 84), (32, 84, 10), (1, 2048, 1000), (8, 1024, 1000),
            (33, 72, 17), (5, 8, 3), (40, 4096, 1000), (16, 25088, 64), (2, 100, 7),
            # long rows: 64 outputs per workgroup, depth split over workgroups
            (32, 25088, 136), (1, 25088, 256), (17, 8192, 4096), (3, 8195, 20), (40, 9000, 72)]


@pytest.mark.parametrize("case", FC_CASES, ids=lambda c: "x".join(map(str, c)))
@pytest.mark.parametrize("out_fp32", [False, True])
def test_fc_parity(part, case, out_fp32):
    N, In, Out = case
    x = inputs.tensor(31, "fcx%d_%d" % (N, In), (N, In), "normal")
    w = inputs.he_normal(31, "fcw%d_%d" % (In, Out), (Out, In))
    b = inputs.bias(31, "fcb%d" % Out, Out)
    relu = not out_fp32
    ref = oracle.fc(x, w, b, relu)
    xd, wd = lowering.to_device_bf16(x, DEV), lowering.to_device_bf16(w, DEV)
    bd = torch.from_numpy(b).to(DEV)
    yd = torch.full((N, Out), -512.0, dtype=torch.float32 if out_fp32 else torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    gpulet.fc(xd, wd, bd, yd, N, In, Out, relu, out_fp32, part.stream)
    part.sync()
    got = yd.to(torch.float32).cpu().numpy().astype(np.float64)
    mag = oracle.fc(np.abs(x), np.abs(w), np.abs(b), False)
    # fp32 output: accumulation error only (half a unit in the last place of an fp32 is 2^-24)
    assert_close(got, ref, mag, tol=1e-5 if out_fp32 else LAYER_TOL, rel=2.0 ** -24 if out_fp32 else 2.0 ** -8)


def test_full_size_vgg_fc6(part):
    # FC 25088 -> 4096 at batch 16: the weight-streaming case
    N, In, Out = 16, 25088, 4096
    x = inputs.tensor(32, "fc6x", (N, In), "uniform")
    w = inputs.he_normal(32, "fc6w", (Out, In))
    b = inputs.bias(32, "fc6b", Out)
    ref = oracle.fc(x, w, b, True)
    xd, wd, bd = lowering.to_device_bf16(x, DEV), lowering.to_device_bf16(w, DEV), torch.from_numpy(b).to(DEV)
    yd = torch.empty((N, Out), dtype=torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    gpulet.fc(xd, wd, bd, yd, N, In, Out, True, False, part.stream)
    part.sync()
    assert_close(yd.to(torch.float32).cpu().numpy().astype(np.float64), ref, oracle.fc(np.abs(x), np.abs(w), np.abs(b), False))


def test_long_row_fc_is_reproducible_and_batch_independent(part):
    # partial tiles of an output group meet in scratch and are added in split order by whichever
    # workgroup arrives last: same bits every time, and the same bits for an image in any batch
    N, In, Out = 32, 25088, 200
    x = inputs.tensor(33, "fcsx", (N, In), "uniform")
    w = inputs.he_normal(33, "fcsw", (Out, In))
    b = inputs.bias(33, "fcsb", Out)
    xd, wd, bd = lowering.to_device_bf16(x, DEV), lowering.to_device_bf16(w, DEV), torch.from_numpy(b).to(DEV)
    runs = []
    for n in (N, N, 16, 1):
        yd = torch.full((n, Out), -512.0, dtype=torch.float32, device=DEV)
        torch.cuda.synchronize()
        gpulet.fc(xd, wd, bd, yd, n, In, Out, False, True, part.stream)
        part.sync()
        runs.append(yd.clone())
    assert torch.equal(runs[0], runs[1])
    assert torch.equal(runs[0][:16], runs[2]) and torch.equal(runs[0][:1], runs[3])
    assert oracle.rel_err(runs[0].cpu().numpy().astype(np.float64), oracle.fc(x, w, b, False))[1] <= 1e-4


def _random_conv_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        kind = rng.integers(0, 5)
        N = int(rng.integers(1, 5))
        H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
        if kind == 0:       # stem-like: few channels
            C, R = int(rng.integers(1, 5)), int(rng.choice([3, 5, 7]))
            K, stride, pad = int(rng.choice([8, 16, 24, 32, 40, 64, 72])), int(rng.integers(1, 3)), int(rng.integers(0, R // 2 + 2))
        elif kind == 1:     # 3x3 over exactly 64 channels
            C, R, stride, pad = 64, 3, 1, 1
            K = int(rng.choice([8, 24, 64, 72, 136]))
        elif kind == 2:     # 1x1 with a short depth
            C, R, stride, pad = int(rng.choice([8, 16, 32, 64, 96, 128])), 1, int(rng.integers(1, 3)), 0
            K = int(rng.choice([8, 20, 64, 100, 136, 264]))
        elif kind == 3:     # 3x3 over multiples of 64 channels (patch kernel)
            C, R, stride, pad = int(rng.choice([64, 128, 192])), 3, 1, 1
            K = int(rng.choice([16, 64, 72]))
        else:               # anything
            C, R = int(rng.integers(1, 80)), int(rng.choice([1, 2, 3, 5]))
            K, stride, pad = int(rng.integers(1, 90)), int(rng.integers(1, 4)), int(rng.integers(0, 3))
        if H + 2 * pad < R or W + 2 * pad < R:
            continue
        cases.append((N, C, H, W, K, R, stride, pad))
    return cases


@pytest.mark.parametrize("case", _random_conv_cases(40, 2024), ids=lambda c: "x".join(map(str, c)))
def test_conv_random_shapes_through_every_kernel_family(part, case):
    # seeded random shapes: automatic selection and every special-purpose kernel forced (a forced
    # kernel that does not apply to a shape falls back to a gathering tile inside the library)
    N, C, H, W, K, R, stride, pad = case
    x, w, b = conv_tensors(29, N, C, H, W, K, R)
    relu = bool((N + K) % 2)
    ref = oracle.conv2d(x, w, b, stride, pad, relu)
    mag = conv_mag(x, w, b, stride, pad)
    for tile in (-1, 7, 8, 9, 10, 11, 3):
        got, _ = gpu_conv(part, x, w, b, stride, pad, relu, tile=tile)
        assert_close(got, ref, mag, what=tile)
