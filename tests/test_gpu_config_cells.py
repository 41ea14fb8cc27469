"""Every (model, batch, gpu-let size) cell of the evaluated configurations against
the fp64 oracle: the kernel chosen for a layer depends on the batch and on the
gpu-let's CU count, so each cell runs tiles that no other cell runs.

  * LeNet-5 shape, batch 32, 100 %
  * the single 3x3 layer (N=32, C=K=256, 14x14) on 20/40/50/60/80/100 %
  * ResNet-50 shape, batch 1/8/32 on 25/50/100 %
  * VGG-16 shape, batch 16 on 50/100 %
  * ResNet-50 shape batch 16 on a 50 % gpu-let next to the GoogLeNet shape batch 32 on the
    complementary 50 % gpu-let, both at full size, outputs checked after the co-run window

Whole models are compared on sampled images of the batch (images are independent; the oracle
needs about a second per image) within 1e-2 normwise; the single layer also element by element.
Oracle results are kept per (model, image) because image i of a seeded batch is the same in
every batch size.
"""

import numpy as np
import pytest
import torch

import oracle
from paper_2109_01611_amd import gpulet, lowering, workloads

from gpu_util import DEV, LAYER_TOL, MODEL_TOL, assert_close, conv_mag, conv_tensors, gpu_conv

pytestmark = pytest.mark.gpu

_models, _refs = {}, {}


def _device_model(name):
    if name not in _models:
        model = getattr(workloads, name)()
        params = workloads.parameters(model, 0)
        _models[name] = (model, params, lowering.DeviceModel(model, params, DEV))
    return _models[name]


def _oracle_logits(name, x, image):
    """The oracle's output for image `image` of the seeded batch (cached)."""
    if (name, image) not in _refs:
        model, params, _ = _device_model(name)
        _refs[(name, image)] = oracle.run_model(model, params, x[image:image + 1]).reshape(-1)
    return _refs[(name, image)]


def _sampled(batch):
    return sorted({0, batch - 1})


def _check_cell(name, batch, pct, which):
    model, params, dm = _device_model(name)
    x = workloads.batch_input(model, batch, 0)
    with gpulet.Partition(0, pct, which) as p:
        y, ms = dm.run(p, dm.input_to_device(x), timed=True)
        assert ms > 0 and p.counters() == (1, batch)
        n_cu = p.n_cu
    got = y.to(torch.float32).cpu().numpy().astype(np.float64).reshape(batch, -1)
    assert np.all(np.isfinite(got))
    worst = 0.0
    for i in _sampled(batch):
        ref = _oracle_logits(name, x, i)
        whole, _ = oracle.rel_err(got[i:i + 1], ref[None])
        worst = max(worst, whole)
        assert whole <= MODEL_TOL, (name, batch, pct, n_cu, i, whole)
    print("%s b%d on %d%% (%d CUs): %.3f ms, worst sampled image %.2e" % (name, batch, pct, n_cu, ms, worst), flush=True)
    return got


def test_lenet5_batch32_whole_gpu():
    _check_cell("lenet5", 32, 100, 0)


@pytest.mark.parametrize("pct,which", [(20, 0), (40, 1), (50, 0), (60, 1), (80, 0), (100, 0)])
def test_single_3x3_layer_on_every_gpulet_size(pct, which):
    x, w, b = conv_tensors(0, 32, 256, 14, 14, 256, 3)
    key = ("single", 0)
    if key not in _refs:
        _refs[key] = (oracle.conv2d(x, w, b, 1, 1, True), conv_mag(x, w, b, 1, 1))
    ref, mag = _refs[key]
    with gpulet.Partition(0, pct, which) as p:
        got, _ = gpu_conv(p, x, w, b, 1, 1, True)
    assert_close(got, ref, mag, tol=LAYER_TOL, what=(pct, which))


@pytest.mark.parametrize("batch", [1, 8, 32])
@pytest.mark.parametrize("pct,which", [(25, 0), (50, 1), (100, 0)])
def test_resnet50_every_batch_and_gpulet_size(batch, pct, which):
    _check_cell("resnet50", batch, pct, which)


@pytest.mark.parametrize("pct,which", [(50, 0), (100, 0)])
def test_vgg16_batch16_on_half_and_whole_gpu(pct, which):
    _check_cell("vgg16", 16, pct, which)


def test_resnet50_and_googlenet_full_size_side_by_side():
    # the co-run configuration at full size: both gpu-lets loop over their batch for the whole
    # window; what the last batch of each left in its output is compared with the oracle
    (ma, _, da), (mb, _, db) = _device_model("resnet50"), _device_model("googlenet")
    ba, bb = 16, 32
    xa, xb = workloads.batch_input(ma, ba, 0), workloads.batch_input(mb, bb, 0)
    xad, xbd = da.input_to_device(xa), db.input_to_device(xb)
    ya, yb = da.alloc_output(ba), db.alloc_output(bb)
    ya.fill_(float("nan"))
    yb.fill_(float("nan"))
    (wsa, na), (wsb, nb) = da.workspace(ba), db.workspace(bb)
    torch.cuda.synchronize()
    with gpulet.Partition(0, 50, 0) as p0, gpulet.Partition(0, 50, 1) as p1:
        la, lb = gpulet.profile_corun((da.desc, ba, p0, xad, ya, wsa, na), (db.desc, bb, p1, xbd, yb, wsb, nb),
                                      warmup=3, window_ms=300.0)
        assert len(la) >= 20 and len(lb) >= 20 and min(la) > 0 and min(lb) > 0
        # the side that was still running when the other left ran one more batch, which is not reported
        extra = [p0.counters()[0] - 3 - len(la), p1.counters()[0] - 3 - len(lb)]
        assert sorted(extra) in ([0, 0], [0, 1])
        assert p0.counters()[1] == ba * p0.counters()[0] and p1.counters()[1] == bb * p1.counters()[0]
        # the same batches alone on the same gpu-lets give the same bits
        ya_alone, _ = da.run(p0, xad)
        yb_alone, _ = db.run(p1, xbd)
    assert torch.equal(ya, ya_alone) and torch.equal(yb, yb_alone)
    for name, y, x, batch in (("resnet50", ya, xa, ba), ("googlenet", yb, xb, bb)):
        got = y.to(torch.float32).cpu().numpy().astype(np.float64).reshape(batch, -1)
        assert np.all(np.isfinite(got))
        for i in _sampled(batch):
            whole, _ = oracle.rel_err(got[i:i + 1], _oracle_logits(name, x, i)[None])
            assert whole <= MODEL_TOL, (name, i, whole)
    print("co-run: %d batches of resnet50 b16 (median %.3f ms), %d of googlenet b32 (median %.3f ms)"
          % (len(la), float(np.median(la)), len(lb), float(np.median(lb))), flush=True)
