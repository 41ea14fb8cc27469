"""Forward pass captured as a HIP graph on a gpu-let: same results as the eager
path on every replay, request counters exact, and the CU mask still honoured."""

import numpy as np
import pytest
import torch

import oracle
from paper_2109_01611_amd import gpulet, lowering, workloads

from gpu_util import DEV, MODEL_TOL
from test_gpu_partition import _placement

pytestmark = pytest.mark.gpu


def test_graph_replays_stay_inside_the_cu_mask():
    with gpulet.Partition(0, 40, 0) as a, gpulet.Partition(0, 60, 1) as b:
        eager_a, eager_b = _placement(a), _placement(b)
        for part, eager in ((a, eager_a), (b, eager_b)):
            out = torch.zeros(2 * 8192, dtype=torch.int32, device=DEV)
            torch.cuda.synchronize()
            part.probe(out, 8192, via_graph=True)
            o = out.cpu().numpy().astype(np.uint32).reshape(8192, 2)
            placed = set(zip((o[:, 0] & 0xF).tolist(), ((o[:, 1] >> 8) & 0xFF).tolist()))
            assert placed <= eager and len(placed) == part.n_cu
        assert not (eager_a & eager_b)


@pytest.mark.parametrize("model,batch", [(workloads.lenet5(), 5),
                                         (workloads.resnet50(width_div=4, in_hw=64, n_class=20, blocks=(1, 2, 1, 1)), 3),
                                         (workloads.googlenet(width_div=4, in_hw=64, n_class=20, n_blocks=2), 2)],
                         ids=lambda v: getattr(v, "name", str(v)))
def test_graph_matches_eager_on_every_replay(model, batch):
    params = workloads.parameters(model, 9)
    x = workloads.batch_input(model, batch, 9)
    dm = lowering.DeviceModel(model, params, DEV)
    other = lowering.DeviceModel(workloads.lenet5(), workloads.parameters(workloads.lenet5(), 1), DEV)
    xo = other.input_to_device(workloads.batch_input(workloads.lenet5(), 4, 1))
    with gpulet.Partition(0, 50, 1) as p:
        xd = dm.input_to_device(x)
        y_eager, _ = dm.run(p, xd)
        ref = y_eager.clone()
        ws, n = dm.workspace(batch)
        y = dm.alloc_output(batch)
        torch.cuda.synchronize()
        with gpulet.ModelGraph(dm.desc, batch, p, xd, y, ws, n) as g:
            before = p.counters()
            for i in range(4):
                y.fill_(-1.0)
                torch.cuda.synchronize()
                ms = g.launch(timed=(i % 2 == 0))
                p.sync()
                assert ms is None or ms > 0
                assert torch.equal(y, ref), i
                other.run(p, xo)                 # eager work between the replays
                torch.cuda.synchronize()
            lat, total = g.profile(2, 5)
            assert len(lat) == 5 and min(lat) > 0 and total >= sum(lat) * 0.5
            assert torch.equal(y, ref)
            after = p.counters()
            # 4 replays + 4 eager LeNet batches of 4 + 7 profiled replays
            assert after[0] - before[0] == 4 + 4 + 7
            assert after[1] - before[1] == (4 + 7) * batch + 4 * 4
        assert gpulet.lib.gpulet_model_graph_destroy(None) == gpulet.EINVAL
    got = ref.to(torch.float32).cpu().numpy().astype(np.float64).reshape(batch, -1)
    want = oracle.run_model(model, params, x).reshape(batch, -1)
    whole, per_img = oracle.rel_err(got, want)
    assert max(whole, per_img) <= MODEL_TOL


def test_graph_with_pools_in_the_convolutions_epilogue_matches_the_two_kernel_path():
    # A captured forward pass whose convolution + max pool pairs run as one launch gives, on every
    # replay, the bits of the eager pass that runs them as two kernels.
    model = workloads.vgg16(width_div=2, in_hw=224, n_class=20)
    batch = 32
    params = workloads.parameters(model, 3)
    dm = lowering.DeviceModel(model, params, DEV)
    with gpulet.Partition(0, 100, 0) as p:
        xd = dm.input_to_device(workloads.batch_input(model, batch, 3))
        try:
            gpulet.set_conv_pool_fusion(False)
            ref, _ = dm.run(p, xd)
            ref = ref.clone()
            n_plain = p.kernel_launches()
        finally:
            gpulet.set_conv_pool_fusion(True)
        y_eager, _ = dm.run(p, xd)
        n_fused = p.kernel_launches() - n_plain
        assert n_plain == dm.desc.n_layers and n_fused < n_plain      # some pairs do share a launch at this size
        assert torch.equal(y_eager, ref)
        ws, n = dm.workspace(batch)
        y = dm.alloc_output(batch)
        torch.cuda.synchronize()
        with gpulet.ModelGraph(dm.desc, batch, p, xd, y, ws, n) as g:
            for i in range(3):
                y.fill_(-1.0)
                torch.cuda.synchronize()
                g.launch()
                p.sync()
                assert torch.equal(y, ref), i
                dm.run(p, xd)                    # eager work between the replays
                torch.cuda.synchronize()
