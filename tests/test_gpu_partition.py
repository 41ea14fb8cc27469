"""gpu-let bookkeeping on the real device: masks honoured by the hardware,
Split partners disjoint, over-subscription refused, request counters exact."""

import collections

import numpy as np
import pytest
import torch

from paper_2109_01611_amd import gpulet

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _placement(part, n_blocks=8192):
    out = torch.zeros(2 * n_blocks, dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()
    part.probe(out, n_blocks)
    o = out.cpu().numpy().astype(np.uint32).reshape(n_blocks, 2)
    xcc = o[:, 0] & 0xF
    # hardware id register: CU in bits 8..11, shader array bit 12, shader engine bits 13..15
    phys = (o[:, 1] >> 8) & 0xFF
    return set(zip(xcc.tolist(), phys.tolist()))


def _popcount(words):
    return sum(bin(w).count("1") for w in words)


@pytest.mark.parametrize("pct", [20, 40, 50, 60, 80])
def test_split_partners_run_on_disjoint_cus(pct):
    with gpulet.Partition(0, pct, 0) as a, gpulet.Partition(0, 100 - pct, 1) as b:
        assert a.n_cu_total == b.n_cu_total == 256
        assert a.n_cu + b.n_cu == 256
        assert _popcount(a.mask) == a.n_cu and _popcount(b.mask) == b.n_cu
        assert all(x & y == 0 for x, y in zip(a.mask, b.mask))
        assert a.query_mask() == a.mask and b.query_mask() == b.mask
        pa, pb = _placement(a), _placement(b)
        assert len(pa) == a.n_cu and len(pb) == b.n_cu
        assert not (pa & pb)
        # the same number of CUs in every die
        for pl, part in ((pa, a), (pb, b)):
            per_die = collections.Counter(x for x, _ in pl)
            assert sorted(per_die) == list(range(8))
            assert set(per_die.values()) == {part.n_cu // 8}
            # ... and the same number in every shader engine of every die
            per_engine = collections.Counter((x, ph >> 5) for x, ph in pl)
            assert len(per_engine) == 32 and set(per_engine.values()) == {part.n_cu // 32}


def test_sizes_and_full_gpu():
    want = {20: 64, 25: 64, 40: 96, 50: 128, 60: 160, 80: 192, 100: 256}
    for pct, n_cu in want.items():
        with gpulet.Partition(0, pct, 0) as p:
            assert (p.pct, p.which, p.n_cu, p.device) == (pct, 0, n_cu, 0)
            assert p.stream
    with gpulet.Partition(0, 100, 0) as p:
        assert len(_placement(p)) == 256


def test_oversubscription_and_handle_errors():
    a = gpulet.Partition(0, 60, 0)
    try:
        for pct, which in [(50, 1), (40, 0), (60, 1)]:     # >100%, same side, >100%
            with pytest.raises(gpulet.GpuletError) as e:
                gpulet.Partition(0, pct, which)
            assert e.value.status == gpulet.EOVERSUB
        b = gpulet.Partition(0, 40, 1)
        with pytest.raises(gpulet.GpuletError) as e:       # a third gpu-let
            gpulet.Partition(0, 1, 0)
        assert e.value.status == gpulet.EOVERSUB
        h = b.handle
        b.destroy()
        assert gpulet.lib.gpulet_partition_destroy(h) == gpulet.EINVAL   # second destroy
        assert gpulet.lib.gpulet_partition_sync(h) == gpulet.EINVAL
        c = gpulet.Partition(0, 40, 1)                      # the share is free again
        c.destroy()
    finally:
        a.destroy()
    with pytest.raises(gpulet.GpuletError):
        gpulet.Partition(7, 50, 0)                          # no such device


def test_request_counters_are_exact():
    from paper_2109_01611_amd import lowering, workloads
    m = workloads.lenet5()
    dm = lowering.DeviceModel(m, workloads.parameters(m, 0), DEV)
    with gpulet.Partition(0, 50, 0) as p:
        assert p.counters() == (0, 0)
        total = 0
        for i, batch in enumerate([1, 7, 32, 5], 1):
            x = dm.input_to_device(workloads.batch_input(m, batch, 0))
            dm.run(p, x)
            total += batch
            assert p.counters() == (i, total)
        x = dm.input_to_device(workloads.batch_input(m, 4, 0))
        ws, n = dm.workspace(4)
        y = dm.alloc_output(4)
        torch.cuda.synchronize()
        lat, tot = gpulet.profile_model(dm.desc, 4, p, x, y, ws, n, warmup=3, iters=10)
        assert len(lat) == 10 and all(v > 0 for v in lat) and tot >= max(lat)
        assert p.counters() == (4 + 13, total + 13 * 4)
        with pytest.raises(gpulet.GpuletError) as e:        # workspace too small
            gpulet.run_model(dm.desc, 4, p, x, y, ws, n - 1)
        assert e.value.status == gpulet.ENOMEM
        assert p.counters() == (17, total + 52)


def test_mfma_rate_probe_scales_with_the_gpulet_and_checks_its_arguments():
    # The matrix-instruction-only probe: a rate below the 2.5 PFLOP/s peak, about half of it on half
    # of the CUs, and no faster on dense operands than on zeros (the power limit works the other way).
    with gpulet.Partition(0, 100, 0) as p:
        p.mfma_rate(0, iters=500, launches=20)                   # clocks up
        _, full_zero = p.mfma_rate(0, iters=500, launches=40)
        _, full_dense = p.mfma_rate(1, iters=500, launches=40)
        for bad in ((0, 3, 10, 1), (0, 8, 0, 1), (0, 8, 10, 0)):
            ms, tf = gpulet.c_float(), gpulet.c_double()
            assert gpulet.lib.gpulet_partition_mfma_rate(p.handle, *bad, gpulet.byref(ms), gpulet.byref(tf)) == gpulet.EINVAL
    with gpulet.Partition(0, 50, 0) as p:
        p.mfma_rate(0, iters=500, launches=20)
        _, half_zero = p.mfma_rate(0, iters=500, launches=40)
    print("mfma probe: %.0f TFLOP/s zeros, %.0f dense, %.0f zeros on 128 CUs" % (full_zero, full_dense, half_zero), flush=True)
    assert 1000.0 < full_zero < 2600.0
    assert 500.0 < full_dense <= 1.02 * full_zero
    assert 0.4 * full_zero < half_zero < 0.6 * full_zero
