"""Host-only check of the model runner's lane schedule (gpulet_model_schedule):
whatever two layers conflict on a buffer - a read after a write, a write after a
read, two writes that are not disjoint slices of one concatenated tensor - must be
ordered by lane order plus the cross-lane waits.  The conflicts are derived here
from the layer table alone, independently of the library's own analysis."""

import pytest

from paper_2109_01611_amd import gpulet, lowering, workloads

MODELS = [
    workloads.googlenet(width_div=4, in_hw=64, n_class=10),
    workloads.resnet50(width_div=8, in_hw=64, n_class=10, blocks=(2, 2, 1, 1)),
    workloads.ssd_mobilenet(width_div=8, in_hw=64, n_class=3),
    workloads.vgg16(width_div=16, in_hw=32, n_class=10),
    workloads.lenet5(),
]


def _happens_before(n, lane, waits):
    """reach[i] = set of layers ordered before layer i."""
    preds = [set() for _ in range(n)]
    last = {}
    for i in range(n):
        if lane[i] in last:
            preds[i].add(last[lane[i]])
        last[lane[i]] = i
    for a, b in waits:
        assert a < b
        preds[b].add(a)
    reach = [set() for _ in range(n)]
    for i in range(n):
        for j in preds[i]:
            reach[i] |= reach[j] | {j}
    return reach


def _writes(L):
    """(buffer, channel slice or None) for everything a layer writes."""
    k1 = L.K - L.K2
    out = [(L.out_buf, (L.out_ch_offset, L.out_ch_offset + k1, L.out_ch_total) if L.out_ch_total > 0 else None)]
    if L.K2 > 0:
        out.append((L.out2_buf, (L.out2_ch_offset, L.out2_ch_offset + L.K2, L.out2_ch_total)
                    if L.out2_ch_total > 0 else None))
    if L.side_pool:
        out.append((L.pool_buf, None))
    return out


def _conflicts(layers):
    """Pairs (i, j), i < j, that must not run concurrently or out of order."""
    out = set()
    for j, Lj in enumerate(layers):
        reads_j = {Lj.in_buf} | ({Lj.res_buf} if Lj.res_buf >= 0 else set())
        for i in range(j):
            Li = layers[i]
            reads_i = {Li.in_buf} | ({Li.res_buf} if Li.res_buf >= 0 else set())
            for bi, si in _writes(Li):
                if bi in reads_j:
                    out.add((i, j))
            for bj, sj in _writes(Lj):
                if bj in reads_i:
                    out.add((i, j))
                for bi, si in _writes(Li):
                    if bi != bj:
                        continue
                    disjoint = (si and sj and si[2] == sj[2] and (si[1] <= sj[0] or sj[1] <= si[0]))
                    # disjoint slices of one tensor are independent only while nobody has read or rewritten
                    # the buffer in between; otherwise j starts a new tensor in a reused buffer
                    between = any(layers[k].in_buf == bi or layers[k].res_buf == bi or
                                  any(b == bi and sl is None for b, sl in _writes(layers[k]))
                                  for k in range(i + 1, j))
                    if not disjoint or between:
                        out.add((i, j))
    return sorted(out)


@pytest.mark.parametrize("model", MODELS, ids=lambda m: m.name)
@pytest.mark.parametrize("reuse", [True, False])
def test_every_buffer_conflict_is_ordered(model, reuse):
    dm = lowering.DeviceModel(model, workloads.parameters(model, 0), "cpu", reuse=reuse)
    layers = list(dm.layers)
    n = len(layers)
    lane, waits = gpulet.model_schedule(dm.desc, 2, lanes=2)
    assert len(lane) == n and set(lane) <= {0, 1}
    reach = _happens_before(n, lane, waits)
    for i, j in _conflicts(layers):
        assert i in reach[j], (i, j, lane[i], lane[j])
    lane1, waits1 = gpulet.model_schedule(dm.desc, 2, lanes=1)
    assert lane1 == [0] * n and waits1 == []
    if model.name.startswith(("googlenet", "ssd")):
        assert 1 in lane            # independent branches really are spread
    if model.name.startswith(("vgg", "lenet")):
        assert lane == [0] * n      # a plain chain stays on the gpu-let's stream


def test_lane_setting():
    gpulet.set_model_lanes(1)
    for bad in (0, 2, 3):            # a second lane is switched off for now
        with pytest.raises(gpulet.GpuletError):
            gpulet.set_model_lanes(bad)
    dm = lowering.DeviceModel(MODELS[-1], workloads.parameters(MODELS[-1], 0), "cpu")
    with pytest.raises(gpulet.GpuletError):
        gpulet.model_schedule(dm.desc, 2, lanes=3)
