"""The FC entry point that allocates nothing (its split-depth scratch is a static
device array of the library) against the ordinary entry point on a gpu-let, whose
scratch the library allocated: same bits, and both within the layer bounds of the
fp64 oracle.  Two calls in a row, the second smaller, so that what the first left
in the shared array cannot leak into the second."""

import numpy as np
import pytest
import torch

import oracle
from paper_2109_01611_amd import gpulet, inputs, lowering

from gpu_util import DEV, LAYER_TOL, assert_close

pytestmark = pytest.mark.gpu


def _case(seed, N, In, Out):
    x = inputs.tensor(seed, "na/x%d_%d" % (N, In), (N, In), "normal")
    w = inputs.he_normal(seed, "na/w%d_%d" % (In, Out), (Out, In))
    b = inputs.bias(seed, "na/b%d" % Out, Out)
    return x, w, b


@pytest.mark.parametrize("out_fp32", [False, True])
def test_fc_with_static_scratch_matches_fc_on_two_calls_in_a_row(out_fp32):
    dt = torch.float32 if out_fp32 else torch.bfloat16
    relu = not out_fp32
    with gpulet.Partition(0, 100, 0) as part:
        # long rows: 16 output groups x 8 depth ranges, then 4 groups x 8 ranges of fewer rows
        for (N, In, Out) in ((32, 8192, 1024), (5, 8200, 200)):
            x, w, b = _case(41, N, In, Out)
            xd, wd = lowering.to_device_bf16(x, DEV), lowering.to_device_bf16(w, DEV)
            bd = torch.from_numpy(b).to(DEV)
            want = torch.full((N, Out), -512.0, dtype=dt, device=DEV)
            got = torch.full((N, Out), -512.0, dtype=dt, device=DEV)
            torch.cuda.synchronize()
            gpulet.fc(xd, wd, bd, want, N, In, Out, relu, out_fp32, part.stream)
            gpulet.fc_static_scratch(xd, wd, bd, got, N, In, Out, relu, out_fp32, part.stream)
            part.sync()
            assert torch.equal(got, want), (N, In, Out)
            ref = oracle.fc(x, w, b, relu)
            mag = oracle.fc(np.abs(x), np.abs(w), np.abs(b), False)
            assert_close(got.to(torch.float32).cpu().numpy().astype(np.float64), ref, mag,
                         tol=1e-5 if out_fp32 else LAYER_TOL, rel=2.0 ** -24 if out_fp32 else 2.0 ** -8,
                         what=(N, In, Out))
        # a layer that needs no scratch goes through the same entry point
        N, In, Out = 7, 400, 120
        x, w, b = _case(42, N, In, Out)
        xd, wd, bd = lowering.to_device_bf16(x, DEV), lowering.to_device_bf16(w, DEV), torch.from_numpy(b).to(DEV)
        want = torch.empty((N, Out), dtype=dt, device=DEV)
        got = torch.empty((N, Out), dtype=dt, device=DEV)
        gpulet.fc(xd, wd, bd, want, N, In, Out, relu, out_fp32, part.stream)
        gpulet.fc_static_scratch(xd, wd, bd, got, N, In, Out, relu, out_fp32, part.stream)
        part.sync()
        assert torch.equal(got, want)


def test_fc_with_static_scratch_checks_its_arguments():
    t = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    for bad in (dict(N=0), dict(In=0), dict(Out=0)):
        a = dict(N=1, In=8, Out=8)
        a.update(bad)
        with pytest.raises(gpulet.GpuletError) as e:
            gpulet.fc_static_scratch(t, t, None, t, a["N"], a["In"], a["Out"], True, False, None)
        assert e.value.status == gpulet.EINVAL
    with pytest.raises(gpulet.GpuletError) as e:
        gpulet.fc_static_scratch(None, t, None, t, 1, 8, 8, True, False, None)
    assert e.value.status == gpulet.EINVAL
