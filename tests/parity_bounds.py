"""Element-wise parity bound used by the GPU tests next to the normwise one.

A layer computed with bf16 operands, fp32 accumulation and one rounding of the
result to bf16 differs from the exact result ``ref`` by at most

    |got - ref| <= 2^-8 |ref|  +  slack * mag          for every element,

where ``mag`` is the same layer evaluated by the oracle on the absolute values
of its operands (the sum of the absolute values of the terms of each output
element): the first term is half a unit in the last place of a bf16 number,
the second bounds what the accumulation in fp32 (in whatever order) and the
rounding of a value that is itself slightly off can add.  A normwise figure
hides a single wrong pixel in a large tensor; this one does not.

Pure numpy, no GPU and no library code, so that the bound itself is tested on
the CPU.
"""

import numpy as np

HALF_ULP_BF16 = 2.0 ** -8
SLACK = 1e-5


def violations(got, ref, mag, slack=SLACK, rel=HALF_ULP_BF16):
    """Boolean array: where ``got`` is further from ``ref`` than the bound allows."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    mag = np.asarray(mag, dtype=np.float64)
    if got.shape != ref.shape or mag.shape != ref.shape:
        raise ValueError("shape mismatch: got %r, ref %r, mag %r" % (got.shape, ref.shape, mag.shape))
    if np.any(mag < 0):
        raise ValueError("the magnitude tensor must be non-negative")
    bound = rel * np.abs(ref) + slack * mag
    bad = ~(np.abs(got - ref) <= bound)      # a NaN in got counts as a violation
    return bad


def assert_elementwise(got, ref, mag, slack=SLACK, rel=HALF_ULP_BF16, what=""):
    bad = violations(got, ref, mag, slack, rel)
    if bad.any():
        idx = tuple(int(i[0]) for i in np.nonzero(bad))
        raise AssertionError(
            "%s%d of %d elements outside |got-ref| <= %.3g|ref| + %.3g*mag; first at %r: got %r, ref %r, mag %r"
            % (what + ": " if what else "", int(bad.sum()), bad.size, rel, slack, idx,
               float(np.asarray(got)[idx]), float(np.asarray(ref)[idx]), float(np.asarray(mag)[idx])))
