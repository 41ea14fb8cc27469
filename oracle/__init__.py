"""fp64 CPU oracle of the CNN forward pass served on a gpu-let.

Test infrastructure only: the tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product never does.
"""

from .reference import (  # noqa: F401
    avgpool, conv2d, depthwise_conv2d, fc, global_avgpool, maxpool, model_flops, model_params, num_threads,
    out_dim, rel_err, run_model)
