"""HBM traffic of the benchmark convolution from hardware counters.

Run once per counter under the profiler (the derived counters FETCH_SIZE and
WRITE_SIZE need separate passes), from a directory the profiler may write to:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -o run -- \\
        python3 /root/repo/paper_2109_01611_amd/traffic.py run
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT2 -o run -- \\
        python3 /root/repo/paper_2109_01611_amd/traffic.py run

then summarise both passes:

    python3 paper_2109_01611_amd/traffic.py parse OUT OUT2

``run`` launches the 3x3 benchmark layer (N=32, C=K=256, 14x14) on the 100%
gpu-let and, as the yardstick, a plain device-to-device copy of 64 MiB (an
the runtime's copy kernel: 64 MiB read, 64 MiB written).  ``parse`` reports
each counter per dispatch for both kernels and scales the convolution's
reading by (known copy bytes) / (counter reading of the copy).
"""

import csv
import glob
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

COPY_BYTES = 64 << 20
CONV_LAUNCHES = 50
COPY_LAUNCHES = 20


def run():
    import torch
    from paper_2109_01611_amd import gpulet, inputs, lowering, workloads
    dev = torch.device("cuda:0")
    model = workloads.single_conv()
    nd = model.nodes[0]
    a = nd.attr
    N, (C, H, W) = 32, model.in_shape
    params = workloads.parameters(model, 0)
    x = lowering.nchw_to_nhwc(workloads.batch_input(model, N, 0), dev)
    w = lowering.kcrs_to_krsc(params[nd.name][0], dev)
    b = torch.from_numpy(params[nd.name][1]).to(dev)
    y = torch.empty((N, H, W, a["K"]), dtype=torch.bfloat16, device=dev)
    src = torch.empty(COPY_BYTES // 2, dtype=torch.bfloat16, device=dev).normal_()
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    with gpulet.Partition(0, 100, 0) as part:
        for _ in range(CONV_LAUNCHES):
            gpulet.conv2d_fwd(x, w, b, y, N, C, H, W, a["K"], a["k"], a["k"], a["stride"], a["pad"], True,
                              part.stream)
        part.sync()
    for _ in range(COPY_LAUNCHES):
        dst.copy_(src)
    torch.cuda.synchronize()
    algorithmic = 2 * (x.numel() + w.numel() + y.numel()) + 4 * b.numel()
    print("conv algorithmic bytes per launch: %d (x %d + w %d + bias %d read, y %d written)"
          % (algorithmic, 2 * x.numel(), 2 * w.numel(), 4 * b.numel(), 2 * y.numel()))


def per_dispatch(out_dir):
    """{counter: {kernel class: (median reading per dispatch, dispatches)}} of one pass."""
    files = glob.glob(os.path.join(out_dir, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit("no counter_collection.csv under %s" % out_dir)
    acc = {}
    for row in csv.DictReader(open(files[0])):
        name = row["Kernel_Name"]
        if "conv3x3_patch_kernel" in name or "conv_igemm_kernel" in name:
            kind = "conv"
        elif "copyBuffer" in name:   # the runtime's device-to-device copy kernel
            kind = "copy"
        else:
            continue
        acc.setdefault(row["Counter_Name"], {}).setdefault(kind, []).append(float(row["Counter_Value"]))
    return {c: {k: (sorted(v)[len(v) // 2], len(v)) for k, v in kinds.items()} for c, kinds in acc.items()}


def parse(dirs):
    for d in dirs:
        for counter, kinds in per_dispatch(d).items():
            if "copy" not in kinds or "conv" not in kinds:
                print("%s: kernels found: %s" % (counter, sorted(kinds)))
                continue
            copy_reading, n_copy = kinds["copy"]
            conv_reading, n_conv = kinds["conv"]
            factor = COPY_BYTES / copy_reading
            print("%s: copy of %d bytes reads %.1f per dispatch (median of %d) -> %.1f bytes per unit; "
                  "conv reads %.1f per dispatch (median of %d) -> %.0f bytes per launch"
                  % (counter, COPY_BYTES, copy_reading, n_copy, factor, conv_reading, n_conv,
                     conv_reading * factor))


if __name__ == "__main__":
    if len(sys.argv) >= 2 and sys.argv[1] == "run":
        run()
    elif len(sys.argv) >= 3 and sys.argv[1] == "parse":
        parse(sys.argv[2:])
    else:
        raise SystemExit(__doc__)
