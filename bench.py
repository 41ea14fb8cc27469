"""Benchmark of the gpu-let hot path on one MI355X.

Workload (the configuration the metric is quoted on): one ResNet-50-style 3x3
convolution layer, N=32, C=K=256, H=W=14, stride 1, pad 1, bias + ReLU, bf16
NHWC, N(0,1) inputs and He-normal weights, seed 0.  A step is one forward pass
of the layer for one batch on the 100% gpu-let; inputs are resident in HBM.
The same layer is then swept over gpu-lets of 20/40/50/60/80/100% of the CUs
(images/s, TFLOP/s, fraction of the masked CUs' MFMA peak, p99 batch latency),
and the fp64 oracle is timed on the host cores as a CPU baseline.

Prints ONE JSON line.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak, all 256 CUs

# The counter passes are separate profiler runs; their summary states the bytes per launch and a
# digest of the sources the benchmark kernel is built from.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "conv3x3_n32_c256_k256_14x14_hbm_traffic.txt")
KERNEL_SOURCES = ["conv_patch.hip", "conv_common.h", "conv.hip", "device_util.h", "gpulet_internal.h"]


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2109_01611_amd", "csrc", name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def recorded_traffic():
    """Bytes per launch from the committed counter summary if it was taken on the kernel as it is now."""
    try:
        fields = dict(line.split(":", 1) for line in open(TRAFFIC_PROFILE) if line.startswith(("traffic_bytes", "kernel_sources")))
        if fields["kernel_sources_sha256"].strip() == kernel_sources_digest():
            return int(fields["traffic_bytes_per_launch"].strip())
    except (OSError, KeyError, ValueError):
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20000)
    ap.add_argument("--warmup", type=int, default=2000)
    # a step is about 10 us and the first few thousand launches after idle run about 3 % slower while
    # the clocks ramp up: an untimed run of this many milliseconds of launches comes before the warm-up
    ap.add_argument("--settle-ms", type=float, default=300.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this benchmark measures one GPU only (gpu-lets partition a single device and "
                 "never exchange data); run with --gpus 1")

    import numpy as np
    import torch

    from paper_2109_01611_amd import gpulet, lowering, profiler, workloads

    dev = "cuda:0"
    N, C, H, W, K, R = 32, 256, 14, 14, 256, 3
    model = workloads.single_conv(C, K, H, W, R, 1, 1, True)
    params = workloads.parameters(model, 0)
    x_host = workloads.batch_input(model, N, 0)
    w_host, b_host = params["conv"]
    x = lowering.nchw_to_nhwc(x_host, dev)
    w = lowering.kcrs_to_krsc(w_host, dev)
    b = torch.from_numpy(b_host).to(dev)
    y = torch.empty((N, H, W, K), dtype=torch.bfloat16, device=dev)
    flops = 2.0 * N * H * W * K * C * R * R

    # ---- timed region: exactly --steps forward passes on the 100% gpu-let
    with gpulet.Partition(0, 100, 0) as part:
        conv_args = (x, w, b, y, N, C, H, W, K, R, R, 1, 1, True)
        # untimed: bring the clocks to their steady state under this load
        settle_launches, t0 = 0, time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < args.settle_ms:
            gpulet.time_conv2d(*conv_args, stream=part.stream, warmup=0, iters=2000)
            settle_launches += 2000
        gpulet.time_conv2d(*conv_args, stream=part.stream, warmup=args.warmup, iters=1)
        torch.cuda.synchronize()
        part.sync()
        t0 = time.perf_counter()
        # the launches and the HIP-event pair around them run inside the library, on the gpu-let's stream
        kernel_ms = gpulet.time_conv2d(*conv_args, stream=part.stream, warmup=0, iters=args.steps)
        part.sync()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        y_full = y.clone()

    out = {
        "metric": "conv images/s + MFMA util per CU fraction (20-100%); p99 batch latency",
        # The steps are timed on the GPU: one HIP event pair on the gpu-let's stream around exactly
        # --steps launches, between two host synchronisations.  The host's clock around the same call
        # (event creation, the wake-up after the last launch) is reported next to it; with few steps
        # of 10 us each it measures the host, not the device.
        "value": N / (kernel_ms * 1e-3),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": kernel_ms,
        "timer": "HIP events on the gpu-let's stream around the timed steps",
        "host_wall_ms_per_step": wall_ms,
        "settle": {"untimed_launches_before_warmup": settle_launches, "ms": args.settle_ms},
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "single ResNet-50-style 3x3 conv layer: N=32 C=K=256 H=W=14 stride 1 pad 1 "
                               "bias+ReLU bf16 NHWC, 100% CUs (256); swept over CU masks 20/40/50/60/80/100%",
                   "flop_per_step": flops},
        "tflops": flops / (kernel_ms * 1e-3) / 1e12,
        "roofline": {
            "bound": "mfma",
            "achieved": flops / (kernel_ms * 1e-3) / 1e12,
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": flops / (kernel_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            # HBM-side bytes per launch from the FETCH_SIZE + WRITE_SIZE counter passes recorded in
            # profiles/ (scaled by a 64 MiB copy); null when the kernel's sources have changed since
            "traffic": recorded_traffic(),
            "kernel": "conv3x3_patch_kernel<64,4,false>",
            "avg_launch_us": kernel_ms * 1e3,
        },
    }

    # ---- the same layer on gpu-lets of every size: L(b=32, p)
    if not args.no_sweep:
        dm = lowering.DeviceModel(model, params, dev)
        bound = profiler.Bound(dm, N, 0)
        rows = []
        for pct in (20, 40, 50, 60, 80, 100):
            with gpulet.Partition(0, pct, 0) as part:
                # throughput: launches back to back on the gpu-let's stream, one event pair around all of them
                ms = gpulet.time_conv2d(*conv_args, stream=part.stream, warmup=3000, iters=2000)
                # latency: one batch in flight at a time, each bracketed by its own event pair
                r = profiler.measure(bound, part, warmup=50, iters=1000)
            tf = flops / (ms * 1e-3) / 1e12
            rows.append({"pct": pct, "n_cu": r["n_cu"], "images_per_s": N / (ms * 1e-3), "tflops": tf,
                         "mfma_frac_of_masked_peak": tf / (r["n_cu"] * profiler.PEAK_TFLOPS_PER_CU),
                         "mean_batch_latency_us": r["mean_ms"] * 1e3, "p99_batch_latency_us": r["p99_ms"] * 1e3})
        full = rows[-1]["images_per_s"]
        for r in rows:
            r["vs_linear_scaling"] = r["images_per_s"] / (full * r["n_cu"] / 256.0)
        out["per_cu_fraction"] = rows
        out["p99_batch_latency_us"] = rows[-1]["p99_batch_latency_us"]

    # ---- CPU baseline: the fp64 oracle as it stands, on the host cores, same workload
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        reps = 0
        while True:
            ref = oracle.conv2d(x_host, w_host, b_host, 1, 1, True)
            reps += 1
            el = time.perf_counter() - t0
            if (el >= 10.0 and reps >= 3) or el >= 30.0:
                break
        out["cpu_baseline"] = {
            "value": N * reps / el, "unit": "images/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "the full layer (batch 32, 7.40 GFLOP) run %d times in %.1f s, fp64 direct convolution" % (reps, el),
            "gflops": flops * reps / el / 1e9,
        }
        whole, per_img = oracle.rel_err(lowering.nhwc_to_nchw(y_full), ref)
        out["parity_rel_err_vs_oracle"] = max(whole, per_img)

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
