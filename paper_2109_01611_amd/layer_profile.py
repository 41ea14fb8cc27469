"""Per-layer roofline table of the convolution kernels from the profiler.

Runs every distinct convolution shape of the served models (Table 4 of the
paper; batch sizes of the evaluated configurations) on the 100% gpu-let, each
shape ``reps`` times back to back, under ``rocprofv3``; the parse steps turn
the profiler's per-dispatch records into one row per shape: which kernel the
library chose, its duration, TFLOP/s, the fraction of the bf16 MFMA peak, and
(from a counter pass) how busy the matrix pipelines were.

    cd /tmp && export TMPDIR=/tmp
    rocprofv3 --kernel-trace --output-format csv -d OUT -o run -- \\
        python3 /root/repo/paper_2109_01611_amd/layer_profile.py run --plan OUT/plan.json
    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 \\
        --output-format csv -d OUT2 -o run -- \\
        python3 /root/repo/paper_2109_01611_amd/layer_profile.py run --plan OUT2/plan.json
    python3 paper_2109_01611_amd/layer_profile.py parse OUT OUT2

``load --shape N,C,H,W,K,R,stride,pad --data normal|relu|zeros --seconds S`` keeps one layer
running so that clocks and power can be read meanwhile; ``mfma --data both|dense|zeros --waves 4|8 --seconds S``
does the same with a probe that issues matrix instructions on register operands and nothing else (the ceiling of
the matrix pipelines for an operand pattern).  ``timeline --shape ... [--tile 7|11]`` prints the wall-clock stamps that the
first workgroups of a launch record about themselves (argument fetch, first data, main loop, epilogue).  ``run`` takes ``--models name:batch,...`` (default: the four ImageNet-size
models at their configurations' batch sizes plus the benchmark layer) and
``--shapes "N,C,H,W,K,R,stride,pad;..."`` for extra layers.  Inputs are dense
N(0,1) values (no zeros), the most power-hungry case for the matrix pipelines;
inside a model the inputs are outputs of a ReLU and a layer runs a few percent
faster.  Dispatches are matched to shapes by their order (one kernel launch
per layer call).

Counters: SQ_VALU_MFMA_BUSY_CYCLES counts, summed over all SIMDs, the cycles a
matrix pipeline executes (32 per 32x32x16 bf16 instruction); SQ_BUSY_CU_CYCLES
the cycles a CU has work, summed over CUs.  busy = MFMA_BUSY / (4 * BUSY_CU) is
the share of the SIMD-cycles of busy CUs in which the matrix pipeline worked;
BUSY_CU / (256 * duration) is the engine clock the kernel ran at when all CUs
are busy for all of it (a lower bound otherwise).
"""

import argparse
import csv
import glob
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

PEAK_TFLOPS = 2500.0
DEFAULT_MODELS = "vgg16:16,resnet50:32,googlenet:32,ssd_mobilenet:32"
BENCH_SHAPE = (32, 256, 14, 14, 256, 3, 1, 1)


def conv_shapes(model, batch):
    """Distinct (N, C, H, W, K, R, stride, pad) of a model's convolutions with their counts, in model order."""
    shape = {"x": tuple(model.in_shape)}
    seen, order = {}, []
    ext = lambda n, k, s, p: (n + 2 * p - k) // s + 1
    for nd in model.nodes:
        a = nd.attr
        if nd.op in ("conv", "dwconv"):
            C, H, W = shape[nd.src]
            K = a["K"] if nd.op == "conv" else C
            shape[nd.dst] = (K, ext(H, a["k"], a["stride"], a["pad"]), ext(W, a["k"], a["stride"], a["pad"]))
            if nd.op == "conv":
                key = (batch, C, H, W, K, a["k"], a["stride"], a["pad"])
                if key not in seen:
                    order.append(key)
                seen[key] = seen.get(key, 0) + 1
        elif nd.op == "maxpool":
            C, H, W = shape[nd.src]
            shape[nd.dst] = (C, ext(H, a["k"], a["stride"], a["pad"]), ext(W, a["k"], a["stride"], a["pad"]))
        elif nd.op == "gavgpool":
            shape[nd.dst] = (shape[nd.src][0], 1, 1)
        elif nd.op == "fc":
            shape[nd.dst] = (a["Out"], 1, 1)
        elif nd.op == "concat":
            parts = [shape[s] for s in nd.src]
            shape[nd.dst] = (sum(p[0] for p in parts),) + parts[0][1:]
    return [(k, seen[k]) for k in order]


def run(args):
    import torch
    from paper_2109_01611_amd import gpulet, workloads
    dev = torch.device("cuda:0")
    plan = []
    todo = [("benchmark layer", BENCH_SHAPE, 1)]
    for item in [m for m in args.models.split(",") if m]:
        name, batch = item.split(":")
        for key, count in conv_shapes(getattr(workloads, name)(), int(batch)):
            todo.append(("%s b%s" % (name, batch), key, count))
    for item in [s for s in args.shapes.split(";") if s]:
        todo.append(("extra", tuple(int(v) for v in item.split(",")), 1))
    gen = torch.Generator(device=dev).manual_seed(0)
    with gpulet.Partition(0, 100, 0) as part:
        for origin, (N, C, H, W, K, R, stride, pad), count in todo:
            P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
            cs = 4 if C == 3 else C            # image stems are stored with their channels padded to four
            x = torch.randn((N, H, W, cs), device=dev, generator=gen).to(torch.bfloat16)
            w = (torch.randn((K, R, R, cs), device=dev, generator=gen) * (2.0 / (C * R * R)) ** 0.5).to(torch.bfloat16)
            if cs != C:
                x[..., C:] = 0
                w[..., C:] = 0
            b = torch.zeros(K, device=dev)
            y = torch.empty((N, P, Q, K), dtype=torch.bfloat16, device=dev)
            torch.cuda.synchronize()
            for _ in range(args.reps):
                gpulet.conv2d_fwd(x, w, b, y, N, cs, H, W, K, R, R, stride, pad, True, part.stream)
            part.sync()
            plan.append({"origin": origin, "shape": [N, C, H, W, K, R, stride, pad], "count": count, "reps": args.reps,
                         "flop": 2.0 * N * P * Q * K * C * R * R})
    with open(args.plan, "w") as fh:
        json.dump(plan, fh)
    print("ran %d shapes x %d launches; plan written to %s" % (len(plan), args.reps, args.plan))


def load(args):
    """Keeps one layer running back to back for ``--seconds`` and prints its rate once a second, so
    that the engine clock and power can be sampled from another shell while it runs
    (``rocm-smi --showclocks --showpower``).  ``--data zeros`` runs the same instructions on
    all-zero operands: the matrix pipelines then draw far less power and the clock stays up."""
    import time
    import torch
    from paper_2109_01611_amd import gpulet
    dev = torch.device("cuda:0")
    N, C, H, W, K, R, stride, pad = (int(v) for v in args.shape.split(","))
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    gen = torch.Generator(device=dev).manual_seed(0)
    x = torch.randn((N, H, W, C), device=dev, generator=gen).to(torch.bfloat16)
    w = (torch.randn((K, R, R, C), device=dev, generator=gen) * (2.0 / (C * R * R)) ** 0.5).to(torch.bfloat16)
    if args.data == "zeros":
        x.zero_()
        w.zero_()
    elif args.data == "relu":
        x = torch.relu(x)
    b = torch.zeros(K, device=dev)
    y = torch.empty((N, P, Q, K), dtype=torch.bfloat16, device=dev)
    flop = 2.0 * N * P * Q * K * C * R * R
    torch.cuda.synchronize()
    with gpulet.Partition(0, 100, 0) as part:
        t_end = time.perf_counter() + args.seconds
        iters = max(50, int(2e11 / flop))
        while time.perf_counter() < t_end:
            ms = gpulet.time_conv2d(x, w, b, y, N, C, H, W, K, R, R, stride, pad, True, stream=part.stream, warmup=0,
                                    iters=iters)
            print("%s data: %.2f us per launch, %.0f TFLOP/s" % (args.data, ms * 1e3, flop / ms / 1e9), flush=True)
            iters = max(50, int(1000.0 / ms))


STAMP_POINTS = ["first instruction", "argument block fetched", "position table complete", "first patch and weights in LDS",
                "end of the main loop", "tile staged", "output stores issued"]


STAMP_POINTS_C64 = ["first instruction", "weights requested", "tile 4: at the patch barrier", "tile 4: patch there",
                    "tile 4: matrix instructions issued", "tile 4: patch released", "tile 4: output stores issued",
                    "tile 5: at the patch barrier"]


def timeline(args):
    """Prints where the first workgroups of a launch spend their time (``gpulet_conv2d_timeline``):
    microseconds from the earliest workgroup's first instruction to each point, next to the
    launch-to-launch time of the same layer measured right before."""
    import torch
    from paper_2109_01611_amd import gpulet
    dev = torch.device("cuda:0")
    N, C, H, W, K, R, stride, pad = (int(v) for v in args.shape.split(","))
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    gen = torch.Generator(device=dev).manual_seed(0)
    x = torch.relu(torch.randn((N, H, W, C), device=dev, generator=gen)).to(torch.bfloat16)
    w = (torch.randn((K, R, R, C), device=dev, generator=gen) * (2.0 / (C * R * R)) ** 0.5).to(torch.bfloat16)
    b = torch.zeros(K, device=dev)
    y = torch.empty((N, P, Q, K), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    with gpulet.Partition(0, 100, 0) as part:
        if args.tile >= 0:
            gpulet.set_conv_tile(args.tile)
        try:
            ms = gpulet.time_conv2d(x, w, b, y, N, C, H, W, K, R, R, stride, pad, True, stream=part.stream, warmup=3000, iters=3000)
            print("shape %s: %.2f us per launch, launch to launch (3000 launches between one event pair)" % (args.shape, ms * 1e3))
            for rep in range(args.reps):
                rows = gpulet.conv2d_timeline(x, w, b, y, N, C, H, W, K, R, R, stride, pad, True, stream=part.stream, warmup=500)
                if not rows:
                    print("the kernel that runs this layer records no stamps")
                    return
                t0 = min(r[0] for r in rows)
                print("launch %d: microseconds since the earliest first instruction of workgroups 0..%d" % (rep, len(rows) - 1))
                names = STAMP_POINTS_C64 if rows[0][7] else STAMP_POINTS   # only the resident-weight kernel uses point 7
                for i, name in enumerate(names):
                    print("  %-34s %s" % (name, " ".join("%6.2f" % ((r[i] - t0) / 100.0) for r in rows)))
        finally:
            gpulet.set_conv_tile(-1)


def mfma(args):
    """Runs the matrix-instruction-only probe (no memory traffic at all) for ``--seconds`` per operand
    pattern and prints its rate once a second: the ceiling of any kernel's matrix throughput at the
    clock the power limit allows for that pattern."""
    import time
    import torch  # noqa: F401  (the binding needs torch's HIP runtime loaded first)
    from paper_2109_01611_amd import gpulet
    with gpulet.Partition(0, 100, 0) as part:
        for dense in ([1] if args.data == "dense" else [0] if args.data == "zeros" else [0, 1]):
            t_end = time.perf_counter() + args.seconds
            while time.perf_counter() < t_end:
                ms, tf = part.mfma_rate(dense, waves_per_cu=args.waves, iters=4000, launches=400)
                print("%s operands, %d wavefronts per CU: %.1f us per launch, %.0f TFLOP/s (%.3f of 2500)"
                      % ("dense" if dense else "zero", args.waves, ms * 1e3, tf, tf / PEAK_TFLOPS), flush=True)


def _conv_dispatches(path, want):
    """Rows of a profiler csv that are convolution kernels of this library, in dispatch order."""
    rows = [r for r in csv.DictReader(open(path)) if "gpulet::conv::" in r["Kernel_Name"] and want(r)]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    return rows


def _short(name):
    name = name.replace("void ", "").replace("gpulet::conv::(anonymous namespace)::", "")
    return name.split("(")[0]


def _median(v):
    v = sorted(v)
    return v[len(v) // 2]


def parse(trace_dir, pmc_dir=None):
    plan = json.load(open(os.path.join(trace_dir, "plan.json")))
    tfile = glob.glob(os.path.join(trace_dir, "**", "*kernel_trace.csv"), recursive=True)
    if not tfile:
        raise SystemExit("no kernel_trace.csv under %s" % trace_dir)
    disp = _conv_dispatches(tfile[0], lambda r: True)
    if len(disp) != sum(p["reps"] for p in plan):
        raise SystemExit("expected %d convolution dispatches, found %d" % (sum(p["reps"] for p in plan), len(disp)))
    busy = {}
    if pmc_dir:
        pplan = json.load(open(os.path.join(pmc_dir, "plan.json")))
        pfile = glob.glob(os.path.join(pmc_dir, "**", "*counter_collection.csv"), recursive=True)[0]
        per = {}
        for name in ("SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES"):
            per[name] = _conv_dispatches(pfile, lambda r, n=name: r["Counter_Name"] == n)
        i = 0
        for e in pplan:
            sl = slice(i + e["reps"] // 2, i + e["reps"])        # second half: warm
            m = [float(r["Counter_Value"]) for r in per["SQ_VALU_MFMA_BUSY_CYCLES"][sl]]
            c = [float(r["Counter_Value"]) for r in per["SQ_BUSY_CU_CYCLES"][sl]]
            d = [int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in per["SQ_BUSY_CU_CYCLES"][sl]]
            busy[tuple(e["shape"])] = (_median(m) / (4.0 * _median(c)), _median(c) / (256.0 * _median(d)))
            i += e["reps"]
    print("| model | N | C | HxW | K | RxS/stride | x | kernel | us | TFLOP/s | of peak | MFMA busy | clock GHz |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    i = 0
    for e in plan:
        rows = disp[i + e["reps"] // 2:i + e["reps"]]
        i += e["reps"]
        us = _median([int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in rows]) / 1e3
        tf = e["flop"] / us / 1e6
        N, C, H, W, K, R, stride, pad = e["shape"]
        b = busy.get(tuple(e["shape"]))
        print("| %s | %d | %d | %dx%d | %d | %dx%d/%d | %d | %s | %.1f | %.0f | %.3f | %s | %s |"
              % (e["origin"], N, C, H, W, K, R, R, stride, e["count"], _short(rows[0]["Kernel_Name"]), us, tf,
                 tf / PEAK_TFLOPS, "%.2f" % b[0] if b else "-", "%.2f" % b[1] if b else "-"))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    r = sub.add_parser("run")
    r.add_argument("--plan", required=True)
    r.add_argument("--models", default=DEFAULT_MODELS)
    r.add_argument("--shapes", default="")
    r.add_argument("--reps", type=int, default=20)
    t = sub.add_parser("timeline")
    t.add_argument("--shape", default=",".join(str(v) for v in BENCH_SHAPE), help="N,C,H,W,K,R,stride,pad")
    t.add_argument("--tile", type=int, default=-1, help="force a tile id (7, 10 and 11 record stamps)")
    t.add_argument("--reps", type=int, default=3)
    m = sub.add_parser("mfma")
    m.add_argument("--data", default="both", choices=["both", "dense", "zeros"])
    m.add_argument("--waves", type=int, default=8, choices=[4, 8])
    m.add_argument("--seconds", type=float, default=3.0)
    l = sub.add_parser("load")
    l.add_argument("--shape", default="16,512,28,28,512,3,1,1", help="N,C,H,W,K,R,stride,pad")
    l.add_argument("--data", default="normal", choices=["normal", "relu", "zeros"])
    l.add_argument("--seconds", type=float, default=5.0)
    p = sub.add_parser("parse")
    p.add_argument("trace_dir")
    p.add_argument("pmc_dir", nargs="?")
    args = ap.parse_args()
    if args.cmd == "run":
        run(args)
    elif args.cmd == "load":
        load(args)
    elif args.cmd == "mfma":
        mfma(args)
    elif args.cmd == "timeline":
        timeline(args)
    else:
        parse(args.trace_dir, args.pmc_dir)


if __name__ == "__main__":
    main()
