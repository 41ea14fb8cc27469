"""Offline profiler: the L(b, p) latency table and co-run interference.

The paper's scheduler consumes, per model, the profiled latency of batch b on
a gpu-let of size p (Sec. 4.1; Table 2; Fig. 3 sweeps batch 1-32 over 20-100%)
and the slowdown two co-located gpu-lets inflict on each other (Sec. 3.2,
Fig. 6).  This module drives the library's profiling calls and writes the
rows; all timing happens inside ``libgpulet.so`` with HIP events on the
gpu-let's stream.

Run ``python -m paper_2109_01611_amd.profiler --help`` for the command line.
"""

import argparse
import json
import os
import sys
import tempfile
import time

from . import gpulet, lowering, scenarios, sched, workloads

# Dense bf16 MFMA peak of one MI355X compute unit: 2.5 PFLOP/s over 256 CUs.
PEAK_TFLOPS_PER_CU = 2500.0 / 256.0

# Models whose batch takes tens of microseconds at most: LeNet and single layers ("conv3x3_...").


def _extent(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


def model_flops(model):
    """2 * multiply-adds of one image (padding taps counted) as (conv, fc)."""
    shape = {"x": tuple(model.in_shape)}
    conv = fc = 0
    for nd in model.nodes:
        a = nd.attr
        if nd.op == "conv":
            C, H, W = shape[nd.src]
            P, Q = _extent(H, a["k"], a["stride"], a["pad"]), _extent(W, a["k"], a["stride"], a["pad"])
            conv += 2 * P * Q * a["K"] * C * a["k"] * a["k"]
            shape[nd.dst] = (a["K"], P, Q)
        elif nd.op == "dwconv":
            C, H, W = shape[nd.src]
            P, Q = _extent(H, a["k"], a["stride"], a["pad"]), _extent(W, a["k"], a["stride"], a["pad"])
            conv += 2 * P * Q * C * a["k"] * a["k"]
            shape[nd.dst] = (C, P, Q)
        elif nd.op == "maxpool":
            C, H, W = shape[nd.src]
            shape[nd.dst] = (C, _extent(H, a["k"], a["stride"], a["pad"]), _extent(W, a["k"], a["stride"], a["pad"]))
        elif nd.op == "gavgpool":
            shape[nd.dst] = (shape[nd.src][0], 1, 1)
        elif nd.op == "fc":
            fc += 2 * a["In"] * a["Out"]
            shape[nd.dst] = (a["Out"], 1, 1)
        elif nd.op == "concat":
            parts = [shape[s] for s in nd.src]
            shape[nd.dst] = (sum(p[0] for p in parts),) + parts[0][1:]
    return conv, fc


def mask_hex(words):
    return "".join("%08x" % w for w in reversed(words))


class Bound:
    """A device model with input, output and workspace for one batch size."""

    def __init__(self, dm, batch, seed=0):
        self.dm, self.batch = dm, batch
        self.x = dm.input_to_device(workloads.batch_input(dm.model, batch, seed))
        self.y = dm.alloc_output(batch)
        self.ws, self.ws_bytes = dm.workspace(batch)

    def args(self, part):
        return (self.dm.desc, self.batch, part, self.x, self.y, self.ws, self.ws_bytes)


def measure(bound, part, warmup=20, iters=200, sync_each=True):
    """One row of the L(b, p) table for ``bound`` on gpu-let ``part``."""
    import torch
    torch.cuda.synchronize()
    lat, _ = gpulet.profile_model(*bound.args(part), warmup=warmup, iters=iters, sync_each=sync_each)
    mean, p50, p99 = gpulet.latency_stats(lat)
    # throughput: batches enqueued back to back inside one event pair (an event record between two
    # batches of a few microseconds would be part of what is measured), at least 100 of them
    n_tp = max(100, iters // 4)
    _, total = gpulet.profile_model(*bound.args(part), warmup=10, iters=n_tp, sync_each=2)
    conv, fc = model_flops(bound.dm.model)
    flops = (conv + fc) * bound.batch
    tp_ms = total / n_tp
    tflops = flops / (tp_ms * 1e-3) / 1e12
    return {
        "model": bound.dm.model.name, "batch": bound.batch, "pct": part.pct, "which": part.which,
        "n_cu": part.n_cu, "mask": mask_hex(part.mask), "iters": iters,
        "mean_ms": mean, "p50_ms": p50, "p99_ms": p99,
        "images_per_s": bound.batch / (tp_ms * 1e-3), "ms_per_batch_back_to_back": tp_ms,
        "tflops": tflops, "mfma_frac_of_masked_peak": tflops / (part.n_cu * PEAK_TFLOPS_PER_CU),
    }


def sweep(model, batches, pcts, seed=0, warmup=20, iters=200, device="cuda:0", log=None):
    """L(b, p) rows of one model over batch sizes and gpu-let sizes (one
    gpu-let per size, every batch size measured on it).  Models whose batch takes
    microseconds (LeNet, the single layer) get at least 1000 timed batches per row, so
    that the 99th percentile rests on more than a handful of samples."""
    if model.name == "lenet5" or model.name.startswith("conv"):
        iters = max(iters, 1000)
    dm = lowering.DeviceModel(model, workloads.parameters(model, seed), device)
    bounds = [Bound(dm, b, seed) for b in batches]
    rows = {}
    for pct in pcts:
        with gpulet.Partition(0, pct, 0) as part:
            for bound in bounds:
                row = measure(bound, part, warmup, iters)
                rows[(bound.batch, pct)] = row
                if log:
                    log("%(model)s b=%(batch)d p=%(pct)d%% (%(n_cu)d CUs): mean %(mean_ms).3f ms  p99 %(p99_ms).3f ms"
                        "  %(images_per_s).0f img/s  %(tflops).1f TFLOP/s  %(mfma_frac_of_masked_peak).3f of masked"
                        " peak" % row)
    return [rows[(b, pct)] for b in batches for pct in pcts]


def latency_table(rows, model, sizes, batches, key="mean_ms"):
    """[size][batch] table of one model out of sweep rows."""
    cell = {(r["pct"], r["batch"]): r[key] for r in rows if r["model"] == model}
    return [[cell[(p, b)] for b in batches] for p in sizes]


def knee_report(table, sizes, batches):
    """SLO by the rule of Table 4, affordable-rate curve, curvature and
    p_eff (Sec. 4.3, Fig. 8) of one model's table; all from the library."""
    slo = scenarios.slo_from_table(table, list(sizes), list(batches))
    curve = sched.rate_curve(batches, table, slo)
    best = [sched.affordable_rate(batches, row, slo)[1] for row in table]
    p_eff, curv = sched.max_efficient_partition(sizes, curve, with_curvature=True)
    return {"slo_ms": slo, "sizes": list(sizes), "rate": curve, "batch": best, "curvature": curv, "p_eff": p_eff}


def schedulability(tables, slos, n_gpu, rate_sets, sizes, batches, merge=True, slowdown=None):
    """Number of rate sets Algorithm 1 can place on ``n_gpu`` GPUs, and the
    mean number of GPUs the schedulable ones occupy."""
    n_ok, gpus = 0, 0
    for rates in rate_sets:
        ok, entries = sched.elastic_partitioning(sizes, batches, tables, rates, slos, n_gpu, slowdown=slowdown,
                                                 merge=merge)
        if ok:
            n_ok += 1
            gpus += len(set(e[0] for e in entries))
    return {"scenarios": len(rate_sets), "schedulable": n_ok, "mean_gpus_used": gpus / n_ok if n_ok else None}


def scheduling_study(rows, names, sizes, batches, n_gpus=(1, 2, 4), slowdown=None):
    """Feeds the measured tables to the scheduler: knees per model, then the
    scenario grid of Sec. 3.1 at the paper's absolute rates and at rates scaled
    to each model's whole-GPU capacity, with and without spatial partitioning
    (the latter: the 100% column only, temporal sharing still allowed).  With a
    ``slowdown`` matrix [victim][aggressor] the interference-aware variant of
    the scheduler (the paper's gpulet+int) is counted too."""
    tables = [latency_table(rows, n, sizes, batches) for n in names]
    knees = {n: knee_report(t, sizes, batches) for n, t in zip(names, tables)}
    slos = [knees[n]["slo_ms"] for n in names]
    whole = [[t[-1]] for t in tables]
    out = {"models": names, "knees": knees, "grids": {}}
    grids = {"paper_rates_0_200_400_600": scenarios.rate_grid(len(names))}
    for frac in (0.25, 0.5, 1.0):
        levels = scenarios.rate_grid(len(names), levels=(0.0, 1.0, 2.0, 3.0))
        cap = [knees[n]["rate"][-1] for n in names]
        grids["capacity_x_%g_levels_0_to_3_thirds" % frac] = [
            [l / 3.0 * frac * c for l, c in zip(lv, cap)] for lv in levels]
    for gname, rate_sets in grids.items():
        for n_gpu in n_gpus:
            out["grids"]["%s/%d_gpu" % (gname, n_gpu)] = {
                "gpulets": schedulability(tables, slos, n_gpu, rate_sets, list(sizes), list(batches)),
                "gpulets_no_merge": schedulability(tables, slos, n_gpu, rate_sets, list(sizes), list(batches),
                                                   False),
                "whole_gpus_only": schedulability(whole, slos, n_gpu, rate_sets, [100], list(batches)),
            }
            if slowdown is not None:
                out["grids"]["%s/%d_gpu" % (gname, n_gpu)]["gpulets_with_interference"] = schedulability(
                    tables, slos, n_gpu, rate_sets, list(sizes), list(batches), True, slowdown)
    return out


def partition_cost(n=20, pct=50):
    """Host wall-clock of creating and destroying a gpu-let (CU-masked stream
    plus its scratch), the counterpart of the paper's 10-15 s partition
    reorganisation (Sec. 5).  Returns (create_ms, destroy_ms) medians."""
    import torch
    torch.cuda.synchronize()
    create, destroy = [], []
    for _ in range(n):
        t0 = time.perf_counter()
        part = gpulet.Partition(0, pct, 0)
        t1 = time.perf_counter()
        part.destroy()
        t2 = time.perf_counter()
        create.append((t1 - t0) * 1e3)
        destroy.append((t2 - t1) * 1e3)
    create.sort()
    destroy.sort()
    return create[n // 2], destroy[n // 2]


def corun(model_a, batch_a, model_b, batch_b, pct_a=50, seed=0, warmup=5, window_ms=2000.0, device="cuda:0"):
    """Two gpu-lets at once: model A on ``pct_a``, model B on the Split partner.
    Returns per-model alone and co-run latency statistics and the slowdown
    (median co-run latency over median alone latency on the same mask)."""
    import torch
    da = lowering.DeviceModel(model_a, workloads.parameters(model_a, seed), device)
    db = lowering.DeviceModel(model_b, workloads.parameters(model_b, seed), device)
    ba, bb = Bound(da, batch_a, seed), Bound(db, batch_b, seed)
    out = {}
    with gpulet.Partition(0, pct_a, 0) as pa, gpulet.Partition(0, 100 - pct_a, 1) as pb:
        torch.cuda.synchronize()
        n_alone = 50
        alone = {}
        for key, bd, part in (("a", ba, pa), ("b", bb, pb)):
            lat, _ = gpulet.profile_model(*bd.args(part), warmup=warmup, iters=n_alone, sync_each=True)
            alone[key] = gpulet.latency_stats(lat)
        la, lb = gpulet.profile_corun(ba.args(pa), bb.args(pb), warmup, window_ms)
        for key, bd, part, lat in (("a", ba, pa, la), ("b", bb, pb, lb)):
            mean, p50, p99 = gpulet.latency_stats(lat)
            am, a50, a99 = alone[key]
            out[key] = {
                "model": bd.dm.model.name, "batch": bd.batch, "pct": part.pct, "n_cu": part.n_cu,
                "mask": mask_hex(part.mask), "alone_p50_ms": a50, "alone_p99_ms": a99, "alone_mean_ms": am,
                "corun_batches": len(lat), "corun_p50_ms": p50, "corun_p99_ms": p99, "corun_mean_ms": mean,
                "slowdown_p50": p50 / a50, "slowdown_p99": p99 / a99,
            }
    return out


def shared_launches(names=("googlenet", "ssd_mobilenet", "resnet50"), batches=(32, 8, 1), pct=100, warmup=50,
                    iters=400, device="cuda:0", log=None):
    """The same models lowered with and without shared launches (stacked sibling layers, riding
    pools, launch groups), alternating twice in one process: launches per batch as counted by the
    gpu-let and milliseconds per batch from back-to-back batches."""
    import torch
    from . import gpulet, lowering
    rows = []
    for name in names:
        model = CONFIGS[name][0]()
        params = workloads.parameters(model, 0)
        for batch in batches:
            for rep in range(2):
                for shared in (False, True):
                    dm = lowering.DeviceModel(model, params, device, merge_siblings=shared)
                    b = Bound(dm, batch, 0)
                    with gpulet.Partition(0, pct, 0) as part:
                        torch.cuda.synchronize()
                        before = part.kernel_launches()
                        gpulet.run_model(*b.args(part))
                        part.sync()
                        launches = part.kernel_launches() - before
                        _, total = gpulet.profile_model(*b.args(part), warmup=warmup, iters=iters, sync_each=False)
                    rows.append({"model": model.name, "batch": batch, "shared": int(shared), "rep": rep,
                                 "launches": int(launches), "ms_per_batch": total / iters})
                    if log:
                        log("%s b=%d %s: %d launches, %.4f ms/batch" % (model.name, batch, "shared launches" if shared
                                                                      else "one launch per layer", launches,
                                                                      total / iters))
    return rows


def write_atomic(path, text):
    """Writes ``text`` to ``path`` through a temporary file and a rename, so a
    killed sweep never leaves a half-written table."""
    d = os.path.dirname(os.path.abspath(path))
    os.makedirs(d, exist_ok=True)
    fd, tmp = tempfile.mkstemp(dir=d, prefix=".tmp_table_")
    with os.fdopen(fd, "w") as fh:
        fh.write(text)
    os.replace(tmp, path)


COLUMNS = ["model", "batch", "pct", "n_cu", "mask", "iters", "mean_ms", "p50_ms", "p99_ms", "images_per_s",
           "tflops", "mfma_frac_of_masked_peak"]


def table_csv(rows):
    lines = [",".join(COLUMNS)]
    for r in rows:
        lines.append(",".join(("%.6g" % r[c]) if isinstance(r[c], float) else str(r[c]) for c in COLUMNS))
    return "\n".join(lines) + "\n"


CONFIGS = {
    "lenet5": (workloads.lenet5, [32], [100]),
    "conv": (workloads.single_conv, [32], [20, 40, 50, 60, 80, 100]),
    "resnet50": (workloads.resnet50, [1, 8, 32], [25, 50, 100]),
    "vgg16": (workloads.vgg16, [16], [50, 100]),
    "googlenet": (workloads.googlenet, [32], [50, 100]),
    "ssd_mobilenet": (workloads.ssd_mobilenet, [32], [50, 100]),
}

# The scheduler's input: every model over the whole profiled grid (Fig. 3).
GRID_MODELS = ("lenet5", "googlenet", "resnet50", "ssd_mobilenet", "vgg16")


def main(argv=None):
    ap = argparse.ArgumentParser(description="L(b, p) latency table and co-run interference on one MI355X")
    ap.add_argument("--config", default="conv", choices=sorted(CONFIGS) + ["corun", "all", "grid", "shared-launches"])
    ap.add_argument("--iters", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--window-ms", type=float, default=2000.0)
    ap.add_argument("--out", default=None, help="CSV (or JSON for corun) path; default prints only")
    args = ap.parse_args(argv)
    log = lambda s: print(s, flush=True)
    if args.config == "shared-launches":
        rows = shared_launches(log=log)
        if args.out:
            write_atomic(args.out, json.dumps(rows, indent=1) + "\n")
        return 0
    if args.config == "grid":
        sizes, batches = list(scenarios.SIZES), list(scenarios.BATCHES)
        rows = []
        for name in GRID_MODELS:
            rows += sweep(CONFIGS[name][0](), batches, sizes, warmup=args.warmup, iters=args.iters, log=log)
            if args.out:
                write_atomic(args.out, table_csv(rows))
        names = [CONFIGS[n][0]().name for n in GRID_MODELS]
        study = scheduling_study(rows, names, sizes, batches)
        study["partition_create_destroy_ms"] = partition_cost()
        for n in names:
            k = study["knees"][n]
            log("%s: SLO %.3f ms, affordable rate per size %s req/s, batch %s, p_eff %d%%"
                % (n, k["slo_ms"], ["%.0f" % r for r in k["rate"]], k["batch"], k["p_eff"]))
        for g, res in study["grids"].items():
            log("%s: %s" % (g, "  ".join("%s %d/%d (%.2f GPUs)" % (k, v["schedulable"], v["scenarios"],
                                                                    v["mean_gpus_used"] or 0.0)
                                         for k, v in res.items())))
        log("gpu-let create %.3f ms, destroy %.3f ms (median)" % tuple(study["partition_create_destroy_ms"]))
        if args.out:
            write_atomic(os.path.splitext(args.out)[0] + "_sched.json", json.dumps(study, indent=1) + "\n")
        return 0
    names = sorted(CONFIGS) if args.config == "all" else [args.config]
    rows = []
    for name in names:
        if name == "corun":
            continue
        make, batches, pcts = CONFIGS[name]
        rows += sweep(make(), batches, pcts, warmup=args.warmup, iters=args.iters, log=log)
        if args.out:
            write_atomic(args.out, table_csv(rows))
    if args.config in ("corun", "all"):
        res = corun(workloads.resnet50(), 16, workloads.googlenet(), 32, 50, window_ms=args.window_ms)
        for k in ("a", "b"):
            log("corun %(model)s b=%(batch)d on %(n_cu)d CUs: alone p50 %(alone_p50_ms).3f ms, co-run p50 "
                "%(corun_p50_ms).3f ms (x%(slowdown_p50).3f), p99 x%(slowdown_p99).3f, %(corun_batches)d batches"
                % res[k])
        if args.out:
            write_atomic(os.path.splitext(args.out)[0] + "_corun.json", json.dumps(res, indent=1) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
