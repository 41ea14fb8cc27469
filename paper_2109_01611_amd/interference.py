"""Interference between two gpu-lets sharing a GPU (paper Sec. 3.2 / Fig. 6) and
the linear model that predicts it (Sec. 4.4 / Fig. 9), measured on one MI355X.

Three measurement steps and two analysis steps; all arithmetic of the method
(utilisation features, co-run factor, training / validation split, fit,
prediction, error and overhead percentiles, slowdown matrix) runs in
``libgpulet.so``; this module reads counter files, marshals and prints:

1. ``solo`` (run under the profiler, once per counter set): every model at every
   batch size on every gpu-let size, alone, so that the per-dispatch counters
   give the L2 requests and memory bytes of a solo run:

       rocprofv3 --pmc FETCH_SIZE TCC_REQ_sum --output-format csv -d OUT_A -o run -- \\
           python3 /root/repo/paper_2109_01611_amd/interference.py solo OUT_A/manifest.json
       rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT_B -o run -- \\
           python3 /root/repo/paper_2109_01611_amd/interference.py solo OUT_B/manifest.json

2. ``features OUT_A OUT_B features.json``: sums the counters of each solo run
   (memory counters scaled by a 64 MiB copy measured in the same pass).

3. ``sweep samples.json``: for every pair of different models, every pair of
   batch sizes and every split of the GPU, the latency of both alone on their
   masks and while running concurrently.

5. ``study grid.csv features.json report.json out.json`` (no GPU needed): turns
   the fitted model into the scheduler's slowdown matrix - for every ordered
   pair of models the largest predicted factor over the profiled batch sizes
   and splits, minus one - and counts schedulable scenarios with and without
   it on the measured L(b, p) grid (the paper's gpulet+int against gpulet).

4. ``fit features.json samples.json report.json``: utilisations = counter totals
   over the solo latency, relative to the whole GPU's L2 request rate and HBM
   bandwidth; a seeded 70/30 split into training and validation samples
   (the paper's 1,750/750); coefficients and the error at the 90th and 95th
   percentile of the validation set.
"""

import csv
import glob
import itertools
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

MODELS = ("lenet5", "googlenet", "resnet50", "ssd_mobilenet", "vgg16")
BATCHES = (2, 4, 8, 16, 32)
SPLITS = (20, 40, 50, 60, 80)       # size of the first gpu-let; the second takes the rest
COPY_BYTES = 64 << 20


def _lowered(names):
    from paper_2109_01611_amd import lowering, profiler, workloads
    out = {}
    for name in names:
        model = profiler.CONFIGS[name][0]()
        dm = lowering.DeviceModel(model, workloads.parameters(model, 0), "cuda:0")
        out[name] = {b: profiler.Bound(dm, b, 0) for b in BATCHES}
    return out


def solo(manifest_path):
    import torch
    from paper_2109_01611_amd import gpulet
    bounds = _lowered(MODELS)
    manifest = []
    for pct in SPLITS:
        with gpulet.Partition(0, pct, 0) as part:
            for name in MODELS:
                for b in BATCHES:
                    bd = bounds[name][b]
                    before = part.kernel_launches()
                    for _ in range(2):          # the second run is the one that counts (weights seen once)
                        gpulet.run_model(*bd.args(part))
                        part.sync()
                    # launches per run (layers that share a launch count once), as the counter pass sees them
                    manifest.append({"model": name, "batch": b, "pct": pct,
                                     "kernels": int(part.kernel_launches() - before) // 2, "runs": 2})
    src = torch.empty(COPY_BYTES // 2, dtype=torch.bfloat16, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(10):
        dst.copy_(src)
    torch.cuda.synchronize()
    with open(manifest_path, "w") as fh:
        json.dump(manifest, fh)
    print("solo: %d runs" % len(manifest))


def _dispatches(out_dir):
    """Counter rows of one pass grouped by dispatch, in launch order:
    [(kernel name, {counter: value})]."""
    files = glob.glob(os.path.join(out_dir, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit("no counter_collection.csv under %s" % out_dir)
    by_id = {}
    for row in csv.DictReader(open(files[0])):
        d = by_id.setdefault(int(row["Dispatch_Id"]), [row["Kernel_Name"], {}])
        d[1][row["Counter_Name"]] = d[1].get(row["Counter_Name"], 0.0) + float(row["Counter_Value"])
    return [tuple(by_id[k]) for k in sorted(by_id)]


def features(dir_a, dir_b, out_path):
    table = {}
    for out_dir in (dir_a, dir_b):
        manifest = json.load(open(os.path.join(out_dir, "manifest.json")))
        rows = _dispatches(out_dir)
        ours = [c for name, c in rows if "gpulet::" in name]
        copies = [c for name, c in rows if "copyBuffer" in name][-10:]   # the yardstick copies come last
        need = sum(m["kernels"] * m["runs"] for m in manifest)
        if len(ours) != need:
            raise SystemExit("%s: %d library dispatches, manifest says %d" % (out_dir, len(ours), need))
        unit = {}
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            vals = sorted(c[counter] for c in copies if counter in c)
            if vals:
                unit[counter] = COPY_BYTES / vals[len(vals) // 2]
        pos = 0
        for m in manifest:
            pos += m["kernels"] * (m["runs"] - 1)
            chunk = ours[pos:pos + m["kernels"]]
            pos += m["kernels"]
            key = "%s/%d/%d" % (m["model"], m["batch"], m["pct"])
            slot = table.setdefault(key, {})
            for counter in chunk[0]:
                total = sum(c[counter] for c in chunk)
                if counter in unit:
                    slot[counter + "_bytes"] = total * unit[counter]
                else:
                    slot[counter] = total
        print("%s: %d dispatches, scale %s" % (out_dir, len(ours), unit))
    with open(out_path, "w") as fh:
        json.dump(table, fh, indent=0)
    print("features for %d solo runs -> %s" % (len(table), out_path))


def sweep(out_path, window_ms=120.0, alone_iters=30):
    from paper_2109_01611_amd import gpulet
    bounds = _lowered(MODELS)
    samples = []
    for pct in SPLITS:
        with gpulet.Partition(0, pct, 0) as pa, gpulet.Partition(0, 100 - pct, 1) as pb:
            alone = {}
            for part, tag in ((pa, "a"), (pb, "b")):
                for name in MODELS:
                    for b in BATCHES:
                        lat, _ = gpulet.profile_model(*bounds[name][b].args(part), warmup=3, iters=alone_iters,
                                                      sync_each=True)
                        alone[(tag, name, b)] = gpulet.latency_stats(lat)[1]
            for ma, mb in itertools.combinations(MODELS, 2):
                for ba in BATCHES:
                    for bb in BATCHES:
                        la, lb = gpulet.profile_corun(bounds[ma][ba].args(pa), bounds[mb][bb].args(pb), 2, window_ms)
                        samples.append({
                            "a": {"model": ma, "batch": ba, "pct": pct, "alone_ms": alone[("a", ma, ba)],
                                  "corun_ms": gpulet.latency_stats(la)[1], "batches": len(la)},
                            "b": {"model": mb, "batch": bb, "pct": 100 - pct, "alone_ms": alone[("b", mb, bb)],
                                  "corun_ms": gpulet.latency_stats(lb)[1], "batches": len(lb)}})
            print("split %d:%d done, %d co-runs so far" % (pct, 100 - pct, len(samples)), flush=True)
            with open(out_path, "w") as fh:
                json.dump(samples, fh)
    print("%d co-runs -> %s" % (len(samples), out_path))


def utilisation(feat, side):
    """(L2 utilisation, memory-bandwidth utilisation) of one solo run, from its counter totals."""
    from paper_2109_01611_amd import sched
    f = feat["%s/%d/%d" % (side["model"], side["batch"], side["pct"])]
    return sched.interference_utilisation(f["TCC_REQ_sum"], f["FETCH_SIZE_bytes"], f["WRITE_SIZE_bytes"],
                                          side["alone_ms"])


def fit(features_path, samples_path, report_path, seed=0):
    import numpy as np
    from paper_2109_01611_amd import inputs, sched
    feat = json.load(open(features_path))
    rows, corun, alone, tags = [], [], [], []
    for s in json.load(open(samples_path)):
        for victim, aggressor in ((s["a"], s["b"]), (s["b"], s["a"])):
            l2v, memv = utilisation(feat, victim)
            l2a, mema = utilisation(feat, aggressor)
            rows.append([l2v, l2a, memv, mema])
            corun.append(victim["corun_ms"])
            alone.append(victim["alone_ms"])
            tags.append("%s b%d %d%% next to %s b%d" % (victim["model"], victim["batch"], victim["pct"],
                                                         aggressor["model"], aggressor["batch"]))
    factors = sched.interference_factor(corun, alone)
    n = len(factors)
    tr, va = sched.interference_split(list(inputs.uniform(seed, "interference/split", n)))
    pick = lambda idx, seq: [seq[i] for i in idx]
    coef = sched.interference_fit(pick(tr, rows), pick(tr, factors))
    qs = (50.0, 90.0, 95.0, 100.0)
    err_val = sched.interference_error(coef, pick(va, rows), pick(va, factors), qs)
    err_train = sched.interference_error(coef, pick(tr, rows), pick(tr, factors), qs)
    const = [0.0, 0.0, 0.0, 0.0, sum(pick(tr, factors)) / len(tr)]       # no-feature baseline: the mean factor
    err_const = sched.interference_error(const, pick(va, rows), pick(va, factors), qs)
    (o50, o90, o99, omax), below18 = sched.interference_overhead(factors, (50.0, 90.0, 99.0, 100.0), 0.18)
    report = {
        "samples": n, "train": int(len(tr)), "validate": int(len(va)),
        "coefficients_c1_c5": coef,
        "validation_error_at_percentile": dict(zip(map(str, qs), err_val)),
        "training_error_at_percentile": dict(zip(map(str, qs), err_train)),
        "mean_factor_baseline_error_at_percentile": dict(zip(map(str, qs), err_const)),
        "overhead_distribution": {"median": o50, "p90": o90, "p99": o99, "max": omax,
                                  "share_below_18_percent": below18},
        "feature_ranges": {"l2": [min(r[0] for r in rows), max(r[0] for r in rows)],
                           "mem": [min(r[2] for r in rows), max(r[2] for r in rows)]},
        "worst_cases": [tags[i] + ": x%.3f" % factors[i] for i in np.argsort(factors)[::-1][:8]],
    }
    with open(report_path, "w") as fh:
        json.dump(report, fh, indent=1)
    print(json.dumps(report, indent=1))


def slowdown_matrix(feat, coef, latency_ms, names):
    """F[victim][aggressor]: worst predicted co-run factor minus one over the
    profiled batch sizes and splits; ``latency_ms[(model, batch, pct)]`` is the
    solo latency the utilisations are taken over."""
    from paper_2109_01611_amd import sched
    F = []
    for v in names:
        row = []
        for a in names:
            rows = []
            for pct in SPLITS:
                for bv in BATCHES:
                    for ba in BATCHES:
                        sv = {"model": v, "batch": bv, "pct": pct, "alone_ms": latency_ms[(v, bv, pct)]}
                        sa = {"model": a, "batch": ba, "pct": 100 - pct, "alone_ms": latency_ms[(a, ba, 100 - pct)]}
                        l2v, memv = utilisation(feat, sv)
                        l2a, mema = utilisation(feat, sa)
                        rows.append([l2v, l2a, memv, mema])
            row.append(sched.interference_worst_slowdown(coef, rows))
        F.append(row)
    return F


def study(grid_csv, features_path, report_path, out_path):
    from paper_2109_01611_amd import profiler, scenarios
    rows = []
    for r in csv.DictReader(open(grid_csv)):
        rows.append({"model": r["model"], "batch": int(r["batch"]), "pct": int(r["pct"]), "mean_ms": float(r["mean_ms"])})
    names = [profiler.CONFIGS[n][0]().name for n in profiler.GRID_MODELS]
    short = dict(zip(names, profiler.GRID_MODELS))
    feat = json.load(open(features_path))
    coef = json.load(open(report_path))["coefficients_c1_c5"]
    lat = {(short[r["model"]], r["batch"], r["pct"]): r["mean_ms"] for r in rows}
    F = slowdown_matrix(feat, coef, lat, [short[n] for n in names])
    out = profiler.scheduling_study(rows, names, list(scenarios.SIZES), list(scenarios.BATCHES), slowdown=F)
    out["slowdown_matrix_victim_by_aggressor"] = {"models": names, "F": F}
    with open(out_path, "w") as fh:
        json.dump(out, fh, indent=1)
    print("slowdown matrix (victim rows, aggressor columns), models %s" % names)
    for n, row in zip(names, F):
        print("  %-14s %s" % (n, " ".join("%.3f" % v for v in row)))
    for g, res in out["grids"].items():
        print("%s: %s" % (g, "  ".join("%s %d/%d (%.2f GPUs)" % (k, v["schedulable"], v["scenarios"],
                                                                 v["mean_gpus_used"] or 0.0)
                                       for k, v in res.items())))


def main(argv):
    if len(argv) == 3 and argv[1] == "solo":
        solo(argv[2])
    elif len(argv) == 5 and argv[1] == "features":
        features(argv[2], argv[3], argv[4])
    elif len(argv) == 3 and argv[1] == "sweep":
        sweep(argv[2])
    elif len(argv) == 5 and argv[1] == "fit":
        fit(argv[2], argv[3], argv[4])
    elif len(argv) == 6 and argv[1] == "study":
        study(argv[2], argv[3], argv[4], argv[5])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv)
