"""Host-side checks of the measurement tools on synthetic profiler output: the arithmetic that turns
rocprofv3 records into the figures under profiles/ (per-layer table, counter-scaled traffic) and the
rule by which the benchmark reports a recorded traffic figure."""

import csv
import json
import os

import pytest

import bench
from paper_2109_01611_amd import layer_profile, traffic, workloads

KNAME = "void gpulet::conv::(anonymous namespace)::conv_igemm_kernel<128, 128, 4, 2, 4, 3, false, false>(gpulet::conv::ConvParams)"


def _write_csv(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as fh:
        w = csv.writer(fh, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(header)
        w.writerows(rows)


def test_conv_shapes_of_resnet50_cover_every_convolution_once():
    shapes = layer_profile.conv_shapes(workloads.resnet50(), 32)
    assert sum(c for _, c in shapes) == 53                      # 1 stem + 16 blocks x 3 + 4 projections
    assert len({k for k, _ in shapes}) == len(shapes)
    assert shapes[0] == ((32, 3, 224, 224, 64, 7, 2, 3), 1)
    assert ((32, 256, 14, 14, 256, 3, 1, 1), 5) in shapes       # the benchmark layer's shape: stage 3 without its strided block
    # multiply-adds of the listed shapes = the published total of the convolutions (4.09 G with the FC's 2 M)
    macs = sum(c * (N // 32) * ((H + 2 * p - R) // s + 1) ** 2 * K * C * R * R for (N, C, H, W, K, R, s, p), c in shapes)
    assert abs(macs - 4.087e9) < 0.01e9


def test_layer_table_arithmetic(tmp_path, capsys):
    # two shapes, four launches each; the second half of each is what counts (medians 20 us and 50 us)
    plan = [{"origin": "m b2", "shape": [2, 64, 8, 8, 64, 3, 1, 1], "count": 3, "reps": 4, "flop": 2.0e9},
            {"origin": "m b2", "shape": [2, 128, 4, 4, 128, 1, 1, 0], "count": 1, "reps": 4, "flop": 1.0e10}]
    durs = [90000, 80000, 20000, 20000, 70000, 60000, 50000, 50000]
    trace, pmc = str(tmp_path / "t"), str(tmp_path / "p")
    hdr = ["Kind", "Kernel_Name", "Start_Timestamp", "End_Timestamp"]
    rows, t = [["KERNEL_DISPATCH", "__amd_rocclr_fillBufferAligned", 1, 2]], 1000
    for d in durs:
        rows.append(["KERNEL_DISPATCH", KNAME, t, t + d])
        t += d + 5000
    _write_csv(os.path.join(trace, "x", "run_kernel_trace.csv"), hdr, rows)
    for d in (trace, pmc):
        os.makedirs(d, exist_ok=True)
        json.dump(plan, open(os.path.join(d, "plan.json"), "w"))
    hdr = ["Kernel_Name", "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]
    rows, t = [], 1000
    for i, d in enumerate(durs):
        busy_cu = 256.0 * d * 2.0 if i < 4 else 128.0 * d * 2.0        # 2 GHz on all / on half of the CUs
        for name, val in (("SQ_VALU_MFMA_BUSY_CYCLES", 4.0 * busy_cu * (0.5 if i < 4 else 0.25)), ("SQ_BUSY_CU_CYCLES", busy_cu),
                          ("SQ_INSTS_VALU_MFMA_MOPS_BF16", 1.0)):
            rows.append([KNAME, name, val, t, t + d])
        t += d + 5000
    _write_csv(os.path.join(pmc, "y", "run_counter_collection.csv"), hdr, rows)
    layer_profile.parse(trace, pmc)
    lines = [l for l in capsys.readouterr().out.splitlines() if l.startswith("| m b2")]
    cells = [[c.strip() for c in l.strip("|").split("|")] for l in lines]
    # model, N, C, HxW, K, RxS/stride, x, kernel, us, TFLOP/s, of peak, MFMA busy, clock GHz
    assert cells[0][:7] == ["m b2", "2", "64", "8x8", "64", "3x3/1", "3"]
    assert cells[0][7] == "conv_igemm_kernel<128, 128, 4, 2, 4, 3, false, false>"
    assert cells[0][8:] == ["20.0", "100", "0.040", "0.50", "2.00"]          # 2e9 FLOP / 20 us = 100 TFLOP/s = 0.04 of 2500
    assert cells[1][8:] == ["50.0", "200", "0.080", "0.25", "1.00"]          # half the CUs busy: "clock" column halves


def test_layer_table_refuses_a_trace_that_does_not_match_its_plan(tmp_path):
    trace = str(tmp_path / "t")
    os.makedirs(trace)
    json.dump([{"origin": "m", "shape": [1] * 8, "count": 1, "reps": 3, "flop": 1.0}], open(os.path.join(trace, "plan.json"), "w"))
    _write_csv(os.path.join(trace, "run_kernel_trace.csv"), ["Kind", "Kernel_Name", "Start_Timestamp", "End_Timestamp"],
               [["KERNEL_DISPATCH", KNAME, 1, 2]])
    with pytest.raises(SystemExit):
        layer_profile.parse(trace)


def test_traffic_is_scaled_by_the_copy_yardstick(tmp_path, capsys):
    # the copy of 64 MiB reads 32768 units -> 2048 bytes per unit; the convolution's median of 6500 units -> 13.3 MB
    hdr = ["Kernel_Name", "Counter_Name", "Counter_Value"]
    rows = [["__amd_rocclr_copyBuffer", "FETCH_SIZE", v] for v in (4.0, 32768.0, 32768.0, 32768.0, 40000.0)]
    rows += [["void gpulet::conv::(anonymous namespace)::conv3x3_patch_kernel<64, 4>(gpulet::conv::ConvParams)", "FETCH_SIZE", v]
             for v in (9000.0, 6500.0, 6500.0, 6400.0, 6600.0)]
    rows += [["some_other_kernel", "FETCH_SIZE", 1e9]]
    _write_csv(str(tmp_path / "a" / "run_counter_collection.csv"), hdr, rows)
    got = traffic.per_dispatch(str(tmp_path / "a"))
    assert got == {"FETCH_SIZE": {"copy": (32768.0, 5), "conv": (6500.0, 5)}}
    traffic.parse([str(tmp_path / "a")])
    out = capsys.readouterr().out
    assert "-> 2048.0 bytes per unit" in out and "-> 13312000 bytes per launch" in out


def test_bench_reports_recorded_traffic_only_for_the_sources_it_was_taken_on(tmp_path, monkeypatch):
    f = tmp_path / "traffic.txt"
    monkeypatch.setattr(bench, "TRAFFIC_PROFILE", str(f))
    assert bench.recorded_traffic() is None                       # no file
    digest = bench.kernel_sources_digest()
    assert len(digest) == 64 and digest == bench.kernel_sources_digest()
    f.write_text("text\nkernel_sources_sha256: %s\ntraffic_bytes_per_launch: 16552374\nmore text\n" % digest)
    assert bench.recorded_traffic() == 16552374
    f.write_text("kernel_sources_sha256: %s\ntraffic_bytes_per_launch: 16552374\n" % ("0" * 64))
    assert bench.recorded_traffic() is None                       # the kernel changed since the counters were read
    f.write_text("kernel_sources_sha256: %s\n" % digest)
    assert bench.recorded_traffic() is None                       # incomplete record
