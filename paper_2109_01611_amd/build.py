"""Compile the HIP sources under ``csrc/`` for gfx950 into ``libgpulet.so``
next to this file.  hipcc cross-compiles without a GPU."""

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgpulet.so")

SOURCES = ["mask.cpp", "partition.cpp", "layers.cpp", "model.cpp", "sched.cpp", "interference.cpp", "conv.hip",
           "conv_igemm.hip", "conv_patch.hip", "conv_tall.hip", "conv_stream.hip", "conv_stem.hip", "conv_pooled.hip", "dwconv.hip",
           "pool.hip", "fc.hip", "probe.hip"]

# The scheduler's fp64 decisions must not depend on fused multiply-adds.
EXTRA = {"sched.cpp": ["-ffp-contract=off"], "interference.cpp": ["-ffp-contract=off"]}

# Packed-fp32 VALU forms are switched off for device code on purpose.
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-Wno-unused-parameter",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src):
    obj = os.path.join(OBJ, src + ".o")
    cmd = ["hipcc"] + COMMON + DEVICE_FLAGS + EXTRA.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass does not know the device-only feature flag; drop that note.
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l).strip()
    return src, obj, r.returncode, err


def build(verbose=False, jobs=8):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(_compile, SOURCES))
    objs = []
    for src, obj, rc, err in results:
        if err and (verbose or rc != 0):
            print("[%s]\n%s" % (src, err), file=sys.stderr, flush=True)
        if rc != 0:
            raise RuntimeError("hipcc failed on %s" % src)
        objs.append(obj)
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs + ["-lpthread"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
