"""Builds libfbsr.so (the C-ABI library of include/fbsr.h) for gfx950 with hipcc, in-tree.

hipcc cross-compiles without a GPU.  Run as `python -m paper_2504_20634_amd.build`.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libfbsr.so")
SOURCES = ["fbsr_api.hip", "fbsr_block.hip", "fbsr_format8.hip", "fbsr_round.hip", "fbsr_round16.hip", "fbsr_qat.hip", "fbsr_sgd.hip", "fbsr_stats.hip", "fbsr_stats8.hip"]
HEADERS = ["fbsr_device.h", "fbsr_launch.h", "fbsr_stats_common.h"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # keep hipcc from forming packed-fp32 instructions out of scalar float code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # no implicit fused multiply-adds: every fma in the kernels is written out
         "-ffp-contract=off",
         "-Wno-unused-command-line-argument"]


def _compile(src):
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    subprocess.check_call([HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj],
                          stderr=subprocess.STDOUT)
    return obj


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    deps += [os.path.join(os.path.dirname(_HERE), "include", h) for h in ("fbsr.h", "fbsr_measure.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True):
    """Compile every translation unit and link the shared library.  Returns its path."""
    if not force and not stale():
        return LIB
    with ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(_compile, SOURCES))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
