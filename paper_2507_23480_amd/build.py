"""Builds the HIP library (csrc/*.hip -> libfastpoint_hip.so) for gfx950 with hipcc.

-ffp-contract=off: every binary32 operation of a squared distance is rounded on
its own (index results are compared bit for bit with a CPU reference).  Packed
fp32 instructions are switched off for all device code."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfastpoint_hip.so")
SOURCES = ["sampler.hip", "ball_query.hip", "knn.hip", "excl_lists.hip", "abi.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", *os.environ.get("FASTPOINT_EXTRA_FLAGS", "").split(), "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    subprocess.run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build(verbose: bool = False) -> str:
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
