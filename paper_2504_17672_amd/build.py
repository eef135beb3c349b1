"""Compile the HIP library for gfx950 into paper_2504_17672_amd/libcocodc.so.

Usage: python -m paper_2504_17672_amd.build [-DCOCODC_TILE=... ...]
hipcc cross-compiles without a GPU.  Extra -D options are passed through (tuning sweeps).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "cocodc.hip")
OUT = os.path.join(HERE, "libcocodc.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-ffp-contract=off",  # explicit fma() only: fused and single-step kernels must round alike
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"),
]


def build(extra=(), out=OUT) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra, "-o", out, SRC]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(extra=sys.argv[1:]))
