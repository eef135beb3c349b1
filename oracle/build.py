"""Compile the CPU oracle (test infrastructure) into oracle/libcocodc_ref.so with g++.

Usage: python oracle/build.py
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cocodc_ref.cpp")
OUT = os.path.join(HERE, "libcocodc_ref.so")

# No fast-math, no FMA contraction: the rounding of every operation is part of the definition.
FLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
         "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= max(
            os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "cocodc_ref.h"))):
        return OUT
    cmd = ["g++", *FLAGS, "-o", OUT, SRC]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
