"""Compiles csrc/*.hip into libhot.so next to this file (hipcc, gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(HERE, "csrc", "hot.hip"), os.path.join(HERE, "csrc", "stats.hip"),
        os.path.join(HERE, "csrc", "linear.hip"), os.path.join(HERE, "csrc", "update.hip")]
LIB = os.path.join(HERE, "libhot.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed fp32 arithmetic is switched off for all device code of this library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-I", os.path.join(ROOT, "include")]


def build_libhot(verbose: bool = False) -> str:
    cmd = [HIPCC] + FLAGS + ["-o", LIB] + SRCS
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose or res.returncode != 0:
        sys.stderr.write(res.stdout)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libhot.so")
    return LIB


if __name__ == "__main__":
    print(build_libhot(verbose=True))
