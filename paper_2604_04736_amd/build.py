"""Compiles csrc/*.hip into libhot.so next to this file (hipcc, gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(HERE, "csrc", name) for name in ("forward.hip", "backward.hip", "hot.hip", "stats.hip", "linear.hip", "update.hip")]
LIB = os.path.join(HERE, "libhot.so")
OBJ_DIR = os.path.join(HERE, "_build")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed fp32 arithmetic is switched off for all device code of this library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-I", os.path.join(ROOT, "include")]


def _run(cmd, verbose):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose or res.returncode != 0:
        sys.stderr.write(res.stdout)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libhot.so: " + " ".join(cmd[-3:]))


def build_libhot(verbose: bool = False) -> str:
    """One object per source file, compiled side by side, then one link."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, os.path.basename(src) + ".o") for src in SRCS]
    with ThreadPoolExecutor(max_workers=len(SRCS)) as pool:
        list(pool.map(lambda so: _run([HIPCC] + FLAGS + ["-c", "-o", so[1], so[0]], verbose), zip(SRCS, objs)))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, verbose)
    return LIB


if __name__ == "__main__":
    print(build_libhot(verbose=True))
