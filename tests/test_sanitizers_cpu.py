"""Host-side code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU (no GPU is touched):

* the C oracle: a driver program calls every oracle function on exactly sized heap buffers and checks
  closed-form values (tests/sanitize/oracle_driver.c), built with gcc -fsanitize=address,undefined;
* the Python oracle pins once more against an oracle library built with -fsanitize=undefined (trapping);
* libhot's host code: the argument validation of every entry point and the host-only queries
  (tests/sanitize/abi_driver.c) against a build of the library whose host side is instrumented (the device
  code is compiled without optimisation and never runs here).
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ORACLE_SRCS = sorted(os.path.join(ROOT, "oracle", f) for f in os.listdir(os.path.join(ROOT, "oracle")) if f.endswith(".c"))


def _run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert res.returncode == 0, " ".join(cmd[:4]) + " ...\n" + res.stdout[-4000:]
    return res.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          "-static-libasan", "-static-libubsan", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra", "-o", exe,
          os.path.join(SAN, "oracle_driver.c")] + ORACLE_SRCS + ["-lm"])
    out = _run([exe], env={**os.environ, "ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "OMP_NUM_THREADS": "4"})
    assert "oracle driver ok" in out


def test_oracle_pins_pass_with_trapping_undefined_behaviour_checks(tmp_path):
    """The pins of tests/test_*oracle_pins.py run again in a child interpreter whose oracle library is built
    with -fsanitize=undefined -fsanitize-trap (signed overflow, misaligned access, out-of-range shifts and
    conversions end the process)."""
    lib = str(tmp_path / "libbbb_oracle_ubsan.so")
    _run(["gcc", "-std=c99", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fsanitize=undefined",
          "-fsanitize-undefined-trap-on-error", "-shared", "-fPIC", "-o", lib] + ORACLE_SRCS + ["-lm"])
    pins = sorted(os.path.join(ROOT, "tests", f) for f in os.listdir(os.path.join(ROOT, "tests")) if f.endswith("oracle_pins.py"))
    out = _run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + pins,
               env={**os.environ, "BBB_ORACLE_LIB": lib}, cwd=ROOT)
    assert " passed" in out and "failed" not in out, out[-2000:]


def test_libhot_host_code_under_sanitizers(tmp_path):
    from paper_2604_04736_amd import build
    flags = ["--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Xarch_device", "-O0", "-Xarch_host", "-O1", "-Xarch_host", "-g",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "include")]
    objs = [str(tmp_path / (os.path.basename(s) + ".o")) for s in build.SRCS]
    with ThreadPoolExecutor(max_workers=len(objs)) as pool:
        list(pool.map(lambda so: _run([build.HIPCC] + flags + ["-c", "-o", so[1], so[0]]), zip(build.SRCS, objs)))
    lib = str(tmp_path / "libhot_san.so")
    _run([build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-o", lib] + objs)
    clang = os.path.join(os.path.dirname(os.path.realpath(build.HIPCC)), "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    exe = str(tmp_path / "abi_driver")
    _run([clang, "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          "-I", os.path.join(ROOT, "include"), "-o", exe, os.path.join(SAN, "abi_driver.c"), lib,
          "-Wl,-rpath," + str(tmp_path)])
    # the HIP runtime's own start-up allocations are not this library's: leak checking stays off
    out = _run([exe], env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0"})
    assert "abi driver ok" in out
