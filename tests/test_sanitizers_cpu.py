"""Sanitizer passes over host code (CPU only).

* the compiled oracle, instrumented with AddressSanitizer and UBSan, driven by
  tests/sanitize/oracle_driver.c (always runs: a few seconds);
* the host side of the library (argument checks, planner, debug switches), instrumented the
  same way, driven by tests/sanitize/host_driver.cpp.  Building the instrumented library takes
  as long as the normal build, so this one only runs when LA_SANITIZE_HOST=1 is set."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-fopenmp"] + SAN + ["-o", exe, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                                             os.path.join(ROOT, "oracle", "la_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(ENV, OMP_NUM_THREADS="4")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    sys.stdout.write(res.stdout)
    sys.stderr.write(res.stderr)
    assert res.returncode == 0 and "oracle sanitizer driver: ok" in res.stdout


@pytest.mark.skipif(os.environ.get("LA_SANITIZE_HOST") != "1",
                    reason="builds a second, instrumented copy of the library: set LA_SANITIZE_HOST=1 to run")
def test_library_host_code_under_address_and_ub_sanitizers(tmp_path):
    from paper_2405_17381_amd import build as _b
    lib = str(tmp_path / "libla_san.so")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    host_san = []
    for flag in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"):
        host_san += ["-Xarch_host", flag]
    cmd = [hipcc] + _b.HIPCC_FLAGS + host_san + ["-o", lib] + _b.SOURCES
    subprocess.run(cmd, check=True, capture_output=True)
    exe = str(tmp_path / "host_san")
    clangxx = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "llvm", "bin", "clang++")
    cmd = [clangxx, "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
           "-fno-sanitize-recover=undefined",
           os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), "-o", exe, lib,
           "-Wl,-rpath," + str(tmp_path)]
    subprocess.run(cmd, check=True, capture_output=True)
    res = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    sys.stdout.write(res.stdout)
    sys.stderr.write(res.stderr)
    assert res.returncode == 0 and "host sanitizer driver: ok" in res.stdout
