"""CPU-only sanitizer runs: the C part of the oracle (gcc) and the host side of the C ABI (the
library's own sources, hipcc with the sanitizers on the host pass only) are built with
AddressSanitizer + UndefinedBehaviorSanitizer and exercised by small drivers under
tests/sanitize/.  No GPU code runs; GPU sanitizers are not used."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
OUT = os.path.join(ROOT, "_build", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="4")


def _run(exe):
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, r.stdout[-4000:]
    return r.stdout


def test_oracle_c_under_asan_and_ubsan():
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_driver")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra",
           os.path.join(ROOT, "oracle", "mquant_oracle.c"), os.path.join(SAN, "oracle_driver.c"), "-o", exe, "-lm"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    assert "oracle sanitizer run ok" in _run(exe)


def test_abi_host_paths_under_asan_and_ubsan():
    """The library's host code (validation, index builder, scale, dispatch planning) with the
    sanitizers on the host pass; the build is kept per source hash since it compiles every kernel."""
    from paper_2502_00425_amd import build as hip_build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "abi_driver_" + hip_build.source_hash())
    driver = os.path.join(SAN, "abi_driver.cpp")
    if not os.path.exists(exe) or os.path.getmtime(exe) < os.path.getmtime(driver):
        for old in os.listdir(OUT):
            if old.startswith("abi_driver_"):
                os.remove(os.path.join(OUT, old))
        flags = [f for f in hip_build.HIPCC_FLAGS if f not in ("-shared", "-O3")]
        cmd = [hipcc, *flags, "-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
               "-Xarch_host", "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"), "-I", hip_build.CSRC,
               *hip_build.sources(), "-x", "hip", driver, "-o", exe]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        assert r.returncode == 0, out[-4000:]
    assert "abi host sanitizer run ok" in _run(exe)
