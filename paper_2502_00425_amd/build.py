"""Build libmquant.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

hipcc cross-compiles without a GPU.  Flags: no FMA contraction and no
fast-math, so the fp32 butterflies and the quantizer multiply are single IEEE
operations; packed-fp32 instructions are switched off.
"""
import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIB_DIR, "libmquant.so")
SOURCES = ["aifs.hip", "hadamard_quant.hip", "w4a8_gemm.hip", "w4a8_gemv.hip", "attention.hip",
           "w4g128_gemm.hip"]
# The benchmark's measurement probes: their own shared object, outside the product's ABI.
PROBES_LIB = os.path.join(LIB_DIR, "libmquant_probes.so")
PROBES_SOURCES = ["probes.hip"]
HEADERS = ["mquant_internal.h", "hadamard_segment.h", "w4a8_common.h", "lds_dma.h", "probes.h"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-inline-asm",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def _deps(srcs):
    return ([os.path.join(CSRC, s) for s in srcs] + [os.path.join(CSRC, h) for h in HEADERS]
            + [os.path.join(ROOT, "include", "mquant.h")])


def source_hash(srcs=None) -> str:
    """Hash of the sources, headers and compiler flags a library is built from.  It is
    compiled into libmquant.so (mquant_build_id) and written next to each library, so that
    staleness is judged by content: file times do not survive every copy of the tree."""
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for d in _deps(SOURCES if srcs is None else srcs):
        h.update(os.path.basename(d).encode())
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def _stale(lib, srcs) -> bool:
    if not os.path.exists(lib) or not os.path.exists(lib + ".id"):
        return True
    with open(lib + ".id") as f:
        return f.read().strip() != source_hash(srcs)


def is_stale() -> bool:
    """True when a library is missing or was built from other sources, headers or flags."""
    return _stale(LIB, SOURCES) or _stale(PROBES_LIB, PROBES_SOURCES)


def _compile(lib, srcs, verbose):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    build_id = source_hash(srcs)
    cmd = [hipcc, *HIPCC_FLAGS, f'-DMQUANT_BUILD_ID="{build_id}"', "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, *[os.path.join(CSRC, s) for s in srcs], "-o", lib]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass prints a harmless "not a recognized feature" line per file
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    with open(lib + ".id", "w") as f:
        f.write(build_id + "\n")


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile libmquant.so and libmquant_probes.so; with force=False only what is stale."""
    os.makedirs(LIB_DIR, exist_ok=True)
    if force or _stale(LIB, SOURCES):
        _compile(LIB, SOURCES, verbose)
    if force or _stale(PROBES_LIB, PROBES_SOURCES):
        _compile(PROBES_LIB, PROBES_SOURCES, verbose)
    return LIB


def ensure_fresh() -> str:
    """What tests, the smoke run and the benchmark call before loading the library: rebuild
    when the sources differ from what the binary was built from, so an edited kernel is never
    checked against an older build.  Where no compiler is present a stale library is an error."""
    if is_stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        if os.path.exists(hipcc):
            build(force=False)
        else:
            raise RuntimeError("libmquant.so is missing or stale and there is no hipcc to build it")
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
