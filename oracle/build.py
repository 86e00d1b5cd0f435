"""Compile the C part of the oracle with gcc into oracle/libmquant_oracle.so.

Flags matter for parity: no fast-math, no FMA contraction, so every fp32
add/sub/multiply in the oracle is one IEEE round-to-nearest-even operation.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "mquant_oracle.c")
LIB = os.path.join(HERE, "libmquant_oracle.so")

CFLAGS = ["-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
          "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", *CFLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
