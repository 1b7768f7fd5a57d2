"""Compile the C oracle into oracle/libagc_oracle.so with gcc.

Test infrastructure only.  Flags: no contraction, no fast-math, so that every
binary32 statement of the C source is one IEEE rounding; -mfma only makes
fmaf() a single instruction (it is a fused operation by definition either way).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "agc_oracle.c")
LIB = os.path.join(HERE, "libagc_oracle.so")

FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
         "-mfma", "-fopenmp", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", *FLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
