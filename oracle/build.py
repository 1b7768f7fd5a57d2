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


SAN_LIB = os.path.join(HERE, "libagc_oracle_san.so")
SAN_FLAGS = ["-O1", "-g", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math", "-mfma",
             "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-fno-omit-frame-pointer", "-Wall", "-Wextra"]


def build_sanitized() -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; the
    process that loads it needs libasan preloaded, see sanitizer_runtime())."""
    subprocess.run(["gcc", *SAN_FLAGS, SRC, "-o", SAN_LIB, "-lm"], check=True)
    return SAN_LIB


def sanitizer_runtime() -> str:
    """Path of gcc's libasan.so, to be put first in LD_PRELOAD of a process that loads a sanitized library."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()


if __name__ == "__main__":
    print(build_sanitized() if "--sanitize" in sys.argv else build(force="--force" in sys.argv))
