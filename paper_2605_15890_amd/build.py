"""Build paper_2605_15890_amd/libagc.so (HIP kernels + C ABI) for gfx950 with hipcc.

The library is built in-tree; nothing is compiled at import time.  Run
`python -m paper_2605_15890_amd.build` after changing a source under csrc/.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libagc.so")
SOURCES = ["agc_kernels.hip", "agc_ls_kernels.hip", "agc_api.cpp", "agc_host.cpp"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",            # every binary32 statement is one rounding; fma only where written
    "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
    "-Wall", "-Wno-unused-function",
]


def hip_runtime_link_flags():
    """The process that loads libagc.so already holds PyTorch's own copy of the HIP runtime
    (its device memory and streams come from there), so the library must bind to that copy and
    not bring a second runtime into the process: link against the libamdhip64.so that ships
    inside the torch package, with the system ROCm directory as a fallback search path."""
    flags = ["-no-hip-rt"]
    try:
        import importlib.util
        spec = importlib.util.find_spec("torch")
        tlib = os.path.join(os.path.dirname(spec.origin), "lib") if spec and spec.origin else None
    except Exception:
        tlib = None
    if tlib and os.path.exists(os.path.join(tlib, "libamdhip64.so")):
        flags += ["-L" + tlib, "-Wl,-rpath," + tlib]
    flags += ["-L/opt/rocm/lib", "-Wl,-rpath,/opt/rocm/lib", "-lamdhip64"]
    return flags


def build(verbose: bool = True, extra=()) -> str:
    cmd = [HIPCC, *FLAGS, *extra, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB,
           *hip_runtime_link_flags()]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(extra=sys.argv[1:])
    print(LIB)
