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
SOURCES = ["agc_kernels.hip", "agc_quantize_b0s.hip", "agc_quantize_b0m.hip", "agc_quantize_b1s.hip",
           "agc_quantize_b1m.hip", "agc_quantize_b2s.hip", "agc_quantize_b2m.hip",
           "agc_ls_kernels.hip", "agc_debug.hip", "agc_api.cpp", "agc_host.cpp"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
OBJ_DIR = os.path.join(HERE, "_build")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
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


def _newest_input():
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "agc.h"), os.path.join(HERE, "..", "include", "agc_debug.h")]
    return max(os.path.getmtime(f) for f in deps)


def build(verbose: bool = True, extra=(), incremental: bool = False) -> str:
    """Compiles every source to an object (in parallel) and links libagc.so.  incremental=True
    skips objects that are newer than every file under csrc/ and the public header (a
    convenience while editing; the default compiles everything)."""
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(OBJ_DIR, exist_ok=True)
    newest = _newest_input()
    jobs = []
    for src in SOURCES:
        obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
        if incremental and not extra and os.path.exists(obj) and os.path.getmtime(obj) > newest:
            continue
        jobs.append([HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    with ThreadPoolExecutor(max_workers=8) as pool:
        list(pool.map(run, jobs))
    objs = [os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o") for src in SOURCES]
    run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB, *hip_runtime_link_flags()])
    return LIB


HOST_SAN_LIB = os.path.join(OBJ_DIR, "libagc_host_san.so")


def build_host_sanitized() -> str:
    """The host-only design routines (csrc/agc_host.cpp: bit allocation, code construction) as a
    library of their own, compiled with plain g++ under AddressSanitizer and
    UndefinedBehaviorSanitizer.  CPU only; no HIP code is involved."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-Wall",
           os.path.join(CSRC, "agc_host.cpp"), "-o", HOST_SAN_LIB]
    subprocess.run(cmd, check=True)
    return HOST_SAN_LIB


if __name__ == "__main__":
    args = sys.argv[1:]
    inc = "--incremental" in args
    build(extra=[a for a in args if a != "--incremental"], incremental=inc)
    print(LIB)
