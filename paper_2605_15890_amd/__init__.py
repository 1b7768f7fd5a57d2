"""MI355X-native hot path of communication-efficient approximate gradient coding:
encode -> stochastic quantize + bit-pack -> masked dequantize + weighted decode.

The compute lives in hand-written HIP kernels behind a C ABI (include/agc.h, built into
paper_2605_15890_amd/libagc.so); `api` is the thin ctypes binding.  Importing this package
does not load the library; `api.load()` does, and fails loudly when it is missing.
"""
__all__ = ["api", "inputs", "build"]
