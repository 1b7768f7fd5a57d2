// Launch interface between the C ABI (agc_api.cpp) and the gfx950 kernels (agc_kernels.hip).
// Plain structs only; every pointer is a device pointer unless it sits inside an argument
// block, which travels to the GPU as kernel arguments.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace agc {

constexpr int kArgWorkers = 256;

struct CodeDev {          // the code matrix B on the device
    const int* row_ptr;   // [n+1]
    const int* col;       // [nnz]
    const float* val;     // [nnz]
    int band;             // 0: generic CSR; s>0: cyclic band with s entries per row
};

struct Workspace {
    float* part_max;      // [nseg][n]   per-segment max |f_i|            (max-abs scale)
    double* part_sq;      // [nseg][n]   per-segment sum of squares       (Euclidean scale)
    double* group_sq;     // [n][ngroup]
    double* super_sq;     // [n][nsuper]
    float* inv16;         // [n]         L_i * 2^16 / scale_i
    int64_t nseg, ngroup, nsuper;
};

struct PerWorkerBits {
    uint8_t bits[kArgWorkers];
};

struct QuantStreams {
    void* codes[kArgWorkers];
    uint8_t bits[kArgWorkers];
};

struct DecodeStreams {
    const void* codes[kArgWorkers];
    float w[kArgWorkers];
    uint8_t bits[kArgWorkers];
    uint8_t mask[kArgWorkers];
};

// K1: per-segment partials of every worker's scale.  scale_mode: 0 Euclidean, 1 max-abs.
hipError_t launch_scale_pass(const float* G, int64_t ldg, int n, int k, int64_t d,
                             const CodeDev& code, int scale_mode, const Workspace& ws,
                             hipStream_t stream);
// K1f: partials -> scales[n] and inv16[n].
hipError_t launch_scale_finalize(int n, int scale_mode, const PerWorkerBits& bits,
                                 const Workspace& ws, float* scales, hipStream_t stream);
// K2: fused encode + stochastic quantize + bit-pack.
hipError_t launch_quantize(const float* G, int64_t ldg, int n, int k, int64_t d,
                           const CodeDev& code, const Workspace& ws, uint64_t seed, uint64_t step,
                           const QuantStreams& out, hipStream_t stream);
// K3: masked dequantize + weighted sum.
hipError_t launch_decode(int n, int64_t d, const DecodeStreams& in, const float* scales,
                         float* ghat, hipStream_t stream);

}  // namespace agc
