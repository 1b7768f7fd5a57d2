// Measurement kernels (include/agc_debug.h): a plain copy of known traffic and the bare access
// pattern of the two streaming passes.  Not part of the method.
#include "agc_device.h"
#include "agc_kernels.h"

namespace agc {

// =======================================================================================
// counter calibration: a copy that moves exactly `bytes` in and `bytes` out
// =======================================================================================
__global__ __launch_bounds__(kWgThreads) void k_calibration_copy(const float4* __restrict__ src,
                                                                 float4* __restrict__ dst, int64_t n16)
{
    const int64_t i = (int64_t)blockIdx.x * kWgThreads + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

hipError_t launch_calibration_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream)
{
    const int64_t n16 = bytes / 16;
    const unsigned grid = (unsigned)((n16 + kWgThreads - 1) / kWgThreads);
    hipLaunchKernelGGL(k_calibration_copy, dim3(grid), dim3(kWgThreads), 0, stream,
                       static_cast<const float4*>(src), static_cast<float4*>(dst), n16);
    return hipGetLastError();
}

// =======================================================================================
// access pattern of the scale pass (reads) and the quantize pass (reads + one small piece per
// row and wave into the row's own output stream)
// =======================================================================================
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) f32x4_t* global_f32x4_w;

// WRITE 0: reads only.  1: every wave writes `pieces` 16-byte pieces to the row's stream right after
// the row.  2: nothing is written until the workgroup has walked all rows; then, after one barrier,
// its four blocks' pieces of every row leave as 4 * pieces contiguous pieces (whole, aligned lines).
// V: neighbouring blocks a wave walks at once (V loads per row, 1 KiB apart); reads-only form.
template <int WRITE, int V>
__global__ __launch_bounds__(kWgThreads) void k_stream_rows(const float* __restrict__ G, int64_t ldg, int k,
                                                            int64_t nblocks, int pieces, f32x4_t* out)
{
    static_assert(V == 1 || WRITE == 0, "several blocks per wave: reads only");
    constexpr int P = V == 1 ? 4 : 2;  // rows in flight, as in the passes
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    const int64_t block = ((int64_t)blockIdx.x * kWavesPerWg + wave) * V;  // the wave's first block
    const int64_t stream_pieces = nblocks * pieces;  // 16-byte pieces per output stream
    float acc = 0.f;
    float4 last = make_float4(0.f, 0.f, 0.f, 0.f);
    if (block + V <= nblocks) {
        LaneCoords lc;
        lc.lane4 = lane;
        lc.byte_off = 16u * (uint32_t)lane;
        lc.nvalid = 4;
        lc.wave_ragged = false;
        const float* row = G + block * (int64_t)kBlockCoords;
        float4 ring[P][V];
#pragma unroll
        for (int r = 0; r < P; ++r)
#pragma unroll
            for (int v = 0; v < V; ++v)
                ring[r][v] = load_row4<false, true>(row + (int64_t)(r < k ? r : k - 1) * ldg + v * kBlockCoords, lc);
        for (int j0 = 0; j0 < k; j0 += P) {
#pragma unroll
            for (int r = 0; r < P; ++r) {
                const int j = j0 + r;
                if (j >= k) break;
                float4 cur[V];
#pragma unroll
                for (int v = 0; v < V; ++v) cur[v] = ring[r][v];
                if (j + P < k) {
#pragma unroll
                    for (int v = 0; v < V; ++v)
                        ring[r][v] = load_row4<false, true>(row + (int64_t)(j + P) * ldg + v * kBlockCoords, lc);
                }
#pragma unroll
                for (int v = 0; v < V; ++v)
                    acc = fmaxf(acc, fmaxf(fmaxf(cur[v].x, cur[v].y), fmaxf(cur[v].z, cur[v].w)));
                last = cur[0];
                if (WRITE == 1 && lane < pieces)
                    __builtin_nontemporal_store(f32x4_t{last.x, last.y, last.z, last.w},
                                                (global_f32x4_w)(out + (int64_t)j * stream_pieces + block * pieces + lane));
            }
        }
    }
    if (WRITE == 2) {
        __syncthreads();
        const int64_t first = (int64_t)blockIdx.x * kWavesPerWg;           // first block of the workgroup
        const int64_t left = nblocks - first;
        const int per_row = pieces * (int)(left < kWavesPerWg ? left : kWavesPerWg);
        const int total = k * per_row;
        for (int q = threadIdx.x; q < total; q += kWgThreads) {
            const int j = q / per_row, r = q - j * per_row;
            __builtin_nontemporal_store(f32x4_t{last.x, last.y, last.z, last.w},
                                        (global_f32x4_w)(out + (int64_t)j * stream_pieces + first * pieces + r));
        }
    }
    if (acc == 1.2345678e37f) out[0] = f32x4_t{acc, acc, acc, acc};  // keeps the loads alive; never true for finite data in practice
}

hipError_t launch_stream_rows(const float* G, int64_t ldg, int k, int64_t d, int piece_bytes, int wg_flush,
                              int blocks_per_wave, void* out, hipStream_t stream)
{
    const int64_t nblocks = d / kBlockCoords;
    const int64_t units = nblocks / blocks_per_wave;  // whole runs of blocks_per_wave blocks
    if (units == 0) return hipSuccess;
    const unsigned grid = (unsigned)((units + kWavesPerWg - 1) / kWavesPerWg);
    f32x4_t* o = static_cast<f32x4_t*>(out);
    if (blocks_per_wave == 2)
        hipLaunchKernelGGL((k_stream_rows<0, 2>), dim3(grid), dim3(kWgThreads), 0, stream, G, ldg, k, nblocks, 0, o);
    else if (piece_bytes == 0)
        hipLaunchKernelGGL((k_stream_rows<0, 1>), dim3(grid), dim3(kWgThreads), 0, stream, G, ldg, k, nblocks, 0, o);
    else if (!wg_flush)
        hipLaunchKernelGGL((k_stream_rows<1, 1>), dim3(grid), dim3(kWgThreads), 0, stream, G, ldg, k, nblocks,
                           piece_bytes / 16, o);
    else
        hipLaunchKernelGGL((k_stream_rows<2, 1>), dim3(grid), dim3(kWgThreads), 0, stream, G, ldg, k, nblocks,
                           piece_bytes / 16, o);
    return hipGetLastError();
}

}  // namespace agc
