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
// OCC: 0, or the number of waves per SIMD the kernel is built for (the quantize pass runs with four).
// FMA: dummy arithmetic between the rows, FMA dependent multiply-adds per row and lane, unrolled (a
// loop of unknown length between the loads would make the compiler wait for all of them); the
// quantize pass issues about ninety vector instructions per row and lane.
template <int WRITE, int V, int OCC, int FMA>
__global__ __launch_bounds__(kWgThreads) __attribute__((amdgpu_waves_per_eu(OCC == 0 ? 1 : OCC, OCC == 0 ? 8 : OCC)))
void k_stream_rows(const float* __restrict__ G, int64_t ldg, int k, int64_t nblocks, int pieces, f32x4_t* out)
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
                last = cur[0];
#pragma unroll
                for (int v = 0; v < V; ++v) {
#pragma unroll
                    for (int it = 0; it < FMA / 4; ++it) {  // each round feeds the next
                        cur[v].x = fmaf(cur[v].x, 1.0001f, cur[v].y);
                        cur[v].y = fmaf(cur[v].y, 0.9999f, cur[v].z);
                        cur[v].z = fmaf(cur[v].z, 1.0002f, cur[v].w);
                        cur[v].w = fmaf(cur[v].w, 0.9998f, cur[v].x);
                    }
                    acc = fmaxf(acc, fmaxf(fmaxf(cur[v].x, cur[v].y), fmaxf(cur[v].z, cur[v].w)));
                }
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

template <int WRITE, int V, int OCC, int FMA>
static void launch_stream_rows_as(unsigned grid, hipStream_t stream, const float* G, int64_t ldg, int k,
                                  int64_t nblocks, int pieces, f32x4_t* o)
{
    hipLaunchKernelGGL((k_stream_rows<WRITE, V, OCC, FMA>), dim3(grid), dim3(kWgThreads), 0, stream, G, ldg, k, nblocks,
                       pieces, o);
}

hipError_t launch_stream_rows(const float* G, int64_t ldg, int k, int64_t d, int piece_bytes, int wg_flush,
                              int blocks_per_wave, int waves_per_simd, int fma_per_row, void* out, hipStream_t stream)
{
    const int64_t nblocks = d / kBlockCoords;
    const int64_t units = nblocks / blocks_per_wave;  // whole runs of blocks_per_wave blocks
    if (units == 0) return hipSuccess;
    const unsigned grid = (unsigned)((units + kWavesPerWg - 1) / kWavesPerWg);
    f32x4_t* o = static_cast<f32x4_t*>(out);
    const int pieces = piece_bytes / 16;
    const bool four = waves_per_simd == 4;
    if (fma_per_row != 0) {  // arithmetic stand-in: the quantize pass's form only
        if (!four || !wg_flush || piece_bytes == 0 || blocks_per_wave != 1) return hipErrorInvalidValue;
        if (fma_per_row == 40) launch_stream_rows_as<2, 1, 4, 40>(grid, stream, G, ldg, k, nblocks, pieces, o);
        else if (fma_per_row == 100) launch_stream_rows_as<2, 1, 4, 100>(grid, stream, G, ldg, k, nblocks, pieces, o);
        else return hipErrorInvalidValue;
    } else if (blocks_per_wave == 2) {
        if (four) launch_stream_rows_as<0, 2, 4, 0>(grid, stream, G, ldg, k, nblocks, 0, o);
        else launch_stream_rows_as<0, 2, 0, 0>(grid, stream, G, ldg, k, nblocks, 0, o);
    } else if (piece_bytes == 0) {
        if (four) launch_stream_rows_as<0, 1, 4, 0>(grid, stream, G, ldg, k, nblocks, 0, o);
        else launch_stream_rows_as<0, 1, 0, 0>(grid, stream, G, ldg, k, nblocks, 0, o);
    } else if (!wg_flush) {
        if (four) launch_stream_rows_as<1, 1, 4, 0>(grid, stream, G, ldg, k, nblocks, pieces, o);
        else launch_stream_rows_as<1, 1, 0, 0>(grid, stream, G, ldg, k, nblocks, pieces, o);
    } else {
        if (four) launch_stream_rows_as<2, 1, 4, 0>(grid, stream, G, ldg, k, nblocks, pieces, o);
        else launch_stream_rows_as<2, 1, 0, 0>(grid, stream, G, ldg, k, nblocks, pieces, o);
    }
    return hipGetLastError();
}

}  // namespace agc
