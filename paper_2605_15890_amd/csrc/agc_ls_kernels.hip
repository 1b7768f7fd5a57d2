// Partial gradients of the least-squares loss for the end-to-end loop: for every data
// partition p (Sec. II-A: g_j = grad L(D_j, beta)),  G[p,:] = X_p^T (X_p w - y_p),
// X in bfloat16 (row-major, n_rows x n_feat), everything else binary32.
//
// One kernel, two sweeps per block of 16 samples:
//   sweep 1  r = X_blk w - y_blk  on the matrix cores: v_mfma_f32_16x16x32_bf16 with the 16
//            samples as M, 32 features as K, and the N columns holding the exact three-way
//            bfloat16 split of the binary32 vector w (w = hi + mid + lo), so that the products
//            are exact and only the binary32 accumulation rounds.  The four waves of the
//            workgroup split the feature range; their partial tiles meet in LDS.
//   sweep 2  g += X_blk^T r  on the vector ALUs: a lane owns 16 features, the 16 residuals are
//            broadcast from LDS; the block is re-read right after sweep 1, i.e. from L2 /
//            Infinity Cache, so HBM sees X once.
// A workgroup walks over a contiguous range of blocks of ONE partition and keeps its part of g
// in registers; a second small kernel adds the workgroups' parts in a fixed order, so the result
// does not depend on scheduling.  The whole stage is bound by the single HBM read of X.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "agc_kernels.h"

namespace agc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kLsThreads = 256;
constexpr int kLsWaves = 4;
constexpr int kLsRows = 16;        // samples per block (M of the MFMA tile)
constexpr int kLsMaxFeat = 8192;   // features handled per workgroup: 2 chunks of 16 per lane

struct LsArgs {
    int64_t n_rows;
    int n_feat;
    int k_parts;
    int wg_per_part;
    int64_t rows_per_part;
    float* resid;    // [n_rows]  r = X w - y
    float* partial;  // [k_parts * wg_per_part][n_feat]
};

__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }

__global__ __launch_bounds__(kLsThreads) void k_ls_partial(const uint16_t* __restrict__ X,
                                                           const float* __restrict__ y,
                                                           const float* __restrict__ w, LsArgs a)
{
    extern __shared__ uint16_t lds_w3[];  // [3][n_feat] bfloat16 pieces of w
    __shared__ float lds_part[kLsWaves][kLsRows];
    __shared__ float lds_r[kLsRows];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int lane = tid % 64;
    const int F = a.n_feat;
    const int part = blockIdx.x / a.wg_per_part;
    const int q = blockIdx.x % a.wg_per_part;

    // exact split w = hi + mid + lo into three bfloat16 numbers (truncation at each step leaves a
    // remainder with eight fewer significant bits, so the third piece is exact)
    for (int f = tid; f < F; f += kLsThreads) {
        const float wf = w[f];
        const float hi = __uint_as_float(__float_as_uint(wf) & 0xFFFF0000u);
        const float rem = wf - hi;
        const float mid = __uint_as_float(__float_as_uint(rem) & 0xFFFF0000u);
        const float lo = rem - mid;
        lds_w3[f] = (uint16_t)(__float_as_uint(hi) >> 16);
        lds_w3[F + f] = (uint16_t)(__float_as_uint(mid) >> 16);
        lds_w3[2 * F + f] = (uint16_t)(__float_as_uint(lo) >> 16);
    }
    __syncthreads();

    float acc[2][16];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;

    const int64_t blocks_per_part = a.rows_per_part / kLsRows;
    const int64_t b0 = blocks_per_part * q / a.wg_per_part;
    const int64_t b1 = blocks_per_part * (q + 1) / a.wg_per_part;
    const int m = lane % 16, kq = lane / 16;           // MFMA operand coordinates of this lane
    const int fw0 = wave * (F / kLsWaves), fw1 = fw0 + F / kLsWaves;

    for (int64_t blk = b0; blk < b1; ++blk) {
        const int64_t row0 = (int64_t)part * a.rows_per_part + blk * kLsRows;
        // ---- sweep 1: residuals on the matrix cores
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
        const uint16_t* xrow = X + (row0 + m) * F + 8 * kq;
        const uint16_t* wcol = lds_w3 + (m < 3 ? m : 0) * F + 8 * kq;
        for (int kk = fw0; kk < fw1; kk += 32) {
            const uint4 xa = *reinterpret_cast<const uint4*>(xrow + kk);
            uint4 wb = *reinterpret_cast<const uint4*>(wcol + kk);
            if (m >= 3) wb = make_uint4(0u, 0u, 0u, 0u);  // only three of the sixteen columns carry data
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa),
                                                        __builtin_bit_cast(bf16x8, wb), d, 0, 0, 0);
        }
        // lane holds D[rows 4*kq .. 4*kq+3][column m]; columns 0,1,2 are the three pieces of w
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float c1 = __shfl_down(d[e], 1, 64), c2 = __shfl_down(d[e], 2, 64);
            if (m == 0) lds_part[wave][4 * kq + e] = (d[e] + c1) + c2;
        }
        __syncthreads();
        if (tid < kLsRows) {
            const float s = ((lds_part[0][tid] + lds_part[1][tid]) + lds_part[2][tid]) + lds_part[3][tid];
            const float r = s - y[row0 + tid];
            lds_r[tid] = r;
            a.resid[row0 + tid] = r;
        }
        __syncthreads();
        // ---- sweep 2: g += X_blk^T r on the vector ALUs (the block comes back from cache)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int f0 = c * (kLsThreads * 16) + tid * 16;
            if (f0 < F) {
#pragma unroll 4
                for (int rr = 0; rr < kLsRows; ++rr) {
                    const float r = lds_r[rr];
                    const uint4* px = reinterpret_cast<const uint4*>(X + (row0 + rr) * F + f0);
                    const uint4 u0 = px[0], u1 = px[1];
                    const uint32_t uu[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        acc[c][2 * e] = fmaf(bf16_lo(uu[e]), r, acc[c][2 * e]);
                        acc[c][2 * e + 1] = fmaf(bf16_hi(uu[e]), r, acc[c][2 * e + 1]);
                    }
                }
            }
        }
        __syncthreads();  // lds_part / lds_r are rewritten by the next block
    }
    float* out = a.partial + (int64_t)blockIdx.x * F;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int f0 = c * (kLsThreads * 16) + tid * 16;
        if (f0 < F) {
#pragma unroll
            for (int e = 0; e < 16; e += 4)
                *reinterpret_cast<float4*>(out + f0 + e) =
                    make_float4(acc[c][e], acc[c][e + 1], acc[c][e + 2], acc[c][e + 3]);
        }
    }
}

// G[p][f] = sum over the partition's workgroups, in workgroup order
__global__ __launch_bounds__(kLsThreads) void k_ls_reduce(const float* __restrict__ partial, int n_feat,
                                                          int wg_per_part, float* G, int64_t ldg)
{
    const int p = blockIdx.y;
    const int f = blockIdx.x * kLsThreads + threadIdx.x;
    if (f >= n_feat) return;
    float s = 0.f;
    for (int qq = 0; qq < wg_per_part; ++qq) s = s + partial[((int64_t)p * wg_per_part + qq) * n_feat + f];
    G[(int64_t)p * ldg + f] = s;
}

__global__ __launch_bounds__(kLsThreads) void k_gd_update(float* beta, const float* __restrict__ ghat,
                                                          float lr, int64_t d)
{
    const int64_t i = (int64_t)blockIdx.x * kLsThreads + threadIdx.x;
    if (i < d) beta[i] = fmaf(-lr, ghat[i], beta[i]);
}

int ls_wg_per_part(int64_t n_rows, int k_parts)
{
    const int64_t blocks = n_rows / k_parts / kLsRows;
    int64_t want = 1024 / (k_parts > 0 ? k_parts : 1);  // about four workgroups per compute unit
    if (want < 1) want = 1;
    return (int)(blocks < want ? blocks : want);
}

hipError_t launch_ls_partial_gradients(const void* X, int64_t n_rows, int n_feat, const float* y,
                                       const float* w, int k_parts, float* G, int64_t ldg,
                                       float* resid, float* partial, hipStream_t stream)
{
    LsArgs a{n_rows, n_feat, k_parts, ls_wg_per_part(n_rows, k_parts), n_rows / k_parts, resid, partial};
    const size_t lds = (size_t)3 * n_feat * sizeof(uint16_t);
    hipLaunchKernelGGL(k_ls_partial, dim3((unsigned)(k_parts * a.wg_per_part)), dim3(kLsThreads), lds, stream,
                       static_cast<const uint16_t*>(X), y, w, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_ls_reduce, dim3((unsigned)((n_feat + kLsThreads - 1) / kLsThreads), (unsigned)k_parts),
                       dim3(kLsThreads), 0, stream, partial, n_feat, a.wg_per_part, G, ldg);
    return hipGetLastError();
}

hipError_t launch_gd_update(float* beta, const float* ghat, float lr, int64_t d, hipStream_t stream)
{
    hipLaunchKernelGGL(k_gd_update, dim3((unsigned)((d + kLsThreads - 1) / kLsThreads)), dim3(kLsThreads), 0,
                       stream, beta, ghat, lr, d);
    return hipGetLastError();
}

}  // namespace agc
