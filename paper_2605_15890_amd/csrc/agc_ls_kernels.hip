// Partial gradients of the least-squares loss for the end-to-end loop: for every data
// partition p (Sec. II-A: g_j = grad L(D_j, beta)),  G[p,:] = X_p^T (X_p w - y_p),
// X in bfloat16 (row-major, n_rows x n_feat), everything else binary32.
//
// The stage is bound by the single HBM read of X (about one flop per byte), so the design keeps a
// block of 16 samples in REGISTERS between its two uses:
//   sweep 1  r = X_blk w - y_blk   (contraction over features)
//   sweep 2  g += X_blk^T r        (contraction over samples)
// k_ls_resident<ROWS, NG>: a lane owns NG groups of eight features of all ROWS samples of the
// block, ROWS * NG = 32 (16 samples x 16 features for n_feat <= 4096, 8 samples x 32 features for
// n_feat <= 8192): 128 VGPRs of packed bfloat16.  Sweep 2 is then a plain per-lane FMA chain.
// Sweep 1 runs on the matrix cores: v_mfma_f32_16x16x32_bf16 with A = the lane's 8 features of
// one sample and B = the lane's own 8 entries of w; the diagonal D[i][i] is the sum over the four
// lanes (i, 0..3) of their own dot products, and the trace over the wave is the wave's share of
// the sample's residual.  w enters as its exact three-way bfloat16 split (w = hi + mid + lo), so
// the products are exact and only the binary32 accumulation rounds.  While sweep 2 consumes a
// sample's registers, the same registers are refilled with the next block's sample, which hides
// the load latency at two waves per SIMD.
// A workgroup walks over a contiguous range of blocks of ONE partition and keeps its part of g in
// registers; a second small kernel adds the workgroups' parts in a fixed order, so the result
// does not depend on scheduling.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "agc_device.h"
#include "agc_kernels.h"

namespace agc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kLsThreads = 256;
constexpr int kLsWaves = 4;
constexpr int kLsRows = 16;        // largest number of samples per block; n_rows is a multiple of it per partition


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

constexpr int kLsResidentFeat = 4096;  // 256 lanes x 16 features

// 16-bit patterns of the exact split wf = hi + mid + lo (truncation at each step leaves a remainder
// with eight fewer significant bits, so the third piece is exact)
__device__ __forceinline__ void split3_bf16(float wf, uint32_t& hi, uint32_t& mid, uint32_t& lo)
{
    const float fh = __uint_as_float(__float_as_uint(wf) & 0xFFFF0000u);
    const float rem = wf - fh;
    const float fm = __uint_as_float(__float_as_uint(rem) & 0xFFFF0000u);
    const float fl = rem - fm;
    hi = __float_as_uint(fh) >> 16;
    mid = __float_as_uint(fm) >> 16;
    lo = __float_as_uint(fl) >> 16;
}

__device__ __forceinline__ float row16_sum(float v)
{
    v = v + __uint_as_float(dpp_u32<kDppQuadSwap1>(__float_as_uint(v)));
    v = v + __uint_as_float(dpp_u32<kDppQuadSwap2>(__float_as_uint(v)));
    v = v + __uint_as_float(dpp_u32<kDppHalfMirror>(__float_as_uint(v)));
    v = v + __uint_as_float(dpp_u32<kDppRowMirror>(__float_as_uint(v)));
    return v;  // every lane of the 16-lane row holds the row's sum
}

// pointer held in scalar registers (the compiler then addresses rows as scalar base + 32-bit lane
// offset instead of one 64-bit address per lane and row)
typedef const __attribute__((address_space(1))) char* global_bytes;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* global_u4;

__device__ __forceinline__ global_bytes uniform_ptr(const void* p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (global_bytes)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ u32x4 load16(global_bytes row, uint32_t byte_off)
{
    // X is read exactly once per call: stream it past the caches (measured: 6.0 -> 6.8 TB/s)
    return __builtin_nontemporal_load((global_u4)(row + byte_off));
}

__device__ __forceinline__ void fma8(float* acc, const u32x4& u, float r)
{
    acc[0] = fmaf(bf16_lo(u.x), r, acc[0]);
    acc[1] = fmaf(bf16_hi(u.x), r, acc[1]);
    acc[2] = fmaf(bf16_lo(u.y), r, acc[2]);
    acc[3] = fmaf(bf16_hi(u.y), r, acc[3]);
    acc[4] = fmaf(bf16_lo(u.z), r, acc[4]);
    acc[5] = fmaf(bf16_hi(u.z), r, acc[5]);
    acc[6] = fmaf(bf16_lo(u.w), r, acc[6]);
    acc[7] = fmaf(bf16_hi(u.w), r, acc[7]);
}

// ROWS samples per block, NG groups of eight features per lane: ROWS * NG = 32 registers of four
// packed words hold the block (16 x 2 for up to 4096 features, 8 x 4 for up to 8192).
template <int ROWS, int NG>
__global__ __launch_bounds__(kLsThreads, 2) void k_ls_resident(const uint16_t* __restrict__ X,
                                                               const float* __restrict__ y,
                                                               const float* __restrict__ w, LsArgs a)
{
    static_assert(ROWS % 4 == 0 && ROWS * NG == 32, "the block must fill 128 registers");
    __shared__ float lds_part[4 * kLsWaves][ROWS];  // [wave * 4 + 16-lane row][sample]
    __shared__ float lds_r[ROWS];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int lane = tid % 64;
    const int F = a.n_feat, H = F / NG;
    const int part = blockIdx.x / a.wg_per_part;
    const int q = blockIdx.x % a.wg_per_part;
    // the lane's NG groups of eight features; lanes beyond the feature range read group 0 and
    // carry zero pieces of w, so they add nothing to sweep 1 and never store their sweep-2 sums
    const bool active = 8 * tid < H;
    uint32_t goff[NG], boff[NG];  // feature offsets of the groups, and the same in bytes
#pragma unroll
    for (int h = 0; h < NG; ++h) {
        goff[h] = active ? (uint32_t)(h * H) + 8u * tid : 0u;
        boff[h] = 2u * goff[h];
    }
    const uint32_t row_bytes = 2u * (uint32_t)F;

    uint4 wp[3][NG];
#pragma unroll
    for (int h = 0; h < NG; ++h) {
        uint32_t pc[3][8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float wf = active ? w[goff[h] + j] : 0.f;
            split3_bf16(wf, pc[0][j], pc[1][j], pc[2][j]);
        }
#pragma unroll
        for (int p = 0; p < 3; ++p)
            wp[p][h] = make_uint4(pc[p][0] | (pc[p][1] << 16), pc[p][2] | (pc[p][3] << 16),
                                  pc[p][4] | (pc[p][5] << 16), pc[p][6] | (pc[p][7] << 16));
    }

    const int64_t blocks_per_part = a.rows_per_part / ROWS;
    const int64_t b0 = blocks_per_part * q / a.wg_per_part;
    const int64_t b1 = blocks_per_part * (q + 1) / a.wg_per_part;
    const uint16_t* base = X + (int64_t)part * a.rows_per_part * F;
    const int64_t row_base = (int64_t)part * a.rows_per_part;

    u32x4 x[ROWS][NG];
    {
        global_bytes blk_ptr = uniform_ptr(base + b0 * ROWS * F);
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
#pragma unroll
            for (int h = 0; h < NG; ++h) x[r][h] = load16(blk_ptr + r * row_bytes, boff[h]);
    }
    float acc[8 * NG];
#pragma unroll
    for (int e = 0; e < 8 * NG; ++e) acc[e] = 0.f;

    // lane (n, g) of the MFMA result holds D[4g .. 4g+3][n]; the diagonal element D[n][n] sits in
    // the lanes with n / 4 == g, at position n % 4
    const int n = lane & 15, g = lane >> 4;
    const bool on_diag = (n >> 2) == g;
    const bool dm0 = on_diag && (n & 3) == 0, dm1 = on_diag && (n & 3) == 1;
    const bool dm2 = on_diag && (n & 3) == 2, dm3 = on_diag && (n & 3) == 3;

    for (int64_t blk = b0; blk < b1; ++blk) {
        const int64_t row0 = row_base + blk * ROWS;
        // ---- sweep 1: the wave's share of the residuals (trace of A B^T per sample)
#pragma unroll
        for (int rg = 0; rg < ROWS; rg += 4) {
            float part_r[4];
            f32x4 d[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) d[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int h = 0; h < NG; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        d[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x[rg + i][h]),
                                                                       __builtin_bit_cast(bf16x8, wp[p][h]), d[i],
                                                                       0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float t = dm0 ? d[i][0] : 0.f;
                t = dm1 ? d[i][1] : t;
                t = dm2 ? d[i][2] : t;
                t = dm3 ? d[i][3] : t;
                part_r[i] = row16_sum(t);
            }
            if (n == 0)
                *reinterpret_cast<float4*>(&lds_part[wave * 4 + g][rg]) =
                    make_float4(part_r[0], part_r[1], part_r[2], part_r[3]);
        }
        __syncthreads();
        if (tid < ROWS) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 4 * kLsWaves; ++e) s = s + lds_part[e][tid];
            const float r = s - y[row0 + tid];
            lds_r[tid] = r;
            a.resid[row0 + tid] = r;
        }
        __syncthreads();
        // ---- sweep 2: g += X_blk^T r from the same registers; each sample's registers are
        // refilled with the next block as soon as they are consumed (the last block is fetched a
        // second time instead of branching)
        const int64_t nb = blk + 1 < b1 ? blk + 1 : blk;
        global_bytes nxt_ptr = uniform_ptr(base + nb * ROWS * F);
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const float rr = lds_r[r];
#pragma unroll
            for (int h = 0; h < NG; ++h) {
                fma8(acc + 8 * h, x[r][h], rr);
                x[r][h] = load16(nxt_ptr + r * row_bytes, boff[h]);
            }
        }
        // the barriers of the next block order the reuse of lds_part and lds_r
    }
    if (active) {
        float* out = a.partial + (int64_t)blockIdx.x * F;
#pragma unroll
        for (int h = 0; h < NG; ++h) {
            *reinterpret_cast<float4*>(out + goff[h]) =
                make_float4(acc[8 * h], acc[8 * h + 1], acc[8 * h + 2], acc[8 * h + 3]);
            *reinterpret_cast<float4*>(out + goff[h] + 4) =
                make_float4(acc[8 * h + 4], acc[8 * h + 5], acc[8 * h + 6], acc[8 * h + 7]);
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

int ls_wg_per_part(int64_t n_rows, int n_feat, int k_parts)
{
    const int64_t blocks = n_rows / k_parts / kLsRows;
    (void)n_feat;
    int64_t want = 512 / (k_parts > 0 ? k_parts : 1);  // two resident workgroups per compute unit
    if (want < 1) want = 1;
    return (int)(blocks < want ? blocks : want);
}

hipError_t launch_ls_partial_gradients(const void* X, int64_t n_rows, int n_feat, const float* y,
                                       const float* w, int k_parts, float* G, int64_t ldg,
                                       float* resid, float* partial, hipStream_t stream)
{
    LsArgs a{n_rows, n_feat, k_parts, ls_wg_per_part(n_rows, n_feat, k_parts), n_rows / k_parts, resid, partial};
    if (n_feat <= kLsResidentFeat / 2 && a.rows_per_part % 32 == 0)  // keeps all lanes busy on short rows
        hipLaunchKernelGGL((k_ls_resident<32, 1>), dim3((unsigned)(k_parts * a.wg_per_part)), dim3(kLsThreads), 0,
                           stream, static_cast<const uint16_t*>(X), y, w, a);
    else if (n_feat <= kLsResidentFeat)
        hipLaunchKernelGGL((k_ls_resident<16, 2>), dim3((unsigned)(k_parts * a.wg_per_part)), dim3(kLsThreads), 0,
                           stream, static_cast<const uint16_t*>(X), y, w, a);
    else
        hipLaunchKernelGGL((k_ls_resident<8, 4>), dim3((unsigned)(k_parts * a.wg_per_part)), dim3(kLsThreads), 0,
                           stream, static_cast<const uint16_t*>(X), y, w, a);
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
