// Partial gradients of the least-squares loss for the end-to-end loop: for every data
// partition p (Sec. II-A: g_j = grad L(D_j, beta)),  G[p,:] = X_p^T (X_p w - y_p),
// X in bfloat16 (row-major, n_rows x n_feat), everything else binary32.
//
// The stage is bound by the single HBM read of X (about one flop per byte), so the design keeps a
// block of 16 samples in REGISTERS between its two uses:
//   sweep 1  r = X_blk w - y_blk   (contraction over features)
//   sweep 2  g += X_blk^T r        (contraction over samples)
// k_ls_resident (n_feat <= 4096): a lane owns 16 features of all 16 samples of the block
// (128 VGPRs of packed bfloat16).  Sweep 2 is then a plain per-lane FMA chain.  Sweep 1 runs on the
// matrix cores: v_mfma_f32_16x16x32_bf16 with A = the lane's 8 features of one sample and B = the
// lane's own 8 entries of w; the diagonal D[i][i] is the sum over the four lanes (i, 0..3) of their
// own dot products, and the trace over the wave is the wave's share of the sample's residual.  w
// enters as its exact three-way bfloat16 split (w = hi + mid + lo), so the products are exact and
// only the binary32 accumulation rounds.  While sweep 2 consumes a sample's registers, the same
// registers are refilled with the next block's sample, which hides the load latency at two waves
// per SIMD.
// k_ls_stream (4096 < n_feat <= 8192): the block does not fit in registers; sweep 1 uses the MFMA
// in its natural layout (16 samples = M, the three pieces of w = three of the N columns) and
// sweep 2 re-reads the block from the caches.
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
constexpr int kLsRows = 16;        // samples per block (M of the MFMA tile)


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

__global__ __launch_bounds__(kLsThreads) void k_ls_stream(const uint16_t* __restrict__ X,
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

__global__ __launch_bounds__(kLsThreads, 2) void k_ls_resident(const uint16_t* __restrict__ X,
                                                               const float* __restrict__ y,
                                                               const float* __restrict__ w, LsArgs a)
{
    __shared__ float lds_part[4 * kLsWaves][kLsRows];  // [wave * 4 + 16-lane row][sample]
    __shared__ float lds_r[kLsRows];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int lane = tid % 64;
    const int F = a.n_feat, H = F / 2;
    const int part = blockIdx.x / a.wg_per_part;
    const int q = blockIdx.x % a.wg_per_part;
    // the lane's two groups of eight features; lanes beyond the feature range read group 0 and
    // carry zero pieces of w, so they add nothing to sweep 1 and never store their sweep-2 sums
    const bool active = 8 * tid < H;
    const uint32_t g0 = active ? 8u * tid : 0u, g1 = active ? (uint32_t)H + 8u * tid : 0u;
    const uint32_t o0 = 2u * g0, o1 = 2u * g1;  // byte offsets inside a row
    const uint32_t row_bytes = 2u * (uint32_t)F;

    uint4 wp[3][2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t pc[3][8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float wf = active ? w[(h ? g1 : g0) + j] : 0.f;
            split3_bf16(wf, pc[0][j], pc[1][j], pc[2][j]);
        }
#pragma unroll
        for (int p = 0; p < 3; ++p)
            wp[p][h] = make_uint4(pc[p][0] | (pc[p][1] << 16), pc[p][2] | (pc[p][3] << 16),
                                  pc[p][4] | (pc[p][5] << 16), pc[p][6] | (pc[p][7] << 16));
    }

    const int64_t blocks_per_part = a.rows_per_part / kLsRows;
    const int64_t b0 = blocks_per_part * q / a.wg_per_part;
    const int64_t b1 = blocks_per_part * (q + 1) / a.wg_per_part;
    const uint16_t* base = X + (int64_t)part * a.rows_per_part * F;
    const int64_t row_base = (int64_t)part * a.rows_per_part;

    u32x4 x[kLsRows][2];
    {
        global_bytes blk_ptr = uniform_ptr(base + b0 * kLsRows * F);
#pragma unroll
        for (int r = 0; r < kLsRows; ++r) {
            x[r][0] = load16(blk_ptr + r * row_bytes, o0);
            x[r][1] = load16(blk_ptr + r * row_bytes, o1);
        }
    }
    float acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;

    // lane (n, g) of the MFMA result holds D[4g .. 4g+3][n]; the diagonal element D[n][n] sits in
    // the lanes with n / 4 == g, at position n % 4
    const int n = lane & 15, g = lane >> 4;
    const bool on_diag = (n >> 2) == g;
    const bool dm0 = on_diag && (n & 3) == 0, dm1 = on_diag && (n & 3) == 1;
    const bool dm2 = on_diag && (n & 3) == 2, dm3 = on_diag && (n & 3) == 3;

    for (int64_t blk = b0; blk < b1; ++blk) {
        const int64_t row0 = row_base + blk * kLsRows;
        // ---- sweep 1: the wave's share of the 16 residuals (trace of A B^T per sample)
#pragma unroll
        for (int rg = 0; rg < kLsRows; rg += 4) {
            float part_r[4];
            f32x4 d[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) d[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int h = 0; h < 2; ++h)
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
        if (tid < kLsRows) {
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
        global_bytes nxt_ptr = uniform_ptr(base + nb * kLsRows * F);
#pragma unroll
        for (int r = 0; r < kLsRows; ++r) {
            const float rr = lds_r[r];
            fma8(acc, x[r][0], rr);
            fma8(acc + 8, x[r][1], rr);
            x[r][0] = load16(nxt_ptr + r * row_bytes, o0);
            x[r][1] = load16(nxt_ptr + r * row_bytes, o1);
        }
        // the barriers of the next block order the reuse of lds_part and lds_r
    }
    if (active) {
        float* out = a.partial + (int64_t)blockIdx.x * F;
        *reinterpret_cast<float4*>(out + g0) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        *reinterpret_cast<float4*>(out + g0 + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
        *reinterpret_cast<float4*>(out + g1) = make_float4(acc[8], acc[9], acc[10], acc[11]);
        *reinterpret_cast<float4*>(out + g1 + 4) = make_float4(acc[12], acc[13], acc[14], acc[15]);
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
    // the register-resident kernel runs two workgroups per compute unit, the streaming one four
    int64_t want = (n_feat <= kLsResidentFeat ? 512 : 1024) / (k_parts > 0 ? k_parts : 1);
    if (want < 1) want = 1;
    return (int)(blocks < want ? blocks : want);
}

hipError_t launch_ls_partial_gradients(const void* X, int64_t n_rows, int n_feat, const float* y,
                                       const float* w, int k_parts, float* G, int64_t ldg,
                                       float* resid, float* partial, hipStream_t stream)
{
    LsArgs a{n_rows, n_feat, k_parts, ls_wg_per_part(n_rows, n_feat, k_parts), n_rows / k_parts, resid, partial};
    const size_t lds = (size_t)3 * n_feat * sizeof(uint16_t);
    if (n_feat <= kLsResidentFeat)
        hipLaunchKernelGGL(k_ls_resident, dim3((unsigned)(k_parts * a.wg_per_part)), dim3(kLsThreads), 0, stream,
                           static_cast<const uint16_t*>(X), y, w, a);
    else
        hipLaunchKernelGGL(k_ls_stream, dim3((unsigned)(k_parts * a.wg_per_part)), dim3(kLsThreads), lds, stream,
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
