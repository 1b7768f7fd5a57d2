// gfx950 kernels of the approximate-gradient-coding hot path.
//
//   k_scale_pass      worker side, pass 1: stream G once, form f_i = sum_j a_ij g_j in registers
//                     (Sec. II-A) and reduce each worker's scale per 1024-coordinate segment
//   k_scale_finalize  fixed-order reduction of the segment partials -> scale_i, inv16_i
//   k_quantize        worker side, pass 2: stream G once more, re-form f_i, stochastic rounding
//                     on the grid {0,1/L,..,1} (Sec. II-B) with Philox draws, variable-width
//                     bit-packing, coalesced stores of the payload
//   k_decode          master side: masked dequantize + weighted sum (Sec. II-A aggregation)
//
// All four are bandwidth/ALU streaming kernels; there is no dense contraction on this path,
// hence no MFMA.
#include "agc_device.h"
#include "agc_kernels.h"

namespace agc {

// =======================================================================================
// K1  scale pass
// =======================================================================================
struct ScaleArgs {
    const float* G;
    int64_t ldg;
    int n, k;
    int64_t d;
    CodeDev code;
    Workspace ws;
};

// epilogue for the largest-magnitude scale: exact and order-free
struct EpiMaxAbs {
    float* acc;  // this wave's LDS slice [n]
    int lane;
    template <bool EVEN>
    __device__ __forceinline__ void worker(int i, const float4& f)
    {
        float a = fmaxf(fmaxf(fabsf(f.x), fabsf(f.y)), fmaxf(fabsf(f.z), fabsf(f.w)));
        a = wave_max_nonneg(a);
        if (lane == 0) acc[i] = fmaxf(acc[i], a);
    }
};

// epilogue for the Euclidean scale: levels 0-2 of the binary64 summation tree (lane value
// (x0^2+x1^2)+(x2^2+x3^2); exchange-add across the 64 lanes; blocks of a segment in order)
struct EpiSumSq {
    double* acc;  // this wave's LDS slice [n]
    int lane;
    template <bool EVEN>
    __device__ __forceinline__ void worker(int i, const float4& f)
    {
        const double x0 = f.x, x1 = f.y, x2 = f.z, x3 = f.w;
        const double s01 = x0 * x0 + x1 * x1;
        const double s23 = x2 * x2 + x3 * x3;
        double q = wave_butterfly_add(s01 + s23);
        if (lane == 0) acc[i] = acc[i] + q;
    }
};

template <int S, int MODE>
__global__ __launch_bounds__(kWgThreads) void k_scale_pass(ScaleArgs a)
{
    __shared__ double lds_acc[kWavesPerWg][kMaxWorkers];
    const int wave = threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    const int64_t seg = (int64_t)blockIdx.x * kWavesPerWg + wave;

    double* accd = lds_acc[wave];
    float* accf = reinterpret_cast<float*>(lds_acc[wave]);
    for (int i = lane; i < a.n; i += kWave) {
        if (MODE == 0) accd[i] = 0.0;
        else accf[i] = 0.f;
    }
    __syncthreads();

    if (seg < a.ws.nseg) {
        for (int blk = 0; blk < kSegBlocks; ++blk) {
            const int64_t base = (seg * kSegBlocks + blk) * (int64_t)kBlockCoords;
            if (base >= a.d) break;
            const LaneCoords lc = lane_coords(base + 4 * lane, a.d);
            if (MODE == 0) {
                EpiSumSq epi{accd, lane};
                if constexpr (S > 0) encode_ring<S>(a.G, a.ldg, a.k, a.code.val, lc, epi);
                else encode_gather(a.G, a.ldg, a.n, CsrView{a.code.row_ptr, a.code.col, a.code.val}, lc, epi);
            } else {
                EpiMaxAbs epi{accf, lane};
                if constexpr (S > 0) encode_ring<S>(a.G, a.ldg, a.k, a.code.val, lc, epi);
                else encode_gather(a.G, a.ldg, a.n, CsrView{a.code.row_ptr, a.code.col, a.code.val}, lc, epi);
            }
        }
    }
    __syncthreads();
    if (seg < a.ws.nseg) {
        for (int i = lane; i < a.n; i += kWave) {
            if (MODE == 0) a.ws.part_sq[seg * a.n + i] = accd[i];
            else a.ws.part_max[seg * a.n + i] = accf[i];
        }
    }
}

template <int S>
static hipError_t launch_scale_pass_s(const ScaleArgs& a, int scale_mode, hipStream_t stream)
{
    const unsigned grid = (unsigned)((a.ws.nseg + kWavesPerWg - 1) / kWavesPerWg);
    if (scale_mode == 0) hipLaunchKernelGGL((k_scale_pass<S, 0>), dim3(grid), dim3(kWgThreads), 0, stream, a);
    else hipLaunchKernelGGL((k_scale_pass<S, 1>), dim3(grid), dim3(kWgThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_scale_pass(const float* G, int64_t ldg, int n, int k, int64_t d,
                             const CodeDev& code, int scale_mode, const Workspace& ws,
                             hipStream_t stream)
{
    ScaleArgs a{G, ldg, n, k, d, code, ws};
    switch (code.band) {
        case 1: return launch_scale_pass_s<1>(a, scale_mode, stream);
        case 2: return launch_scale_pass_s<2>(a, scale_mode, stream);
        case 3: return launch_scale_pass_s<3>(a, scale_mode, stream);
        case 4: return launch_scale_pass_s<4>(a, scale_mode, stream);
        case 5: return launch_scale_pass_s<5>(a, scale_mode, stream);
        case 6: return launch_scale_pass_s<6>(a, scale_mode, stream);
        case 7: return launch_scale_pass_s<7>(a, scale_mode, stream);
        case 8: return launch_scale_pass_s<8>(a, scale_mode, stream);
        default: return launch_scale_pass_s<0>(a, scale_mode, stream);
    }
}

// =======================================================================================
// K1f  scale finalize: one workgroup per worker
// =======================================================================================
__device__ __forceinline__ float inv16_of(float scale, int bits)
{
    if (!(scale > 0.f)) return 0.f;
    const double num = bits >= 2 ? (double)((1 << (bits - 1)) - 1) * 65536.0 : 32768.0;
    const float q = (float)(num / (double)scale);
    return (q <= 3.402823466e+38f) ? q : 0.f;
}

template <int MODE>
__global__ __launch_bounds__(kWgThreads) void k_scale_finalize(int n, PerWorkerBits bits,
                                                               Workspace ws, float* scales)
{
    const int i = blockIdx.x;
    const int tid = threadIdx.x;
    __shared__ float red[kWgThreads];
    float scale;
    if (MODE == 1) {
        float m = 0.f;
        for (int64_t s = tid; s < ws.nseg; s += kWgThreads) m = fmaxf(m, ws.part_max[s * n + i]);
        red[tid] = m;
        __syncthreads();
        for (int h = kWgThreads / 2; h > 0; h >>= 1) {
            if (tid < h) red[tid] = fmaxf(red[tid], red[tid + h]);
            __syncthreads();
        }
        scale = red[0];
    } else {
        // level 3: 64 segments -> group, in order
        for (int64_t g = tid; g < ws.ngroup; g += kWgThreads) {
            double acc = 0.0;
            const int64_t s1 = (g + 1) * kGroupSegs < ws.nseg ? (g + 1) * kGroupSegs : ws.nseg;
            for (int64_t s = g * kGroupSegs; s < s1; ++s) acc = acc + ws.part_sq[s * n + i];
            ws.group_sq[(int64_t)i * ws.ngroup + g] = acc;
        }
        __syncthreads();
        // level 4: 64 groups -> supergroup, in order
        for (int64_t u = tid; u < ws.nsuper; u += kWgThreads) {
            double acc = 0.0;
            const int64_t g1 = (u + 1) * kGroupSegs < ws.ngroup ? (u + 1) * kGroupSegs : ws.ngroup;
            for (int64_t g = u * kGroupSegs; g < g1; ++g) acc = acc + ws.group_sq[(int64_t)i * ws.ngroup + g];
            ws.super_sq[(int64_t)i * ws.nsuper + u] = acc;
        }
        __syncthreads();
        // level 5: supergroups in order
        double total = 0.0;
        if (tid == 0) {
            for (int64_t u = 0; u < ws.nsuper; ++u) total = total + ws.super_sq[(int64_t)i * ws.nsuper + u];
            red[0] = (float)sqrt(total);
        }
        __syncthreads();
        scale = red[0];
    }
    if (tid == 0) {
        scales[i] = scale;
        ws.inv16[i] = inv16_of(scale, bits.bits[i]);
    }
}

hipError_t launch_scale_finalize(int n, int scale_mode, const PerWorkerBits& bits,
                                 const Workspace& ws, float* scales, hipStream_t stream)
{
    if (scale_mode == 0) hipLaunchKernelGGL((k_scale_finalize<0>), dim3(n), dim3(kWgThreads), 0, stream, n, bits, ws, scales);
    else hipLaunchKernelGGL((k_scale_finalize<1>), dim3(n), dim3(kWgThreads), 0, stream, n, bits, ws, scales);
    return hipGetLastError();
}

// =======================================================================================
// K2  encode + stochastic quantize + bit-pack
// =======================================================================================
struct QuantArgs {
    const float* G;
    int64_t ldg;
    int n, k;
    int64_t d;
    CodeDev code;
    const float* inv16;
    uint32_t key0, key1, step_lo, step_hi;
    QuantStreams out;
};

constexpr int kStageWords = 8 * 16 + 2;  // 256 codes of up to 16 bits, plus spill of zero bits

// One rounding decision (Sec. II-B): T is the grid position scaled by 2^16; the cell is
// T >> 16, the low 16 bits are the first 16 bits of the round-up probability, compared with
// the 16-bit primary draw; equality is a tie, resolved later by a secondary draw.
__device__ __forceinline__ uint32_t round_primary(float T, uint32_t u16, uint32_t L, bool& tie)
{
    const uint32_t Ti = (uint32_t)T;
    const uint32_t lo = Ti >> 16, Fi = Ti & 0xFFFFu;
    tie = (u16 == Fi);
    const uint32_t level = lo + (u16 < Fi ? 1u : 0u);
    return level < L ? level : L;
}

// the same decision for a coordinate whose primary draw tied: U < (Fi+g)/2^16 <=> r2 < g*2^32
__device__ __forceinline__ uint32_t round_tied(float T, uint32_t r2, uint32_t L)
{
    const uint32_t Ti = (uint32_t)T;
    const float g = T - (float)Ti;
    const uint32_t up = ((double)r2 < (double)g * 4294967296.0) ? 1u : 0u;
    const uint32_t level = (Ti >> 16) + up;
    return level < L ? level : L;
}

template <bool ONEBIT>
__device__ __forceinline__ float grid_pos(float f, float inv)
{
    if (ONEBIT) return fmaxf(fmaf(f, inv, 32768.0f), 0.0f);
    return fabsf(f) * inv;
}

struct EpiQuant {
    const QuantArgs& a;
    uint32_t* stage;     // this wave's LDS staging words, all zero between workers
    int lane;
    int64_t block;       // index of this wave's 256-coordinate block
    uint32_t ctr0;       // m >> 2 of this lane's coordinates
    int nvalid;
    bool wave_has_pad;   // wave-uniform: some lane has coordinates >= d
    uint32_t keep2, keep3;  // second half of the Philox block, for the odd worker of the pair

    template <bool ONEBIT>
    __device__ __forceinline__ void codes4(int i, const float4& f, float inv, int b, uint32_t wa,
                                           uint32_t wb, uint32_t (&c)[4])
    {
        const uint32_t L = ONEBIT ? 1u : ((1u << (b - 1)) - 1u);
        const float fv[4] = {f.x, f.y, f.z, f.w};
        const uint32_t u[4] = {wa & 0xFFFFu, wa >> 16, wb & 0xFFFFu, wb >> 16};
        bool tie[4];
        float T[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            T[q] = grid_pos<ONEBIT>(fv[q], inv);
            c[q] = round_primary(T[q], u[q], L, tie[q]);
        }
        if (__any(tie[0] | tie[1] | tie[2] | tie[3])) {  // about one wave pass in 250
            uint32_t r2[4];
            philox4x32_10(ctr0, 0x80000000u | (uint32_t)i, a.step_lo, a.step_hi, a.key0, a.key1, r2);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (tie[q]) c[q] = round_tied(T[q], r2[q], L);
        }
        if (!ONEBIT) {
            const uint32_t signbit = 1u << (b - 1);
#pragma unroll
            for (int q = 0; q < 4; ++q) c[q] |= (__float_as_uint(fv[q]) >> (32 - b)) & signbit;
        }
        if (wave_has_pad) {  // codes of coordinates >= d are zero padding
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (q >= nvalid) c[q] = 0u;
        }
    }

    template <bool EVEN>
    __device__ __forceinline__ void worker(int i, const float4& f)
    {
        uint32_t wa, wb;
        if (EVEN) {
            uint32_t o[4];
            philox4x32_10(ctr0, (uint32_t)i >> 1, a.step_lo, a.step_hi, a.key0, a.key1, o);
            wa = o[0];
            wb = o[1];
            keep2 = o[2];
            keep3 = o[3];
        } else {
            wa = keep2;
            wb = keep3;
        }
        const int b = a.out.bits[i];
        const float inv = a.inv16[i];
        uint32_t c[4];
        if (b >= 2) codes4<false>(i, f, inv, b, wa, wb, c);
        else codes4<true>(i, f, inv, b, wa, wb, c);

        // bit-pack: this lane's four codes start at bit lane*4b of the block's 256*b bits
        const uint32_t bitpos = (uint32_t)lane * 4u * (uint32_t)b;
        const uint32_t word = bitpos >> 5, sh = bitpos & 31u;
        if (b <= 8) {
            const uint32_t chunk = c[0] | (c[1] << b) | (c[2] << (2 * b)) | (c[3] << (3 * b));
            const uint64_t v = (uint64_t)chunk << sh;
            atomicOr(&stage[word], (uint32_t)v);
            atomicOr(&stage[word + 1], (uint32_t)(v >> 32));
        } else {
            const uint64_t chunk = (uint64_t)c[0] | ((uint64_t)c[1] << b) | ((uint64_t)c[2] << (2 * b)) |
                                   ((uint64_t)c[3] << (3 * b));
            const uint64_t v = chunk << sh;
            const uint32_t top = sh ? (uint32_t)(chunk >> (64 - sh)) : 0u;
            atomicOr(&stage[word], (uint32_t)v);
            atomicOr(&stage[word + 1], (uint32_t)(v >> 32));
            atomicOr(&stage[word + 2], top);
        }
        // LDS operations of one wave execute in issue order; the fences only stop the compiler
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int nwords = 8 * b;
        const int64_t total_words = ((a.d + 127) / 128) * 4 * b;
        uint32_t* dst = reinterpret_cast<uint32_t*>(a.out.codes[i]);
        for (int w = lane; w < nwords; w += kWave) {
            const uint32_t v = stage[w];
            stage[w] = 0u;
            const int64_t gi = block * nwords + w;
            if (gi < total_words) dst[gi] = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
};

template <int S>
__global__ __launch_bounds__(kWgThreads) void k_quantize(QuantArgs a)
{
    __shared__ uint32_t lds_stage[kWavesPerWg][kStageWords];
    const int wave = threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    const int64_t block = (int64_t)blockIdx.x * kWavesPerWg + wave;
    const int64_t base = block * (int64_t)kBlockCoords;
    for (int w = lane; w < kStageWords; w += kWave) lds_stage[wave][w] = 0u;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (base >= a.d) return;
    const LaneCoords lc = lane_coords(base + 4 * lane, a.d);
    EpiQuant epi{a, lds_stage[wave], lane, block, (uint32_t)((base + 4 * lane) >> 2), lc.nvalid,
                 __any(lc.nvalid < 4) != 0, 0u, 0u};
    if constexpr (S > 0) encode_ring<S>(a.G, a.ldg, a.k, a.code.val, lc, epi);
    else encode_gather(a.G, a.ldg, a.n, CsrView{a.code.row_ptr, a.code.col, a.code.val}, lc, epi);
}

template <int S>
static hipError_t launch_quantize_s(const QuantArgs& a, hipStream_t stream)
{
    const int64_t nblocks = (a.d + kBlockCoords - 1) / kBlockCoords;
    const unsigned grid = (unsigned)((nblocks + kWavesPerWg - 1) / kWavesPerWg);
    hipLaunchKernelGGL((k_quantize<S>), dim3(grid), dim3(kWgThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_quantize(const float* G, int64_t ldg, int n, int k, int64_t d,
                           const CodeDev& code, const Workspace& ws, uint64_t seed, uint64_t step,
                           const QuantStreams& out, hipStream_t stream)
{
    QuantArgs a{G, ldg, n, k, d, code, ws.inv16, (uint32_t)seed, (uint32_t)(seed >> 32),
                (uint32_t)step, (uint32_t)(step >> 32), out};
    switch (code.band) {
        case 1: return launch_quantize_s<1>(a, stream);
        case 2: return launch_quantize_s<2>(a, stream);
        case 3: return launch_quantize_s<3>(a, stream);
        case 4: return launch_quantize_s<4>(a, stream);
        case 5: return launch_quantize_s<5>(a, stream);
        case 6: return launch_quantize_s<6>(a, stream);
        case 7: return launch_quantize_s<7>(a, stream);
        case 8: return launch_quantize_s<8>(a, stream);
        default: return launch_quantize_s<0>(a, stream);
    }
}

// =======================================================================================
// K3  masked dequantize + weighted sum
// =======================================================================================
// A lane owns 32 consecutive coordinates: for a b-bit worker these are exactly b consecutive
// 32-bit words of the stream, so unpacking needs no cross-lane traffic and every shift is a
// compile-time constant.
constexpr int kDecCoords = 32;

struct DecodeArgs {
    int n;
    int64_t d;
    const float* scales;
    float* ghat;
    DecodeStreams in;
};

template <int B>
__device__ __forceinline__ void decode_words(const uint32_t* __restrict__ src, float coef,
                                             float (&acc)[kDecCoords])
{
    uint32_t w[B];
#pragma unroll
    for (int t = 0; t < B; ++t) w[t] = src[t];
#pragma unroll
    for (int q = 0; q < kDecCoords; ++q) {
        const int bit = q * B;
        const int wi = bit >> 5, sh = bit & 31;
        uint32_t code = w[wi] >> sh;
        if (sh + B > 32) code |= w[wi + 1] << (32 - sh);
        float v;
        if (B == 1) {
            v = (code & 1u) ? 1.0f : -1.0f;
        } else {
            const uint32_t level = code & ((1u << (B - 1)) - 1u);
            const uint32_t sign = (code << (32 - B)) & 0x80000000u;
            v = __uint_as_float(__float_as_uint((float)level) | sign);
        }
        acc[q] = fmaf(coef, v, acc[q]);
    }
}

__global__ __launch_bounds__(kWgThreads) void k_decode(DecodeArgs a)
{
    __shared__ float lds_coef[kMaxWorkers];
    // weight of one grid unit of worker i: w_i * scale_i / L_i, binary64 then one rounding
    for (int i = threadIdx.x; i < a.n; i += kWgThreads) {
        const int b = a.in.bits[i];
        const double L = b >= 2 ? (double)((1 << (b - 1)) - 1) : 1.0;
        lds_coef[i] = (float)(((double)a.in.w[i] * (double)a.scales[i]) / L);
    }
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * kWgThreads + threadIdx.x;
    const int64_t m0 = t * kDecCoords;
    if (m0 >= a.d) return;
    float acc[kDecCoords];
#pragma unroll
    for (int q = 0; q < kDecCoords; ++q) acc[q] = 0.f;
    for (int i = 0; i < a.n; ++i) {
        if (!a.in.mask[i]) continue;
        const int b = a.in.bits[i];
        const float coef = lds_coef[i];
        const uint32_t* src = reinterpret_cast<const uint32_t*>(a.in.codes[i]) + t * b;
        switch (b) {
            case 1: decode_words<1>(src, coef, acc); break;
            case 2: decode_words<2>(src, coef, acc); break;
            case 3: decode_words<3>(src, coef, acc); break;
            case 4: decode_words<4>(src, coef, acc); break;
            case 5: decode_words<5>(src, coef, acc); break;
            case 6: decode_words<6>(src, coef, acc); break;
            case 7: decode_words<7>(src, coef, acc); break;
            case 8: decode_words<8>(src, coef, acc); break;
            case 9: decode_words<9>(src, coef, acc); break;
            case 10: decode_words<10>(src, coef, acc); break;
            case 11: decode_words<11>(src, coef, acc); break;
            case 12: decode_words<12>(src, coef, acc); break;
            case 13: decode_words<13>(src, coef, acc); break;
            case 14: decode_words<14>(src, coef, acc); break;
            case 15: decode_words<15>(src, coef, acc); break;
            default: decode_words<16>(src, coef, acc); break;
        }
    }
    float* dst = a.ghat + m0;
    if (m0 + kDecCoords <= a.d) {
#pragma unroll
        for (int q = 0; q < kDecCoords; q += 4)
            *reinterpret_cast<float4*>(dst + q) = make_float4(acc[q], acc[q + 1], acc[q + 2], acc[q + 3]);
    } else {
#pragma unroll
        for (int q = 0; q < kDecCoords; ++q)
            if (m0 + q < a.d) dst[q] = acc[q];
    }
}

hipError_t launch_decode(int n, int64_t d, const DecodeStreams& in, const float* scales,
                         float* ghat, hipStream_t stream)
{
    DecodeArgs a{n, d, scales, ghat, in};
    const int64_t nthreads = (d + kDecCoords - 1) / kDecCoords;
    const unsigned grid = (unsigned)((nthreads + kWgThreads - 1) / kWgThreads);
    hipLaunchKernelGGL(k_decode, dim3(grid), dim3(kWgThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace agc
