// K2 of the worker side: streaming encode + stochastic quantize + bit-pack (+ the fused estimate).
// Template code only; agc_quantize_b<0|1|2><s|m>.hip instantiate it for the three ways a block gets
// its multiplier and for one or several fills of the staging area, so that the sets of kernels
// compile in parallel.
#pragma once

#include "agc_device.h"
#include "agc_kernels.h"

namespace agc {

// =======================================================================================
// K2  encode + stochastic quantize + bit-pack
// =======================================================================================
struct QuantArgs {
    int64_t ldg;
    int n, k;
    int64_t d;
    uint32_t key0, key1, step_lo, step_hi;
    float* scales;  // bucket-wise scales only: n x nb
    int64_t nb;
    float* ghat;    // fused step only
    const WindowRec* win;  // monotone-interval codes only; filled in by the launcher
    int stage_bits;        // largest sum of bit-widths one fill of the staging area holds (<= kStageBits)
    int stage_fills;       // how many fills the workers need (1 unless the widths sum to more than kStageBits)
    const uint8_t* block_layer;  // layer-wise scales only: the layer of every block; wq is then [layer][n]
};

typedef __attribute__((address_space(1))) uint32_t global_u32;  // a pointer known to be device memory
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // one 16-byte piece of a stream

// Waves (= 256-coordinate blocks) per workgroup of the quantize pass.  A worker's codes leave in
// pieces of 32 * kQuantWaves * b contiguous bytes; the staging area grows by the same factor.
#ifndef AGC_K2_WG_WAVES
#define AGC_K2_WG_WAVES 4
#endif
constexpr int kQuantWaves = AGC_K2_WG_WAVES;
constexpr int kQuantThreads = kWave * kQuantWaves;
static_assert(kQuantWaves % 4 == 0 && kQuantWaves <= 16, "the per-worker table counts pieces for four waves");

// LDS staging area of a workgroup, in 16-byte pieces: 2 * kQuantWaves * bits pieces per worker
// (the blocks of the workgroup, 2 * bits pieces each), plus one piece that takes the zero bits the
// packer spills past a block's last word
__host__ __device__ constexpr int stage_pieces(int stage_bits) { return 2 * kQuantWaves * stage_bits + 1; }

// raw buffer descriptor, last word: 32-bit untyped data format of this target; the bounds check is
// on the byte offset against num_records (stride 0)
constexpr int kBufferRsrcFlags = 0x00020000;
// cache-policy operand of the payload stores: bit 1 = non-temporal, bit 4 = sc1 (written through to
// memory), bit 0 = sc0.  Measured on the metric workload: plain 1.50 ms, sc0 1.51, sc1 1.45,
// non-temporal 1.42, non-temporal + sc1 1.41.
#ifndef AGC_PAYLOAD_POLICY
#define AGC_PAYLOAD_POLICY 18
#endif
constexpr int kPayloadStorePolicy = AGC_PAYLOAD_POLICY;

// cache-policy operand of the store of the fused estimate: sc1 alone (written through).  Next to
// the payload stores: plain 1.41-1.42 ms, non-temporal 1.43, sc1 1.40-1.41.
#ifndef AGC_ESTIMATE_POLICY
#define AGC_ESTIMATE_POLICY 16
#endif
constexpr int kEstimateStorePolicy = AGC_ESTIMATE_POLICY;

// buffer descriptor over `bytes` bytes at a wave-uniform address (the hardware drops accesses at
// offsets >= bytes).  The two halves of the address go through readfirstlane as unsigned words:
// the builtin returns a signed int, and a sign-extended low word would corrupt the high one.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t uniform_buffer(const void* p, int bytes)
{
    const uint64_t bits = (uint64_t)p;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)bits);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(bits >> 32));
    return __builtin_amdgcn_make_buffer_rsrc((char*)(((uint64_t)hi << 32) | (uint64_t)lo), 0,
                                             __builtin_amdgcn_readfirstlane(bytes), kBufferRsrcFlags);
}

// One rounding decision (Sec. II-B): T is the grid position scaled by 2^16; the cell is
// T >> 16, the low 16 bits are the first 16 bits of the round-up probability, compared with
// the 16-bit primary draw; equality is a tie, resolved later by a secondary draw.
__device__ __forceinline__ uint32_t round_primary(float T, uint32_t u16, uint32_t L, bool& tie)
{
    const uint32_t Ti = (uint32_t)T;
    tie = (u16 == (Ti & 0xFFFFu));
    // up <=> u16 < Fi <=> Fi + (0xFFFF - u16) carries into bit 16: one add and one shift
    const uint32_t level = (Ti + (0xFFFFu - u16)) >> 16;
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

// BUCKET 0: the worker's multiplier comes from the table (one scale per vector).
// BUCKET 1 / 2: one scale per 256-coordinate block, derived here from the block itself (largest
// magnitude / Euclidean norm), stored by lane 0, and turned into the multiplier with one binary32
// division (Sec. II-B names the bucket-wise extension; this is its single-pass form).
// FUSE: the pass also accumulates the master's estimate (Sec. II-A aggregation) from the codes it
// has just formed: arrived workers in ascending order, one fused multiply-add each from 0, the
// arithmetic of the stand-alone decode kernel, so both give the same bits.
// Payload path: a worker's codes are not stored when they are formed.  Every wave ORs its block's
// 8b words into the workgroup's LDS staging area (worker-major, then block, so that the four
// blocks of a worker lie in stream order); when the area is full, or after the last worker, the
// workgroup meets at a barrier and writes each worker's 128*b bytes as one contiguous, line-aligned
// piece of its stream.  Stores of 64..96 bytes per wave and worker, as a wave alone would issue
// them, reach memory as partial lines and cost several times their bytes on this memory system.
// MULTI: the workers need more than one fill of the area, so it is also written out between
// workers, inside the streaming loop.  Without MULTI (the common case: widths sum to at most
// kStageBits) the loop over the workers contains no store at all and the kernel writes the area
// out once, after the loop; the encode drivers then keep their rolling prefetch.
template <int BUCKET, bool FUSE, bool MULTI>
struct EpiQuant {
    static constexpr bool kStoresPerWorker = MULTI;  // stores inside the worker loop (a flush between workers)
    static constexpr int kPrefetchRows = AGC_PREFETCH_ROWS;
    const WorkerQ* __restrict__ wq;
    uint32_t key0, key1, step_lo, step_hi;
    uint32_t* stage;     // the workgroup's LDS staging area, all zero between fills
    float* stage_scales; // bucket-wise scales: [n][kQuantWaves] floats behind the staging area
    int lane;
    int wave;            // this wave's block inside the workgroup
    int n;               // workers
    int64_t wg;          // index of the workgroup = index of its group of four blocks
    int wg_groups;       // 128-code groups of the workgroup's blocks that exist in the streams (1..2*kQuantWaves)
    int64_t block;       // index of this wave's 256-coordinate block
    uint32_t ctr0;       // m >> 2 of this lane's coordinates
    int nvalid;
    bool wave_ragged;    // wave-uniform: some lane has coordinates >= d
    uint32_t keep2, keep3;  // second half of the Philox block, for the odd worker of the pair
    float* scales;          // bucket-wise scales: n x nb
    int64_t nb;
    int group_first;        // first worker of the fill that is being staged
    float acc[4];           // fused step: this lane's four coordinates of the estimate
    WorkerQ pend;           // record of the worker that comes next, requested one worker early

    // The workgroup writes out the fill that ends with worker `last`.  Every wave of the
    // workgroup calls this for the same workers in the same order (also a wave whose block lies
    // past the end of the vector), so the barriers match.  The waves share the workers of the
    // fill; a worker's 8b pieces leave as one store of 128*b contiguous bytes through a buffer
    // descriptor that covers exactly the bytes of the stream that exist, so the hardware's range
    // check drops the pieces past the end of the vector.  Pieces are handed back zeroed.
    __device__ __forceinline__ void flush_fill(int last)
    {
        __syncthreads();
        u32x4_t* pieces = reinterpret_cast<u32x4_t*>(stage);
        for (int j = group_first + wave; j <= last; j += kQuantWaves) {
            const WorkerQ w = load_uniform(wq + j);
            const int b = (int)w.bits;
            const int np = 2 * kQuantWaves * b;  // pieces of this worker in the area
            const __amdgpu_buffer_rsrc_t rsrc = uniform_buffer(
                (const char*)w.codes + (uint64_t)wg * (uint64_t)(32 * kQuantWaves * b), 16 * b * wg_groups);
            const uint32_t first = w.stage_piece * (uint32_t)(kQuantWaves / 4);  // the table counts for four waves
            for (int off = 0; off < np; off += kWave) {
                const int piece = off + lane;
                u32x4_t v = u32x4_t{0u, 0u, 0u, 0u};
                if (piece < np) {
                    u32x4_t* sp = pieces + (first + (uint32_t)piece);
                    v = *sp;
                    *sp = u32x4_t{0u, 0u, 0u, 0u};
                }
                // lanes with piece >= np lie at or past the worker's bytes >= valid_bytes: dropped by the range check
#ifndef AGC_ABLATE_STORES
                __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, 16 * piece, 0, kPayloadStorePolicy);
#endif
            }
        }
        group_first = last + 1;
        if (last + 1 < n) {
            __syncthreads();  // the area is reused by the next fill
        } else if (BUCKET != 0) {
            // after the last worker: the scales of all workers for the workgroup's blocks, one run of
            // kQuantWaves floats per worker (the barrier above made every wave's entries visible)
            const int64_t first_block = wg * kQuantWaves;
            const int have = nb - first_block >= kQuantWaves ? kQuantWaves : (int)(nb - first_block);
            for (int t = wave * kWave + lane; t < n; t += kQuantThreads) {
                __attribute__((address_space(1))) float* dst =
                    (__attribute__((address_space(1))) float*)scales + ((int64_t)t * nb + first_block);
                if (have == kQuantWaves) {  // one run per worker, dword-aligned (a row of scales starts anywhere)
                    typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
#pragma unroll
                    for (int u = 0; u < kQuantWaves; u += 4)
                        *(__attribute__((address_space(1))) f32x4_a4*)(dst + u) =
                            f32x4_a4{stage_scales[t * kQuantWaves + u], stage_scales[t * kQuantWaves + u + 1],
                                     stage_scales[t * kQuantWaves + u + 2], stage_scales[t * kQuantWaves + u + 3]};
                } else {
#pragma unroll
                    for (int u = 0; u < kQuantWaves; ++u)
                        if (u < have) dst[u] = stage_scales[t * kQuantWaves + u];
                }
            }
        }
    }

    // a wave without a block (past the end of the vector) still takes part in every flush
    __device__ __forceinline__ void flush_only()
    {
        for (int i = 0; i < n; ++i) {
            const WorkerQ w = load_uniform(wq + i);
            if (w.flush) flush_fill(i);
        }
    }

    __device__ __forceinline__ float block_multiplier(int i, const float4& f, float num, float& scale)
    {
        if (BUCKET == 1) {
            const float a = fmaxf(fmaxf(fabsf(f.x), fabsf(f.y)), fmaxf(fabsf(f.z), fabsf(f.w)));
            scale = __uint_as_float(wave_max_nonneg_bits(a));
        } else {
            const double x0 = f.x, x1 = f.y, x2 = f.z, x3 = f.w;
            const double s01 = x0 * x0 + x1 * x1;
            const double s23 = x2 * x2 + x3 * x3;
            scale = (float)sqrt(wave_butterfly_add(s01 + s23));
        }
        // the block's scale waits in LDS next to the codes ([worker][block of the workgroup]) and
        // leaves with the last flush: 4-byte stores scattered over n rows cost far more than their bytes
        if (lane == 0) stage_scales[i * kQuantWaves + wave] = scale;
        // num = L * 2^16 (2^15 for a one-bit worker) comes with the worker's record
        const float q = num / scale;  // correctly rounded binary32 division
        return q <= 3.402823466e+38f ? q : 0.0f;  // scale == 0 gives +inf and ends here too
    }

    // four rounding decisions; only the grid position differs between the regular grid
    // (b >= 2) and the two-point grid of a one-bit worker
    __device__ __forceinline__ void codes4(int i, const float4& f, float inv, int b, uint32_t wa,
                                           uint32_t wb, uint32_t (&c)[4], uint32_t (&lev)[4])
    {
        const float fv[4] = {f.x, f.y, f.z, f.w};
        const uint32_t u[4] = {wa & 0xFFFFu, wa >> 16, wb & 0xFFFFu, wb >> 16};
        const uint32_t L = (b >= 2) ? ((1u << (b - 1)) - 1u) : 1u;
        const uint32_t signbit = (b >= 2) ? (1u << (b - 1)) : 0u;
        bool tie[4];
        float T[4];
#ifdef AGC_ABLATE_QUANT  // measurement build: no rounding arithmetic, codes are arbitrary bits
#pragma unroll
        for (int q = 0; q < 4; ++q) lev[q] = c[q] = (__float_as_uint(fv[q]) >> 9) & L;
        (void)tie; (void)T; (void)u; (void)signbit; (void)inv;
        return;
#endif
        if (b >= 2) {
#pragma unroll
            for (int q = 0; q < 4; ++q) T[q] = grid_pos<false>(fv[q], inv);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) T[q] = grid_pos<true>(fv[q], inv);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) c[q] = round_primary(T[q], u[q], L, tie[q]);
        if (__any(tie[0] | tie[1] | tie[2] | tie[3])) {  // about one wave pass in 250
            uint32_t r2[4];
            philox4x32_10(ctr0, 0x80000000u | (uint32_t)i, step_lo, step_hi, key0, key1, r2);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (tie[q]) c[q] = round_tied(T[q], r2[q], L);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) lev[q] = c[q];
#pragma unroll
        for (int q = 0; q < 4; ++q) c[q] |= (__float_as_uint(fv[q]) >> ((32 - b) & 31)) & signbit;
        if (wave_ragged) {  // codes of coordinates >= d are zero padding
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (q >= nvalid) c[q] = 0u;
        }
    }

    // the worker's parity known at compile time (ring and gather drivers)
    template <bool EVEN>
    __device__ __forceinline__ void worker(int i, const float4& f)
    {
        uint32_t wa, wb;
        if (EVEN) {
            uint32_t o[4];
            philox4x32_10(ctr0, (uint32_t)i >> 1, step_lo, step_hi, key0, key1, o);
            wa = o[0];
            wb = o[1];
            keep2 = o[2];
            keep3 = o[3];
        } else {
            wa = keep2;
            wb = keep3;
        }
        finish(i, f, wa, wb);
    }

    // the worker's parity known only at run time (window driver); workers still come in
    // ascending order, so an odd worker finds the second half of its pair's Philox block
    __device__ __forceinline__ void worker_any(int i, const float4& f)
    {
        uint32_t wa = keep2, wb = keep3;
        if ((i & 1) == 0) {  // wave-uniform
            uint32_t o[4];
            philox4x32_10(ctr0, (uint32_t)i >> 1, step_lo, step_hi, key0, key1, o);
            wa = o[0];
            wb = o[1];
            keep2 = o[2];
            keep3 = o[3];
        }
        finish(i, f, wa, wb);
    }

    __device__ __forceinline__ void finish(int i, const float4& f, uint32_t wa, uint32_t wb)
    {
        // wave-uniform scalar reads; workers come in ascending order, so the record of this one
        // was requested while the previous one was quantized
        const WorkerQ q = pend;
        pend = load_uniform(wq + (i + 1 < n ? i + 1 : i));
        const int b = (int)q.bits;
        uint32_t c[4], lev[4];
        float scale = 0.f;
        const float inv = BUCKET == 0 ? q.inv16 : block_multiplier(i, f, q.inv16, scale);
        codes4(i, f, inv, b, wa, wb, c, lev);
        if constexpr (FUSE) {
            if (q.arrived) {  // wave-uniform
                const float coef = BUCKET == 0 ? q.coef : q.coef * scale;
                const float fv[4] = {f.x, f.y, f.z, f.w};
                // the decoded value: +-level (the level as a float with the sign bit of f), or +-1
                // for a one-bit worker; one fused multiply-add per coordinate either way
                float v[4];
                if (b >= 2) {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        v[t] = __uint_as_float(__float_as_uint((float)lev[t]) | (__float_as_uint(fv[t]) & 0x80000000u));
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) v[t] = lev[t] ? 1.0f : -1.0f;
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) acc[t] = fmaf(coef, v[t], acc[t]);
            }
        }

        // bit-pack: this lane's four codes start at bit lane*4b of the block's 256*b bits, the block's
        // 8b words start at piece q.stage_piece + wave*2b of the staging area
        const uint32_t bitpos = __umul24((uint32_t)lane, 4u * (uint32_t)b);
        uint32_t* slot = stage + 4u * (q.stage_piece * (uint32_t)(kQuantWaves / 4) + (uint32_t)wave * 2u * (uint32_t)b) +
                         (bitpos >> 5);
        const uint32_t sh = bitpos & 31u;
#ifdef AGC_ABLATE_PACK
        if (c[0] + c[1] + c[2] + c[3] + sh == 0xFFFFFFF0u) atomicOr(slot, 1u);
        else
#endif
        if (b <= 8) {
            const uint32_t chunk = c[0] | (c[1] << b) | (c[2] << (2 * b)) | (c[3] << (3 * b));
            const uint64_t v = (uint64_t)chunk << sh;
            atomicOr(slot, (uint32_t)v);
            atomicOr(slot + 1, (uint32_t)(v >> 32));
        } else {
            const uint64_t chunk = (uint64_t)c[0] | ((uint64_t)c[1] << b) | ((uint64_t)c[2] << (2 * b)) |
                                   ((uint64_t)c[3] << (3 * b));
            const uint64_t v = chunk << sh;
            const uint32_t top = sh ? (uint32_t)(chunk >> (64 - sh)) : 0u;
            atomicOr(slot, (uint32_t)v);
            atomicOr(slot + 1, (uint32_t)(v >> 32));
            atomicOr(slot + 2, top);
        }
        if constexpr (MULTI) {
            if (q.flush) flush_fill(i);  // wave-uniform, and the same for every wave of the workgroup
        }
    }
};

template <int S, int BUCKET, bool FUSE, bool MULTI>
// The compiler is told to plan for four waves per SIMD: with a register count just under the
// five-wave limit it otherwise schedules for five and gives up instruction-level parallelism;
// measured 1.45 ms against 1.51 ms on the metric workload (three: 1.51 ms).  The gather driver
// (S == 0) lives on occupancy instead and keeps the default.
#ifndef AGC_K2_WAVES
#define AGC_K2_WAVES 4
#endif
__global__ __launch_bounds__(kQuantThreads) __attribute__((amdgpu_waves_per_eu(S == 0 ? 1 : AGC_K2_WAVES, S == 0 ? 8 : AGC_K2_WAVES))) void k_quantize(const float* __restrict__ G,
                                                         const int* __restrict__ row_ptr,
                                                         const int* __restrict__ col,
                                                         const float* __restrict__ val,
                                                         const WorkerQ* __restrict__ wq, QuantArgs a)
{
    // stage_pieces(a.stage_bits) pieces, then (bucket-wise scales) n * kQuantWaves floats
    extern __shared__ __attribute__((aligned(16))) uint32_t lds_stage[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // wave-uniform by construction
    const int lane = threadIdx.x % kWave;
#ifdef AGC_XCD_ORDER
    int64_t wg = blockIdx.x;
    {
        const int64_t per = gridDim.x / 8;
        if (wg < per * 8) wg = (wg % 8) * per + wg / 8;
    }
#elif defined(AGC_REVERSE_ORDER)
    const int64_t wg = (int64_t)gridDim.x - 1 - blockIdx.x;
#else
    const int64_t wg = blockIdx.x;
#endif
    const int64_t block = wg * kQuantWaves + wave;
    const int64_t base = block * (int64_t)kBlockCoords;
    {
        u32x4_t* pieces = reinterpret_cast<u32x4_t*>(lds_stage);
        const int np = stage_pieces(a.stage_bits);
        for (int p = threadIdx.x; p < np; p += kQuantThreads) pieces[p] = u32x4_t{0u, 0u, 0u, 0u};
    }
    __syncthreads();
    const int64_t groups_left = (a.d + 127) / 128 - 2 * kQuantWaves * wg;  // >= 1: the workgroup's first block exists
    const bool has_block = base < a.d;
    LaneCoords lc{};
    if (has_block) lc = lane_coords(base, lane, a.d);
    // layer-wise scales: the table of the block's layer (multiplier and decode weight differ from
    // layer to layer; bit-width, stream and staging place are the same in every table, so the
    // waves of a workgroup may hold different tables when they meet at a flush)
    if (a.block_layer && has_block) wq += (int64_t)__builtin_amdgcn_readfirstlane((int)a.block_layer[block]) * a.n;
    EpiQuant<BUCKET, FUSE, MULTI> epi{wq, a.key0, a.key1, a.step_lo, a.step_hi, lds_stage,
                               reinterpret_cast<float*>(lds_stage + 4 * stage_pieces(a.stage_bits)), lane, wave, a.n, wg,
                               groups_left >= 2 * kQuantWaves ? 2 * kQuantWaves : (int)groups_left, block, (uint32_t)((base + 4 * lane) >> 2),
                               lc.nvalid, lc.wave_ragged, 0u, 0u, a.scales, a.nb, 0, {0.f, 0.f, 0.f, 0.f},
                               load_uniform(wq)};
    if (!has_block) {  // nothing to encode, but the other waves of the workgroup wait at the flushes
        if constexpr (MULTI) epi.flush_only();
        else epi.flush_fill(a.n - 1);
        return;
    }
    encode_block<S>(G + base, a.ldg, a.n, a.k, CsrView{row_ptr, col, val, a.win}, lc, epi);
    if constexpr (!MULTI) epi.flush_fill(a.n - 1);  // the one fill: all workers, written out after the loop
    if constexpr (FUSE) {
        float* dst = a.ghat + base + 4 * lane;
        if (lc.nvalid == 4) {
            const __amdgpu_buffer_rsrc_t rs = uniform_buffer(a.ghat + base, 4 * kBlockCoords);
            __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{__float_as_uint(epi.acc[0]), __float_as_uint(epi.acc[1]),
                                                           __float_as_uint(epi.acc[2]), __float_as_uint(epi.acc[3])},
                                                   rs, 16 * lane, 0, kEstimateStorePolicy);
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (t < lc.nvalid) dst[t] = epi.acc[t];
        }
    }
}

template <int S, int BUCKET, bool MULTI>
static hipError_t launch_quantize_s(const float* G, const CodeDev& code, const Workspace& ws,
                                    const QuantArgs& args, hipStream_t stream)
{
    QuantArgs a = args;
    a.win = code.win;
    if (S < 0 && !a.win) return hipErrorInvalidValue;  // the window driver reads the records
    const int64_t nblocks = (a.d + kBlockCoords - 1) / kBlockCoords;
    const unsigned grid = (unsigned)((nblocks + kQuantWaves - 1) / kQuantWaves);
    if (a.stage_bits < 1 || a.stage_bits > kStageBits) return hipErrorInvalidValue;
    if (MULTI ? a.stage_fills < 2 : a.stage_fills != 1) return hipErrorInvalidValue;
    const unsigned lds_bytes = 16u * (unsigned)stage_pieces(a.stage_bits) +
                               (BUCKET != 0 ? (unsigned)(sizeof(float) * kQuantWaves * a.n) : 0u);
    const dim3 g(grid), b(kQuantThreads);
    if (a.ghat)
        hipLaunchKernelGGL((k_quantize<S, BUCKET, true, MULTI>), g, b, lds_bytes, stream, G, code.row_ptr, code.col,
                           code.val, ws.wq, a);
    else
        hipLaunchKernelGGL((k_quantize<S, BUCKET, false, MULTI>), g, b, lds_bytes, stream, G, code.row_ptr, code.col,
                           code.val, ws.wq, a);
    return hipGetLastError();
}

template <int BUCKET, bool MULTI>
static inline hipError_t launch_quantize_band(const float* G, const CodeDev& code, const Workspace& ws,
                                              const QuantArgs& a, hipStream_t stream)
{
    switch (code.band) {
        case 1: return launch_quantize_s<1, BUCKET, MULTI>(G, code, ws, a, stream);
        case 2: return launch_quantize_s<2, BUCKET, MULTI>(G, code, ws, a, stream);
        case 3: return launch_quantize_s<3, BUCKET, MULTI>(G, code, ws, a, stream);
        case 4: return launch_quantize_s<4, BUCKET, MULTI>(G, code, ws, a, stream);
        case 5: return launch_quantize_s<5, BUCKET, MULTI>(G, code, ws, a, stream);
        case 6: return launch_quantize_s<6, BUCKET, MULTI>(G, code, ws, a, stream);
        case 7: return launch_quantize_s<7, BUCKET, MULTI>(G, code, ws, a, stream);
        case 8: return launch_quantize_s<8, BUCKET, MULTI>(G, code, ws, a, stream);
        case -2: return launch_quantize_s<-2, BUCKET, MULTI>(G, code, ws, a, stream);
        case -4: return launch_quantize_s<-4, BUCKET, MULTI>(G, code, ws, a, stream);
        case -8: return launch_quantize_s<-8, BUCKET, MULTI>(G, code, ws, a, stream);
        default: return launch_quantize_s<0, BUCKET, MULTI>(G, code, ws, a, stream);
    }
}

// One entry point per instantiation unit (agc_quantize_b<BUCKET><s|m>.hip: the way a block gets its
// multiplier, and one fill or several), so that the sets of kernels compile in parallel.
#define AGC_QUANT_UNIT(NAME) \
    hipError_t NAME(const float* G, const CodeDev& code, const Workspace& ws, const QuantArgs& a, hipStream_t stream)
AGC_QUANT_UNIT(launch_quantize_band0s);
AGC_QUANT_UNIT(launch_quantize_band0m);
AGC_QUANT_UNIT(launch_quantize_band1s);
AGC_QUANT_UNIT(launch_quantize_band1m);
AGC_QUANT_UNIT(launch_quantize_band2s);
AGC_QUANT_UNIT(launch_quantize_band2m);

}  // namespace agc
