// gfx950 kernels of the approximate-gradient-coding hot path.
//
//   k_scale_pass      worker side, pass 1: stream G once, form f_i = sum_j a_ij g_j in registers
//                     (Sec. II-A) and reduce each worker's scale: running maxima in a small
//                     array (max-abs, also per layer), sums of squares per 1024-coordinate
//                     segment (Euclidean)
//   k_scale_finalize  the maxima, or a fixed-order reduction of the segment sums -> scale_i and
//   (.._layers)       the per-worker table (inv16_i, b_i, stream pointer) of the next pass
//   k_quantize        worker side, pass 2: stream G once more, re-form f_i, stochastic rounding
//                     on the grid {0,1/L,..,1} (Sec. II-B) with Philox draws, variable-width
//                     bit-packing, coalesced stores of the payload
//   k_decode_table    master side prologue: table of the arrived workers with their weights
//   k_decode          master side: masked dequantize + weighted sum (Sec. II-A aggregation)
//
// All of them are bandwidth/ALU streaming kernels; there is no dense contraction on this
// path, hence no MFMA.  Per-worker parameters are read with scalar loads from small device
// tables, never with vector loads, so that waiting for them does not drain the queue of
// outstanding row loads.
#include <mutex>

#include "agc_device.h"
#include "agc_kernels.h"
#include "agc_quantize.h"

namespace agc {

// =======================================================================================
// K1  scale pass
// =======================================================================================
// Pointers that the kernels only read are separate __restrict__ kernel parameters: that is
// what lets the compiler keep wave-uniform reads (code coefficients, per-worker tables) on the
// scalar unit even though the same kernel stores through other pointers.
struct ScaleArgs {
    int64_t ldg;
    int n, k;
    int64_t d;
    int64_t nseg;
    uint32_t* part_max;
    double* part_sq;
    const WindowRec* win;  // monotone-interval codes only
    const uint8_t* block_layer;  // layer-wise scales only (max-abs): the layer of every block
    const int* seg_first;        // layer-wise Euclidean scales only: the segments of the layers
    const uint8_t* seg_blocks;
};

// the same 32-bit word seen as device memory (store without address-space checks)
typedef __attribute__((address_space(1))) uint32_t global_word;

// epilogue for the largest-magnitude scale: exact and order-free
struct EpiMaxAbs {
    static constexpr bool kStoresPerWorker = false;
    static constexpr int kPrefetchRows = AGC_SCALE_PREFETCH_ROWS;
    uint32_t* acc;  // this wave's LDS slice [n], bit patterns of non-negative floats
    int lane;
    static __device__ __forceinline__ float max_abs4(const float4& f)
    {
        return fmaxf(fmaxf(fabsf(f.x), fabsf(f.y)), fmaxf(fabsf(f.z), fabsf(f.w)));
    }
    template <bool EVEN>
    __device__ __forceinline__ void worker(int i, const float4& f)
    {
        const uint32_t m = wave_max_nonneg_bits(max_abs4(f));
        if (lane == 0) acc[i] = m;
    }
    template <bool EVEN, int V>
    __device__ __forceinline__ void worker(int i, const RowN<V>& f)  // V blocks, one reduction
    {
        float a = max_abs4(f.v[0]);
#pragma unroll
        for (int t = 1; t < V; ++t) a = fmaxf(a, max_abs4(f.v[t]));
        const uint32_t m = wave_max_nonneg_bits(a);
        if (lane == 0) acc[i] = m;
    }
    template <class Row>
    __device__ __forceinline__ void worker_any(int i, const Row& f) { worker<true>(i, f); }
};

// epilogue for the Euclidean scale: levels 0 and 1 of the binary64 summation tree (lane value
// (x0^2+x1^2)+(x2^2+x3^2); exchange-add across the 64 lanes)
struct EpiSumSq {
    static constexpr bool kStoresPerWorker = false;
    static constexpr int kPrefetchRows = AGC_SCALE_PREFETCH_ROWS;
    double* acc;  // this wave's LDS slice [n]
    int lane;
    template <bool EVEN>
    __device__ __forceinline__ void worker(int i, const float4& f)
    {
        const double x0 = f.x, x1 = f.y, x2 = f.z, x3 = f.w;
        const double s01 = x0 * x0 + x1 * x1;
        const double s23 = x2 * x2 + x3 * x3;
        const double q = wave_butterfly_add(s01 + s23);
        if (lane == 0) acc[i] = q;
    }
    __device__ __forceinline__ void worker_any(int i, const float4& f) { worker<true>(i, f); }
};

// The norm's workgroups are the four blocks of a segment of its summation tree; the max-abs pass
// is free in its workgroup size (4 and 8 waves measured within 1 % of each other, 16 waves 2 %
// slower) and, with two blocks per wave, in its prefetch distance (2 to 8 rows within 1 %).
#ifndef AGC_SCALE_WAVES
#define AGC_SCALE_WAVES 8
#endif
#ifndef AGC_SCALE_PREFETCH_ROWS2
#define AGC_SCALE_PREFETCH_ROWS2 2  // rows ahead in the two-block ring: four loads in flight per lane
#endif
// below this many blocks the two-block form would leave compute units without a wave
// (256 units x 4 SIMDs x 5 resident waves of two blocks each, twice over)
constexpr int64_t kTwoBlockMin = 2 * 2 * 256 * 4 * 5;
// Euclidean scale: one workgroup per 1024-coordinate segment, one wave per 256-coordinate block of
// it.  The four block values of every worker meet in LDS and are combined in block order (level 2
// of the tree), which keeps the result independent of how the waves were scheduled.
// Max-abs scale: the maximum is exact and order-free.  A wave takes V neighbouring blocks (V = 2:
// both at once through the two-block register ring when they lie wholly inside the vector and the
// code has a ring driver, else one after the other) and folds its n maxima into the workgroup's
// LDS array with LDS atomics; the last wave of the workgroup to finish folds that array into one
// of kMaxSlots rows of a small array in memory ([slot][worker]) with one integer atomic-max
// instruction (bit patterns of non-negative floats order like the floats).  No wave waits for
// another, and the pass writes no partial results to memory (stores mixed into the read stream
// cost far more than their bytes on this memory system; even the atomics, performed in memory,
// cost 22 us at one per wave and worker).  The finalize kernel reads the rows and hands them back
// zeroed.
template <int S, int MODE, int WAVES, int V>
__global__ __launch_bounds__(kWave * WAVES) void k_scale_pass(const float* __restrict__ G,
                                                              const int* __restrict__ row_ptr,
                                                              const int* __restrict__ col,
                                                              const float* __restrict__ val,
                                                              ScaleArgs a)
{
    static_assert(MODE == 1 || (WAVES == kSegBlocks && V == 1), "the norm's tree fixes four blocks per workgroup");
    static_assert(V == 1 || V == 2 || V == 4, "one, two or four blocks per wave");
    __shared__ double lds_acc[WAVES][kMaxWorkers];
    // the wave index is the same for all lanes: tell the compiler, so that everything derived
    // from it (block base, pointers) lives in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    const int64_t seg = blockIdx.x;
    const int64_t blk = seg * WAVES + wave;  // max-abs: index of the wave's run of V blocks
    const int64_t base = blk * (int64_t)(V * kBlockCoords);
    const CsrView B{row_ptr, col, val, a.win};

    double* accd = lds_acc[wave];
    uint32_t* accu = reinterpret_cast<uint32_t*>(lds_acc[wave]);
    if (MODE == 1) {
        // the workgroup's running maxima and the count of waves that have delivered theirs
        __shared__ uint32_t wg_max[kMaxWorkers];
        __shared__ uint32_t wg_done;
        for (int i = threadIdx.x; i < a.n; i += kWave * WAVES) wg_max[i] = 0u;
        if (threadIdx.x == 0) wg_done = 0u;
        __syncthreads();  // the only barrier: at the start, where no wave has anything to wait for
        EpiMaxAbs epi{accu, lane};
        // Layer-wise scales (Sec. II-B names the layer-wise granularity): layer l owns rows
        // l*kLayerSub .. l*kLayerSub+kLayerSub-1 of the slot array (several rows, so that the
        // workgroups that walk one layer at the same time do not all hit the same words).  The
        // workgroup's LDS array collects the layer of the workgroup's first block; a wave whose
        // blocks lie in another layer (a workgroup that straddles a boundary) hands its maxima to
        // that layer's row itself.
        const int64_t last_block = (a.d - 1) / kBlockCoords;
        const int64_t wg_first = (int64_t)blockIdx.x * (WAVES * V);
        const int layer0 = a.block_layer
                               ? __builtin_amdgcn_readfirstlane((int)a.block_layer[wg_first < last_block ? wg_first : last_block])
                               : 0;
        const int sub = (int)(blockIdx.x % kLayerSub);
        auto fold = [&](int layer) {  // accu[i] was written by this wave's lane 0
            if (layer == layer0) {
                for (int i = lane; i < a.n; i += kWave)
                    (void)__hip_atomic_fetch_max(wg_max + i, accu[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            } else {
                uint32_t* dst = a.part_max + ((int64_t)layer * kLayerSub + sub) * a.n;
                for (int i = lane; i < a.n; i += kWave)
                    (void)__hip_atomic_fetch_max(dst + i, accu[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        };
        auto layer_of = [&](int64_t first_coord) {
            return a.block_layer ? __builtin_amdgcn_readfirstlane((int)a.block_layer[first_coord / kBlockCoords]) : 0;
        };
        if (base < a.d) {
            bool together = V > 1 && S != 0 && base + V * kBlockCoords <= a.d;
            if (together && a.block_layer) {  // all V blocks in one layer
                for (int u = 1; u < V; ++u)
                    together = together && layer_of(base + (int64_t)u * kBlockCoords) == layer_of(base);
            }
            if (together) {
                const LaneCoords lc = lane_coords(base, lane, a.d);  // every lane whole, in all V blocks
                if constexpr (S > 0) encode_ring<S, AGC_SCALE_PREFETCH_ROWS2, RowN<V>>(G + base, a.ldg, a.k, val, lc, epi);
                else if constexpr (S < 0) encode_window<-S, AGC_SCALE_PREFETCH_ROWS2, RowN<V>>(G + base, a.ldg, a.k, B, lc, epi);
                fold(layer_of(base));
            } else {
                for (int u = 0; u < V; ++u) {
                    const int64_t b = base + (int64_t)u * kBlockCoords;
                    if (b < a.d) {
                        const LaneCoords lc = lane_coords(b, lane, a.d);
                        encode_block<S>(G + b, a.ldg, a.n, a.k, B, lc, epi);
                        fold(layer_of(b));
                    }
                }
            }
        }
        // Nobody waits for anybody: a wave that is done makes sure its maxima have reached wg_max
        // (release fence: the wave's LDS operations have completed) and adds itself to the count;
        // the wave that finds itself last hands the workgroup's maxima to the slot array - one
        // memory-side atomic per worker and workgroup instead of one per wave.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        uint32_t before = 0u;
        if (lane == 0) before = __hip_atomic_fetch_add(&wg_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        before = (uint32_t)__builtin_amdgcn_readfirstlane((int)before);
        if (before == (uint32_t)(WAVES - 1)) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            uint32_t* dst = a.part_max + (a.block_layer ? (int64_t)layer0 * kLayerSub + sub
                                                        : ((int64_t)blockIdx.x & (kMaxSlots - 1))) * a.n;
            for (int i = lane; i < a.n; i += kWave) {
                const uint32_t m = __hip_atomic_load(wg_max + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (m != 0u) (void)__hip_atomic_fetch_max(dst + i, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        return;
    }
    // Euclidean scale per layer: segment `seg` is the table's run of up to four blocks (the tree of
    // a layer starts at the layer's first block); a wave past the run contributes nothing
    int64_t sq_base = base;
    bool sq_has = base < a.d;
    if (a.seg_first) {
        sq_base = ((int64_t)a.seg_first[seg] + wave) * (int64_t)kBlockCoords;
        sq_has = wave < (int)a.seg_blocks[seg];
    }
    if (sq_has) {
        const LaneCoords lc = lane_coords(sq_base, lane, a.d);
        EpiSumSq epi{accd, lane};
        encode_block<S>(G + sq_base, a.ldg, a.n, a.k, B, lc, epi);
    } else {  // a block past the end of the vector (or of the layer's last segment) contributes nothing
        for (int i = lane; i < a.n; i += kWave) accd[i] = 0.0;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < a.n; i += kWave * WAVES) {
        double sum = 0.0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum = sum + lds_acc[w][i];
        // [segment][worker]: one coalesced row per workgroup, non-temporal (a plain store costs the
        // pass 30 us more: the dirty lines leave the cache in the middle of the read stream)
        __builtin_nontemporal_store(sum, a.part_sq + seg * (int64_t)a.n + i);
    }
}

// rows of the max-abs slot array back to zero (context creation does it with a memset; this
// kernel serves a call that follows one whose launches failed half-way)
__global__ __launch_bounds__(kWgThreads) void k_scale_clear_slots(uint32_t* slots, int count)
{
    const int t = blockIdx.x * kWgThreads + threadIdx.x;
    if (t < count) slots[t] = 0u;
}

hipError_t launch_scale_clear_slots(int n, const Workspace& ws, hipStream_t stream)
{
    const int count = n * ws.max_rows;
    hipLaunchKernelGGL(k_scale_clear_slots, dim3((count + kWgThreads - 1) / kWgThreads), dim3(kWgThreads), 0, stream,
                       ws.part_max, count);
    return hipGetLastError();
}

#ifndef AGC_SCALE_BLOCKS_PER_WAVE
#define AGC_SCALE_BLOCKS_PER_WAVE 2
#endif
template <int S, int V>
static void launch_scale_max(const float* G, const CodeDev& code, const ScaleArgs& a, hipStream_t stream)
{
    // the widest two-block rings leave room for three waves per SIMD: workgroups of four waves
    // then fill a compute unit (three of them), workgroups of eight would not (one)
    constexpr int W = (V > 1 && S >= 7) ? 4 : AGC_SCALE_WAVES;
    const int64_t nblocks = (a.d + kBlockCoords - 1) / kBlockCoords;
    const int64_t per_wg = (int64_t)W * V;
    hipLaunchKernelGGL((k_scale_pass<S, 1, W, V>), dim3((unsigned)((nblocks + per_wg - 1) / per_wg)), dim3(kWave * W),
                       0, stream, G, code.row_ptr, code.col, code.val, a);
}

template <int S>
static hipError_t launch_scale_pass_s(const float* G, const CodeDev& code, const ScaleArgs& a,
                                      int scale_mode, hipStream_t stream)
{
    if (scale_mode == 0) {
        hipLaunchKernelGGL((k_scale_pass<S, 0, kSegBlocks, 1>), dim3((unsigned)a.nseg), dim3(kWgThreads), 0, stream, G,
                           code.row_ptr, code.col, code.val, a);
    } else {
        // two blocks per wave where a ring driver serves the code and the vector is long enough
        // to fill the chip with half as many waves
        const int64_t nblocks = (a.d + kBlockCoords - 1) / kBlockCoords;
        if (S != 0 && AGC_SCALE_BLOCKS_PER_WAVE > 1 && nblocks >= kTwoBlockMin) launch_scale_max<S, AGC_SCALE_BLOCKS_PER_WAVE>(G, code, a, stream);
        else launch_scale_max<S, 1>(G, code, a, stream);
    }
    return hipGetLastError();
}

hipError_t launch_scale_pass(const float* G, int64_t ldg, int n, int k, int64_t d,
                             const CodeDev& code, int scale_mode, const Workspace& ws,
                             hipStream_t stream)
{
    const bool layers = ws.n_layers > 0;
    ScaleArgs a{ldg, n, k, d, layers && scale_mode == 0 ? ws.nseg_layers : ws.nseg, ws.part_max, ws.part_sq, code.win,
                layers && scale_mode == 1 ? ws.block_layer : nullptr,
                layers && scale_mode == 0 ? ws.seg_first : nullptr, layers && scale_mode == 0 ? ws.seg_blocks : nullptr};
    if (code.band < 0 && !code.win) return hipErrorInvalidValue;  // the window driver reads the records
    switch (code.band) {
        case 1: return launch_scale_pass_s<1>(G, code, a, scale_mode, stream);
        case 2: return launch_scale_pass_s<2>(G, code, a, scale_mode, stream);
        case 3: return launch_scale_pass_s<3>(G, code, a, scale_mode, stream);
        case 4: return launch_scale_pass_s<4>(G, code, a, scale_mode, stream);
        case 5: return launch_scale_pass_s<5>(G, code, a, scale_mode, stream);
        case 6: return launch_scale_pass_s<6>(G, code, a, scale_mode, stream);
        case 7: return launch_scale_pass_s<7>(G, code, a, scale_mode, stream);
        case 8: return launch_scale_pass_s<8>(G, code, a, scale_mode, stream);
        case -2: return launch_scale_pass_s<-2>(G, code, a, scale_mode, stream);
        case -4: return launch_scale_pass_s<-4>(G, code, a, scale_mode, stream);
        case -8: return launch_scale_pass_s<-8>(G, code, a, scale_mode, stream);
        default: return launch_scale_pass_s<0>(G, code, a, scale_mode, stream);
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

// Euclidean scale, level 3 of the tree: one workgroup per group of 64 segments, thread t follows
// worker t through the group's rows of [segment][worker] (coalesced) and adds them in segment order.
__global__ __launch_bounds__(kWgThreads) void k_scale_groups(int n, Workspace ws)
{
    const int64_t g = blockIdx.x;
    const int64_t s1 = (g + 1) * kGroupSegs < ws.nseg ? (g + 1) * kGroupSegs : ws.nseg;
    for (int i = threadIdx.x; i < n; i += kWgThreads) {
        const double* part = ws.part_sq + i;
        double acc = 0.0;
        for (int64_t s0 = g * kGroupSegs; s0 < s1; s0 += 8) {
            double v[8];  // loads first, then the additions in segment order
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = s0 + u < s1 ? part[(s0 + u) * n] : 0.0;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < s1) acc = acc + v[u];
        }
        ws.group_sq[(int64_t)i * ws.ngroup + g] = acc;
    }
}

template <int MODE>
__global__ __launch_bounds__(kWgThreads) void k_scale_finalize(int n, QuantStreams out, StepWeights sw,
                                                               Workspace ws, float* scales)
{
    const int i = blockIdx.x;
    const int tid = threadIdx.x;
    __shared__ uint32_t red[kWgThreads];
    float scale;
    if (MODE == 1) {
        // this worker's column of the slot array: read it with loads that see the atomics of the
        // scale pass (they were performed in memory, past the caches), and leave zeros behind
        uint32_t m = 0u;
        for (int sl = tid; sl < kMaxSlots; sl += kWgThreads) {
            uint32_t* p = ws.part_max + (int64_t)sl * n + i;
            m = max(m, __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            __hip_atomic_store(p, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        red[tid] = m;
        __syncthreads();
        for (int h = kWgThreads / 2; h > 0; h >>= 1) {
            if (tid < h) red[tid] = max(red[tid], red[tid + h]);
            __syncthreads();
        }
        scale = __uint_as_float(red[0]);
    } else {
        // level 3 (64 segments -> group) was formed by k_scale_groups
        // level 4: 64 groups -> supergroup, in order
        for (int64_t u = tid; u < ws.nsuper; u += kWgThreads) {
            double acc = 0.0;
            const int64_t g1 = (u + 1) * kGroupSegs < ws.ngroup ? (u + 1) * kGroupSegs : ws.ngroup;
            for (int64_t g = u * kGroupSegs; g < g1; ++g) acc = acc + ws.group_sq[(int64_t)i * ws.ngroup + g];
            ws.super_sq[(int64_t)i * ws.nsuper + u] = acc;
        }
        __syncthreads();
        // level 5: supergroups in order
        if (tid == 0) {
            double total = 0.0;
            for (int64_t u = 0; u < ws.nsuper; ++u) total = total + ws.super_sq[(int64_t)i * ws.nsuper + u];
            red[0] = __float_as_uint((float)sqrt(total));
        }
        __syncthreads();
        scale = __uint_as_float(red[0]);
    }
    if (tid == 0) {
        scales[i] = scale;
        const int b = out.bits[i];
        // the staging area is written out after the last worker and before every worker that starts a new fill
        const uint32_t flush = (i == n - 1 || out.stage_start[i + 1] == 0) ? 1u : 0u;
        WorkerQ e{inv16_of(scale, b), (uint32_t)b, out.codes[i], 0.f, 0u, 8u * out.stage_start[i], flush};
        if (sw.fuse) {  // decode weight of one grid unit, as the decode prologue forms it
            const double L = b >= 2 ? (double)((1 << (b - 1)) - 1) : 1.0;
            e.coef = (float)(((double)sw.w[i] * (double)scale) / L);
            e.arrived = (uint32_t)sw.arrived[i];
        }
        ws.wq[i] = e;
    }
}

// Layer-wise scales: workgroup l, thread i.  The kLayerSub rows of layer l in the slot array hold
// the layer's maxima; every (worker, layer) gets its scale, and table l of the quantize pass gets the
// worker's record with the multiplier and the decode weight of that layer (the formulas of the
// per-vector case with the layer's scale).  The rows are handed back zeroed.
// Euclidean scale (MODE 0): thread i walks the layer's segment sums [segment][worker] in the order of
// the tree - 64 segments into a group, 64 groups into a supergroup, supergroups into the total,
// every sum from 0.0 in index order - with the loads of eight segments requested together.
template <int MODE>
__global__ __launch_bounds__(kWgThreads) void k_scale_finalize_layers(int n, QuantStreams out, StepWeights sw,
                                                                      Workspace ws, float* scales)
{
    const int l = blockIdx.x;
    for (int i = threadIdx.x; i < n; i += kWgThreads) {
        float scale;
        if (MODE == 1) {
            uint32_t m = 0u;
            for (int r = 0; r < kLayerSub; ++r) {
                uint32_t* p = ws.part_max + ((int64_t)l * kLayerSub + r) * n + i;
                m = max(m, __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                __hip_atomic_store(p, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            scale = __uint_as_float(m);
        } else {
            const int64_t s_begin = ws.layer_seg[l], s_end = ws.layer_seg[l + 1];
            const double* part = ws.part_sq + i;
            double total = 0.0;
            for (int64_t u0 = s_begin; u0 < s_end; u0 += (int64_t)kGroupSegs * kGroupSegs) {  // supergroups
                const int64_t u1 = u0 + (int64_t)kGroupSegs * kGroupSegs < s_end ? u0 + (int64_t)kGroupSegs * kGroupSegs : s_end;
                double super = 0.0;
                for (int64_t g0 = u0; g0 < u1; g0 += kGroupSegs) {  // groups
                    const int64_t g1 = g0 + kGroupSegs < u1 ? g0 + kGroupSegs : u1;
                    double group = 0.0;
                    for (int64_t s0 = g0; s0 < g1; s0 += 8) {
                        double v[8];
#pragma unroll
                        for (int t = 0; t < 8; ++t) v[t] = s0 + t < g1 ? part[(s0 + t) * n] : 0.0;
#pragma unroll
                        for (int t = 0; t < 8; ++t)
                            if (s0 + t < g1) group = group + v[t];
                    }
                    super = super + group;
                }
                total = total + super;
            }
            scale = (float)sqrt(total);
        }
        scales[(int64_t)i * ws.n_layers + l] = scale;
        const int b = out.bits[i];
        const uint32_t flush = (i == n - 1 || out.stage_start[i + 1] == 0) ? 1u : 0u;
        WorkerQ e{inv16_of(scale, b), (uint32_t)b, out.codes[i], 0.f, 0u, 8u * out.stage_start[i], flush};
        if (sw.fuse) {
            const double L = b >= 2 ? (double)((1 << (b - 1)) - 1) : 1.0;
            e.coef = (float)(((double)sw.w[i] * (double)scale) / L);
            e.arrived = (uint32_t)sw.arrived[i];
        }
        ws.wq[(int64_t)l * n + i] = e;
    }
}

hipError_t launch_scale_finalize(int n, int scale_mode, const QuantStreams& out, const StepWeights& sw,
                                 const Workspace& ws, float* scales, hipStream_t stream)
{
    if (ws.n_layers > 0) {
        if (scale_mode == 1)
            hipLaunchKernelGGL((k_scale_finalize_layers<1>), dim3(ws.n_layers), dim3(kWgThreads), 0, stream, n, out, sw,
                               ws, scales);
        else
            hipLaunchKernelGGL((k_scale_finalize_layers<0>), dim3(ws.n_layers), dim3(kWgThreads), 0, stream, n, out, sw,
                               ws, scales);
        return hipGetLastError();
    }
    if (scale_mode == 0) {
        hipLaunchKernelGGL(k_scale_groups, dim3((unsigned)ws.ngroup), dim3(kWgThreads), 0, stream, n, ws);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((k_scale_finalize<0>), dim3(n), dim3(kWgThreads), 0, stream, n, out, sw, ws, scales);
    } else
        hipLaunchKernelGGL((k_scale_finalize<1>), dim3(n), dim3(kWgThreads), 0, stream, n, out, sw, ws, scales);
    return hipGetLastError();
}

// =======================================================================================
// K2  encode + stochastic quantize + bit-pack: kernels in agc_quantize.h, instantiated in
// agc_quantize_b0/b1/b2.hip; here the table prologue and the launch entry points
// =======================================================================================
// table of the bucket-wise pass: bit-width and stream of every worker (the multiplier is
// found per block inside the pass)
__global__ __launch_bounds__(kWgThreads) void k_quant_table(int n, QuantStreams out, StepWeights sw, WorkerQ* wq)
{
    const int i = threadIdx.x;
    if (i >= n) return;
    const int b = out.bits[i];
    // bucket-wise scales: the multiplier is num / scale with the block's own scale; the record
    // carries the numerator L * 2^16 (2^15 for a one-bit worker)
    const float num = b >= 2 ? (float)(((1u << (b - 1)) - 1u) << 16) : 32768.0f;
    const uint32_t flush = (i == n - 1 || out.stage_start[i + 1] == 0) ? 1u : 0u;
    WorkerQ e{num, (uint32_t)b, out.codes[i], 0.f, 0u, 8u * out.stage_start[i], flush};
    if (sw.fuse) {
        const double L = b >= 2 ? (double)((1 << (b - 1)) - 1) : 1.0;
        e.coef = (float)((double)sw.w[i] / L);
        e.arrived = (uint32_t)sw.arrived[i];
    }
    wq[i] = e;
}

hipError_t launch_quantize_bucket(const float* G, int64_t ldg, int n, int k, int64_t d, const CodeDev& code,
                                  int scale_mode, const QuantStreams& out, const StepWeights& sw,
                                  const Workspace& ws, float* scales, uint64_t seed, uint64_t step, float* ghat,
                                  hipStream_t stream)
{
    hipLaunchKernelGGL(k_quant_table, dim3(1), dim3(kWgThreads), 0, stream, n, out, sw, ws.wq);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    QuantArgs a{ldg, n, k, d, (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)(step >> 32),
                scales, (d + kBlockCoords - 1) / kBlockCoords, ghat, nullptr, stage_bits_needed(out.bits, n), stage_fills(out.bits, n),
                nullptr};
    if (a.stage_fills > 1)
        return scale_mode == 0 ? launch_quantize_band2m(G, code, ws, a, stream)
                               : launch_quantize_band1m(G, code, ws, a, stream);
    return scale_mode == 0 ? launch_quantize_band2s(G, code, ws, a, stream)
                           : launch_quantize_band1s(G, code, ws, a, stream);
}

hipError_t launch_quantize(const float* G, int64_t ldg, int n, int k, int64_t d,
                           const CodeDev& code, const Workspace& ws, const uint8_t* bits, uint64_t seed,
                           uint64_t step, float* ghat, hipStream_t stream)
{
    QuantArgs a{ldg, n, k, d, (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)(step >> 32),
                nullptr, 0, ghat, nullptr, stage_bits_needed(bits, n), stage_fills(bits, n),
                ws.n_layers > 0 ? ws.block_layer : nullptr};
    return a.stage_fills > 1 ? launch_quantize_band0m(G, code, ws, a, stream)
                             : launch_quantize_band0s(G, code, ws, a, stream);
}

// =======================================================================================
// K3  masked dequantize + weighted sum
// =======================================================================================
// A lane owns 32 consecutive coordinates: for a b-bit worker these are exactly b consecutive
// 32-bit words of the stream, so unpacking needs no cross-lane traffic and every shift is a
// compile-time constant.
constexpr int kDecCoords = 32;

// prologue: one entry per ARRIVED worker, in ascending worker order
// nb == 0: one scale per worker, folded into the weight here.  nb > 0: bucket-wise scales; the
// table holds w_i / L_i and the worker's row of scales, the product is formed per bucket.
__global__ __launch_bounds__(kWgThreads) void k_decode_table(int n, DecodeStreams in,
                                                             const float* scales, int64_t nb, WorkerD* wd,
                                                             const float** srow)
{
    const int i = threadIdx.x;
    if (i >= n) return;
    const uint32_t slot = in.slot[i];
    if (slot == 0xFFFFu) return;
    const int b = in.bits[i];
    // weight of one grid unit of worker i: w_i * scale_i / L_i, binary64 then one rounding
    const double L = b >= 2 ? (double)((1 << (b - 1)) - 1) : 1.0;
    if (nb == 0) {
        wd[slot] = WorkerD{in.codes[i], (float)(((double)in.w[i] * (double)scales[i]) / L), (uint32_t)b};
    } else {
        wd[slot] = WorkerD{in.codes[i], (float)((double)in.w[i] / L), (uint32_t)b};
        srow[slot] = scales + (int64_t)i * nb;
    }
}

// second table of the two-track decode: weight of one grid unit of worker i under the
// second decoding vector, v_i * scale_i / L_i, same rounding as the first
__global__ __launch_bounds__(kWgThreads) void k_decode_table2(int n, DecodeSecond in, const float* scales,
                                                              int64_t nb, float* coef2)
{
    const int i = threadIdx.x;
    if (i >= n) return;
    const uint32_t slot = in.slot[i];
    if (slot == 0xFFFFu) return;
    const int b = in.bits[i];
    const double L = b >= 2 ? (double)((1 << (b - 1)) - 1) : 1.0;
    coef2[slot] = nb == 0 ? (float)(((double)in.v[i] * (double)scales[i]) / L) : (float)((double)in.v[i] / L);
}

template <int B, bool TWO>
__device__ __forceinline__ void decode_words(const global_u32* __restrict__ src, float coef, float coef2,
                                             float (&acc)[kDecCoords], float (&acc2)[TWO ? kDecCoords : 1])
{
    uint32_t w[B];
#pragma unroll
    for (int t = 0; t < B; ++t) w[t] = __builtin_nontemporal_load(src + t);  // each code word is read once
#pragma unroll
    for (int q = 0; q < kDecCoords; ++q) {
        const int bit = q * B;
        const int wi = bit >> 5, sh = bit & 31;
        float v;
        if (B == 1) {
            v = ((w[wi] >> sh) & 1u) ? 1.0f : -1.0f;
        } else {
            // the code's low B-1 bits are the level, its top bit the sign
            uint32_t x = w[wi];
            int s = sh;
            if (sh + B > 32) {  // the code straddles two words: bring it down to bit 0
                x = __builtin_amdgcn_alignbit(w[(wi + 1) < B ? (wi + 1) : wi], w[wi], sh);
                s = 0;
            }
            const uint32_t level = (x >> s) & ((1u << (B - 1)) - 1u);
            const uint32_t sign = (x << (32 - B - s)) & 0x80000000u;
            v = __uint_as_float(__float_as_uint((float)level) | sign);
        }
        acc[q] = fmaf(coef, v, acc[q]);
        if (TWO) acc2[TWO ? q : 0] = fmaf(coef2, v, acc2[TWO ? q : 0]);
    }
}

// Two-bit workers (sign + one level bit; most workers of a tight budget): shifted to the top of a
// word, the code's two bits are the sign and the leading exponent bit of a float, i.e. the values
// +0, +2, -0, -2 = twice the decoded value.  With half the weight the fused multiply-add has the
// same exact product and therefore the same rounded result as fma(coef, +-level, acc): three
// vector instructions per code (shift, mask, fma) instead of five.  The caller guarantees that
// halving the weights is exact (they are zero or normal numbers above the smallest exponent).
template <bool TWO>
__device__ __forceinline__ void decode_words_2bit(const global_u32* __restrict__ src, float half_coef,
                                                  float half_coef2, float (&acc)[kDecCoords],
                                                  float (&acc2)[TWO ? kDecCoords : 1])
{
    uint32_t w[2];
    w[0] = __builtin_nontemporal_load(src);
    w[1] = __builtin_nontemporal_load(src + 1);
#pragma unroll
    for (int q = 0; q < kDecCoords; ++q) {
        const int sh = 30 - 2 * (q & 15);  // brings code q of its word to bits 31..30
        const float v2 = __uint_as_float((w[q >> 4] << sh) & 0xC0000000u);
        acc[q] = fmaf(half_coef, v2, acc[q]);
        if (TWO) acc2[TWO ? q : 0] = fmaf(half_coef2, v2, acc2[TWO ? q : 0]);
    }
}

// true when x / 2 is exact in binary32: zero, or a normal number that stays normal
__device__ __forceinline__ bool halves_exactly(float x)
{
    const uint32_t e = (__float_as_uint(x) >> 23) & 0xFFu;
    return x == 0.0f || (e >= 2u && e != 0xFFu);
}

struct DecodeArgs {
    int n_arrived;
    int64_t d;
    float* ghat;
    float* ghat2;  // second track (two-track decode only)
    // layer-wise scales only: the layer of every block and the weights [layer][arrived slot]
    const uint8_t* block_layer;
    const float* coef_layer;
    const float* coef2_layer;
};

__device__ __forceinline__ void store_coords(float* dst, const float (&acc)[kDecCoords], int64_t m0, int64_t d)
{
    if (m0 + kDecCoords <= d) {
#pragma unroll
        for (int q = 0; q < kDecCoords; q += 4)
            *reinterpret_cast<float4*>(dst + q) = make_float4(acc[q], acc[q + 1], acc[q + 2], acc[q + 3]);
    } else {
#pragma unroll
        for (int q = 0; q < kDecCoords; ++q)
            if (m0 + q < d) dst[q] = acc[q];
    }
}

// Planned for six waves per SIMD (77 registers instead of 82): the kernel is short (12 waves per
// SIMD at the metric size), so one more resident wave shortens its last, partly filled round;
// measured 0.175 -> 0.168 ms.  Eight would spill.
// SCALES 0: one scale per worker (the weight of the table).  1: bucket-wise (weight of the table
// times the bucket's scale).  2: layer-wise (the weight of the lane's layer, read from the
// [layer][slot] table; a lane's 32 coordinates lie in one block and therefore in one layer).
template <bool TWO, int SCALES>
__global__ __launch_bounds__(kWgThreads) __attribute__((amdgpu_waves_per_eu(TWO ? 1 : 6, TWO ? 8 : 6))) void k_decode(const WorkerD* __restrict__ wd,
                                                       const float* __restrict__ coef2,
                                                       const float* const* __restrict__ srow, DecodeArgs a)
{
    const int64_t t = (int64_t)blockIdx.x * kWgThreads + threadIdx.x;
    const int64_t m0 = t * kDecCoords;
    if (m0 >= a.d) return;
    float acc[kDecCoords];
    float acc2[TWO ? kDecCoords : 1];
#pragma unroll
    for (int q = 0; q < kDecCoords; ++q) acc[q] = 0.f;
#pragma unroll
    for (int q = 0; q < (TWO ? kDecCoords : 1); ++q) acc2[q] = 0.f;
    constexpr bool BUCKET = SCALES != 0;  // the weights differ from lane to lane
    int64_t layer_row = 0;
    if (SCALES == 2) layer_row = (int64_t)a.block_layer[t >> 3] * a.n_arrived;
    for (int e = 0; e < a.n_arrived; ++e) {
        const WorkerD wk = wd[e];  // wave-uniform: one scalar 16-byte load
        float c1 = wk.coef;
        float c2 = TWO ? coef2[e] : 0.f;
        if (SCALES == 1) {  // the lane's 32 coordinates lie in one 256-coordinate bucket
            const float sc = ((const __attribute__((address_space(1))) float*)srow[e])[t >> 3];
            c1 = c1 * sc;
            c2 = c2 * sc;
        } else if (SCALES == 2) {
            c1 = a.coef_layer[layer_row + e];
            if (TWO) c2 = a.coef2_layer[layer_row + e];
        }
        const int b = (int)wk.bits;
        const global_u32* src = (const global_u32*)wk.codes + t * b;
        switch (b) {
            case 1: decode_words<1, TWO>(src, c1, c2, acc, acc2); break;
            case 2:
                // wave-uniform choice (without bucket-wise scales the weights are per worker)
                if (!BUCKET && halves_exactly(c1) && (!TWO || halves_exactly(c2)))
                    decode_words_2bit<TWO>(src, 0.5f * c1, 0.5f * c2, acc, acc2);
                else
                    decode_words<2, TWO>(src, c1, c2, acc, acc2);
                break;
            case 3: decode_words<3, TWO>(src, c1, c2, acc, acc2); break;
            case 4: decode_words<4, TWO>(src, c1, c2, acc, acc2); break;
            case 5: decode_words<5, TWO>(src, c1, c2, acc, acc2); break;
            case 6: decode_words<6, TWO>(src, c1, c2, acc, acc2); break;
            case 7: decode_words<7, TWO>(src, c1, c2, acc, acc2); break;
            case 8: decode_words<8, TWO>(src, c1, c2, acc, acc2); break;
            case 9: decode_words<9, TWO>(src, c1, c2, acc, acc2); break;
            case 10: decode_words<10, TWO>(src, c1, c2, acc, acc2); break;
            case 11: decode_words<11, TWO>(src, c1, c2, acc, acc2); break;
            case 12: decode_words<12, TWO>(src, c1, c2, acc, acc2); break;
            case 13: decode_words<13, TWO>(src, c1, c2, acc, acc2); break;
            case 14: decode_words<14, TWO>(src, c1, c2, acc, acc2); break;
            case 15: decode_words<15, TWO>(src, c1, c2, acc, acc2); break;
            default: decode_words<16, TWO>(src, c1, c2, acc, acc2); break;
        }
    }
    store_coords(a.ghat + m0, acc, m0, a.d);
    if constexpr (TWO) store_coords(a.ghat2 + m0, acc2, m0, a.d);
}

template <bool TWO>
static void launch_decode_kernel(int scales_kind, unsigned grid, hipStream_t stream, const Workspace& ws,
                                 const DecodeArgs& a)
{
    const float* c2 = TWO ? ws.coef2 : nullptr;
    if (scales_kind == 2)
        hipLaunchKernelGGL((k_decode<TWO, 2>), dim3(grid), dim3(kWgThreads), 0, stream, ws.wd, c2,
                           (const float* const*)nullptr, a);
    else if (scales_kind == 1)
        hipLaunchKernelGGL((k_decode<TWO, 1>), dim3(grid), dim3(kWgThreads), 0, stream, ws.wd, c2,
                           (const float* const*)ws.srow, a);
    else
        hipLaunchKernelGGL((k_decode<TWO, 0>), dim3(grid), dim3(kWgThreads), 0, stream, ws.wd, c2,
                           (const float* const*)nullptr, a);
}

// Layer-wise scales, prologue: workgroup l, thread i.  The weight of arrived worker i in layer l,
// w_i * scale_il / L_i (binary64, one rounding: the per-vector formula with the layer's scale),
// goes to [l][slot]; workgroup 0 also writes the table of streams and bit-widths.
__global__ __launch_bounds__(kWgThreads) void k_decode_table_layers(int n, int n_layers, int n_arrived,
                                                                    DecodeStreams in, const float* scales,
                                                                    WorkerD* wd, float* coef_layer)
{
    const int l = blockIdx.x;
    for (int i = threadIdx.x; i < n; i += kWgThreads) {
        const uint32_t slot = in.slot[i];
        if (slot == 0xFFFFu) continue;
        const int b = in.bits[i];
        const double L = b >= 2 ? (double)((1 << (b - 1)) - 1) : 1.0;
        coef_layer[(int64_t)l * n_arrived + slot] =
            (float)(((double)in.w[i] * (double)scales[(int64_t)i * n_layers + l]) / L);
        if (l == 0) wd[slot] = WorkerD{in.codes[i], 0.f, (uint32_t)b};
    }
}

// the same for the second decoding vector of the two-track decode
__global__ __launch_bounds__(kWgThreads) void k_decode_table2_layers(int n, int n_layers, int n_arrived,
                                                                     DecodeSecond in, const float* scales,
                                                                     float* coef2_layer)
{
    const int l = blockIdx.x;
    for (int i = threadIdx.x; i < n; i += kWgThreads) {
        const uint32_t slot = in.slot[i];
        if (slot == 0xFFFFu) continue;
        const int b = in.bits[i];
        const double L = b >= 2 ? (double)((1 << (b - 1)) - 1) : 1.0;
        coef2_layer[(int64_t)l * n_arrived + slot] =
            (float)(((double)in.v[i] * (double)scales[(int64_t)i * n_layers + l]) / L);
    }
}

hipError_t launch_decode(int n, int n_arrived, int64_t d, const DecodeStreams& in,
                         const float* scales, int64_t nb, const Workspace& ws, float* ghat,
                         hipStream_t stream)
{
    const bool layers = ws.n_layers > 0;
    if (layers)
        hipLaunchKernelGGL(k_decode_table_layers, dim3(ws.n_layers), dim3(kWgThreads), 0, stream, n, ws.n_layers,
                           n_arrived, in, scales, ws.wd, ws.coef_layer);
    else
        hipLaunchKernelGGL(k_decode_table, dim3(1), dim3(kWgThreads), 0, stream, n, in, scales, nb, ws.wd, ws.srow);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    DecodeArgs a{n_arrived, d, ghat, nullptr, ws.block_layer, ws.coef_layer, nullptr};
    const int64_t nthreads = (d + kDecCoords - 1) / kDecCoords;
    const unsigned grid = (unsigned)((nthreads + kWgThreads - 1) / kWgThreads);
    launch_decode_kernel<false>(layers ? 2 : (nb > 0 ? 1 : 0), grid, stream, ws, a);
    return hipGetLastError();
}

hipError_t launch_decode2(int n, int n_arrived, int64_t d, const DecodeStreams& in, const DecodeSecond& second,
                          const float* scales, int64_t nb, const Workspace& ws, float* ghat, float* ghat2,
                          hipStream_t stream)
{
    const bool layers = ws.n_layers > 0;
    if (layers)
        hipLaunchKernelGGL(k_decode_table_layers, dim3(ws.n_layers), dim3(kWgThreads), 0, stream, n, ws.n_layers,
                           n_arrived, in, scales, ws.wd, ws.coef_layer);
    else
        hipLaunchKernelGGL(k_decode_table, dim3(1), dim3(kWgThreads), 0, stream, n, in, scales, nb, ws.wd, ws.srow);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (layers)
        hipLaunchKernelGGL(k_decode_table2_layers, dim3(ws.n_layers), dim3(kWgThreads), 0, stream, n, ws.n_layers,
                           n_arrived, second, scales, ws.coef2_layer);
    else
        hipLaunchKernelGGL(k_decode_table2, dim3(1), dim3(kWgThreads), 0, stream, n, second, scales, nb, ws.coef2);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    DecodeArgs a{n_arrived, d, ghat, ghat2, ws.block_layer, ws.coef_layer, ws.coef2_layer};
    const int64_t nthreads = (d + kDecCoords - 1) / kDecCoords;
    const unsigned grid = (unsigned)((nthreads + kWgThreads - 1) / kWgThreads);
    launch_decode_kernel<true>(layers ? 2 : (nb > 0 ? 1 : 0), grid, stream, ws, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Decode for callers that cannot allocate (HIP graph capture, tight serving loops): the table
// of arrived workers and their rows of bucket-wise scales, which agc_decode keeps in the
// context's workspace, live in a fixed device array instead.  Each GPU holds its own copy of
// the array at its own address; host code only ever uses the address that
// hipGetSymbolAddress returned for the device that was current.
// ---------------------------------------------------------------------------------------
constexpr size_t kScratchTableBytes = sizeof(WorkerD) * kMaxWorkers;          // 4096
constexpr size_t kScratchRowsBytes = sizeof(const float*) * kMaxWorkers;      // 2048
constexpr size_t kScratchBytes = kScratchTableBytes + kScratchRowsBytes;
static_assert(kScratchBytes == kStaticScratchBytes, "size stated in the launch interface");
static_assert(kScratchTableBytes % 256 == 0, "the rows of scales start on an aligned offset");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices];  // per device: the device address of `scratch`, null = not resolved yet
}  // namespace

hipError_t launch_decode_static(int n, int n_arrived, int64_t d, const DecodeStreams& in, const float* scales,
                                int64_t nb, float* ghat, hipStream_t stream)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* base = nullptr;
    {
        std::lock_guard<std::mutex> hold(g_scratch_lock);
        if (!g_scratch_ptr[dev]) {  // first call on this device, which is the current one
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev] = p;
        }
        base = g_scratch_ptr[dev];
    }
    WorkerD* wd = reinterpret_cast<WorkerD*>(base);
    const float** srow = reinterpret_cast<const float**>(static_cast<unsigned char*>(base) + kScratchTableBytes);
    // the prologue rewrites every entry that the decode kernel reads (slots 0..n_arrived-1), so
    // nothing of the previous call's contents has to be cleared
    hipLaunchKernelGGL(k_decode_table, dim3(1), dim3(kWgThreads), 0, stream, n, in, scales, nb, wd, srow);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    DecodeArgs a{n_arrived, d, ghat, nullptr, nullptr, nullptr, nullptr};
    const int64_t nthreads = (d + kDecCoords - 1) / kDecCoords;
    const unsigned grid = (unsigned)((nthreads + kWgThreads - 1) / kWgThreads);
    if (nb > 0)
        hipLaunchKernelGGL((k_decode<false, 1>), dim3(grid), dim3(kWgThreads), 0, stream, wd, (const float*)nullptr,
                           (const float* const*)srow, a);
    else
        hipLaunchKernelGGL((k_decode<false, 0>), dim3(grid), dim3(kWgThreads), 0, stream, wd,
                           (const float*)nullptr, (const float* const*)nullptr, a);
    return hipGetLastError();
}

// Adam with the two-track estimates (Sec. V): first moment from the unbiased estimate, second
// moment from the square of the variance-reduced one.  corr1 = 1 - beta1^t, corr2 = 1 - beta2^t.
__global__ __launch_bounds__(kWgThreads) void k_adam_update(float* beta, float* m1, float* m2,
                                                            const float* __restrict__ ghat,
                                                            const float* __restrict__ ghat2, float lr, float beta1,
                                                            float beta2, float eps, float corr1, float corr2,
                                                            int64_t d)
{
    const int64_t i = (int64_t)blockIdx.x * kWgThreads + threadIdx.x;
    if (i >= d) return;
    const float g = ghat[i], h = ghat2[i];
    const float a = fmaf(beta1, m1[i], (1.0f - beta1) * g);
    const float b = fmaf(beta2, m2[i], (1.0f - beta2) * (h * h));
    m1[i] = a;
    m2[i] = b;
    beta[i] = beta[i] - lr * (a / corr1) / (sqrtf(b / corr2) + eps);
}

hipError_t launch_adam_update(float* beta, float* m1, float* m2, const float* ghat, const float* ghat2,
                              float lr, float beta1, float beta2, float eps, float corr1, float corr2,
                              int64_t d, hipStream_t stream)
{
    hipLaunchKernelGGL(k_adam_update, dim3((unsigned)((d + kWgThreads - 1) / kWgThreads)), dim3(kWgThreads), 0,
                       stream, beta, m1, m2, ghat, ghat2, lr, beta1, beta2, eps, corr1, corr2, d);
    return hipGetLastError();
}

}  // namespace agc
