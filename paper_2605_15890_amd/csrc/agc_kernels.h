// Launch interface between the C ABI (agc_api.cpp) and the gfx950 kernels (agc_kernels.hip).
// Plain structs only; every pointer is a device pointer unless it sits inside an argument
// block, which travels to the GPU as kernel arguments.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace agc {

constexpr int kArgWorkers = 256;

// Row i of a monotone-interval code as one 64-byte record, so that a kernel reads a worker's
// structure with scalar loads whose address depends on i alone (no row_ptr -> col -> val chain).
// Record n is a sentinel whose lo matches no row.
struct WindowRec {
    int lo;               // first column of the run
    int len;              // 1..8 stored entries
    int pad[6];
    float val[8];         // the entries in stored order; unused ones are 0 and never read
};
static_assert(sizeof(WindowRec) == 64, "one record is 64 bytes");

struct CodeDev {          // the code matrix B on the device
    const int* row_ptr;   // [n+1]
    const int* col;       // [nnz]
    const float* val;     // [nnz]
    int band;             // 0: generic CSR; s>0: cyclic band with s entries per row; -W: monotone intervals
    const WindowRec* win; // [n+1], monotone-interval codes only (else null)
};

// what the quantize pass needs to know about worker i, read with one scalar 32-byte load
struct WorkerQ {
    float inv16;          // L_i * 2^16 / scale_i (2^15 / scale_i for a one-bit worker); with bucket-wise
                          // scales the numerator alone, the division happens per block
    uint32_t bits;
    void* codes;          // packed stream of the worker
    // fused quantize+decode pass only: the decode weight of worker i (w_i * scale_i / L_i; with
    // bucket-wise scales w_i / L_i) and whether it arrived
    float coef;
    uint32_t arrived;
    // where the worker's codes wait in the workgroup's LDS staging area before they leave as whole
    // 128-byte lines: first 16-byte piece of the worker (a workgroup stages 8 * bits pieces per
    // worker: four blocks of 2 * bits), and whether the area is written out after this worker
    uint32_t stage_piece;
    uint32_t flush;
};
static_assert(sizeof(WorkerQ) == 32, "one record is two 16-byte scalar loads");

// The staging area of a workgroup holds the codes of consecutive workers whose bit-widths sum to
// at most kStageBits (8 * kStageBits pieces of 16 bytes); workers beyond that start a new fill.
constexpr int kStageBits = 256;

// Places the workers in the staging area (host side): start[i] = sum of the bit-widths staged
// before worker i in its fill (< kStageBits, fits a byte); a fill ends before the worker that
// would overflow it, and that worker starts the next one at 0.
inline void stage_starts(const uint8_t* bits, int n, uint8_t* start)
{
    int acc = 0;
    for (int j = 0; j < n; ++j) {
        if (acc + bits[j] > kStageBits) acc = 0;
        start[j] = (uint8_t)acc;
        acc += bits[j];
    }
}
// number of fills the workers need
inline int stage_fills(const uint8_t* bits, int n)
{
    int acc = 0, fills = n > 0 ? 1 : 0;
    for (int j = 0; j < n; ++j) {
        if (acc + bits[j] > kStageBits) {
            acc = 0;
            ++fills;
        }
        acc += bits[j];
    }
    return fills;
}
// largest fill over all groups, in bits (host side: sizes the LDS area of a launch)
inline int stage_bits_needed(const uint8_t* bits, int n)
{
    int acc = 0, most = 0;
    for (int j = 0; j < n; ++j) {
        if (acc + bits[j] > kStageBits) acc = 0;
        acc += bits[j];
        if (acc > most) most = acc;
    }
    return most;
}

// one arrived worker as the decode pass sees it
struct WorkerD {
    const void* codes;
    float coef;           // w_i * scale_i / L_i
    uint32_t bits;
};

struct Workspace {
    uint32_t* part_max;   // [max_rows][n] running max |f_i| as bit patterns, all zero between steps (max-abs scale)
    int max_rows;         // kMaxSlots, or n_layers * kLayerSub if that is more
    double* part_sq;      // [nseg][n]   per-segment sum of squares             (Euclidean scale)
    double* group_sq;     // [n][ngroup]
    double* super_sq;     // [n][nsuper]
    WorkerQ* wq;          // [n]  written by the scale finalize
    WorkerD* wd;          // [n]  arrived workers, compacted, written by the decode prologue
    float* coef2;         // [n]  second-track weights v_i * scale_i / L_i of the arrived workers
    const float** srow;   // [n]  bucket-wise scales: row of scales of every arrived worker
    int64_t nseg, ngroup, nsuper;
    // layer-wise scales (n_layers > 0; max-abs only): the layer of every 256-coordinate block, and
    // the decode weights w_i * scale_il / L_i (and v_i * ...) of the arrived workers, [layer][slot].
    // wq then holds one table per layer, [layer][n].
    const uint8_t* block_layer;  // [ceil(d/256)]
    int n_layers;
    // Euclidean scale per layer: the summation tree starts anew in every layer, so the segments
    // (up to four blocks) are counted from each layer's first block
    const int* seg_first;        // [nseg_layers] first block of the segment
    const uint8_t* seg_blocks;   // [nseg_layers] its number of blocks, 1..4
    const int* layer_seg;        // [n_layers + 1] first segment of every layer
    int64_t nseg_layers;
    float* coef_layer;    // [n_layers][n]
    float* coef2_layer;   // [n_layers][n]
};

constexpr int kMaxSlots = 256;  // rows of the max-abs array; a block folds into row (block mod kMaxSlots)
constexpr int kMaxLayers = 256;  // layer-wise scales: a block's layer fits a byte
constexpr int kLayerSub = 16;    // with layer-wise scales layer l owns rows l*kLayerSub .. +kLayerSub-1 of the array

struct QuantStreams {      // host arrays of the encode call, as kernel arguments of the finalize
    void* codes[kArgWorkers];
    uint8_t bits[kArgWorkers];
    uint8_t stage_start[kArgWorkers];  // stage_starts() of the bit-widths
};

struct StepWeights {       // decode side of a fused step, as kernel arguments of the table kernels
    float w[kArgWorkers];
    uint8_t arrived[kArgWorkers];
    int fuse;              // 0: plain encode+quantize, the two arrays are ignored
};

struct DecodeStreams {     // host arrays of the decode call, as kernel arguments of its prologue
    const void* codes[kArgWorkers];
    float w[kArgWorkers];
    uint8_t bits[kArgWorkers];
    uint16_t slot[kArgWorkers];  // position among the arrived workers, 0xFFFF for a straggler
};

struct DecodeSecond {      // second decoding vector of the two-track decode (Sec. V)
    float v[kArgWorkers];
    uint8_t bits[kArgWorkers];
    uint16_t slot[kArgWorkers];
};

// K1: partial results of every worker's scale (max-abs: running maxima in ws.part_max, per layer
// with layer-wise scales; Euclidean: per-segment sums of squares).  scale_mode: 0 Euclidean, 1 max-abs.
hipError_t launch_scale_pass(const float* G, int64_t ldg, int n, int k, int64_t d,
                             const CodeDev& code, int scale_mode, const Workspace& ws,
                             hipStream_t stream);
// all rows of the max-abs slot array back to zero
hipError_t launch_scale_clear_slots(int n, const Workspace& ws, hipStream_t stream);
// K1f: partials -> scales[n] and the per-worker table of the quantize pass (with layer-wise scales:
// scales[n][n_layers] and one table per layer).
// sw.fuse != 0: the quantize pass that follows also forms the estimate (ghat) from the codes it
// has just produced, in the same order and arithmetic as the decode kernel.
hipError_t launch_scale_finalize(int n, int scale_mode, const QuantStreams& out, const StepWeights& sw,
                                 const Workspace& ws, float* scales, hipStream_t stream);
// K2: fused encode + stochastic quantize + bit-pack.
// ghat != nullptr: fused step (the table must have been written with sw.fuse != 0).
// bits: host array of the n bit-widths (sizes the LDS staging area; the table holds them too).
hipError_t launch_quantize(const float* G, int64_t ldg, int n, int k, int64_t d,
                           const CodeDev& code, const Workspace& ws, const uint8_t* bits, uint64_t seed,
                           uint64_t step, float* ghat, hipStream_t stream);
// Bucket-wise scales (one per 256-coordinate block and worker): a table prologue, then ONE pass
// over G that derives each block's scale from the block itself.  scales: n x nb, nb = ceil(d/256).
hipError_t launch_quantize_bucket(const float* G, int64_t ldg, int n, int k, int64_t d, const CodeDev& code,
                                  int scale_mode, const QuantStreams& out, const StepWeights& sw,
                                  const Workspace& ws, float* scales, uint64_t seed, uint64_t step, float* ghat,
                                  hipStream_t stream);
// K3: table of the arrived workers (a one-workgroup prologue), then masked dequantize +
// weighted sum.
// nb = 0: one scale per worker; nb > 0: scales is n x nb, one scale per 256-coordinate bucket.
hipError_t launch_decode(int n, int n_arrived, int64_t d, const DecodeStreams& in,
                         const float* scales, int64_t nb, const Workspace& ws, float* ghat,
                         hipStream_t stream);
// Two-track variant: the same read of the codes feeds a second weighted sum with weights v.
hipError_t launch_decode2(int n, int n_arrived, int64_t d, const DecodeStreams& in, const DecodeSecond& second,
                          const float* scales, int64_t nb, const Workspace& ws, float* ghat, float* ghat2,
                          hipStream_t stream);
// The decode of launch_decode with its two small tables (arrived workers, their rows of
// bucket-wise scales) in a fixed device array of kStaticScratchBytes bytes instead of a context's
// workspace: no allocation anywhere, n <= 256.  Calls on one GPU share the array.
constexpr size_t kStaticScratchBytes = 6144;
hipError_t launch_decode_static(int n, int n_arrived, int64_t d, const DecodeStreams& in, const float* scales,
                                int64_t nb, float* ghat, hipStream_t stream);
// Adam update that takes its first moment from ghat and its second moment from ghat2.
hipError_t launch_adam_update(float* beta, float* m1, float* m2, const float* ghat, const float* ghat2,
                              float lr, float beta1, float beta2, float eps, float corr1, float corr2,
                              int64_t d, hipStream_t stream);

// Least-squares partial gradients G[p,:] = X_p^T (X_p w - y_p) (X bfloat16) and the descent update.
int ls_wg_per_part(int64_t n_rows, int n_feat, int k_parts);
hipError_t launch_ls_partial_gradients(const void* X, int64_t n_rows, int n_feat, const float* y,
                                       const float* w, int k_parts, float* G, int64_t ldg,
                                       float* resid, float* partial, hipStream_t stream);
hipError_t launch_gd_update(float* beta, const float* ghat, float lr, int64_t d, hipStream_t stream);

// measurement kernels (agc_debug.hip): plain streaming copy of `bytes` (multiple of 16) bytes, and
// the bare row-walk access pattern of the streaming passes (piece_bytes = 0: reads only)
hipError_t launch_calibration_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream);
hipError_t launch_stream_rows(const float* G, int64_t ldg, int k, int64_t d, int piece_bytes, int wg_flush,
                              int blocks_per_wave, int waves_per_simd, int fma_per_row, void* out, hipStream_t stream);

}  // namespace agc
