// C ABI of the hot path (include/agc.h): context management, synchronous argument
// validation, kernel launches on the caller's stream, optional per-kernel event timing.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <algorithm>
#include <cmath>
#include <vector>

#include "../../include/agc.h"
#include "../../include/agc_debug.h"
#include "agc_kernels.h"

namespace {

constexpr int kEventRing = 128;

struct EventPair {
    hipEvent_t beg = nullptr, end = nullptr;
};

}  // namespace

struct agc_ctx {
    int n = 0, k = 0;
    int64_t d = 0;
    agc_opts opts{};
    int device = 0;
    // code matrix
    bool slots_dirty = false;  // a scale pass may have run without its finalize (a launch failed in between)
    bool has_code = false;
    int nnz = 0;
    int* d_row_ptr = nullptr;
    int* d_col = nullptr;
    float* d_val = nullptr;
    agc::WindowRec* d_win = nullptr;   // monotone-interval codes only
    int band = 0;
    // workspace
    agc::Workspace ws{};
    // profiling
    bool profiling = false;
    std::vector<EventPair> events[AGC_NUM_KERNELS];
    int ev_head[AGC_NUM_KERNELS] = {0, 0, 0, 0};   // next slot to record
    int ev_count[AGC_NUM_KERNELS] = {0, 0, 0, 0};  // recorded, not yet drained
    double ev_ms[AGC_NUM_KERNELS] = {0, 0, 0, 0};
    int64_t ev_launches[AGC_NUM_KERNELS] = {0, 0, 0, 0};
    std::string err;
};

namespace {

thread_local std::string g_err;  // failures that have no context to hang on (agc_create)

agc_status fail(agc_ctx* ctx, agc_status st, const std::string& msg)
{
    if (ctx) ctx->err = msg;
    else g_err = msg;
    return st;
}

agc_status hip_fail(agc_ctx* ctx, hipError_t e, const char* what)
{
    return fail(ctx, AGC_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

template <class T>
hipError_t dev_alloc(T** p, size_t count)
{
    return hipMalloc(reinterpret_cast<void**>(p), count * sizeof(T));
}

void free_layers(agc_ctx* c)
{
    if (c->ws.block_layer) (void)hipFree(const_cast<uint8_t*>(c->ws.block_layer));
    if (c->ws.seg_first) (void)hipFree(const_cast<int*>(c->ws.seg_first));
    if (c->ws.seg_blocks) (void)hipFree(const_cast<uint8_t*>(c->ws.seg_blocks));
    if (c->ws.layer_seg) (void)hipFree(const_cast<int*>(c->ws.layer_seg));
    c->ws.seg_first = nullptr;
    c->ws.seg_blocks = nullptr;
    c->ws.layer_seg = nullptr;
    c->ws.nseg_layers = 0;
    if (c->ws.coef_layer) (void)hipFree(c->ws.coef_layer);
    if (c->ws.coef2_layer) (void)hipFree(c->ws.coef2_layer);
    c->ws.block_layer = nullptr;
    c->ws.coef_layer = nullptr;
    c->ws.coef2_layer = nullptr;
    c->ws.n_layers = 0;
}

void free_code(agc_ctx* c)
{
    if (c->d_row_ptr) (void)hipFree(c->d_row_ptr);
    if (c->d_col) (void)hipFree(c->d_col);
    if (c->d_val) (void)hipFree(c->d_val);
    if (c->d_win) (void)hipFree(c->d_win);
    c->d_win = nullptr;
    c->d_row_ptr = nullptr;
    c->d_col = nullptr;
    c->d_val = nullptr;
    c->has_code = false;
}

// drains the oldest recorded pair of kernel j into the totals
agc_status drain_one(agc_ctx* c, int j)
{
    const int slot = (c->ev_head[j] - c->ev_count[j] + kEventRing) % kEventRing;
    EventPair& ep = c->events[j][slot];
    hipError_t e = hipEventSynchronize(ep.end);
    if (e != hipSuccess) return hip_fail(c, e, "hipEventSynchronize");
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, ep.beg, ep.end);
    if (e != hipSuccess) return hip_fail(c, e, "hipEventElapsedTime");
    c->ev_ms[j] += ms;
    c->ev_launches[j] += 1;
    c->ev_count[j] -= 1;
    return AGC_OK;
}

struct KernelTimer {
    agc_ctx* c;
    int j;
    hipStream_t stream;
    EventPair* ep = nullptr;
    agc_status begin()
    {
        if (!c->profiling) return AGC_OK;
        if (c->ev_count[j] == kEventRing) {
            agc_status st = drain_one(c, j);
            if (st != AGC_OK) return st;
        }
        ep = &c->events[j][c->ev_head[j]];
        hipError_t e = hipEventRecord(ep->beg, stream);
        if (e != hipSuccess) return hip_fail(c, e, "hipEventRecord");
        return AGC_OK;
    }
    agc_status end()
    {
        if (!c->profiling) return AGC_OK;
        hipError_t e = hipEventRecord(ep->end, stream);
        if (e != hipSuccess) return hip_fail(c, e, "hipEventRecord");
        c->ev_head[j] = (c->ev_head[j] + 1) % kEventRing;
        c->ev_count[j] += 1;
        return AGC_OK;
    }
};

agc_status check_bits(agc_ctx* c, const uint8_t* bits)
{
    for (int i = 0; i < c->n; ++i) {
        const int b = bits[i];
        if (b > AGC_MAX_BITS || b < 1 || (b == 1 && !c->opts.allow_1bit))
            return fail(c, AGC_EBITS, "bit-width of worker " + std::to_string(i) + " is " +
                                          std::to_string(b) + " (allowed: " +
                                          (c->opts.allow_1bit ? "1" : "2") + "..16)");
    }
    return AGC_OK;
}

agc_status check_streams(agc_ctx* c, void* const* codes)
{
    for (int i = 0; i < c->n; ++i) {
        if (!codes[i]) return fail(c, AGC_EINVAL, "codes_dev[" + std::to_string(i) + "] is null");
        if (reinterpret_cast<uintptr_t>(codes[i]) & 15u)
            return fail(c, AGC_EALIGN, "codes_dev[" + std::to_string(i) + "] is not 16-byte aligned");
    }
    return AGC_OK;
}

agc::CodeDev code_dev(const agc_ctx* c)
{
    return agc::CodeDev{c->d_row_ptr, c->d_col, c->d_val, c->opts.force_generic ? 0 : c->band, c->d_win};
}

}  // namespace

extern "C" {

int64_t agc_code_bytes(int64_t d, int bits)
{
    if (d <= 0 || bits < 1 || bits > AGC_MAX_BITS) return 0;
    return ((d + 127) / 128) * 16 * (int64_t)bits;
}

int64_t agc_scales_per_worker(const agc_ctx* ctx)
{
    if (!ctx) return 0;
    if (ctx->opts.bucket) return (ctx->d + 255) / 256;
    return ctx->ws.n_layers > 0 ? ctx->ws.n_layers : 1;
}

const char* agc_last_error(const agc_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

agc_status agc_create(agc_ctx** out, int n, int k, int64_t d, const agc_opts* opts)
{
    if (!out) return AGC_EINVAL;
    *out = nullptr;
    if (n < 1 || n > AGC_MAX_WORKERS || k < 1 || k > 65536 || d < 1 || d > ((int64_t)1 << 33))
        return AGC_ESHAPE;
    agc_opts o{};
    o.scale_mode = AGC_SCALE_MAXABS;
    if (opts) {
        o = *opts;
        if (o.scale_mode != AGC_SCALE_L2 && o.scale_mode != AGC_SCALE_MAXABS) return AGC_EINVAL;
        if (o.bucket != 0 && o.bucket != 256) return AGC_EINVAL;
        for (int r : o.reserved)
            if (r != 0) return AGC_EINVAL;
    }
    agc_ctx* c = new (std::nothrow) agc_ctx;
    if (!c) return AGC_ENOMEM;
    c->n = n;
    c->k = k;
    c->d = d;
    c->opts = o;
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) {
        delete c;
        return hip_fail(nullptr, e, "hipGetDevice");
    }
    const int64_t nblocks = (d + 255) / 256;
    c->ws.nseg = (nblocks + 3) / 4;
    c->ws.ngroup = (c->ws.nseg + 63) / 64;
    c->ws.nsuper = (c->ws.ngroup + 63) / 64;
    if (o.bucket) {
        e = dev_alloc(&c->ws.srow, (size_t)n);  // the scales need no reduction workspace
    } else if (o.scale_mode == AGC_SCALE_MAXABS) {
        c->ws.max_rows = agc::kMaxSlots;
        e = dev_alloc(&c->ws.part_max, (size_t)agc::kMaxSlots * n);
        if (e == hipSuccess) e = hipMemset(c->ws.part_max, 0, sizeof(uint32_t) * (size_t)agc::kMaxSlots * n);
        // the first scale pass may run on any stream of the caller, also one that does not order
        // itself after the default stream: the zeros must be in memory before this call returns
        if (e == hipSuccess) e = hipDeviceSynchronize();
    } else {
        e = dev_alloc(&c->ws.part_sq, (size_t)c->ws.nseg * n);
        if (e == hipSuccess) e = dev_alloc(&c->ws.group_sq, (size_t)c->ws.ngroup * n);
        if (e == hipSuccess) e = dev_alloc(&c->ws.super_sq, (size_t)c->ws.nsuper * n);
    }
    if (e == hipSuccess) e = dev_alloc(&c->ws.wq, (size_t)n);
    if (e == hipSuccess) e = dev_alloc(&c->ws.wd, (size_t)n);
    if (e == hipSuccess) e = dev_alloc(&c->ws.coef2, (size_t)n);
    if (e != hipSuccess) {
        agc_destroy(c);
        return fail(nullptr, e == hipErrorOutOfMemory ? AGC_ENOMEM : AGC_EHIP,
                    std::string("workspace allocation: ") + hipGetErrorString(e));
    }
    *out = c;
    return AGC_OK;
}

void agc_destroy(agc_ctx* c)
{
    if (!c) return;
    free_code(c);
    free_layers(c);
    if (c->ws.part_max) (void)hipFree(c->ws.part_max);
    if (c->ws.part_sq) (void)hipFree(c->ws.part_sq);
    if (c->ws.group_sq) (void)hipFree(c->ws.group_sq);
    if (c->ws.super_sq) (void)hipFree(c->ws.super_sq);
    if (c->ws.wq) (void)hipFree(c->ws.wq);
    if (c->ws.wd) (void)hipFree(c->ws.wd);
    if (c->ws.coef2) (void)hipFree(c->ws.coef2);
    if (c->ws.srow) (void)hipFree(c->ws.srow);
    for (auto& ring : c->events)
        for (auto& ep : ring) {
            if (ep.beg) (void)hipEventDestroy(ep.beg);
            if (ep.end) (void)hipEventDestroy(ep.end);
        }
    delete c;
}

agc_status agc_set_code(agc_ctx* c, const int32_t* row_ptr, const int32_t* col, const float* val)
{
    if (!c) return AGC_EINVAL;
    if (!row_ptr) return fail(c, AGC_EINVAL, "row_ptr is null");
    if (row_ptr[0] != 0) return fail(c, AGC_ESHAPE, "row_ptr[0] must be 0");
    for (int i = 0; i < c->n; ++i)
        if (row_ptr[i + 1] < row_ptr[i]) return fail(c, AGC_ESHAPE, "row_ptr must be non-decreasing");
    const int nnz = row_ptr[c->n];
    if (nnz > 0 && (!col || !val)) return fail(c, AGC_EINVAL, "col/val are null");
    for (int e = 0; e < nnz; ++e)
        if (col[e] < 0 || col[e] >= c->k)
            return fail(c, AGC_ESHAPE, "column index " + std::to_string(col[e]) + " out of range");
    // cyclic band: n == k and row i stores exactly s entries (i+u) mod k, u = 0..s-1, in order
    int band = 0;
    if (c->n == c->k && nnz > 0 && nnz % c->n == 0) {
        const int s = nnz / c->n;
        bool ok = s >= 1 && s <= 8 && s <= c->k;
        for (int i = 0; ok && i < c->n; ++i) {
            ok = row_ptr[i] == i * s;
            for (int u = 0; ok && u < s; ++u) ok = col[i * s + u] == (i + u) % c->k;
        }
        if (ok) band = s;
    }
    // monotone intervals (the shape of the paper's sparse construction): every row stores a run of
    // consecutive ascending columns, at most 8 of them, and neither end of the run decreases from
    // one worker to the next.  Stored as -W, W the window (2, 4 or 8) that holds the longest run.
    if (band == 0 && nnz > 0) {
        bool ok = true;
        int longest = 0, prev_lo = 0, prev_hi = 0;
        for (int i = 0; ok && i < c->n; ++i) {
            const int e0 = row_ptr[i], len = row_ptr[i + 1] - e0;
            ok = len >= 1 && len <= 8;
            for (int u = 1; ok && u < len; ++u) ok = col[e0 + u] == col[e0] + u;
            if (!ok) break;
            const int lo = col[e0], hi = lo + len - 1;
            if (i > 0) ok = lo >= prev_lo && hi >= prev_hi;
            prev_lo = lo;
            prev_hi = hi;
            longest = std::max(longest, len);
        }
        if (ok) band = -(longest <= 2 ? 2 : (longest <= 4 ? 4 : 8));
    }
    free_code(c);
    hipError_t e = dev_alloc(&c->d_row_ptr, (size_t)c->n + 1);
    if (e == hipSuccess) e = dev_alloc(&c->d_col, (size_t)(nnz > 0 ? nnz : 1));
    if (e == hipSuccess) e = dev_alloc(&c->d_val, (size_t)(nnz > 0 ? nnz : 1));
    if (e == hipSuccess) e = hipMemcpy(c->d_row_ptr, row_ptr, sizeof(int) * ((size_t)c->n + 1), hipMemcpyHostToDevice);
    if (e == hipSuccess && nnz > 0) e = hipMemcpy(c->d_col, col, sizeof(int) * (size_t)nnz, hipMemcpyHostToDevice);
    if (e == hipSuccess && nnz > 0) e = hipMemcpy(c->d_val, val, sizeof(float) * (size_t)nnz, hipMemcpyHostToDevice);
    if (e == hipSuccess && band < 0) {  // one record per row plus the sentinel
        std::vector<agc::WindowRec> win((size_t)c->n + 1);
        for (int i = 0; i <= c->n; ++i) {
            agc::WindowRec r{};
            if (i < c->n) {
                const int e0 = row_ptr[i];
                r.lo = col[e0];
                r.len = row_ptr[i + 1] - e0;
                for (int u = 0; u < r.len; ++u) r.val[u] = val[e0 + u];
            } else {
                r.lo = INT32_MAX;
            }
            win[(size_t)i] = r;
        }
        e = dev_alloc(&c->d_win, win.size());
        if (e == hipSuccess) e = hipMemcpy(c->d_win, win.data(), sizeof(agc::WindowRec) * win.size(), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        free_code(c);
        return hip_fail(c, e, "uploading the code matrix");
    }
    c->nnz = nnz;
    c->band = band;
    c->has_code = true;
    return AGC_OK;
}

agc_status agc_set_layers(agc_ctx* c, int n_layers, const int64_t* layer_end)
{
    if (!c) return AGC_EINVAL;
    if (n_layers < 0 || n_layers > AGC_MAX_LAYERS)
        return fail(c, AGC_ESHAPE, "n_layers must lie in 0.." + std::to_string(AGC_MAX_LAYERS));
    // nothing of the old tables may still be in use by a kernel when they are replaced
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return hip_fail(c, e, "hipDeviceSynchronize");
    if (n_layers == 0) {
        free_layers(c);
        return AGC_OK;
    }
    if (c->opts.bucket) return fail(c, AGC_EINVAL, "layer-wise scales need bucket == 0");
    if (!layer_end) return fail(c, AGC_EINVAL, "layer_end is null");
    int64_t prev = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int64_t end = layer_end[l];
        if (end <= prev) return fail(c, AGC_ESHAPE, "layer ends must be positive and strictly ascending");
        if (l + 1 < n_layers && (end & 255))
            return fail(c, AGC_ESHAPE, "layer end " + std::to_string(end) + " is not a multiple of 256");
        prev = end;
    }
    if (prev != c->d) return fail(c, AGC_ESHAPE, "the last layer must end at d");
    const int64_t nblocks = (c->d + 255) / 256;
    std::vector<uint8_t> layer_of((size_t)nblocks);
    {
        int l = 0;
        for (int64_t blk = 0; blk < nblocks; ++blk) {
            while (blk * 256 >= layer_end[l]) ++l;  // ends before the last are block boundaries
            layer_of[(size_t)blk] = (uint8_t)l;
        }
    }
    // Euclidean scale: the segments of every layer's own summation tree
    const bool l2 = c->opts.scale_mode == AGC_SCALE_L2;
    std::vector<int> seg_first, layer_seg;
    std::vector<uint8_t> seg_blocks;
    if (l2) {
        int64_t first = 0;
        for (int l = 0; l < n_layers; ++l) {
            const int64_t end_block = (layer_end[l] + 255) / 256;  // one past the layer's last block
            layer_seg.push_back((int)seg_first.size());
            for (int64_t blk = first; blk < end_block; blk += 4) {
                seg_first.push_back((int)blk);
                seg_blocks.push_back((uint8_t)std::min<int64_t>(4, end_block - blk));
            }
            first = end_block;
        }
        layer_seg.push_back((int)seg_first.size());
    }
    int* d_seg_first = nullptr;
    uint8_t* d_seg_blocks = nullptr;
    int* d_layer_seg = nullptr;
    double* d_part_sq = nullptr;
    uint8_t* d_layer = nullptr;
    agc::WorkerQ* d_wq = nullptr;
    float *d_c1 = nullptr, *d_c2 = nullptr;
    uint32_t* d_max = nullptr;
    const size_t entries = (size_t)c->n * (size_t)n_layers;
    const int rows = std::max(agc::kMaxSlots, n_layers * agc::kLayerSub);
    e = dev_alloc(&d_layer, (size_t)nblocks);
    if (e == hipSuccess && !l2 && rows > c->ws.max_rows) {  // several rows of running maxima per layer
        e = dev_alloc(&d_max, (size_t)rows * c->n);
        if (e == hipSuccess) e = hipMemset(d_max, 0, sizeof(uint32_t) * (size_t)rows * c->n);
        if (e == hipSuccess) e = hipDeviceSynchronize();
    }
    if (e == hipSuccess && l2) {
        e = dev_alloc(&d_seg_first, seg_first.size());
        if (e == hipSuccess) e = dev_alloc(&d_seg_blocks, seg_blocks.size());
        if (e == hipSuccess) e = dev_alloc(&d_layer_seg, layer_seg.size());
        if (e == hipSuccess) e = dev_alloc(&d_part_sq, seg_first.size() * (size_t)c->n);
        if (e == hipSuccess) e = hipMemcpy(d_seg_first, seg_first.data(), sizeof(int) * seg_first.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(d_seg_blocks, seg_blocks.data(), seg_blocks.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(d_layer_seg, layer_seg.data(), sizeof(int) * layer_seg.size(), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = dev_alloc(&d_wq, entries);
    if (e == hipSuccess) e = dev_alloc(&d_c1, entries);
    if (e == hipSuccess) e = dev_alloc(&d_c2, entries);
    if (e == hipSuccess) e = hipMemcpy(d_layer, layer_of.data(), (size_t)nblocks, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (d_layer) (void)hipFree(d_layer);
        if (d_seg_first) (void)hipFree(d_seg_first);
        if (d_seg_blocks) (void)hipFree(d_seg_blocks);
        if (d_layer_seg) (void)hipFree(d_layer_seg);
        if (d_part_sq) (void)hipFree(d_part_sq);
        if (d_max) (void)hipFree(d_max);
        if (d_wq) (void)hipFree(d_wq);
        if (d_c1) (void)hipFree(d_c1);
        if (d_c2) (void)hipFree(d_c2);
        return fail(c, e == hipErrorOutOfMemory ? AGC_ENOMEM : AGC_EHIP,
                    std::string("layer tables: ") + hipGetErrorString(e));
    }
    free_layers(c);
    if (c->ws.wq) (void)hipFree(c->ws.wq);
    c->ws.wq = d_wq;  // one table per layer; a later return to one scale per vector uses the first
    if (d_max) {      // the larger array also serves the per-vector pass (its first kMaxSlots rows)
        (void)hipFree(c->ws.part_max);
        c->ws.part_max = d_max;
        c->ws.max_rows = rows;
    }
    c->ws.block_layer = d_layer;
    if (l2) {  // at least as many segments as the per-vector tree has: the array serves both
        (void)hipFree(c->ws.part_sq);
        c->ws.part_sq = d_part_sq;
        c->ws.seg_first = d_seg_first;
        c->ws.seg_blocks = d_seg_blocks;
        c->ws.layer_seg = d_layer_seg;
        c->ws.nseg_layers = (int64_t)seg_first.size();
    }
    c->ws.coef_layer = d_c1;
    c->ws.coef2_layer = d_c2;
    c->ws.n_layers = n_layers;
    return AGC_OK;
}

int agc_code_path(const agc_ctx* c)
{
    if (!c || !c->has_code) return -1;
    if (c->opts.force_generic) return 0;
    return c->band >= 0 ? c->band : 100 - c->band;
}

}  // extern "C"

namespace {

// Worker side of a step.  sw.fuse != 0 (agc_step): the quantize pass also forms ghat.
agc_status encode_quantize_impl(agc_ctx* c, const float* G, int64_t ldg, const uint8_t* bits,
                                uint64_t seed, uint64_t step, void* const* codes, float* scales,
                                const agc::StepWeights& sw, float* ghat, void* hip_stream)
{
    if (!c) return AGC_EINVAL;
    if (!c->has_code) return fail(c, AGC_ESTATE, "agc_set_code() has not been called");
    if (!G || !bits || !codes || !scales) return fail(c, AGC_EINVAL, "null argument");
    if (ldg < c->d || (ldg & 3)) return fail(c, AGC_EALIGN, "ldg must be >= d and a multiple of 4");
    if (reinterpret_cast<uintptr_t>(G) & 15u) return fail(c, AGC_EALIGN, "G_dev is not 16-byte aligned");
    if (reinterpret_cast<uintptr_t>(scales) & 3u) return fail(c, AGC_EALIGN, "scales_dev is not 4-byte aligned");
    agc_status st = check_bits(c, bits);
    if (st != AGC_OK) return st;
    st = check_streams(c, codes);
    if (st != AGC_OK) return st;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    const agc::CodeDev code = code_dev(c);
    agc::QuantStreams qs{};
    for (int i = 0; i < c->n; ++i) {
        qs.bits[i] = bits[i];
        qs.codes[i] = codes[i];
    }
    agc::stage_starts(qs.bits, c->n, qs.stage_start);
    hipError_t e;
    if (c->opts.bucket) {  // one pass: every block finds its own scale
        KernelTimer t{c, 2, stream};
        if ((st = t.begin()) != AGC_OK) return st;
        e = agc::launch_quantize_bucket(G, ldg, c->n, c->k, c->d, code, c->opts.scale_mode, qs, sw, c->ws, scales,
                                        seed, step, ghat, stream);
        if (e != hipSuccess) return hip_fail(c, e, "bucket-wise quantize launch");
        return t.end();
    }
    const bool maxabs = c->opts.scale_mode == AGC_SCALE_MAXABS;
    if (maxabs && c->slots_dirty) {  // the finalize hands the running maxima back zeroed; restore that after a failure
        e = agc::launch_scale_clear_slots(c->n, c->ws, stream);
        if (e != hipSuccess) return hip_fail(c, e, "clearing the scale workspace");
        c->slots_dirty = false;
    }
    {
        KernelTimer t{c, 0, stream};
        if ((st = t.begin()) != AGC_OK) return st;
        c->slots_dirty = maxabs;
        e = agc::launch_scale_pass(G, ldg, c->n, c->k, c->d, code, c->opts.scale_mode, c->ws, stream);
        if (e != hipSuccess) return hip_fail(c, e, "scale pass launch");
        if ((st = t.end()) != AGC_OK) return st;
    }
    {
        KernelTimer t{c, 1, stream};
        if ((st = t.begin()) != AGC_OK) return st;
        e = agc::launch_scale_finalize(c->n, c->opts.scale_mode, qs, sw, c->ws, scales, stream);
        if (e != hipSuccess) return hip_fail(c, e, "scale finalize launch");
        c->slots_dirty = false;
        if ((st = t.end()) != AGC_OK) return st;
    }
    {
        KernelTimer t{c, 2, stream};
        if ((st = t.begin()) != AGC_OK) return st;
        e = agc::launch_quantize(G, ldg, c->n, c->k, c->d, code, c->ws, qs.bits, seed, step, ghat, stream);
        if (e != hipSuccess) return hip_fail(c, e, "quantize launch");
        if ((st = t.end()) != AGC_OK) return st;
    }
    return AGC_OK;
}

}  // namespace

extern "C" {

agc_status agc_encode_quantize(agc_ctx* c, const float* G, int64_t ldg, const uint8_t* bits,
                               uint64_t seed, uint64_t step, void* const* codes, float* scales,
                               void* hip_stream)
{
    agc::StepWeights sw{};
    return encode_quantize_impl(c, G, ldg, bits, seed, step, codes, scales, sw, nullptr, hip_stream);
}

agc_status agc_decode(agc_ctx* c, void* const* codes, const float* scales, const uint8_t* bits,
                      const float* w, const uint8_t* mask, float* ghat, void* hip_stream)
{
    if (!c) return AGC_EINVAL;
    if (!codes || !scales || !bits || !w || !mask || !ghat) return fail(c, AGC_EINVAL, "null argument");
    if (reinterpret_cast<uintptr_t>(ghat) & 15u) return fail(c, AGC_EALIGN, "ghat_dev is not 16-byte aligned");
    agc_status st = check_bits(c, bits);
    if (st != AGC_OK) return st;
    st = check_streams(c, codes);
    if (st != AGC_OK) return st;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    agc::DecodeStreams ds{};
    int n_arrived = 0;
    for (int i = 0; i < c->n; ++i) {
        ds.codes[i] = codes[i];
        ds.w[i] = w[i];
        ds.bits[i] = bits[i];
        ds.slot[i] = mask[i] ? (uint16_t)n_arrived++ : (uint16_t)0xFFFF;
    }
    KernelTimer t{c, 3, stream};
    if ((st = t.begin()) != AGC_OK) return st;
    hipError_t e = agc::launch_decode(c->n, n_arrived, c->d, ds, scales, c->opts.bucket ? (c->d + 255) / 256 : 0, c->ws, ghat, stream);
    if (e != hipSuccess) return hip_fail(c, e, "decode launch");
    return t.end();
}

agc_status agc_decode2(agc_ctx* c, void* const* codes, const float* scales, const uint8_t* bits,
                       const float* w, const float* v, const uint8_t* mask, float* ghat, float* ghat2,
                       void* hip_stream)
{
    if (!c) return AGC_EINVAL;
    if (!codes || !scales || !bits || !w || !v || !mask || !ghat || !ghat2)
        return fail(c, AGC_EINVAL, "null argument");
    if ((reinterpret_cast<uintptr_t>(ghat) & 15u) || (reinterpret_cast<uintptr_t>(ghat2) & 15u))
        return fail(c, AGC_EALIGN, "ghat_dev / ghat2_dev is not 16-byte aligned");
    if (ghat == ghat2) return fail(c, AGC_EINVAL, "ghat_dev and ghat2_dev must be different buffers");
    agc_status st = check_bits(c, bits);
    if (st != AGC_OK) return st;
    st = check_streams(c, codes);
    if (st != AGC_OK) return st;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    agc::DecodeStreams ds{};
    agc::DecodeSecond d2{};
    int n_arrived = 0;
    for (int i = 0; i < c->n; ++i) {
        ds.codes[i] = codes[i];
        ds.w[i] = w[i];
        d2.v[i] = v[i];
        ds.bits[i] = d2.bits[i] = bits[i];
        ds.slot[i] = d2.slot[i] = mask[i] ? (uint16_t)n_arrived++ : (uint16_t)0xFFFF;
    }
    KernelTimer t{c, 3, stream};
    if ((st = t.begin()) != AGC_OK) return st;
    hipError_t e = agc::launch_decode2(c->n, n_arrived, c->d, ds, d2, scales, c->opts.bucket ? (c->d + 255) / 256 : 0, c->ws, ghat, ghat2, stream);
    if (e != hipSuccess) return hip_fail(c, e, "two-track decode launch");
    return t.end();
}

agc_status agc_decode_noalloc(int n, int64_t d, int bucket, void* const* codes, const float* scales,
                              const uint8_t* bits, const float* w, const uint8_t* mask, float* ghat,
                              void* hip_stream)
{
    if (n < 1 || d < 1 || d > ((int64_t)1 << 33)) return fail(nullptr, AGC_ESHAPE, "n_workers and d must be positive, d <= 2^33");
    if (n > AGC_MAX_WORKERS)
        return fail(nullptr, AGC_ESHAPE, "agc_decode_noalloc: n_workers = " + std::to_string(n) +
                                             " exceeds the " + std::to_string(AGC_MAX_WORKERS) +
                                             " workers the fixed device scratch array holds");
    if (bucket != 0 && bucket != 256) return fail(nullptr, AGC_EINVAL, "bucket must be 0 or 256");
    if (!codes || !scales || !bits || !w || !mask || !ghat) return fail(nullptr, AGC_EINVAL, "null argument");
    if (reinterpret_cast<uintptr_t>(ghat) & 15u) return fail(nullptr, AGC_EALIGN, "ghat_dev is not 16-byte aligned");
    agc::DecodeStreams ds{};
    int n_arrived = 0;
    for (int i = 0; i < n; ++i) {
        if (bits[i] < 1 || bits[i] > AGC_MAX_BITS)
            return fail(nullptr, AGC_EBITS, "bit-width of worker " + std::to_string(i) + " is " +
                                                std::to_string((int)bits[i]) + " (allowed: 1..16)");
        if (!codes[i]) return fail(nullptr, AGC_EINVAL, "codes_dev[" + std::to_string(i) + "] is null");
        if (reinterpret_cast<uintptr_t>(codes[i]) & 15u)
            return fail(nullptr, AGC_EALIGN, "codes_dev[" + std::to_string(i) + "] is not 16-byte aligned");
        ds.codes[i] = codes[i];
        ds.w[i] = w[i];
        ds.bits[i] = bits[i];
        ds.slot[i] = mask[i] ? (uint16_t)n_arrived++ : (uint16_t)0xFFFF;
    }
    hipError_t e = agc::launch_decode_static(n, n_arrived, d, ds, scales, bucket ? (d + 255) / 256 : 0, ghat,
                                             reinterpret_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(nullptr, e, "allocation-free decode");
    return AGC_OK;
}

agc_status agc_adam_update(float* beta_dev, float* m1_dev, float* m2_dev, const float* ghat_dev,
                           const float* ghat2_dev, float lr, float beta1, float beta2, float eps,
                           int64_t t, int64_t d, void* hip_stream)
{
    if (!beta_dev || !m1_dev || !m2_dev || !ghat_dev || !ghat2_dev || d <= 0 || t <= 0) return AGC_EINVAL;
    if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f)) return AGC_EINVAL;
    const float corr1 = (float)(1.0 - std::pow((double)beta1, (double)t));
    const float corr2 = (float)(1.0 - std::pow((double)beta2, (double)t));
    hipError_t e = agc::launch_adam_update(beta_dev, m1_dev, m2_dev, ghat_dev, ghat2_dev, lr, beta1, beta2, eps,
                                           corr1, corr2, d, reinterpret_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? AGC_OK : AGC_EHIP;
}

agc_status agc_step(agc_ctx* c, const float* G, int64_t ldg, const uint8_t* bits, const float* w,
                    const uint8_t* mask, uint64_t seed, uint64_t step, void* const* codes,
                    float* scales, float* ghat, void* hip_stream)
{
    if (!c) return AGC_EINVAL;
    // validate the decode arguments before anything is enqueued
    if (!w || !mask || !ghat) return fail(c, AGC_EINVAL, "null argument");
    if (reinterpret_cast<uintptr_t>(ghat) & 15u) return fail(c, AGC_EALIGN, "ghat_dev is not 16-byte aligned");
    if (c->opts.unfused_step) {
        agc_status st = agc_encode_quantize(c, G, ldg, bits, seed, step, codes, scales, hip_stream);
        if (st != AGC_OK) return st;
        return agc_decode(c, codes, scales, bits, w, mask, ghat, hip_stream);
    }
    // fused: the quantize pass forms the estimate from the codes it has just produced (the codes
    // are still written: they are the payload), which saves the decode kernel's read of them
    agc::StepWeights sw{};
    sw.fuse = 1;
    for (int i = 0; i < c->n; ++i) {
        sw.w[i] = w[i];
        sw.arrived[i] = mask[i] ? 1 : 0;
    }
    return encode_quantize_impl(c, G, ldg, bits, seed, step, codes, scales, sw, ghat, hip_stream);
}

int64_t agc_ls_workspace_floats(int64_t n_rows, int n_feat, int k_parts)
{
    if (n_rows <= 0 || n_feat <= 0 || k_parts <= 0) return 0;
    return (int64_t)k_parts * agc::ls_wg_per_part(n_rows, n_feat, k_parts) * n_feat;
}

agc_status agc_ls_partial_gradients(const void* X_dev, int64_t n_rows, int n_feat, const float* y_dev,
                                    const float* w_dev, int k_parts, float* G_dev, int64_t ldg,
                                    float* resid_dev, float* workspace_dev, void* hip_stream)
{
    if (!X_dev || !y_dev || !w_dev || !G_dev || !resid_dev || !workspace_dev) return AGC_EINVAL;
    if (n_rows <= 0 || k_parts <= 0 || n_feat <= 0 || n_feat > 8192 || (n_feat % 128) != 0) return AGC_ESHAPE;
    if (n_rows % ((int64_t)k_parts * 16) != 0 || ldg < n_feat) return AGC_ESHAPE;
    if ((reinterpret_cast<uintptr_t>(X_dev) & 15u) || (reinterpret_cast<uintptr_t>(workspace_dev) & 15u) ||
        (reinterpret_cast<uintptr_t>(G_dev) & 3u))
        return AGC_EALIGN;
    hipError_t e = agc::launch_ls_partial_gradients(X_dev, n_rows, n_feat, y_dev, w_dev, k_parts, G_dev, ldg,
                                                    resid_dev, workspace_dev,
                                                    reinterpret_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? AGC_OK : AGC_EHIP;
}

agc_status agc_gd_update(float* beta_dev, const float* ghat_dev, float lr, int64_t d, void* hip_stream)
{
    if (!beta_dev || !ghat_dev || d <= 0) return AGC_EINVAL;
    hipError_t e = agc::launch_gd_update(beta_dev, ghat_dev, lr, d, reinterpret_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? AGC_OK : AGC_EHIP;
}

agc_status agc_calibration_copy(void* dst_dev, const void* src_dev, int64_t bytes, void* hip_stream)
{
    if (!dst_dev || !src_dev || bytes <= 0) return AGC_EINVAL;
    if ((bytes & 15) || (reinterpret_cast<uintptr_t>(dst_dev) & 15u) || (reinterpret_cast<uintptr_t>(src_dev) & 15u))
        return AGC_EALIGN;
    if (bytes / 16 / 256 >= ((int64_t)1 << 31)) return AGC_ESHAPE;
    hipError_t e = agc::launch_calibration_copy(dst_dev, src_dev, bytes, reinterpret_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? AGC_OK : AGC_EHIP;
}

agc_status agc_debug_stream_rows(const float* G_dev, int64_t ldg, int k, int64_t d, int piece_bytes, int wg_flush,
                                 int blocks_per_wave, int waves_per_simd, int fma_per_row, void* out_dev,
                                 void* hip_stream)
{
    if (waves_per_simd != 0 && waves_per_simd != 4) return AGC_EINVAL;
    if (fma_per_row != 0 && fma_per_row != 40 && fma_per_row != 100) return AGC_EINVAL;
    if (fma_per_row != 0 && (waves_per_simd != 4 || !wg_flush || piece_bytes == 0 || blocks_per_wave != 1))
        return AGC_EINVAL;
    if (!G_dev || !out_dev) return AGC_EINVAL;
    if (k < 1 || k > 65536 || d < 1 || d > ((int64_t)1 << 33)) return AGC_ESHAPE;
    if (piece_bytes < 0 || piece_bytes > 1024 || (piece_bytes & 15)) return AGC_EINVAL;
    if (blocks_per_wave != 1 && !(blocks_per_wave == 2 && piece_bytes == 0)) return AGC_EINVAL;
    if (ldg < d || (ldg & 3) || (reinterpret_cast<uintptr_t>(G_dev) & 15u) || (reinterpret_cast<uintptr_t>(out_dev) & 15u))
        return AGC_EALIGN;
    hipError_t e = agc::launch_stream_rows(G_dev, ldg, k, d, piece_bytes, wg_flush != 0, blocks_per_wave,
                                           waves_per_simd, fma_per_row, out_dev,
                                           reinterpret_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? AGC_OK : AGC_EHIP;
}

agc_status agc_profile_enable(agc_ctx* c, int on)
{
    if (!c) return AGC_EINVAL;
    if (on && c->events[0].empty()) {
        for (auto& ring : c->events) {
            ring.resize(kEventRing);
            for (auto& ep : ring) {
                hipError_t e = hipEventCreate(&ep.beg);
                if (e == hipSuccess) e = hipEventCreate(&ep.end);
                if (e != hipSuccess) return hip_fail(c, e, "hipEventCreate");
            }
        }
    }
    c->profiling = on != 0;
    return AGC_OK;
}

agc_status agc_profile_read(agc_ctx* c, double total_ms[AGC_NUM_KERNELS],
                            int64_t launches[AGC_NUM_KERNELS])
{
    if (!c || !total_ms || !launches) return AGC_EINVAL;
    for (int j = 0; j < AGC_NUM_KERNELS; ++j) {
        while (c->ev_count[j] > 0) {
            agc_status st = drain_one(c, j);
            if (st != AGC_OK) return st;
        }
        total_ms[j] = c->ev_ms[j];
        launches[j] = c->ev_launches[j];
        c->ev_ms[j] = 0.0;
        c->ev_launches[j] = 0;
    }
    return AGC_OK;
}

}  // extern "C"
