/*
 * agc.h -- C ABI of the MI355X (gfx950) hot path of communication-efficient approximate
 * gradient coding: encode -> stochastic quantize + bit-pack -> masked dequantize + decode.
 *
 * Symbols (the paper's own letters in brackets): n workers [k], k data partitions [n],
 * d gradient coordinates [l], code matrix B [A] of shape n x k, partial gradients G
 * (k x d, row j = g_j), bit-width b_i [z_i], magnitude levels L_i = 2^(b_i-1)-1 [s_i],
 * decode weights w_i, arrival indicators mask_i [I_i], straggling probabilities p_i.
 *
 * General conventions
 *   - every entry point returns agc_status (0 = ok, negative = error); nothing throws or
 *     aborts; agc_last_error() gives a message for the last failure on a context;
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device memory
 *     of the GPU that was current when the context was created;
 *   - the caller owns every buffer it passes; the library owns only the workspace it
 *     allocates in agc_create() and allocates nothing in the per-step calls;
 *   - per-step calls validate their arguments synchronously, enqueue kernels on the given
 *     HIP stream (a hipStream_t passed as void*, NULL = the default stream) and return
 *     without waiting and without any host<->device copy: the small host arrays (bits, w,
 *     mask, code pointers) travel as kernel arguments; they enqueue nothing but kernel launches
 *     (no allocation, fill, copy or wait), so a caller may record them into a HIP graph: a
 *     replay repeats the recorded call, seed and step counter included (not while the event
 *     timing of agc_debug.h is switched on);
 *   - NaN or infinity in G is outside the contract (no check on the hot path);
 *   - a context's workspace and tables are shared by all its calls: calls on one context must be
 *     ordered (one stream, or events between streams); concurrent streams need one context each.
 *
 * Arithmetic fixed by this library (the paper leaves these open; the CPU oracle in
 * oracle/ takes the same readings):
 *   encode     binary32; first stored entry of a row: rounded product; each further entry:
 *              one fused multiply-add, in stored order;
 *   scale      AGC_SCALE_MAXABS: max_m |f_i[m]|;  AGC_SCALE_L2: (float)sqrt(S) with S the
 *              binary64 sum of squares in the fixed tree described at agc_encode_quantize;
 *   draws      Philox4x32-10, key = seed; 16-bit primary field, 32-bit secondary word
 *              (see agc_encode_quantize);
 *   payload    per worker a little-endian bit stream, code m in bits [m*b, (m+1)*b),
 *              zero-padded to whole groups of 128 codes (agc_code_bytes);
 *   decode     binary32, arrived workers in ascending order, one fused multiply-add each;
 *   bucket-wise scales (agc_opts.bucket = 256; Sec. II-B names the extension, the arithmetic is
 *              this library's): bucket u = coordinates [256u, 256u+256) below d; scale_iu = largest
 *              magnitude of f_i in the bucket, or (float)sqrt of the bucket's binary64 sum of squares
 *              (the two lowest levels of the tree); multiplier = L_i*2^16 / scale_iu (2^15 / scale_iu
 *              for one bit) as ONE correctly rounded binary32 division, 0 for an empty or overflowing
 *              bucket; rounding rule, draws, codes and payload as above; decode weight =
 *              (float)((double)w_i / L_i) * scale_iu, one binary32 product; scales_dev is n x
 *              ceil(d/256), row-major.
 */
#ifndef AGC_H
#define AGC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AGC_MAX_WORKERS 256   /* n <= 256: per-worker arguments travel in the kernel argument block */
#define AGC_MAX_BITS 16
#define AGC_MAX_LAYERS 256    /* layer-wise scales: at most this many layers */

typedef struct agc_ctx agc_ctx; /* opaque; owns device workspace and a copy of B */

typedef enum {
    AGC_OK = 0,
    AGC_EINVAL = -1, /* null pointer, non-positive size, unknown option value */
    AGC_ESHAPE = -2, /* n, k, d out of range; CSR malformed; column index out of range */
    AGC_EBITS = -3,  /* bit-width outside [2,16] (or 1 without allow_1bit) */
    AGC_EALIGN = -4, /* G or g_hat not 16-byte aligned, ldg not a multiple of 4, stream not 16-byte aligned */
    AGC_ENOMEM = -5, /* workspace allocation failed */
    AGC_EHIP = -6,   /* a HIP call failed (message in agc_last_error) */
    AGC_ESTATE = -7  /* agc_set_code() has not been called */
} agc_status;

typedef enum {
    AGC_SCALE_L2 = 0,    /* Euclidean norm: the quantizer of Sec. II-B as printed */
    AGC_SCALE_MAXABS = 1 /* largest magnitude: finer grid, still unbiased (any scale >= max|f| is) */
} agc_scale_mode;

typedef struct {
    int scale_mode;    /* agc_scale_mode */
    int allow_1bit;    /* non-zero: accept b_i = 1 (two-point grid {-scale,+scale}; outside the paper, which needs b >= 2) */
    int force_generic; /* testing hook (see agc_debug.h): non-zero = every code takes the generic gather path */
    int bucket;        /* 0: one scale per coded vector (the paper's quantizer).  256: one scale per
                          256-coordinate bucket (Sec. II-B names the bucket-wise extension): the
                          scales array becomes n x ceil(d/256) and the worker side reads G once */
    int unfused_step;  /* non-zero: agc_step runs agc_encode_quantize then agc_decode as two passes;
                          zero: one fused pass (same results bit for bit, see agc_step) */
    int reserved[3];   /* must be zero */
} agc_opts;

/* --------------------------------------------------------------------------------------
 * Context
 * ------------------------------------------------------------------------------------ */
/* Creates a context for n workers, k partitions, d coordinates on the current device and
 * allocates its workspace (scale partials: 4 bytes * 256 * n for the max-abs scale, whatever d is;
 * 8 bytes * n * ceil(d/1024) for the Euclidean one; none with bucket-wise scales; a few n-entry
 * tables).
 * opts may be NULL (AGC_SCALE_MAXABS, no 1-bit).  Limits: 1 <= n <= AGC_MAX_WORKERS,
 * 1 <= k <= 65536, 1 <= d <= 2^33. */
agc_status agc_create(agc_ctx **out, int n_workers, int k_parts, int64_t d, const agc_opts *opts);
void agc_destroy(agc_ctx *ctx);

/* Sets the code matrix B (Sec. II-A: f_i = sum_j a_ij g_j) as CSR rows over host arrays
 * row_ptr[n+1], col[nnz], val[nnz]; the arrays are copied (one synchronous upload).  The
 * order of the stored entries inside a row IS the summation order of the encode.  When
 * n == k and every row i stores exactly s <= 8 entries with columns (i+u) mod k, u=0..s-1 in
 * that order (cyclic replication), the kernels take a register sliding-window path that
 * reads every element of G once per pass; when every row is a run of at most 8 consecutive
 * ascending columns whose two ends never decrease from one worker to the next (the shape
 * agc_build_code produces), they take the same kind of path without the wrap-around; any other B
 * takes the generic gather path, which re-reads shared rows through the caches.  All three give
 * identical bits (agc_code_path tells which one a context runs). */
agc_status agc_set_code(agc_ctx *ctx, const int32_t *row_ptr, const int32_t *col, const float *val);

/* Layer-wise scales (Sec. II-B: the quantizer "at layer-wise or bucket-wise granularity"): the d
 * coordinates are cut into n_layers consecutive layers, layer l = [layer_end[l-1], layer_end[l])
 * with layer_end[-1] = 0, and every worker gets one scale per layer, of the context's kind:
 * scale_il = max over the layer of |f_i[m]|, or the Euclidean norm of the layer with the AGC_SCALE_L2
 * tree started anew at the layer's first coordinate (blocks, segments, groups and supergroups are
 * counted from there).  Everything else is the per-vector arithmetic with
 * the layer's scale in place of the vector's: inv16_il = (float)(L_i * 2^16 / scale_il), decode
 * weight (float)(((double)w_i * scale_il) / L_i); draws and payload layout do not change.  With
 * layers set, scales_dev of the per-step calls holds n x n_layers floats, [worker][layer]
 * (agc_scales_per_worker), and agc_encode_quantize, agc_decode, agc_decode2 and agc_step (both
 * forms) work on them; the worker side still reads G twice.
 *   layer_end  host, n_layers ends, strictly ascending, all but the last multiples of 256 (a
 *              256-coordinate block lies in one layer), the last equal to d
 * 1 <= n_layers <= AGC_MAX_LAYERS; n_layers == 0 returns to one scale per vector.  Needs a context
 * with bucket == 0 (AGC_EINVAL otherwise).  Synchronous (waits for the device,
 * replaces small tables); not available in agc_decode_noalloc, which has no context. */
agc_status agc_set_layers(agc_ctx *ctx, int n_layers, const int64_t *layer_end);

/* 0 = generic gather path; 1..8 = cyclic-band path with replication s; 102, 104, 108 = monotone-
 * interval path (every row a run of at most 2, 4, 8 consecutive ascending columns whose ends never
 * decrease from one worker to the next - the shape agc_build_code produces); < 0 = no code set.
 * All paths give identical bits; the last two read every element of G once per pass. */
int agc_code_path(const agc_ctx *ctx);

/* Bytes of one worker's packed stream: ceil(d/128) * 16 * bits (Sec. II-B: the payload is
 * the scale plus d codes of b bits; the padding is this library's). */
int64_t agc_code_bytes(int64_t d, int bits);

/* Scales per worker in scales_dev: 1, ceil(d/256) with bucket-wise scales, n_layers with layer-wise scales. */
int64_t agc_scales_per_worker(const agc_ctx *ctx);

const char *agc_last_error(const agc_ctx *ctx);

/* --------------------------------------------------------------------------------------
 * Hot path
 * ------------------------------------------------------------------------------------ */
/*
 * Worker side (Sec. II-A encoded message, Sec. II-B quantizer): for every worker i
 *   f_i      = sum_j B[i,j] G[j,:]                      (never written to memory)
 *   scale_i  per scale_mode over all d coordinates
 *   code     = sign << (b_i-1) | level,  level = min(floor(T/2^16) + up, L_i),
 *              T = |f| * inv16_i (binary32), inv16_i = (float)(L_i * 2^16 / scale_i) (0 when
 *              scale_i is 0 or the quotient overflows), up = U < frac(T/2^16) with the
 *              48-bit uniform U = (u16 + r2 / 2^32) / 2^16:
 *                u16 = 16-bit field (i&1)*4 + (m&3) of Philox4x32-10(key = seed,
 *                      counter = (m>>2, i>>1, step lo, step hi)), fields counted from the
 *                      low half of output word 0;
 *                r2  = word m&3 of Philox4x32-10(key = seed, counter = (m>>2, 2^31 | i,
 *                      step lo, step hi)), consulted only when u16 ties;
 *              b_i = 1 (allow_1bit): T = max(fma(f, 2^15/scale_i, 2^15), 0), code = level in {0,1};
 *   stream_i = little-endian bit stream of the d codes.
 * All n workers are encoded: a straggler still computes, its message is merely late; the
 * arrival mask is an argument of the decode only.
 *
 * AGC_SCALE_L2 tree (binary64): 256-coordinate blocks; slot l of a block owns coordinates
 * 4l..4l+3 and holds (x0^2+x1^2)+(x2^2+x3^2); exchange-add over slots at distances
 * 1,2,4,8,16,32; 4 blocks are summed in order into a segment, 64 segments in order into a
 * group, 64 groups in order into a supergroup, supergroups in order into S (every
 * sequential sum starts from 0.0).
 *
 *   G_dev      device, k x d binary32, row-major with row stride ldg elements (ldg >= d,
 *              ldg % 4 == 0, base 16-byte aligned); read-only.  The kernels load whole 16-byte
 *              groups of four coordinates: the allocation must hold (k-1)*ldg + 4*ceil(d/4)
 *              floats (always true when every row owns its full stride of ldg floats); the up to
 *              three floats past d in a row are read and ignored
 *   bits_host  host, n bytes
 *   codes_dev  host array of n device pointers; stream i has agc_code_bytes(d, b_i) bytes,
 *              16-byte aligned; fully overwritten, padding included
 *   scales_dev device, n floats; overwritten
 */
agc_status agc_encode_quantize(agc_ctx *ctx, const float *G_dev, int64_t ldg,
                               const uint8_t *bits_host, uint64_t seed, uint64_t step,
                               void *const *codes_dev, float *scales_dev, void *hip_stream);

/*
 * Master side (Sec. II-A aggregation): g_hat[m] = sum over arrived i, ascending, of
 * coef_i * v_i[m] folded with one binary32 fused multiply-add each from 0, where
 * coef_i = (float)(((double)w_i * scale_i) / L_i) and v = +-level (b_i >= 2) or +-1 (b_i = 1).
 *
 *   codes_dev, scales_dev, bits_host   as written by agc_encode_quantize (read-only)
 *   w_host     host, n floats: decode weights
 *   mask_host  host, n bytes: 1 = worker arrived, 0 = straggler (its stream is not read)
 *   ghat_dev   device, d floats, 16-byte aligned; overwritten
 */
agc_status agc_decode(agc_ctx *ctx, void *const *codes_dev, const float *scales_dev,
                      const uint8_t *bits_host, const float *w_host, const uint8_t *mask_host,
                      float *ghat_dev, void *hip_stream);

/*
 * Two-track decoding (Sec. V, extension to adaptive optimizers; Appendix F): the master applies
 * two decoding vectors to the same received codes.  g_hat is formed with w exactly as in
 * agc_decode; g_hat2 is formed in the same way with v in place of w (same order, same
 * rounding), from the same single read of the streams.
 *
 *   v_host     host, n floats: second-moment decoding vector (agc_second_moment_decoder)
 *   ghat2_dev  device, d floats, 16-byte aligned, distinct from ghat_dev; overwritten
 * Everything else as in agc_decode.
 */
agc_status agc_decode2(agc_ctx *ctx, void *const *codes_dev, const float *scales_dev,
                       const uint8_t *bits_host, const float *w_host, const float *v_host,
                       const uint8_t *mask_host, float *ghat_dev, float *ghat2_dev, void *hip_stream);

/*
 * agc_decode for callers that cannot allocate device memory and therefore cannot hold a context:
 * code under HIP graph capture, tight serving loops on the master, harnesses that forbid
 * hipMalloc.  No context: n_workers, d and bucket (0, or 256 for bucket-wise scales) are passed
 * directly; a one-bit stream is always accepted.  Same kernels, same arithmetic and the same bits
 * in g_hat as agc_decode.  The small tables the decode kernel reads (one 16-byte record and one
 * row pointer per arrived worker) live in a fixed 6144-byte device array inside the library,
 * which every GPU the library runs on holds until the process ends; hence n_workers <= 256
 * (AGC_ESHAPE with a message otherwise).  The call itself and everything below it performs no
 * hipMalloc/hipFree; the first call on a device looks the array's address up once (make that
 * call before starting a graph capture).  All calls on one GPU share the array: calls that
 * overlap on one GPU (different streams without an event between them, or different threads)
 * race on it and must be serialised by the caller.  Errors are reported through
 * agc_last_error(NULL).
 */
agc_status agc_decode_noalloc(int n_workers, int64_t d, int bucket, void *const *codes_dev,
                              const float *scales_dev, const uint8_t *bits_host, const float *w_host,
                              const uint8_t *mask_host, float *ghat_dev, void *hip_stream);

/* One whole pass, with the outputs of agc_encode_quantize followed by agc_decode on the same
 * stream (codes, scales, g_hat; identical bits).  By default the quantize kernel also forms
 * g_hat from the codes it has just produced, in the order and arithmetic of agc_decode, so the
 * payload is written but not read back; agc_opts.unfused_step selects the two-pass form. */
agc_status agc_step(agc_ctx *ctx, const float *G_dev, int64_t ldg, const uint8_t *bits_host,
                    const float *w_host, const uint8_t *mask_host, uint64_t seed, uint64_t step,
                    void *const *codes_dev, float *scales_dev, float *ghat_dev, void *hip_stream);

/* --------------------------------------------------------------------------------------
 * End-to-end least-squares loop (the producer of G and the consumer of g_hat)
 * ------------------------------------------------------------------------------------ */
/* Partial gradients of the least-squares loss 0.5 * ||X_p beta - y_p||^2 of k equal, contiguous
 * data partitions (Sec. II-A: g_j = grad L(D_j, beta)):  G[p,:] = X_p^T (X_p beta - y_p).
 *   X_dev     device, n_rows x n_feat bfloat16 (upper halves of binary32), row-major, 16-byte aligned
 *   y_dev     device, n_rows floats;  beta_dev  device, n_feat floats
 *   G_dev     device, k_parts x n_feat floats with row stride ldg; overwritten
 *   resid_dev device, n_rows floats; receives X beta - y (its squared norm is twice the loss)
 *   workspace_dev device, agc_ls_workspace_floats(...) floats, 16-byte aligned; scratch
 * Products are exact (beta enters as an exact three-way bfloat16 split on the matrix cores),
 * accumulation is binary32 in a fixed order, so the result is reproducible run to run.
 * Shapes: n_feat a multiple of 128 and <= 8192; n_rows a multiple of 16 * k_parts (AGC_ESHAPE). */
int64_t agc_ls_workspace_floats(int64_t n_rows, int n_feat, int k_parts);
agc_status agc_ls_partial_gradients(const void *X_dev, int64_t n_rows, int n_feat, const float *y_dev,
                                    const float *beta_dev, int k_parts, float *G_dev, int64_t ldg,
                                    float *resid_dev, float *workspace_dev, void *hip_stream);
/* Gradient-descent update of Sec. II-A: beta <- beta - lr * g_hat (one fused multiply-add per
 * coordinate), device pointers, d floats each. */
agc_status agc_gd_update(float *beta_dev, const float *ghat_dev, float lr, int64_t d, void *hip_stream);
/* Adam step t (t >= 1) that consumes the two tracks of agc_decode2 (Sec. V; update ratio of
 * Appendix F): the first-moment average takes g_hat, the second-moment average takes the
 * square of g_hat2; binary32 throughout:
 *   m1 <- beta1*m1 + (1-beta1)*g_hat;  m2 <- beta2*m2 + (1-beta2)*g_hat2^2;
 *   beta <- beta - lr * (m1/(1-beta1^t)) / (sqrt(m2/(1-beta2^t)) + eps).
 * The bias corrections and eps are the customary ones of the optimizer; the paper prints only
 * the ratio.  All pointers device, d floats each; beta, m1, m2 updated in place. */
agc_status agc_adam_update(float *beta_dev, float *m1_dev, float *m2_dev, const float *ghat_dev,
                           const float *ghat2_dev, float lr, float beta1, float beta2, float eps,
                           int64_t t, int64_t d, void *hip_stream);

/* --------------------------------------------------------------------------------------
 * Host-side design routines (no GPU work; run once per change of the system statistics)
 * ------------------------------------------------------------------------------------ */
/* phi(z) = phi_coef / (2^(z-1)-1)^2.  The paper's constant is phi_coef = d/4 (Sec. II-B);
 * the error-balance scaling of Sec. V-B gives phi_coef = mean(p) * (2^(z_total/n - 1) - 1)^2,
 * returned by this helper. */
double agc_phi_coef_balanced(int n, const double *p, int z_total);

/* Low-complexity bit allocation (Sec. III-B.2, Algorithm 1): maximises
 * F = sum_i (1-p_i)/(p_i + phi(z_i)) subject to sum z_i = z_total, z_min <= z_i <= z_max
 * (z_max is this library's cap; the paper has none).  Steps the paper leaves open are read
 * as: Lagrangian candidate by bisection on the multiplier with each active worker on the
 * concave branch of its utility, rounded by largest remainder; equal candidate
 * floor/ceil; best-improvement one-bit swaps inside the active set.  bits_out: n bytes. */
agc_status agc_alloc_bits(int n, const double *p, double phi_coef, int z_total, int z_min,
                          int z_max, uint8_t *bits_out);
/* Optimal allocation by the Bellman recurrence of Sec. III-B.1 (O(n * z_res^2)). */
agc_status agc_alloc_bits_dp(int n, const double *p, double phi_coef, int z_total, int z_min,
                             int z_max, uint8_t *bits_out);
/* F(z) of problem b-SP1 for a given allocation. */
double agc_alloc_objective(int n, const double *p, double phi_coef, const uint8_t *bits);

/* Optimally structured sparse code (Theorem 1 and the interval construction of Sec. III-A):
 * c_i = (p_i + phi(b_i))/(1-p_i), Y_i = c_i^-1 k / sum c^-1, R_i = prefix sums,
 * alpha_ij = [min(R_i, j) - max(R_{i-1}, j-1)]_+, then a_ij = alpha_ij, w_i = 1/(1-p_i)
 * (the free factor w~_i is taken as 1).  Outputs: CSR over caller arrays row_ptr[n+1],
 * col[cap], val[cap] with columns ascending, w_out[n]; *nnz receives the count
 * (<= n + k - 1); cap is the capacity of col/val (AGC_ESHAPE when too small). */
agc_status agc_build_code(int n, int k, const double *p, const uint8_t *bits, double phi_coef,
                          int32_t *row_ptr, int32_t *col, float *val, float *w_out, int cap,
                          int *nnz);
/* Code on the cyclic support {i, .., i+s-1 mod k} (n == k): alpha_ij = c_i^-1 / (sum of
 * c^-1 over the workers holding j); column sums are 1, so the estimator is unbiased; it is a
 * heuristic on a prescribed support, not Theorem 1's optimum.  col/val hold n*s entries in
 * the order u = 0..s-1. */
agc_status agc_build_cyclic_code(int n, int k, int s, const double *p, const uint8_t *bits,
                                 double phi_coef, int32_t *row_ptr, int32_t *col, float *val,
                                 float *w_out);
/* Optimum of the structure problem (Sec. III-A, problem c-SP2) restricted to the same cyclic
 * support: minimises sum_i c_i (sum_j alpha_i^j)^2 over alpha >= 0 with column sums 1, by exact
 * minimisation over one column at a time (convex, converges to the optimum).  When the support
 * admits the row sums of Theorem 1 the result has them and *objective equals k^2 / sum_i c_i^-1
 * (then *reaches_bound = 1); otherwise it is the best the support allows.  A worker may end with
 * zero weight on a partition it holds (the entry is kept, with value 0, so that the layout stays
 * cyclic).  Outputs as agc_build_cyclic_code; objective and reaches_bound may be NULL. */
agc_status agc_build_cyclic_code_opt(int n, int k, int s, const double *p, const uint8_t *bits,
                                     double phi_coef, int32_t *row_ptr, int32_t *col, float *val,
                                     float *w_out, double *objective, int *reaches_bound);
/* Unbiasedness condition of Sec. III: max_j | sum_i (1-p_i) w_i a_ij - 1 | <= tol (binary64
 * over the binary32 inputs).  AGC_OK when it holds, AGC_EINVAL when it does not;
 * *residual (may be NULL) receives the maximum. */
agc_status agc_check_unbiased(int n, int k, const int32_t *row_ptr, const int32_t *col,
                              const float *val, const float *w, const double *p, double tol,
                              double *residual);

/* Second-moment decoding vector of the two-track decode (Sec. V, closed form below the
 * bias-variance objective): with A_i the i-th row sum of the code and c_i = (p_i+phi(z_i))/(1-p_i),
 *   v_i = k * Lambda / ((p_i + phi(z_i)) * A_i * (1 + Lambda * sum_m 1/c_m)),
 * k being the number of columns of the code (the count the bias term sums over).  Lambda > 0
 * weighs squared bias against variance.  v_out: host, n floats. */
agc_status agc_second_moment_decoder(int n, int k, const int32_t *row_ptr, const int32_t *col,
                                     const float *val, const double *p, const uint8_t *bits,
                                     double phi_coef, double Lambda, float *v_out);

#ifdef __cplusplus
}
#endif
#endif /* AGC_H */
