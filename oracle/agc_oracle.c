/*
 * agc_oracle.c -- CPU oracle for the approximate-gradient-coding hot path
 *                 (encode -> stochastic quantize + bit-pack -> masked decode).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, single-pass
 * implementation written from the paper's definitions; it shares no code,
 * header, table or helper with the HIP library and must never be called from
 * the product path.  Only the tests, the smoke check and the bench's
 * cpu_baseline leg may load it.
 *
 * Notation (repo/ABI symbols; the paper's letters in brackets):
 *   n workers [k], k partitions [n], d coordinates [l], code matrix B [A],
 *   bit-width b_i [z_i], magnitude levels L_i = 2^(b_i-1)-1 [s_i],
 *   decode weight w_i, arrival indicator mask_i [I_i].
 *
 * What the paper fixes and what it leaves open
 *   - Sec. II-A: coded gradient f_i = sum_j a_ij g_j; master estimate
 *     g_hat = sum_i I_i w_i Q_i(f_i)                          (fixed)
 *   - Sec. II-B: Q_i(x)_m = scale * sign(x_m) * xi, xi on the grid
 *     {0,1/L,..,1}, rounded up with probability L*u - floor(L*u), u=|x_m|/scale;
 *     scale is the Euclidean norm of x; b_i >= 2                (fixed)
 *   - floating-point precision, summation order, the random generator, the
 *     resolution of the uniform draw, the wire layout of the payload: the
 *     paper is silent.  The readings taken here are stated at each function.
 *
 * Every floating-point operation below that decides a code is IEEE binary32
 * (one rounding per statement; the file must be compiled with
 * -ffp-contract=off and without fast-math).  Accumulations that only feed a
 * norm are IEEE binary64 in a fixed tree.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* Counter-based random numbers: Philox4x32 with 10 rounds                     */
/* (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3", */
/*  SC'11).  The paper only asks for "lightweight shared random seeds"        */
/*  (Sec. II-B, last paragraph); the generator is this build's choice.        */
/* ------------------------------------------------------------------------- */
void agc_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                              uint32_t out[4])
{
    const uint32_t MUL_A = 0xD2511F53u; /* multiplies word 0 */
    const uint32_t MUL_B = 0xCD9E8D57u; /* multiplies word 2 */
    const uint32_t WEYL_0 = 0x9E3779B9u;
    const uint32_t WEYL_1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += WEYL_0;
            k1 += WEYL_1;
        }
        uint64_t pa = (uint64_t)MUL_A * (uint64_t)c0;
        uint64_t pb = (uint64_t)MUL_B * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)pb;
        uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)pa;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * The two uniform draws of (worker i, coordinate m) at (seed, step).
 *
 * Reading (paper silent): the rounding decision uses a 48-bit uniform,
 * delivered lazily as a 16-bit primary field u16 and a 32-bit secondary word
 * r2 that only matters when the primary field ties (see quantize_one).
 *
 *   primary  : key = (seed lo, seed hi), counter = (m>>2, i>>1, step lo, step hi);
 *              the 128 output bits are eight 16-bit fields; field number
 *              (i&1)*4 + (m&3), counted from the low half of word 0 upward.
 *   secondary: same key, counter = (m>>2, 2^31 | i, step lo, step hi); word m&3.
 * One primary block therefore serves 4 coordinates of 2 consecutive workers.
 */
void agc_oracle_draw(uint64_t seed, uint64_t step, uint32_t worker, uint64_t m,
                     uint32_t *u16, uint32_t *r2)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4], out[4];
    ctr[0] = (uint32_t)(m >> 2);
    ctr[2] = (uint32_t)step;
    ctr[3] = (uint32_t)(step >> 32);

    ctr[1] = worker >> 1;
    agc_oracle_philox4x32_10(ctr, key, out);
    uint32_t field = (worker & 1u) * 4u + (uint32_t)(m & 3u);
    uint32_t word = out[field >> 1];
    *u16 = (field & 1u) ? (word >> 16) : (word & 0xFFFFu);

    ctr[1] = 0x80000000u | worker;
    agc_oracle_philox4x32_10(ctr, key, out);
    *r2 = out[m & 3u];
}

/* ------------------------------------------------------------------------- */
/* Encode: f_i[m] = sum_j B[i,j] G[j,m]            (Sec. II-A, encoded message) */
/* ------------------------------------------------------------------------- */
/*
 * B is given as CSR rows (row_ptr, col, val).  Reading (paper silent on
 * arithmetic): binary32; the first stored entry contributes a rounded product,
 * every further stored entry is folded in with one fused multiply-add, in the
 * stored order of the row.  An empty row gives 0.
 */
float agc_oracle_encode_one(const float *G, int64_t ldg, const int32_t *row_ptr,
                            const int32_t *col, const float *val, int i, int64_t m)
{
    int e0 = row_ptr[i], e1 = row_ptr[i + 1];
    if (e0 >= e1) return 0.0f;
    float acc = val[e0] * G[(int64_t)col[e0] * ldg + m];
    for (int e = e0 + 1; e < e1; ++e)
        acc = fmaf(val[e], G[(int64_t)col[e] * ldg + m], acc);
    return acc;
}

void agc_oracle_encode_range(const float *G, int64_t ldg, const int32_t *row_ptr,
                             const int32_t *col, const float *val, int i,
                             int64_t m0, int64_t m1, float *f_out)
{
    for (int64_t m = m0; m < m1; ++m)
        f_out[m - m0] = agc_oracle_encode_one(G, ldg, row_ptr, col, val, i, m);
}

/* ------------------------------------------------------------------------- */
/* Scale of a coded vector                     (Sec. II-B, quantizer definition) */
/* ------------------------------------------------------------------------- */
/* mode 1: largest magnitude (exact, order-free).  Any scale >= max|f| keeps the
 * normalised magnitude in [0,1], so the quantizer stays unbiased.            */
float agc_oracle_scale_maxabs(const float *f, int64_t d)
{
    float mx = 0.0f;
    for (int64_t m = 0; m < d; ++m) {
        float a = fabsf(f[m]);
        if (a > mx) mx = a;
    }
    return mx;
}

/*
 * mode 0: the Euclidean norm, as the paper defines the quantizer.  Binary64
 * accumulation of exact squares in a fixed tree, so that the value does not
 * depend on who computes it:
 *   level 0  a block is 256 consecutive coordinates, slot l (0..63) owns the
 *            four coordinates 4l..4l+3 of the block; coordinates >= d count 0;
 *            slot value = (x0^2 + x1^2) + (x2^2 + x3^2);
 *   level 1  exchange-add over slots with distances 1,2,4,8,16,32
 *            (v[l] <- v[l] + v[l xor h]); block value = v[0];
 *   level 2  4 consecutive blocks form a segment: sequential sum from 0.0;
 *   level 3  64 consecutive segments form a group: sequential sum from 0.0;
 *   level 4  64 consecutive groups form a supergroup: sequential sum from 0.0;
 *   level 5  supergroups: sequential sum from 0.0.
 * scale = (float) sqrt(total).
 */
static double l2_block(const float *f, int64_t d, int64_t block)
{
    double v[64], t[64];
    for (int l = 0; l < 64; ++l) {
        double x[4];
        for (int c = 0; c < 4; ++c) {
            int64_t m = block * 256 + 4 * l + c;
            x[c] = (m < d) ? (double)f[m] : 0.0;
        }
        double s01 = x[0] * x[0] + x[1] * x[1];
        double s23 = x[2] * x[2] + x[3] * x[3];
        v[l] = s01 + s23;
    }
    for (int h = 1; h < 64; h <<= 1) {
        for (int l = 0; l < 64; ++l) t[l] = v[l] + v[l ^ h];
        memcpy(v, t, sizeof v);
    }
    return v[0];
}

double agc_oracle_sumsq_tree(const float *f, int64_t d)
{
    int64_t nblocks = (d + 255) / 256;
    int64_t nsegs = (nblocks + 3) / 4;
    int64_t ngroups = (nsegs + 63) / 64;
    int64_t nsuper = (ngroups + 63) / 64;
    double total = 0.0;
    for (int64_t u = 0; u < nsuper; ++u) {
        double usum = 0.0;
        for (int64_t g = u * 64; g < (u + 1) * 64 && g < ngroups; ++g) {
            double gsum = 0.0;
            for (int64_t s = g * 64; s < (g + 1) * 64 && s < nsegs; ++s) {
                double ssum = 0.0;
                for (int64_t b = s * 4; b < (s + 1) * 4 && b < nblocks; ++b)
                    ssum = ssum + l2_block(f, d, b);
                gsum = gsum + ssum;
            }
            usum = usum + gsum;
        }
        total = total + usum;
    }
    return total;
}

float agc_oracle_scale_l2(const float *f, int64_t d)
{
    return (float)sqrt(agc_oracle_sumsq_tree(f, d));
}

/* ------------------------------------------------------------------------- */
/* Quantizer                         (Sec. II-B, stochastic-rounding rule)      */
/* ------------------------------------------------------------------------- */
/* number of magnitude levels: 2^(b-1)-1 for b >= 2 (paper); the one-bit
 * extension (not in the paper, which requires b >= 2) uses the two-point grid
 * {-scale,+scale} and is given L = 1 here. */
int agc_oracle_levels(int bits)
{
    return bits >= 2 ? (1 << (bits - 1)) - 1 : 1;
}

/*
 * Multiplier that maps a coordinate to its position on the grid, pre-scaled by
 * 2^16 so that the integer part of T = |f|*inv16 carries the grid cell in its
 * high bits and the first 16 bits of the round-up probability in its low bits.
 *   b >= 2 : inv16 = L * 2^16 / scale
 *   b == 1 : inv16 =     2^15 / scale
 * evaluated in binary64 and rounded once to binary32; 0 when scale is 0 or
 * the quotient is not finite in binary32 (vector treated as all-zero).
 */
float agc_oracle_inv16(float scale, int bits)
{
    if (!(scale > 0.0f)) return 0.0f;
    double num = bits >= 2 ? (double)agc_oracle_levels(bits) * 65536.0 : 32768.0;
    float q = (float)(num / (double)scale);
    if (!(q <= 3.402823466e+38f)) return 0.0f;
    return q;
}

/* grid position of one coordinate, binary32: T = |f|*inv16 (b>=2) or
 * max(fma(f, inv16, 2^15), 0) (b==1: position of (1+f/scale)/2 on [0,1]). */
float agc_oracle_grid_pos(float f, float inv16, int bits)
{
    if (bits >= 2) return fabsf(f) * inv16;
    float t = fmaf(f, inv16, 32768.0f);
    return t > 0.0f ? t : 0.0f;
}

/*
 * One rounding decision.  Ti = floor(T); cell lo = Ti >> 16; the probability of
 * rounding up is (T - lo*2^16)/2^16 = (Fi + g)/2^16 with Fi = Ti & 0xFFFF and
 * g = T - Ti in [0,1).  With U = (u16 + r2/2^32)/2^16 uniform on [0,1):
 *   up  <=>  U < (Fi+g)/2^16  <=>  u16 < Fi  or  (u16 == Fi and r2 < g*2^32).
 * level = min(lo + up, L)  (the clamp only acts when binary32 rounding pushed
 * T past L*2^16, e.g. at |f| == scale).  For b >= 2 the code is
 * sign << (b-1) | level with sign = sign bit of f; for b == 1 the code is level.
 */
uint32_t agc_oracle_quantize_one(float f, float inv16, int bits, uint32_t u16,
                                 uint32_t r2)
{
    float T = agc_oracle_grid_pos(f, inv16, bits);
    uint32_t Ti = (uint32_t)T;
    float g = T - (float)Ti;
    uint32_t lo = Ti >> 16, Fi = Ti & 0xFFFFu;
    int up = (u16 < Fi) || (u16 == Fi && (double)r2 < (double)g * 4294967296.0);
    uint32_t L = (uint32_t)agc_oracle_levels(bits);
    uint32_t level = lo + (uint32_t)up;
    if (level > L) level = L;
    if (bits == 1) return level;
    uint32_t sign = signbit(f) ? 1u : 0u;
    return (sign << (bits - 1)) | level;
}

/* The cell and the exact round-up probability of that decision (binary64),
 * for the enumeration tests. */
void agc_oracle_quantize_prob(float f, float inv16, int bits, uint32_t *lo_out,
                              double *p_up)
{
    float T = agc_oracle_grid_pos(f, inv16, bits);
    uint32_t Ti = (uint32_t)T;
    float g = T - (float)Ti;
    *lo_out = Ti >> 16;
    *p_up = ((double)(Ti & 0xFFFFu) + (double)g) / 65536.0;
}

/* ------------------------------------------------------------------------- */
/* Payload layout                         (Sec. II-B: norm + quantized coords)  */
/* ------------------------------------------------------------------------- */
/* Reading (paper silent): worker i's codes form a little-endian bit stream;
 * code m occupies bits [m*b, (m+1)*b); bit q of the stream is bit (q & 7) of
 * byte (q >> 3).  The stream is zero-padded to whole groups of 128 codes,
 * i.e. to ceil(d/128) * 16 * b bytes. */
int64_t agc_oracle_code_bytes(int64_t d, int bits)
{
    return ((d + 127) / 128) * 16 * (int64_t)bits;
}

void agc_oracle_pack(const uint32_t *codes, int64_t d, int bits, uint8_t *stream)
{
    memset(stream, 0, (size_t)agc_oracle_code_bytes(d, bits));
    for (int64_t m = 0; m < d; ++m)
        for (int t = 0; t < bits; ++t)
            if ((codes[m] >> t) & 1u) {
                int64_t q = m * bits + t;
                stream[q >> 3] |= (uint8_t)(1u << (q & 7));
            }
}

uint32_t agc_oracle_unpack_one(const uint8_t *stream, int bits, int64_t m)
{
    uint32_t code = 0;
    for (int t = 0; t < bits; ++t) {
        int64_t q = m * bits + t;
        code |= (uint32_t)((stream[q >> 3] >> (q & 7)) & 1u) << t;
    }
    return code;
}

void agc_oracle_unpack_range(const uint8_t *stream, int bits, int64_t m0, int64_t m1,
                             uint32_t *codes)
{
    for (int64_t m = m0; m < m1; ++m) codes[m - m0] = agc_oracle_unpack_one(stream, bits, m);
}

void agc_oracle_unpack(const uint8_t *stream, int64_t d, int bits, uint32_t *codes)
{
    for (int64_t m = 0; m < d; ++m) codes[m] = agc_oracle_unpack_one(stream, bits, m);
}

/* ------------------------------------------------------------------------- */
/* Decode: g_hat = sum_i I_i w_i Q_i(f_i)       (Sec. II-A, master aggregation)  */
/* ------------------------------------------------------------------------- */
/* dequantized value of a code in units of scale/L: +-level (b>=2), +-1 (b==1) */
float agc_oracle_code_value(uint32_t code, int bits)
{
    if (bits == 1) return code ? 1.0f : -1.0f;
    uint32_t level = code & ((1u << (bits - 1)) - 1u);
    float v = (float)level;
    return ((code >> (bits - 1)) & 1u) ? -v : v;
}

/* weight of one grid unit of worker i in the estimate: w*scale/L, product and
 * quotient in binary64, rounded once to binary32 */
float agc_oracle_coef(float w, float scale, int bits)
{
    return (float)(((double)w * (double)scale) / (double)agc_oracle_levels(bits));
}

/* Reading (paper silent on arithmetic): binary32, arrived workers folded in
 * ascending worker order with one fused multiply-add each, starting from 0. */
void agc_oracle_decode_range(int n, const uint8_t *const *streams,
                             const float *scales, const uint8_t *bits,
                             const float *w, const uint8_t *mask, int64_t m0,
                             int64_t m1, float *ghat_out)
{
    float *coef = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    for (int i = 0; i < n; ++i) coef[i] = agc_oracle_coef(w[i], scales[i], bits[i]);
    for (int64_t m = m0; m < m1; ++m) {
        float acc = 0.0f;
        for (int i = 0; i < n; ++i) {
            if (!mask[i]) continue;
            float v = agc_oracle_code_value(
                agc_oracle_unpack_one(streams[i], bits[i], m), bits[i]);
            acc = fmaf(coef[i], v, acc);
        }
        ghat_out[m - m0] = acc;
    }
    free(coef);
}

/* ------------------------------------------------------------------------- */
/* Whole stages                                                                */
/* ------------------------------------------------------------------------- */
/* scales of all workers (a full pass over d).  scale_mode: 0 = Euclidean norm,
 * 1 = largest magnitude. */
void agc_oracle_scales(int n, int64_t d, const float *G, int64_t ldg,
                       const int32_t *row_ptr, const int32_t *col,
                       const float *val, int scale_mode, float *scales_out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        float *f = (float *)malloc(sizeof(float) * (size_t)d);
        agc_oracle_encode_range(G, ldg, row_ptr, col, val, i, 0, d, f);
        scales_out[i] = scale_mode == 0 ? agc_oracle_scale_l2(f, d)
                                        : agc_oracle_scale_maxabs(f, d);
        free(f);
    }
}

/* codes of worker i for coordinates [m0, m1), unpacked, given its scale */
void agc_oracle_codes_range(const float *G, int64_t ldg, const int32_t *row_ptr,
                            const int32_t *col, const float *val, int i, int bits,
                            float scale, uint64_t seed, uint64_t step, int64_t m0,
                            int64_t m1, uint32_t *codes_out)
{
    float inv16 = agc_oracle_inv16(scale, bits);
    for (int64_t m = m0; m < m1; ++m) {
        float f = agc_oracle_encode_one(G, ldg, row_ptr, col, val, i, m);
        uint32_t u16, r2;
        agc_oracle_draw(seed, step, (uint32_t)i, (uint64_t)m, &u16, &r2);
        codes_out[m - m0] = agc_oracle_quantize_one(f, inv16, bits, u16, r2);
    }
}

/*
 * Exact second moments of worker i's message (b >= 2), for the Monte-Carlo checks of the
 * residual error (proof of Lemma 1, before any bounding):
 *   *sumsq = sum_m f_i[m]^2                       (enters the straggler term p_i ||f_i||^2)
 *   *var_q = sum_m Var[Q_i(f_i)_m | f_i]
 *          = (scale/L)^2 * sum_m pu_m (1 - pu_m)  over coordinates whose cell lies below L,
 * pu_m being the round-up probability of the rounding rule of Sec. II-B as quantize_prob
 * returns it (at the top cell the clamp leaves nothing random).  Binary64 sums; the order of
 * the additions is not fixed (nothing is decided by these values).
 * Returns 0, or -1 for a one-bit worker (outside the paper; not covered here).
 */
int agc_oracle_worker_moments(const float *G, int64_t ldg, const int32_t *row_ptr,
                              const int32_t *col, const float *val, int i, int bits,
                              float scale, int64_t d, double *sumsq, double *var_q)
{
    if (bits < 2) return -1;
    float inv16 = agc_oracle_inv16(scale, bits);
    uint32_t L = (uint32_t)agc_oracle_levels(bits);
    double unit = (double)scale / (double)L;
    double ss = 0.0, vq = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : ss, vq)
    for (int64_t m = 0; m < d; ++m) {
        float f = agc_oracle_encode_one(G, ldg, row_ptr, col, val, i, m);
        uint32_t lo;
        double pu;
        agc_oracle_quantize_prob(f, inv16, bits, &lo, &pu);
        ss += (double)f * (double)f;
        if (lo < L) vq += pu * (1.0 - pu);
    }
    *sumsq = ss;
    *var_q = unit * unit * vq;
    return 0;
}

/* encode + quantize + pack for all workers.  scales_in == NULL: scales are
 * computed (and returned in scales_out); otherwise scales_in is used as given
 * and copied to scales_out. */
void agc_oracle_encode_quantize(int n, int64_t d, const float *G, int64_t ldg,
                                const int32_t *row_ptr, const int32_t *col,
                                const float *val, const uint8_t *bits,
                                uint64_t seed, uint64_t step, int scale_mode,
                                const float *scales_in, uint8_t *const *streams_out,
                                float *scales_out)
{
    if (scales_in)
        memcpy(scales_out, scales_in, sizeof(float) * (size_t)n);
    else
        agc_oracle_scales(n, d, G, ldg, row_ptr, col, val, scale_mode, scales_out);
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        uint32_t *codes = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)d);
        agc_oracle_codes_range(G, ldg, row_ptr, col, val, i, bits[i], scales_out[i],
                               seed, step, 0, d, codes);
        agc_oracle_pack(codes, d, bits[i], streams_out[i]);
        free(codes);
    }
}

/* one whole pass: encode + quantize + pack, then masked decode */
void agc_oracle_step(int n, int64_t d, const float *G, int64_t ldg,
                     const int32_t *row_ptr, const int32_t *col, const float *val,
                     const uint8_t *bits, const float *w, const uint8_t *mask,
                     uint64_t seed, uint64_t step, int scale_mode,
                     uint8_t *const *streams_out, float *scales_out, float *ghat_out)
{
    agc_oracle_encode_quantize(n, d, G, ldg, row_ptr, col, val, bits, seed, step,
                               scale_mode, NULL, streams_out, scales_out);
    int64_t chunk = 4096;
    int64_t nchunks = (d + chunk - 1) / chunk;
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < nchunks; ++c) {
        int64_t m0 = c * chunk, m1 = m0 + chunk < d ? m0 + chunk : d;
        agc_oracle_decode_range(n, (const uint8_t *const *)streams_out, scales_out,
                                bits, w, mask, m0, m1, ghat_out + m0);
    }
}

/* ------------------------------------------------------------------------- */
/* Bucket-wise granularity            (Sec. II-B: the extension the paper calls */
/* straightforward; one scale per 256-coordinate bucket instead of one per      */
/* vector, at the price of transmitting d/256 scales per worker)                */
/* ------------------------------------------------------------------------- */
/* Readings fixed here (the paper gives no arithmetic for the extension):
 *   bucket u      = coordinates [256u, 256u+256) that are < d;
 *   scale         = largest magnitude in the bucket (mode 1), or the Euclidean
 *                   norm of the bucket (mode 0): levels 0 and 1 of the binary64
 *                   tree above, square root, one rounding to binary32;
 *   multiplier    = L*2^16 / scale (b >= 2), 2^15 / scale (b == 1): ONE binary32
 *                   division (the dividend is exact in binary32); 0 when the
 *                   scale is 0 or the quotient overflows;
 *   rounding rule, draws, codes, payload: exactly as for the global scale;
 *   decode weight = wl_i * scale_iu, ONE binary32 product, with
 *                   wl_i = (float)((double)w_i / L_i);  then as before: arrived
 *                   workers ascending, one fused multiply-add each from 0.     */
int64_t agc_oracle_num_buckets(int64_t d) { return (d + 255) / 256; }

/* scale of one bucket given as its own short array fb[0..cnt), cnt <= 256 */
static float bucket_scale_local(const float *fb, int cnt, int scale_mode)
{
    if (scale_mode == 0) return (float)sqrt(l2_block(fb, cnt, 0));
    return agc_oracle_scale_maxabs(fb, cnt);
}

float agc_oracle_bucket_scale(const float *f, int64_t d, int64_t u, int scale_mode)
{
    int64_t a = u * 256, b = a + 256 < d ? a + 256 : d;
    return bucket_scale_local(f + a, (int)(b - a), scale_mode);
}

float agc_oracle_inv16_bucket(float scale, int bits)
{
    if (!(scale > 0.0f)) return 0.0f;
    float num = bits >= 2 ? (float)agc_oracle_levels(bits) * 65536.0f : 32768.0f;
    float q = num / scale;
    if (!(q <= 3.402823466e+38f)) return 0.0f;
    return q;
}

float agc_oracle_wl_bucket(float w, int bits)
{
    return (float)((double)w / (double)agc_oracle_levels(bits));
}

/* scales [nb] and unpacked codes [m1-m0] of worker i for the buckets that cover
 * [m0, m1); m0 must be a multiple of 256.  scales_out may be NULL. */
void agc_oracle_codes_bucket_range(const float *G, int64_t ldg, const int32_t *row_ptr,
                                   const int32_t *col, const float *val, int i, int bits,
                                   int scale_mode, uint64_t seed, uint64_t step, int64_t d,
                                   int64_t m0, int64_t m1, uint32_t *codes_out,
                                   float *scales_out)
{
    float f[256];
    for (int64_t u = m0 / 256; u * 256 < m1; ++u) {
        int64_t a = u * 256, b = a + 256 < d ? a + 256 : d;
        /* the bucket's scale needs the whole bucket, also past m1 */
        agc_oracle_encode_range(G, ldg, row_ptr, col, val, i, a, b, f);
        float scale = bucket_scale_local(f, (int)(b - a), scale_mode);
        if (scales_out) scales_out[u - m0 / 256] = scale;
        float inv16 = agc_oracle_inv16_bucket(scale, bits);
        for (int64_t m = a; m < b && m < m1; ++m) {
            uint32_t u16, r2;
            agc_oracle_draw(seed, step, (uint32_t)i, (uint64_t)m, &u16, &r2);
            codes_out[m - m0] = agc_oracle_quantize_one(f[m - a], inv16, bits, u16, r2);
        }
    }
}

/* encode + quantize + pack for all workers; scales_out is n x nb, row-major */
void agc_oracle_encode_quantize_bucket(int n, int64_t d, const float *G, int64_t ldg,
                                       const int32_t *row_ptr, const int32_t *col,
                                       const float *val, const uint8_t *bits,
                                       uint64_t seed, uint64_t step, int scale_mode,
                                       uint8_t *const *streams_out, float *scales_out)
{
    int64_t nb = agc_oracle_num_buckets(d);
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        uint32_t *codes = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(d > 0 ? d : 1));
        agc_oracle_codes_bucket_range(G, ldg, row_ptr, col, val, i, bits[i], scale_mode, seed,
                                      step, d, 0, d, codes, scales_out + (int64_t)i * nb);
        agc_oracle_pack(codes, d, bits[i], streams_out[i]);
        free(codes);
    }
}

void agc_oracle_decode_bucket_range(int n, const uint8_t *const *streams,
                                    const float *scales, int64_t nb, const uint8_t *bits,
                                    const float *w, const uint8_t *mask, int64_t m0,
                                    int64_t m1, float *ghat_out)
{
    for (int64_t m = m0; m < m1; ++m) {
        float acc = 0.0f;
        for (int i = 0; i < n; ++i) {
            if (!mask[i]) continue;
            float coef = agc_oracle_wl_bucket(w[i], bits[i]) * scales[(int64_t)i * nb + m / 256];
            float v = agc_oracle_code_value(
                agc_oracle_unpack_one(streams[i], bits[i], m), bits[i]);
            acc = fmaf(coef, v, acc);
        }
        ghat_out[m - m0] = acc;
    }
}

void agc_oracle_step_bucket(int n, int64_t d, const float *G, int64_t ldg,
                            const int32_t *row_ptr, const int32_t *col, const float *val,
                            const uint8_t *bits, const float *w, const uint8_t *mask,
                            uint64_t seed, uint64_t step, int scale_mode,
                            uint8_t *const *streams_out, float *scales_out, float *ghat_out)
{
    agc_oracle_encode_quantize_bucket(n, d, G, ldg, row_ptr, col, val, bits, seed, step,
                                      scale_mode, streams_out, scales_out);
    int64_t nb = agc_oracle_num_buckets(d);
    int64_t chunk = 4096;
    int64_t nchunks = (d + chunk - 1) / chunk;
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < nchunks; ++c) {
        int64_t m0 = c * chunk, m1 = m0 + chunk < d ? m0 + chunk : d;
        agc_oracle_decode_bucket_range(n, (const uint8_t *const *)streams_out, scales_out, nb,
                                       bits, w, mask, m0, m1, ghat_out + m0);
    }
}

/* number of threads the parallel loops above may use from now on (timing runs only) */
void agc_oracle_set_threads(int count)
{
#ifdef _OPENMP
    if (count >= 1) omp_set_num_threads(count);
#else
    (void)count;
#endif
}

int agc_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
