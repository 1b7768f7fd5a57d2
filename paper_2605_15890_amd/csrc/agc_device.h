// Device-side building blocks of the gfx950 kernels: Philox4x32-10, DPP wave reductions and
// the two encode drivers (cyclic-band register ring, generic CSR gather).
//
// Thread geometry shared by the scale pass and the encode+quantize+pack pass: a wave covers
// one block of 256 consecutive coordinates, lane l owning the float4 at coordinates 4l..4l+3
// (the max-abs scale pass may give a wave two neighbouring blocks at once); a workgroup is
// four waves unless a kernel says otherwise.  Every lane walks over all workers for its
// coordinates, so the coded gradient f_i = sum_j a_ij g_j (Sec. II-A) only ever lives in
// registers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

#include "agc_kernels.h"

namespace agc {

constexpr int kMaxWorkers = 256;
constexpr int kWave = 64;
constexpr int kBlockCoords = 256;  // coordinates per wave pass
constexpr int kWavesPerWg = 4;
constexpr int kWgThreads = kWave * kWavesPerWg;
constexpr int kSegBlocks = 4;   // blocks per segment of the norm's summation tree
constexpr int kGroupSegs = 64;  // segments per group, groups per supergroup
constexpr int kMaxBand = 8;     // largest replication factor served by the register ring

// ---------------------------------------------------------------------------------------
// Philox4x32 with ten rounds (Salmon et al., SC'11).  Round: the two 32x32->64 products of
// counter words 0 and 2 with fixed odd multipliers; high halves are mixed with words 1 and 3
// and the round key; the key advances by Weyl constants.  On gfx950 the wide product is one
// full-rate v_mad_u64_u32 and the two mixes are one three-input xor each, so a block costs
// about 40 vector instructions.
// ---------------------------------------------------------------------------------------
// a ^ b ^ c in one instruction (gfx950's three-input bitwise op; truth table 0x96 = parity)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return (uint32_t)__builtin_amdgcn_bitop3_b32((int)a, (int)b, (int)c, 0x96);
}

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#ifdef AGC_ABLATE_PHILOX
    constexpr int kRounds = 1;
#else
    constexpr int kRounds = 10;
#endif
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const uint64_t pa = (uint64_t)0xD2511F53u * c0;
        const uint64_t pb = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = xor3((uint32_t)(pb >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(pa >> 32), c3, k1);
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

// ---------------------------------------------------------------------------------------
// wave-wide reductions on the DPP cross-lane network (no LDS traffic)
// ---------------------------------------------------------------------------------------
constexpr int kDppQuadSwap1 = 0xB1;     // quad_perm [1,0,3,2]: partner l ^ 1
constexpr int kDppQuadSwap2 = 0x4E;     // quad_perm [2,3,0,1]: partner l ^ 2
constexpr int kDppHalfMirror = 0x141;   // l -> 7 - l within 8 lanes: a partner in the other quad
constexpr int kDppRowMirror = 0x140;    // l -> 15 - l within 16 lanes: a partner in the other half

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

// maximum over the wave of non-negative floats, returned as a wave-uniform bit pattern
// (non-negative floats order like their bit patterns)
__device__ __forceinline__ uint32_t wave_max_nonneg_bits(float x)
{
    uint32_t v = __float_as_uint(x);
    v = max(v, dpp_u32<kDppQuadSwap1>(v));
    v = max(v, dpp_u32<kDppQuadSwap2>(v));
    v = max(v, dpp_u32<kDppHalfMirror>(v));
    v = max(v, dpp_u32<kDppRowMirror>(v));  // every 16-lane row now holds its maximum
    const uint32_t r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
    const uint32_t r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
    // the four row maxima are wave-uniform: combine them on the scalar unit (left to itself the
    // compiler moves them back into vector registers for a three-operand maximum)
    uint32_t a, b, m;
    asm("s_max_u32 %0, %1, %2" : "=s"(a) : "s"(r0), "s"(r1) : "scc");
    asm("s_max_u32 %0, %1, %2" : "=s"(b) : "s"(r2), "s"(r3) : "scc");
    asm("s_max_u32 %0, %1, %2" : "=s"(m) : "s"(a), "s"(b) : "scc");
    return m;
}

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v)
{
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = dpp_u32<CTRL>((uint32_t)b), hi = dpp_u32<CTRL>((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

__device__ __forceinline__ double readlane_f64(double v, int lane)
{
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)b, lane);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(b >> 32), lane);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// Exchange-add over lanes at distances 1,2,4,8,16,32 (second level of the norm's tree),
// result wave-uniform.  After the steps at distance 1 and 2 every quad is uniform, so the
// mirror partners used for distances 4 and 8 hold exactly the value of lane l^4 and l^8; after
// distance 8 every 16-lane row is uniform and the last two steps are (r0+r1)+(r2+r3) on the
// four row values, which is what lanes of rows 0 and 1 compute in the exchange (rows 2 and 3
// compute the commuted, identical sum).
__device__ __forceinline__ double wave_butterfly_add(double v)
{
    v = v + dpp_f64<kDppQuadSwap1>(v);
    v = v + dpp_f64<kDppQuadSwap2>(v);
    v = v + dpp_f64<kDppHalfMirror>(v);
    v = v + dpp_f64<kDppRowMirror>(v);
    const double r0 = readlane_f64(v, 0), r1 = readlane_f64(v, 16);
    const double r2 = readlane_f64(v, 32), r3 = readlane_f64(v, 48);
    const double a = r0 + r1, b = r2 + r3;
    return a + b;
}

// ---------------------------------------------------------------------------------------
// loads of one lane's float4
// ---------------------------------------------------------------------------------------
struct LaneCoords {
    int lane4;         // which float4 of the block the lane loads (clamped into the vector for lanes past d)
    uint32_t byte_off; // 16 * lane4: the lane's offset inside the block, as the 32-bit part of the address
    int nvalid;        // how many of the lane's four coordinates are < d (0..4)
    bool wave_ragged;  // wave-uniform: some lane of this wave has nvalid < 4
};

// base: first coordinate of the wave's block (wave-uniform, < d)
__device__ __forceinline__ LaneCoords lane_coords(int64_t base, int lane, int64_t d)
{
    LaneCoords lc;
    const int64_t left = d - base - 4 * lane;
    lc.nvalid = left >= 4 ? 4 : (left > 0 ? (int)left : 0);
    const int64_t last4 = (d - 1 - base) >> 2;  // last float4 of the block that holds a coordinate < d
    lc.lane4 = last4 < lane ? (int)last4 : lane;
    lc.byte_off = 16u * (uint32_t)lc.lane4;
    lc.wave_ragged = __any(lc.nvalid < 4) != 0;
    return lc;
}

// `row` points at the block's first coordinate inside one row of G and is wave-uniform, so
// the load is a scalar base plus a 32-bit lane offset.  Every lane loads (lanes past d re-read
// the last float4), so there is no per-lane predicate; with RAGGED the coordinates >= d are
// zeroed, without it the caller guarantees that the whole block lies inside the vector.
// STREAM: the element is used once per pass (register-ring driver); a non-temporal load keeps it
// from displacing anything in the caches (measured: 9 % off the scale pass).  The gather driver
// re-reads rows and wants them cached.
template <bool RAGGED, bool STREAM = false>
__device__ __forceinline__ float4 load_row4(const float* __restrict__ row, const LaneCoords& lc)
{
    // scalar row pointer + zero-extended 32-bit lane offset: the form the hardware addresses
    // without any per-lane 64-bit arithmetic
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(1))) char* global_bytes_t;
    typedef const __attribute__((address_space(1))) f32x4_t* global_f32x4_t;
    const global_f32x4_t src = (global_f32x4_t)((global_bytes_t)row + lc.byte_off);
#ifdef AGC_PLAIN_ROW_LOADS
    const f32x4_t t = *src;
#else
    const f32x4_t t = STREAM ? __builtin_nontemporal_load(src) : *src;
#endif
    float4 v = make_float4(t.x, t.y, t.z, t.w);
    if (RAGGED) {
        if (lc.nvalid < 1) v.x = 0.f;
        if (lc.nvalid < 2) v.y = 0.f;
        if (lc.nvalid < 3) v.z = 0.f;
        if (lc.nvalid < 4) v.w = 0.f;
    }
    return v;
}

__device__ __forceinline__ float4 mul4(float a, const float4& g)
{
    return make_float4(a * g.x, a * g.y, a * g.z, a * g.w);
}
__device__ __forceinline__ float4 fma4(float a, const float4& g, const float4& c)
{
    return make_float4(fmaf(a, g.x, c.x), fmaf(a, g.y, c.y), fmaf(a, g.z, c.z), fmaf(a, g.w, c.w));
}

// What a lane holds of one row of G while it streams through a register ring: its float4 of one
// block (float4 itself), or its float4s of V neighbouring blocks (RowN<V>; the wave then covers
// 256 V consecutive coordinates and issues V loads per row, 1 KiB apart).  The multi-block form
// divides the number of row walks and of per-worker reductions by V; it is used where registers
// allow it (the max-abs scale pass).  All forms perform the same arithmetic on every coordinate.
template <int V>
struct RowN {
    float4 v[V];
};
typedef RowN<2> Row2;
template <int V>
__device__ __forceinline__ RowN<V> mul4(float c, const RowN<V>& g)
{
    RowN<V> r;
#pragma unroll
    for (int t = 0; t < V; ++t) r.v[t] = mul4(c, g.v[t]);
    return r;
}
template <int V>
__device__ __forceinline__ RowN<V> fma4(float c, const RowN<V>& g, const RowN<V>& f)
{
    RowN<V> r;
#pragma unroll
    for (int t = 0; t < V; ++t) r.v[t] = fma4(c, g.v[t], f.v[t]);
    return r;
}

// Row -> number of blocks
template <class Row>
struct RowBlocks {
    static constexpr int value = sizeof(Row) / sizeof(float4);
};

template <class Row>
__device__ __forceinline__ Row zero_row()
{
    Row r;
    float4* p = reinterpret_cast<float4*>(&r);
#pragma unroll
    for (int t = 0; t < RowBlocks<Row>::value; ++t) p[t] = make_float4(0.f, 0.f, 0.f, 0.f);
    return r;
}

// streaming load of a lane's part of a row whose blocks lie wholly inside the vector
template <class Row>
__device__ __forceinline__ Row load_row(const float* __restrict__ row, const LaneCoords& lc)
{
    Row r;
    float4* p = reinterpret_cast<float4*>(&r);
#pragma unroll
    for (int t = 0; t < RowBlocks<Row>::value; ++t) p[t] = load_row4<false, true>(row + t * kBlockCoords, lc);
    return r;
}

// ---------------------------------------------------------------------------------------
// Encode driver 1: cyclic band.  n == k, worker i stores columns (i+u) mod k, u = 0..S-1.
// Rows stream once through a ring of R = S + P row registers (P rows of prefetch); worker
// i is formed when row i+S-1 has arrived.  The first S-1 rows are kept in a register stash
// for the last S-1 workers, which wrap around, so every element of G is read exactly once.
// R is even so that the parity of the worker handled at each unrolled position is known at
// compile time (the quantizer shares one Philox block between workers 2q and 2q+1).  The
// epilogue is called for workers 0..n-1 in ascending order.
// ---------------------------------------------------------------------------------------
// PF = requested prefetch distance in rows (made one larger when S + PF would be odd)
template <int S, int PF>
struct RingShapeT {
    static constexpr int P = ((S + PF) & 1) ? PF + 1 : PF;
    static constexpr int R = S + P;
    static constexpr int NSTASH = S > 1 ? S - 1 : 1;
};
// The prefetch distance is a property of the epilogue (Epi::kPrefetchRows).  Quantize pass: two
// rows ahead (measured 2/3/4/6/8/10 rows: 1.393/1.402/1.400/1.411/1.419/1.414 ms on the metric
// workload, two rows also best on the smaller ones: deeper prefetch only costs registers, the
// pass does not wait for its loads).  One-block scale pass: two as well (Euclidean scale at the
// metric size: 0.972 ms against 0.983 ms with four).
#ifndef AGC_PREFETCH_ROWS
#define AGC_PREFETCH_ROWS 2
#endif
#ifndef AGC_SCALE_PREFETCH_ROWS
#define AGC_SCALE_PREFETCH_ROWS 2
#endif

// value select (the operands are read before the choice, so the choice is between registers)
__device__ __forceinline__ float4 sel4(bool c, const float4 a, const float4 b)
{
    return make_float4(c ? a.x : b.x, c ? a.y : b.y, c ? a.z : b.z, c ? a.w : b.w);
}
template <int V>
__device__ __forceinline__ RowN<V> sel4(bool c, const RowN<V>& a, const RowN<V>& b)
{
    RowN<V> r;
#pragma unroll
    for (int t = 0; t < V; ++t) r.v[t] = sel4(c, a.v[t], b.v[t]);
    return r;
}

// stash helpers with compile-time indices (so the stash stays in registers)
template <int S, int PF, class Row, int... Us>
__device__ __forceinline__ Row stash_pick(const Row (&stash)[(RingShapeT<S, PF>::NSTASH)], int idx,
                                             std::integer_sequence<int, Us...>)
{
    Row v = stash[0];
    ((v = sel4(idx == Us + 1, stash[(Us + 1) < RingShapeT<S, PF>::NSTASH ? (Us + 1) : 0], v)), ...);
    return v;
}

template <int S, int PF, class Row, int r, int... Us>
__device__ __forceinline__ void stash_fill(Row (&stash)[(RingShapeT<S, PF>::NSTASH)],
                                           const Row (&ring)[(RingShapeT<S, PF>::R)],
                                           std::integer_sequence<int, Us...>)
{
    constexpr int R = RingShapeT<S, PF>::R;
    ((stash[Us] = ring[(r + R - (S - 1) + Us) % R]), ...);
}

// One row arrival.  STEADY rounds are straight-line code: every prefetch is issued (past the
// last row the last row is re-read, a cache hit whose value is never used), every worker index
// is valid and no wrapped row is involved, so the compiler can count outstanding loads exactly
// and let P of them stay in flight.  The first round and the last one or two (GENERAL) carry
// the conditions: workers that do not exist yet, the stash fill, the wrapped rows.
template <int S, int PF, class Row, int r, bool STEADY, class Epi>
__device__ __forceinline__ void ring_step(Row (&ring)[(RingShapeT<S, PF>::R)],
                                          Row (&stash)[(RingShapeT<S, PF>::NSTASH)],
                                          const float*& next_row, int64_t ldg, int k,
                                          const float* __restrict__ bval, const LaneCoords& lc,
                                          int j0, float (&coef)[S], Epi& epi)
{
    constexpr int P = RingShapeT<S, PF>::P;
    constexpr int R = RingShapeT<S, PF>::R;
    const int j = j0 + r;
    if (STEADY) {
        ring[(r + P) % R] = load_row<Row>(next_row, lc);
        next_row += (j + P + 1 < k) ? ldg : 0;  // stays on the last row once it is reached
    } else {
        if (j + P < k) {  // prefetch the row that arrives P steps from now
            ring[(r + P) % R] = load_row<Row>(next_row, lc);
            next_row += (j + P + 1 < k) ? ldg : 0;
        }
        if (S > 1 && j >= k && j < k + S - 1)  // arrivals k..k+S-2 are rows 0..S-2, kept in the stash
            ring[r] = stash_pick<S, PF, Row>(stash, j - k, std::make_integer_sequence<int, (S > 2 ? S - 2 : 0)>{});
    }
    const int i = j - (S - 1);
    if (STEADY || (i >= 0 && i < k)) {
        if (!STEADY && S > 1 && i == 0)
            stash_fill<S, PF, Row, r>(stash, ring, std::make_integer_sequence<int, (S > 1 ? S - 1 : 0)>{});
        // the worker's coefficients were requested one worker earlier (the scalar read is then
        // over by the time they are used); request the next worker's now
        float next[S];
        const float* bv = bval + (int64_t)(i + 1 < k ? i + 1 : i) * S;
#pragma unroll
        for (int u = 0; u < S; ++u) next[u] = bv[u];
        Row f = mul4(coef[0], ring[(r + R - (S - 1)) % R]);
#pragma unroll
        for (int u = 1; u < S; ++u) f = fma4(coef[u], ring[(r + R - (S - 1) + u) % R], f);
        epi.template worker<(((r + R - (S - 1)) & 1) == 0)>(i, f);
#pragma unroll
        for (int u = 0; u < S; ++u) coef[u] = next[u];
    }
}

template <int S, int PF, class Row, bool STEADY, class Epi, int... Rs>
__device__ __forceinline__ void ring_round(Row (&ring)[(RingShapeT<S, PF>::R)],
                                           Row (&stash)[(RingShapeT<S, PF>::NSTASH)],
                                           const float*& next_row, int64_t ldg, int k,
                                           const float* __restrict__ bval, const LaneCoords& lc,
                                           int j0, float (&coef)[S], Epi& epi, std::integer_sequence<int, Rs...>)
{
    (ring_step<S, PF, Row, Rs, STEADY>(ring, stash, next_row, ldg, k, bval, lc, j0, coef, epi), ...);
}

template <int S, int PF, class Row, class Epi>
__device__ __forceinline__ void encode_ring(const float* __restrict__ G, int64_t ldg, int k,
                                            const float* __restrict__ bval, const LaneCoords& lc,
                                            Epi& epi)
{
    constexpr int P = RingShapeT<S, PF>::P;
    constexpr int R = RingShapeT<S, PF>::R;
    static_assert(R % 2 == 0, "ring length must be even");
    constexpr auto seq = std::make_integer_sequence<int, R>{};
    const int steps = k + S - 1;  // row arrivals, the last S-1 being the wrapped rows
    Row ring[R];
    Row stash[(RingShapeT<S, PF>::NSTASH)];
    const float* next_row = G;  // G already points at the block's first coordinate in row 0
#pragma unroll
    for (int r = 0; r < R; ++r) ring[r] = zero_row<Row>();
    stash[0] = zero_row<Row>();
#pragma unroll
    for (int r = 0; r < P; ++r) {
        if (r < k) {
            ring[r] = load_row<Row>(next_row, lc);
            next_row += (r + 1 < k) ? ldg : 0;
        }
    }
    float coef[S];  // coefficients of the worker that is formed next
#pragma unroll
    for (int u = 0; u < S; ++u) coef[u] = bval[u];
    int j0 = 0;
    ring_round<S, PF, Row, false>(ring, stash, next_row, ldg, k, bval, lc, j0, coef, epi, seq);
    for (j0 = R; j0 + R - 1 < k; j0 += R)
        ring_round<S, PF, Row, true>(ring, stash, next_row, ldg, k, bval, lc, j0, coef, epi, seq);
    for (; j0 < steps; j0 += R)
        ring_round<S, PF, Row, false>(ring, stash, next_row, ldg, k, bval, lc, j0, coef, epi, seq);
}

// ---------------------------------------------------------------------------------------
// Encode driver 2: any CSR code.  Each worker gathers its rows straight from memory; rows
// shared by neighbouring workers are served by the caches.
// ---------------------------------------------------------------------------------------
// Wave-uniform read of a small read-only table (code structure, per-worker records).  Tagging the
// address as constant memory keeps the read on the scalar path even in a kernel that also stores:
// otherwise the compiler must assume its own stores may have changed the table, reads it with a
// vector load and waits for every outstanding load and store.  Nothing writes these tables while
// a kernel that reads them runs.
template <class T>
__device__ __forceinline__ T load_uniform(const T* p)
{
    static_assert(sizeof(T) % 4 == 0, "whole dwords");
    constexpr int N = sizeof(T) / 4;
    const __attribute__((address_space(4))) uint32_t* q = (const __attribute__((address_space(4))) uint32_t*)p;
    uint32_t w[N];
#pragma unroll
    for (int t = 0; t < N; ++t) w[t] = q[t];
    T out;
    __builtin_memcpy(&out, w, sizeof(T));
    return out;
}

struct CsrView {
    const int* __restrict__ row_ptr;
    const int* __restrict__ col;
    const float* __restrict__ val;
    const WindowRec* __restrict__ win;  // monotone-interval codes: one record per row + sentinel
};

template <bool RAGGED>
__device__ __forceinline__ float4 encode_gather_one(const float* __restrict__ G, int64_t ldg,
                                                    const CsrView& B, int i, const LaneCoords& lc)
{
    const int e0 = B.row_ptr[i], e1 = B.row_ptr[i + 1];
    float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
    if (e0 < e1) {
        f = mul4(B.val[e0], load_row4<RAGGED>(G + (int64_t)B.col[e0] * ldg, lc));
        for (int e = e0 + 1; e < e1; ++e)
            f = fma4(B.val[e], load_row4<RAGGED>(G + (int64_t)B.col[e] * ldg, lc), f);
    }
    return f;
}

template <bool RAGGED, class Epi>
__device__ __forceinline__ void encode_gather(const float* __restrict__ G, int64_t ldg, int n,
                                              const CsrView& B, const LaneCoords& lc, Epi& epi)
{
    for (int i = 0; i < n; i += 2) {
        epi.template worker<true>(i, encode_gather_one<RAGGED>(G, ldg, B, i, lc));
        if (i + 1 < n) epi.template worker<false>(i + 1, encode_gather_one<RAGGED>(G, ldg, B, i + 1, lc));
    }
}

// ---------------------------------------------------------------------------------------
// Encode driver 3: monotone intervals.  Every worker stores a run of consecutive columns
// lo_i .. lo_i+len_i-1 (ascending, len_i <= W) and neither lo_i nor lo_i+len_i-1 decreases with i
// - the shape of the paper's sparse construction (Sec. III-A: contiguous allocation segments on
// the partition axis).  Rows stream once through the same register ring as the cyclic band; a
// worker is formed when row lo_i + W - 1 arrives, so that row lo_i + u sits at a ring position
// that is known at compile time; entries u >= len_i are skipped by wave-uniform branches (not
// multiplied by zero: the sum must have exactly the stored terms).  Several workers, or none, may
// be anchored at the same row.
// ---------------------------------------------------------------------------------------
// the part of a row's record the driver keeps in scalar registers
struct WindowCur {
    int lo, len;
    float val[8];
};

__device__ __forceinline__ WindowCur load_window_rec(const WindowRec* rec)
{
    struct Head { int lo, len; };
    struct Vals { float v[8]; };
    const Head h = load_uniform(reinterpret_cast<const Head*>(rec));
    const Vals v = load_uniform(reinterpret_cast<const Vals*>(rec->val));
    WindowCur c;
    c.lo = h.lo;
    c.len = h.len;
#pragma unroll
    for (int u = 0; u < 8; ++u) c.val[u] = v.v[u];
    return c;
}

template <int W, int PF, class Row, int r, bool STEADY, class Epi>
__device__ __forceinline__ void window_step(Row (&ring)[(RingShapeT<W, PF>::R)], const float*& next_row,
                                            int64_t ldg, int k, const CsrView& B, const LaneCoords& lc,
                                            int j0, int& i, WindowCur& cur, Epi& epi)
{
    constexpr int P = RingShapeT<W, PF>::P;
    constexpr int R = RingShapeT<W, PF>::R;
    const int j = j0 + r;
    if (STEADY || j + P < k) {  // prefetch the row that arrives P steps from now
        ring[(r + P) % R] = load_row<Row>(next_row, lc);
        next_row += (j + P + 1 < k) ? ldg : 0;
    }
    const int lo = j - (W - 1);
    while (cur.lo == lo) {  // the sentinel record ends the last run
        const WindowCur nxt = load_window_rec(B.win + i + 1);
        Row f = mul4(cur.val[0], ring[(r + R - (W - 1)) % R]);
#pragma unroll
        for (int u = 1; u < W; ++u)
            if (u < cur.len) f = fma4(cur.val[u], ring[(r + R - (W - 1) + u) % R], f);
        epi.worker_any(i, f);
        cur = nxt;
        ++i;
    }
}

template <int W, int PF, class Row, bool STEADY, class Epi, int... Rs>
__device__ __forceinline__ void window_round(Row (&ring)[(RingShapeT<W, PF>::R)], const float*& next_row,
                                             int64_t ldg, int k, const CsrView& B, const LaneCoords& lc,
                                             int j0, int& i, WindowCur& cur, Epi& epi,
                                             std::integer_sequence<int, Rs...>)
{
    (window_step<W, PF, Row, Rs, STEADY>(ring, next_row, ldg, k, B, lc, j0, i, cur, epi), ...);
}

template <int W, int PF, class Row, class Epi>
__device__ __forceinline__ void encode_window(const float* __restrict__ G, int64_t ldg, int k,
                                              const CsrView& B, const LaneCoords& lc, Epi& epi)
{
    constexpr int P = RingShapeT<W, PF>::P;
    constexpr int R = RingShapeT<W, PF>::R;
    constexpr auto seq = std::make_integer_sequence<int, R>{};
    Row ring[R];
    const float* next_row = G;
#pragma unroll
    for (int r = 0; r < R; ++r) ring[r] = zero_row<Row>();
#pragma unroll
    for (int r = 0; r < P; ++r) {
        if (r < k) {
            ring[r] = load_row<Row>(next_row, lc);
            next_row += (r + 1 < k) ? ldg : 0;
        }
    }
    int i = 0;
    WindowCur cur = load_window_rec(B.win);
    int j0 = 0;
    const int steps = k + W - 1;  // the last worker may be anchored at row k-1
    for (; j0 + R - 1 + P < k; j0 += R)  // every prefetch of the round exists
        window_round<W, PF, Row, true>(ring, next_row, ldg, k, B, lc, j0, i, cur, epi, seq);
    for (; j0 < steps; j0 += R)
        window_round<W, PF, Row, false>(ring, next_row, ldg, k, B, lc, j0, i, cur, epi, seq);
}

// The same driver for epilogues that store inside the worker loop (the quantize pass).  Stores
// and loads share one outstanding-operation counter on this hardware, so behind a loop of unknown
// length the compiler can only wait for everything; a rolling prefetch would be drained at every
// row.  Here the rows arrive in batches of BT: while the BT row steps of one batch run, the next
// batch is in flight; it is waited for as a whole when its turn comes.  The ring holds the
// current batch, the next one and the up to W-1 older rows a worker may still need, rounded up to
// whole batches so that all positions stay compile-time.  The structure of worker i comes from
// its 64-byte record, read one worker ahead.
template <int W>
struct BatchShape {
    static constexpr int BT = 4;                                   // rows per batch
    static constexpr int R = ((2 * BT + W - 1 + BT - 1) / BT) * BT;  // current + next batch + W-1 older rows
    static constexpr int NB = R / BT;
};

template <int W, int H>
__device__ __forceinline__ void window_request(float4 (&ring)[BatchShape<W>::R], const float* __restrict__ G,
                                               int64_t ldg, int k, const LaneCoords& lc, int row0)
{
    constexpr int BT = BatchShape<W>::BT;
    if (row0 < k) {  // one straight run of loads; a batch that straddles the end repeats row k-1
#pragma unroll
        for (int r = 0; r < BT; ++r) {
            const int row = row0 + r < k ? row0 + r : k - 1;
            ring[H * BT + r] = load_row4<false, true>(G + (int64_t)row * ldg, lc);
        }
    }
}

template <int W, int H, class Epi>
__device__ __forceinline__ void window_batch(float4 (&ring)[BatchShape<W>::R], const float* __restrict__ G,
                                             int64_t ldg, int k, const CsrView& B, const LaneCoords& lc,
                                             int row0, int& i, WindowCur& cur, Epi& epi)
{
    constexpr int BT = BatchShape<W>::BT;
    constexpr int R = BatchShape<W>::R;
    constexpr int NB = BatchShape<W>::NB;
    // the batch requested one round ago has to be here now.  The empty asm makes its registers
    // plain values for the compiler from here on: without it every later row step waits for all
    // outstanding operations, the stores of the step before included.
#pragma unroll
    for (int r = 0; r < BT; ++r) {
        float4& x = ring[H * BT + r];
        asm volatile("" : "+v"(x.x), "+v"(x.y), "+v"(x.z), "+v"(x.w));
    }
    window_request<W, (H + 1) % NB>(ring, G, ldg, k, lc, row0 + BT);
#pragma unroll
    for (int r = 0; r < BT; ++r) {
        const int lo = row0 + r - (W - 1);
        while (cur.lo == lo) {  // the sentinel record ends the last run
            const WindowCur nxt = load_window_rec(B.win + i + 1);  // in flight during this worker
            float4 f = mul4(cur.val[0], ring[(H * BT + r + R - (W - 1)) % R]);
#pragma unroll
            for (int u = 1; u < W; ++u)
                if (u < cur.len) f = fma4(cur.val[u], ring[(H * BT + r + R - (W - 1) + u) % R], f);
            epi.worker_any(i, f);
            cur = nxt;
            ++i;
        }
    }
}

template <int W, int H, class Epi>
__device__ __forceinline__ void window_batches(float4 (&ring)[BatchShape<W>::R], const float* __restrict__ G,
                                               int64_t ldg, int k, const CsrView& B, const LaneCoords& lc,
                                               int row0, int steps, int& i, WindowCur& cur, Epi& epi)
{
    if constexpr (H < BatchShape<W>::NB) {
        if (row0 < steps) {
            window_batch<W, H>(ring, G, ldg, k, B, lc, row0, i, cur, epi);
            window_batches<W, H + 1>(ring, G, ldg, k, B, lc, row0 + BatchShape<W>::BT, steps, i, cur, epi);
        }
    }
}

template <int W, class Epi>
__device__ __forceinline__ void encode_window_batched(const float* __restrict__ G, int64_t ldg, int k,
                                                      const CsrView& B, const LaneCoords& lc, Epi& epi)
{
    constexpr int R = BatchShape<W>::R;
    float4 ring[R];
#pragma unroll
    for (int r = 0; r < R; ++r) ring[r] = make_float4(0.f, 0.f, 0.f, 0.f);
    int i = 0;
    WindowCur cur = load_window_rec(B.win);
    const int steps = k + W - 1;  // the last worker may be anchored at row k-1
    window_request<W, 0>(ring, G, ldg, k, lc, 0);
    for (int row0 = 0; row0 < steps; row0 += R)
        window_batches<W, 0>(ring, G, ldg, k, B, lc, row0, steps, i, cur, epi);
}

// One block of 256 coordinates for all workers.  S > 0: cyclic band of width S; S < 0: monotone
// intervals of at most -S columns; S == 0: any code.  The register ring serves whole blocks; the
// one block that straddles d (and any other code) goes through the gather driver, which masks
// the coordinates past the end.  All give identical bits.
template <int S, class Epi>
__device__ __forceinline__ void encode_block(const float* __restrict__ G, int64_t ldg, int n, int k,
                                             const CsrView& B, const LaneCoords& lc, Epi& epi)
{
    if constexpr (S > 0) {
        if (!lc.wave_ragged) encode_ring<S, Epi::kPrefetchRows, float4>(G, ldg, k, B.val, lc, epi);
        else encode_gather<true>(G, ldg, n, B, lc, epi);
    } else if constexpr (S < 0) {  // monotone intervals of at most -S columns
        if (lc.wave_ragged) encode_gather<true>(G, ldg, n, B, lc, epi);
        else if constexpr (Epi::kStoresPerWorker) encode_window_batched<-S>(G, ldg, k, B, lc, epi);
        else encode_window<-S, Epi::kPrefetchRows, float4>(G, ldg, k, B, lc, epi);
    } else {
        if (!lc.wave_ragged) encode_gather<false>(G, ldg, n, B, lc, epi);
        else encode_gather<true>(G, ldg, n, B, lc, epi);
    }
}

}  // namespace agc
