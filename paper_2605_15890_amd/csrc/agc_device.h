// Device-side building blocks of the gfx950 kernels: Philox4x32-10, wave reductions and the
// two encode drivers (cyclic-band register ring, generic CSR gather).
//
// Thread geometry shared by the scale pass and the encode+quantize+pack pass: a wave covers
// one block of 256 consecutive coordinates, lane l owning the float4 at coordinates 4l..4l+3;
// a workgroup is four waves.  Every lane walks over all workers for its four coordinates, so
// the coded gradient f_i = sum_j a_ij g_j (Sec. II-A) only ever lives in registers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

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
// and the round key; the key advances by Weyl constants.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t pa = (uint64_t)0xD2511F53u * c0;
        const uint64_t pb = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
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
// wave-wide reductions (all lanes receive the result)
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_max_nonneg(float v)
{
    // non-negative floats order like their bit patterns
#pragma unroll
    for (int h = 1; h < kWave; h <<= 1) v = fmaxf(v, __shfl_xor(v, h, kWave));
    return v;
}

// exchange-add over lanes at distances 1,2,4,8,16,32: the second level of the norm's tree
__device__ __forceinline__ double wave_butterfly_add(double v)
{
#pragma unroll
    for (int h = 1; h < kWave; h <<= 1) v = v + __shfl_xor(v, h, kWave);
    return v;
}

// ---------------------------------------------------------------------------------------
// loads of one lane's float4 of row `row`
// ---------------------------------------------------------------------------------------
struct LaneCoords {
    int64_t m0;         // first coordinate of the lane
    int nvalid;         // how many of m0..m0+3 are < d (0..4)
    bool wave_partial;  // wave-uniform: some lane of this wave has 0 < nvalid < 4
};

__device__ __forceinline__ LaneCoords lane_coords(int64_t m0, int64_t d)
{
    LaneCoords lc;
    lc.m0 = m0;
    const int64_t left = d - m0;
    lc.nvalid = left >= 4 ? 4 : (left > 0 ? (int)left : 0);
    lc.wave_partial = __any(lc.nvalid > 0 && lc.nvalid < 4) != 0;
    return lc;
}

__device__ __forceinline__ float4 load_row4(const float* __restrict__ G, int64_t ldg, int row,
                                            const LaneCoords& lc)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (lc.nvalid > 0) {
        v = *reinterpret_cast<const float4*>(G + (int64_t)row * ldg + lc.m0);
    }
    if (lc.wave_partial) {  // the one float4 that straddles d: coordinates >= d count as 0
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

// ---------------------------------------------------------------------------------------
// Encode driver 1: cyclic band.  n == k, worker i stores columns (i+u) mod k, u = 0..S-1.
// Rows stream once through a ring of R = S + P float4 registers (P rows of prefetch); worker
// i is formed when row i+S-1 has arrived; the last S-1 workers wrap around and re-read rows
// 0..S-2.  R is even so that the parity of the worker handled at each unrolled position is
// known at compile time (the quantizer shares one Philox block between workers 2q and 2q+1).
// The epilogue is called for workers 0..n-1 in ascending order.
// ---------------------------------------------------------------------------------------
template <int S>
struct RingShape {
    static constexpr int P = ((S + 4) & 1) ? 5 : 4;
    static constexpr int R = S + P;
};

template <int S, int r, class Epi>
__device__ __forceinline__ void ring_step(float4 (&ring)[RingShape<S>::R], const float* __restrict__ G,
                                          int64_t ldg, int k, const float* __restrict__ bval,
                                          const LaneCoords& lc, int j0, int steps, Epi& epi)
{
    constexpr int P = RingShape<S>::P;
    constexpr int R = RingShape<S>::R;
    const int j = j0 + r;
    int jn = j + P;  // prefetch; past the end the last row is re-read (harmless, cached)
    jn = jn < steps ? jn : steps - 1;
    ring[(r + P) % R] = load_row4(G, ldg, jn < k ? jn : jn - k, lc);
    const int i = j - (S - 1);
    if (i >= 0 && i < k) {
        const float* bv = bval + (int64_t)i * S;
        float4 f = mul4(bv[0], ring[(r + R - (S - 1)) % R]);
#pragma unroll
        for (int u = 1; u < S; ++u) f = fma4(bv[u], ring[(r + R - (S - 1) + u) % R], f);
        epi.template worker<(((r + R - (S - 1)) & 1) == 0)>(i, f);
    }
}

template <int S, class Epi, int... Rs>
__device__ __forceinline__ void ring_round(float4 (&ring)[RingShape<S>::R], const float* __restrict__ G,
                                           int64_t ldg, int k, const float* __restrict__ bval,
                                           const LaneCoords& lc, int j0, int steps, Epi& epi,
                                           std::integer_sequence<int, Rs...>)
{
    (ring_step<S, Rs>(ring, G, ldg, k, bval, lc, j0, steps, epi), ...);
}

template <int S, class Epi>
__device__ __forceinline__ void encode_ring(const float* __restrict__ G, int64_t ldg, int k,
                                            const float* __restrict__ bval, const LaneCoords& lc,
                                            Epi& epi)
{
    constexpr int P = RingShape<S>::P;
    constexpr int R = RingShape<S>::R;
    static_assert(R % 2 == 0, "ring length must be even");
    const int steps = k + S - 1;  // row arrivals, the last S-1 being the wrapped rows
    float4 ring[R];
#pragma unroll
    for (int r = 0; r < P; ++r) {
        const int j = r < steps ? r : steps - 1;
        ring[r] = load_row4(G, ldg, j < k ? j : j - k, lc);
    }
#pragma unroll
    for (int r = P; r < R; ++r) ring[r] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j0 = 0; j0 < steps; j0 += R)
        ring_round<S>(ring, G, ldg, k, bval, lc, j0, steps, epi, std::make_integer_sequence<int, R>{});
}

// ---------------------------------------------------------------------------------------
// Encode driver 2: any CSR code.  Each worker gathers its rows straight from memory; rows
// shared by neighbouring workers are served by the caches.
// ---------------------------------------------------------------------------------------
struct CsrView {
    const int* __restrict__ row_ptr;
    const int* __restrict__ col;
    const float* __restrict__ val;
};

__device__ __forceinline__ float4 encode_gather_one(const float* __restrict__ G, int64_t ldg,
                                                    const CsrView& B, int i, const LaneCoords& lc)
{
    const int e0 = B.row_ptr[i], e1 = B.row_ptr[i + 1];
    float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
    if (e0 < e1) {
        f = mul4(B.val[e0], load_row4(G, ldg, B.col[e0], lc));
        for (int e = e0 + 1; e < e1; ++e) f = fma4(B.val[e], load_row4(G, ldg, B.col[e], lc), f);
    }
    return f;
}

template <class Epi>
__device__ __forceinline__ void encode_gather(const float* __restrict__ G, int64_t ldg, int n,
                                              const CsrView& B, const LaneCoords& lc, Epi& epi)
{
    for (int i = 0; i < n; i += 2) {
        epi.template worker<true>(i, encode_gather_one(G, ldg, B, i, lc));
        if (i + 1 < n) epi.template worker<false>(i + 1, encode_gather_one(G, ldg, B, i + 1, lc));
    }
}

}  // namespace agc
