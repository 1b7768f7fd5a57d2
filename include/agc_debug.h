/*
 * agc_debug.h -- measurement and testing hooks of libagc.so.  Nothing here is part of the method
 * (include/agc.h is); these entry points exist so that benchmarks and tests can time the
 * library's kernels one by one, scale hardware counters against a kernel of known traffic,
 * measure what the memory system delivers for the access pattern of the two streaming passes,
 * and force a code onto the slow general path.
 */
#ifndef AGC_DEBUG_H
#define AGC_DEBUG_H

#include "agc.h"

#ifdef __cplusplus
extern "C" {
#endif

#define AGC_NUM_KERNELS 4     /* scale pass, scale finalize, encode+quantize+pack, decode */

/* Testing hook in agc_opts: force_generic != 0 makes agc_set_code ignore the structure of the
 * code (cyclic band, monotone intervals) so that the general gather driver runs; results are
 * the same bits, only slower. */

/* --------------------------------------------------------------------------------------
 * Per-kernel timing (HIP events recorded on the caller's stream around each kernel)
 * ------------------------------------------------------------------------------------ */
/* on != 0: the following hot-path calls bracket each of their kernels with a pair of events
 * (a ring of 128 pairs per kernel; when the ring is full the oldest pair is drained with one
 * event synchronisation).  Kernel indices: 0 scale pass, 1 scale finalize,
 * 2 encode+quantize+pack, 3 decode.  The event records cost about 20 microseconds per step. */
agc_status agc_profile_enable(agc_ctx *ctx, int on);
/* Waits for the recorded events, adds them up and clears the ring: total_ms[j] and
 * launches[j] for each kernel index j since the previous read. */
agc_status agc_profile_read(agc_ctx *ctx, double total_ms[AGC_NUM_KERNELS],
                            int64_t launches[AGC_NUM_KERNELS]);

/* A plain copy kernel that reads `bytes` and writes `bytes` (device pointers, 16-byte aligned,
 * bytes a multiple of 16).  Profiling runs use it as the kernel of known size against which the
 * memory-traffic counters are scaled; timed, it is a measured copy ceiling of the device. */
agc_status agc_calibration_copy(void *dst_dev, const void *src_dev, int64_t bytes, void *hip_stream);

/*
 * The bare memory access pattern of the scale pass and of the quantize pass, with no
 * arithmetic worth the name: one wave per 256 consecutive coordinates walks over the k rows of G
 * (16 bytes per lane and row, non-temporal, four rows in flight) exactly as the register-ring
 * driver does.  piece_bytes == 0: reads only (the scale pass).  piece_bytes > 0 (a multiple of 16,
 * at most 1024): the kernel also writes piece_bytes bytes per block and row, non-temporal, to that
 * row's own output stream, the way the quantize pass writes a b-bit worker's 32*b bytes per block;
 * out_dev then holds k streams of floor(d/256) * piece_bytes bytes each, back to back.
 *   wg_flush == 0: every wave stores its piece right after the row (what a wave on its own would do:
 *                  64..96-byte stores that reach memory as partial lines);
 *   wg_flush != 0: a workgroup (four blocks) keeps its pieces until it has walked all rows and then,
 *                  after one barrier, writes 4 * piece_bytes contiguous bytes per row (what the
 *                  quantize pass does through its LDS staging area).
 *   blocks_per_wave: 1, or 2 with piece_bytes == 0: a wave walks two neighbouring blocks at once
 *                  (two loads per row, 1 KiB apart, two rows in flight), the form of the max-abs
 *                  scale pass on long vectors; only whole pairs of blocks are read then.
 *   waves_per_simd: 0 = whatever fits (eight), 4 = the kernel is built for four waves per SIMD, the
 *                  occupancy the quantize pass runs at (the memory system delivers most there);
 *   fma_per_row:   0, 40 or 100: that many dependent multiply-adds per row and lane between the
 *                  loads, standing in for the arithmetic of a pass (the quantize pass issues about
 *                  ninety vector instructions per row and lane); only with waves_per_simd == 4,
 *                  wg_flush != 0, piece_bytes > 0 and blocks_per_wave == 1.
 * Only whole blocks are touched (floor(d/256) of them).  What this kernel reaches is what the
 * memory system delivers for that traffic, whatever the arithmetic on top of it.
 *   G_dev    device, k x d binary32, row stride ldg (multiple of 4), 16-byte aligned; read-only
 *   out_dev  device, 16-byte aligned, at least max(16, k * floor(d/256) * piece_bytes) bytes
 */
agc_status agc_debug_stream_rows(const float *G_dev, int64_t ldg, int k, int64_t d, int piece_bytes,
                                 int wg_flush, int blocks_per_wave, int waves_per_simd, int fma_per_row,
                                 void *out_dev, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* AGC_DEBUG_H */
