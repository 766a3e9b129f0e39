/*
 * lsr_head_measure.h - measurement aids of the MI355X sparse-lexical LM head library.
 *
 * Not part of the product boundary (that is lsr_head.h): these entry points exist for the benchmark,
 * the profiles and the host-logic tests.  Same conventions as lsr_head.h, except that the *_profiled
 * variants and the probe synchronise `stream` and write to HOST arrays.
 */
#ifndef LSR_HEAD_MEASURE_H
#define LSR_HEAD_MEASURE_H

#include "lsr_head.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Same work as the calls above, with each kernel bracketed by HIP events on `stream`.  The call
 * synchronises the stream and writes the per-kernel times in milliseconds to the HOST array
 * kernel_ms (LSR_PROFILE_SLOTS floats; unused slots are set to 0).  For measurement only.
 *   forward : [0] mask compaction and packing  [1] fused GEMM + max/argmax + activation
 *             [2] join of the sequences cut by a chunk boundary
 *   backward: [0] bucket count     [1] bucket scan   [2] bucket placement
 *             [3] dH gather        [4] dW/db gather
 */
#define LSR_PROFILE_SLOTS 8
int lsr_head_forward_profiled(const lsr_head_desc* desc,
                              const void* H, const void* W, const float* bias, const uint8_t* mask,
                              float* Y, int32_t* I,
                              void* workspace, size_t workspace_bytes, lsr_stream_t stream,
                              float* kernel_ms);
int lsr_head_backward_profiled(const lsr_head_desc* desc,
                               const void* H, const void* W,
                               const float* dY, const float* Y, const int32_t* I,
                               float* dH, float* dW, float* db,
                               void* workspace, size_t workspace_bytes, lsr_stream_t stream,
                               float* kernel_ms);

/*
 * Measurement aid, not part of the head: what the matrix cores of the current device deliver on
 * bf16 32x32x16 MFMAs issued from registers alone (no memory traffic), at the clock the part
 * sustains under that load.  Runs `launches` back-to-back launches of `iters` rounds per wave on
 * `stream` (two waves per SIMD, four independent accumulator chains each), times the last one with
 * events, synchronises, and writes dense TFLOP/s to the HOST double *tflops.  `sink` is a DEVICE
 * pointer to 4 writable bytes (never written in practice; it keeps the arithmetic alive).
 * iters in [1, 2^24], launches in [1, 64].
 */
int lsr_mfma_peak_probe(int64_t iters, int launches, void* sink, double* tflops, lsr_stream_t stream);

/*
 * Measurement aids, not part of the head: reference rates the benchmark quotes beside the backward's
 * gathers.  Both run `launches` back-to-back launches on `stream` (1..64), time the last one with events,
 * synchronise, and write a rate in GB/s (1e9 bytes per second) to the HOST double *gbytes_per_s.
 *
 * lsr_copy_probe: a plain copy of `bytes` (a multiple of 16) from the DEVICE buffer src to the DEVICE
 *   buffer dst; the rate counts bytes read plus bytes written.  Also the known-size reference for the
 *   profiler's FETCH_SIZE / WRITE_SIZE counters.
 * lsr_gather_probe: 128-byte row pieces gathered at pseudo-random rows of the first window_bytes (a
 *   multiple of 128) of the DEVICE buffer `table`, eight lanes per piece, four pieces in flight per
 *   lane, `steps` rounds per lane, fp32 FMAs on the bf16 payload - the access pattern of the backward's
 *   sliced gathers without their index lists.  The rate counts gathered bytes.  `out` is a DEVICE buffer
 *   of at least CUs * 16 * 256 * 32 bytes (32 MiB on 256 compute units; LSR_ERR_WORKSPACE if out_bytes
 *   is smaller); it receives the partial sums.
 */
int lsr_copy_probe(void* dst, const void* src, size_t bytes, int launches, double* gbytes_per_s, lsr_stream_t stream);
int lsr_gather_probe(const void* table, size_t window_bytes, int steps, int launches, void* out, size_t out_bytes,
                     double* gbytes_per_s, lsr_stream_t stream);

/*
 * The launch plan the host derives from a shape alone, for inspection and tests (no device needed,
 * nothing is launched).  Writes LSR_PLAN_SLOTS int32 values to the HOST array `plan`:
 *   [0] most tiles per chunk of the packed forward    [1] segments of the bucket sort per sequence
 *   [2] vocabulary entries per sort segment       [3] 1 if the sort places through LDS, else 0
 *   [4] vocabulary chunks of the dH gather        [5] vocabulary entries per chunk
 *   [6] buckets per wave in the sliced dH gather (0: whole-row dH kernel, D not a multiple of 64)
 *   [7] rows of the sliced dW gather's staging tile (0: whole-row dW kernel)
 *   [8] sequences per launch of the sliced dW gather (B: one launch)
 *   [9] chunks the forward grid provides for (the longest token list the shape allows)
 *   [10] rows per segment of the packed token list (32, or 8 for batches of short sequences)
 *   [11] 1 if the forward runs one resident workgroup per CU over its units (shallow problems), else 0
 *   [12] 1 if the column slices of the sliced dH gather are owned by XCDs (small batches), else 0
 *   [13] copy passes per tile of the LDS-tile dW kernel (ceil(S / 128)), 0 when the gathers of [7] / [8] run
 *        instead (the kernel applies to bfloat16 shapes with 128 <= S <= 512 and enough vocabulary rows to
 *        give every CU a workgroup; it also needs dW to be requested)
 */
#define LSR_PLAN_SLOTS 14
int lsr_head_plan(const lsr_head_desc* desc, int32_t* plan);

#ifdef __cplusplus
}
#endif
#endif /* LSR_HEAD_MEASURE_H */
