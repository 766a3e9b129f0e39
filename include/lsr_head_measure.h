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
 *   forward : [0] mask compaction  [1] fused GEMM + max/argmax + activation
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
 * The launch plan the host derives from a shape alone, for inspection and tests (no device needed,
 * nothing is launched).  Writes LSR_PLAN_SLOTS int32 values to the HOST array `plan`:
 *   [0] row groups of the packed forward          [1] segments of the bucket sort per sequence
 *   [2] vocabulary entries per sort segment       [3] 1 if the sort places through LDS, else 0
 *   [4] vocabulary chunks of the dH gather        [5] vocabulary entries per chunk
 *   [6] buckets per wave in the sliced dH gather (0: whole-row dH kernel, D not a multiple of 64)
 *   [7] rows of the sliced dW gather's staging tile (0: whole-row dW kernel)
 *   [8] sequences per launch of the sliced dW gather (B: one launch)
 */
#define LSR_PLAN_SLOTS 9
int lsr_head_plan(const lsr_head_desc* desc, int32_t* plan);

#ifdef __cplusplus
}
#endif
#endif /* LSR_HEAD_MEASURE_H */
