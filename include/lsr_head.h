/*
 * lsr_head.h - C ABI of the MI355X (gfx950) sparse-lexical LM head.
 *
 * The head maps hidden states to one non-negative score per vocabulary entry
 * (paper Sec. 2, Eq. 1):
 *
 *     Y[b,v] = max over valid s of  log(1 + ReLU( sum_d H[b,s,d] * W[v,d] + bias[v] ))
 *
 * computed as in Sec. 3 "Forward Pass": the activation is monotone, so the maximum is
 * taken over raw logit tiles on chip and the activation is applied once to the B x V result;
 * the B x S x V logit tensor is never written to memory.  The backward follows Sec. 3
 * "Backward Pass" / Alg. 3: only (Y, I) are saved, the upstream gradient is gated by
 * exp(-Y) where Y > 0 and routed to the single position I[b,v].
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller, contiguous row-major,
 *     16-byte aligned.  The library never allocates, frees or keeps device memory.  Its only
 *     state is, per device, one auxiliary stream and two events created by the first backward
 *     call that uses them (small problems run the dW gather beside the dH chain; the work is
 *     forked from and joined back into `stream`, so the caller sees ordinary stream order).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null stream)
 *     and the call returns without synchronising, except the *_profiled variants.
 *     Both calls can be recorded into a HIP graph on a capturing stream; make one backward call
 *     on the device before capturing, so that the auxiliary stream and events already exist.
 *   - Outputs are overwritten; nothing has to be zeroed by the caller.
 *   - All argument checks run on the host before anything is enqueued; on error nothing has
 *     been launched.  The return value is an lsr_status; no exceptions, no abort().
 *   - Inputs must be finite.  The mask may be arbitrary (not only padding at the end).
 */
#ifndef LSR_HEAD_H
#define LSR_HEAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LSR_OK = 0,
    LSR_ERR_NULL = 1,       /* a required pointer is NULL                               */
    LSR_ERR_SHAPE = 2,      /* B,S,D,V out of the supported range (see lsr_head_desc)   */
    LSR_ERR_DTYPE = 3,      /* unknown hw_dtype                                         */
    LSR_ERR_ALIGN = 4,      /* a pointer is not 16-byte aligned                         */
    LSR_ERR_WORKSPACE = 5,  /* workspace NULL or smaller than lsr_head_workspace_bytes  */
    LSR_ERR_ARCH = 6,       /* no usable device, or the current device is not gfx950    */
    LSR_ERR_LAUNCH = 7      /* the HIP runtime reported a launch/event error            */
} lsr_status;

typedef enum { LSR_F32 = 0, LSR_BF16 = 1 } lsr_dtype;

/*
 * Problem shape (paper Sec. 2: H in R^{B x S x D}, E (here W) in R^{|V| x D}, b in R^{|V|},
 * M in {0,1}^{B x S}).  H and W share hw_dtype; bias, Y and all gradients are float32; I is int32.
 * Limits: 1 <= B,S,D,V;  B <= 65535;  B*S < 2^31;  B*V < 2^31;  D a multiple of 8 and D <= 8192;
 * S <= 32768 (backward: S <= 8192 and B <= 6144).  LSR_BF16 runs the MFMA kernel; LSR_F32 is a
 * plain reference-precision path meant for small problems.
 */
typedef struct {
    int64_t B, S, D, V;
    int32_t hw_dtype;   /* lsr_dtype */
} lsr_head_desc;

/* Bytes of device scratch the forward (for_backward = 0) or backward (!= 0) call needs for
 * this shape: O(B*S) for the forward, O(B*V + B*S) for the backward (8*B*V bytes of sorted
 * (v, g) pairs, count tables of at most 4*B*V, and 4*B*S*(c+1) for a vocabulary gathered in
 * c <= 64 chunks).  Returns 0 for an invalid desc. */
size_t lsr_head_workspace_bytes(const lsr_head_desc* desc, int for_backward);

/*
 * Forward (Eq. 1 via the streaming max of Sec. 3; result of Alg. 2).
 *   H    [B,S,D] hw_dtype      W [V,D] hw_dtype      bias [V] f32
 *   mask [B,S] uint8, non-zero = valid token.  Masked positions are excluded from the maximum.
 *   Y    [B,V] f32 out.  Rows without any valid token give 0.
 *   I    [B,V] int32 out, may be NULL (then no index is tracked).  I[b,v] is the sequence
 *        position of the maximum logit; the lowest position wins exact ties; 0 for rows without
 *        valid tokens.
 */
int lsr_head_forward(const lsr_head_desc* desc,
                     const void* H, const void* W, const float* bias, const uint8_t* mask,
                     float* Y, int32_t* I,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward (Sec. 3 "Backward Pass", Alg. 3), from the saved (Y, I) of the forward:
 *   g[b,v]    = dY[b,v] * exp(-Y[b,v]) if Y[b,v] > 0 else 0
 *   db[v]     = sum_b g[b,v]                       (bias gradient; chain rule, not in Alg. 3)
 *   dW[v,:]   = sum_b g[b,v] * H[b, I[b,v], :]
 *   dH[b,s,:] = sum over v with I[b,v] = s of g[b,v] * W[v,:]     (0 for unselected positions)
 * dH [B,S,D], dW [V,D], db [V] are float32 outputs; each may be NULL to skip it.  Every
 * requested output is fully overwritten.  Summation order is fixed, so results are
 * bit-reproducible from call to call.  I must hold values in [0,S).
 */
int lsr_head_backward(const lsr_head_desc* desc,
                      const void* H, const void* W,
                      const float* dY, const float* Y, const int32_t* I,
                      float* dH, float* dW, float* db,
                      void* workspace, size_t workspace_bytes, void* stream);

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
                              void* workspace, size_t workspace_bytes, void* stream,
                              float* kernel_ms);
int lsr_head_backward_profiled(const lsr_head_desc* desc,
                               const void* H, const void* W,
                               const float* dY, const float* Y, const int32_t* I,
                               float* dH, float* dW, float* db,
                               void* workspace, size_t workspace_bytes, void* stream,
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
int lsr_mfma_peak_probe(int64_t iters, int launches, void* sink, double* tflops, void* stream);

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

/* Static, NUL-terminated description of a status code. */
const char* lsr_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* LSR_HEAD_H */
