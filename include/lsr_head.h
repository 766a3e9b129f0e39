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
 *     16-byte aligned.  The library never allocates, frees or keeps device memory; scratch comes in
 *     as a caller-owned workspace (lsr_head_workspace_bytes states its size).
 *   - Work is enqueued on `stream` (lsr_stream_t is HIP's hipStream_t; NULL = the null stream)
 *     and the call returns without synchronising.
 *   - State.  The library keeps no per-problem state.  Per device it keeps one auxiliary stream and
 *     two events, created by the first backward call that uses them and kept until the process ends:
 *     small problems run the dW/db gather on that stream beside the dH chain, forked from and
 *     joined back into `stream`, so the caller sees ordinary stream order.  The fork..join enqueue is
 *     serialised per device by a mutex inside the library, so any number of host threads may call
 *     into the library concurrently, each on its own stream and buffers (their dW gathers then
 *     queue up on the one auxiliary stream).  Two calls that share a workspace or an output buffer
 *     must be ordered by the caller, as for any other stream work.
 *   - Both calls can be recorded into a HIP graph on a capturing stream; make one backward call
 *     on the device before capturing, so that the auxiliary stream and events already exist.
 *   - Outputs are overwritten; nothing has to be zeroed by the caller.
 *   - All argument checks run on the host before anything is enqueued; an error from a check
 *     (every status except LSR_ERR_LAUNCH) means nothing has been launched.  LSR_ERR_LAUNCH reports
 *     a failure of the HIP runtime in the middle of the sequence: earlier kernels of the call may
 *     have been enqueued, the auxiliary stream has been joined back, outputs are undefined.
 *     The return value is an lsr_status; no exceptions, no abort().
 *   - Inputs must be finite.  The mask may be arbitrary (not only padding at the end).
 *
 * Measurement aids (per-kernel timing, the launch plan, a matrix-core probe) are declared in
 * lsr_head_measure.h; they are not part of the product boundary.
 */
#ifndef LSR_HEAD_H
#define LSR_HEAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* HIP's stream handle (hipStream_t is a pointer to this same opaque struct), declared here so that
 * the header needs no HIP include and stays plain C. */
struct ihipStream_t;
typedef struct ihipStream_t* lsr_stream_t;

typedef enum {
    LSR_OK = 0,
    LSR_ERR_NULL = 1,       /* a required pointer is NULL                               */
    LSR_ERR_SHAPE = 2,      /* B,S,D,V out of the supported range (see lsr_head_desc)   */
    LSR_ERR_DTYPE = 3,      /* unknown hw_dtype                                         */
    LSR_ERR_ALIGN = 4,      /* a pointer is not 16-byte aligned                         */
    LSR_ERR_WORKSPACE = 5,  /* workspace NULL or smaller than lsr_head_workspace_bytes  */
    LSR_ERR_ARCH = 6,       /* no usable device, or the current device is not gfx950    */
    LSR_ERR_LAUNCH = 7,     /* the HIP runtime reported a launch/event error            */
    LSR_ERR_STATIC_SCRATCH = 8  /* lsr_head_forward_static: the shape needs more scratch than
                                   LSR_STATIC_SCRATCH_BYTES                              */
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
                     void* workspace, size_t workspace_bytes, lsr_stream_t stream);

/*
 * The forward for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same
 * kernels, same results as lsr_head_forward; the scratch that call takes as `workspace` lives here in
 * a static device array of LSR_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until
 * the process ends).  The call allocates and frees nothing.  A shape whose forward scratch
 * (lsr_head_workspace_bytes(desc, 0)) exceeds the array is rejected with LSR_ERR_STATIC_SCRATCH before
 * anything is enqueued.  All calls on one GPU share the one array: calls that may overlap on the
 * device (different streams, or different host threads) race on it and must be ordered by the caller;
 * calls on one stream are ordered by the stream.  Nothing in the array has to survive between calls.
 */
#define LSR_STATIC_SCRATCH_BYTES (16u << 20)
int lsr_head_forward_static(const lsr_head_desc* desc,
                            const void* H, const void* W, const float* bias, const uint8_t* mask,
                            float* Y, int32_t* I, lsr_stream_t stream);

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
                      void* workspace, size_t workspace_bytes, lsr_stream_t stream);

/*
 * The backward with options (Sec. 5 trains through the head: gradients usually go straight into
 * bfloat16 parameter gradients, and are accumulated over micro-batches).
 *   grad_dtype  LSR_F32: dH and dW are float32 (as lsr_head_backward).  LSR_BF16 (needs hw_dtype =
 *               LSR_BF16): dH [B,S,D] and dW [V,D] are bfloat16.  Sums are formed in float32 in the same
 *               order as for float32 outputs and rounded to nearest-even once, when the final value is
 *               stored; a result that several launches add up keeps its float32 partial sums in the
 *               workspace meanwhile.  db is float32 in both cases.
 *   accumulate  0: every requested output is overwritten.  1: the gradients are added to what dH, dW and
 *               db hold on entry (out = out + gradient, one rounding for bfloat16); positions of dH that
 *               receive no gradient are left as they are.
 * opts == NULL means {LSR_F32, 0}.  The workspace size for given options comes from
 * lsr_head_backward_ex_workspace_bytes (0 for an invalid desc or option); for {LSR_F32, any} it equals
 * lsr_head_workspace_bytes(desc, 1).  Everything else as lsr_head_backward.
 */
typedef struct {
    int32_t grad_dtype;   /* lsr_dtype of dH and dW */
    int32_t accumulate;   /* 0 or 1 */
} lsr_backward_opts;

size_t lsr_head_backward_ex_workspace_bytes(const lsr_head_desc* desc, const lsr_backward_opts* opts);

int lsr_head_backward_ex(const lsr_head_desc* desc,
                         const void* H, const void* W,
                         const float* dY, const float* Y, const int32_t* I,
                         void* dH, void* dW, float* db,
                         const lsr_backward_opts* opts,
                         void* workspace, size_t workspace_bytes, lsr_stream_t stream);

/* Static, NUL-terminated description of a status code. */
const char* lsr_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* LSR_HEAD_H */
