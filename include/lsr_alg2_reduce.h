/*
 * lsr_alg2_reduce.h - the reduce step of the paper's hybrid forward (Sec. 3, Alg. 2), as a benchmark
 * comparator.  NOT part of the product: the product is the fused kernel behind lsr_head.h, which
 * never writes logits to memory.  Alg. 2 runs, per tile of the vocabulary, a library GEMM that writes
 * the tile's logits to memory and then a small kernel that takes the masked maximum and arg-max over
 * the sequence and applies ReLU and log1p; this header declares that small kernel, so that the
 * benchmark can time "library GEMM + reduce" on the same inputs as the fused kernel.
 */
#ifndef LSR_ALG2_REDUCE_H
#define LSR_ALG2_REDUCE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

struct ihipStream_t;

/*
 * One vocabulary tile of Alg. 2's reduce.  All pointers are DEVICE pointers owned by the caller.
 *   logits    [M, C] row-major with leading dimension ldl (elements): the tile's logits for the M packed
 *             valid tokens of the batch (rows of sequence b are seq_row0[b] .. seq_row0[b+1]-1, in
 *             ascending position), float32 (logits_bf16 = 0) or bfloat16 (logits_bf16 = 1)
 *   seq_row0  [B+1] int32     row_pos [M] int32: sequence position of every packed row
 *   bias      [V] float32 (the whole vocabulary; the tile starts at v0)
 *   Y [B,V] float32, I [B,V] int32: columns v0 .. v0+C-1 are written:
 *             Y = log1p(max(0, max_row logit + bias)), I = position of the first row attaining the
 *             maximum; 0 and 0 for a sequence without rows.
 * Enqueued on `stream`, no synchronisation.  Returns 0, or 1 for a bad argument (NULL pointer, C < 1,
 * C odd, ldl < C, v0 + C > V), 2 if the launch failed.
 */
int lsr_alg2_reduce(const void* logits, int logits_bf16, int64_t ldl,
                    const int32_t* seq_row0, const int32_t* row_pos, const float* bias,
                    float* Y, int32_t* I, int B, int64_t V, int64_t v0, int C,
                    struct ihipStream_t* stream);

#ifdef __cplusplus
}
#endif
#endif /* LSR_ALG2_REDUCE_H */
