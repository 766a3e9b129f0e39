// Reduce step of the paper's hybrid forward (Sec. 3, Alg. 2) as a benchmark comparator: reads one
// vocabulary tile of logits that a library GEMM wrote to memory, takes the maximum and arg-max over each
// sequence's rows, applies bias, ReLU and log1p.  Bandwidth-bound by construction (every logit is read
// once); the product's fused kernel exists so that this read, and the write before it, never happen.
#include "lsr_alg2_reduce.h"

#include <hip/hip_runtime.h>

namespace {

constexpr int RED_THREADS = 256;      // 4 waves: wave w takes rows w, w+4, ... of the sequence
constexpr int RED_COLS = 128;         // columns per workgroup: 64 lanes x 2

template <bool BF16>
__device__ __forceinline__ float2 load2(const void* base, size_t elem) {
    if (BF16) {
        const uint32_t u = *reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(base) + elem);
        return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xffff0000u));
    }
    return *reinterpret_cast<const float2*>(static_cast<const float*>(base) + elem);
}

template <bool BF16>
__global__ __launch_bounds__(RED_THREADS) void alg2_reduce_kernel(const void* __restrict__ logits, size_t ldl,
                                                                  const int* __restrict__ seq_row0,
                                                                  const int* __restrict__ row_pos,
                                                                  const float* __restrict__ bias,
                                                                  float* __restrict__ Y, int* __restrict__ I,
                                                                  size_t V, size_t v0, int C) {
    __shared__ float s_m[4][RED_COLS];
    __shared__ int s_r[4][RED_COLS];
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x * RED_COLS + lane * 2;
    const int r0 = seq_row0[b], r1 = seq_row0[b + 1];
    float m[2] = {-INFINITY, -INFINITY};
    int a[2] = {r0, r0};
    if (c < C) {
        // four rows in flight per lane; rows ascend, so a strict comparison keeps the first maximum
        for (int r = r0 + wave; r < r1; r += 16) {
            float2 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int rr = r + 4 * u;
                x[u] = rr < r1 ? load2<BF16>(logits, (size_t)rr * ldl + c) : make_float2(-INFINITY, -INFINITY);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (x[u].x > m[0]) { m[0] = x[u].x; a[0] = r + 4 * u; }
                if (x[u].y > m[1]) { m[1] = x[u].y; a[1] = r + 4 * u; }
            }
        }
    }
    s_m[wave][lane * 2] = m[0];
    s_m[wave][lane * 2 + 1] = m[1];
    s_r[wave][lane * 2] = a[0];
    s_r[wave][lane * 2 + 1] = a[1];
    __syncthreads();
    if (threadIdx.x < RED_COLS) {
        const int cc = blockIdx.x * RED_COLS + threadIdx.x;
        if (cc < C) {
            float best = s_m[0][threadIdx.x];
            int row = s_r[0][threadIdx.x];
#pragma unroll
            for (int w = 1; w < 4; ++w) {
                const float mw = s_m[w][threadIdx.x];
                const int rw = s_r[w][threadIdx.x];
                if (mw > best || (mw == best && rw < row)) { best = mw; row = rw; }
            }
            const size_t o = (size_t)b * V + v0 + cc;
            const bool any = r1 > r0;
            Y[o] = any ? log1pf(fmaxf(best + bias[v0 + cc], 0.f)) : 0.f;
            I[o] = any ? row_pos[row] : 0;
        }
    }
}

}  // namespace

extern "C" int lsr_alg2_reduce(const void* logits, int logits_bf16, int64_t ldl, const int32_t* seq_row0,
                               const int32_t* row_pos, const float* bias, float* Y, int32_t* I, int B, int64_t V,
                               int64_t v0, int C, struct ihipStream_t* stream) {
    if (!logits || !seq_row0 || !row_pos || !bias || !Y || !I) return 1;
    if (B < 1 || B > 65535 || C < 1 || (C & 1) || ldl < C || (ldl & 1) || v0 < 0 || v0 + C > V) return 1;
    const dim3 grid((C + RED_COLS - 1) / RED_COLS, B);
    if (logits_bf16)
        hipLaunchKernelGGL(alg2_reduce_kernel<true>, grid, dim3(RED_THREADS), 0, stream, logits, (size_t)ldl, seq_row0, row_pos,
                           bias, Y, I, (size_t)V, (size_t)v0, C);
    else
        hipLaunchKernelGGL(alg2_reduce_kernel<false>, grid, dim3(RED_THREADS), 0, stream, logits, (size_t)ldl, seq_row0, row_pos,
                           bias, Y, I, (size_t)V, (size_t)v0, C);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
