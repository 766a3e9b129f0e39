// Mask compaction (feeds the fused forward) and the plain fp32 forward used for small problems.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lsr {

constexpr int PREP_THREADS = 256;

// One workgroup per sequence: len[b] = number of valid tokens, pos[b, 0..len) = their positions in
// ascending order.  The attention mask M of Sec. 2 may be arbitrary, so this is a stream
// compaction (ballot + popcount prefix), not a search for the first padding token.
__global__ __launch_bounds__(PREP_THREADS) void fwd_prep_kernel(const uint8_t* __restrict__ mask,
                                                                 int* __restrict__ len,
                                                                 int* __restrict__ pos, int S) {
    __shared__ int s_wave_total[PREP_THREADS / 64];
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const uint8_t* mrow = mask + (size_t)b * S;
    int* prow = pos + (size_t)b * S;
    int base = 0;
    for (int s0 = 0; s0 < S; s0 += PREP_THREADS) {
        const int s = s0 + tid;
        const bool flag = s < S && mrow[s] != 0;
        const unsigned long long bal = __ballot(flag);
        const int rank = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) s_wave_total[wave] = __popcll(bal);
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < PREP_THREADS / 64; ++w) {
            const int t = s_wave_total[w];
            before += w < wave ? t : 0;
            total += t;
        }
        if (flag) prow[base + before + rank] = s;
        base += total;
        __syncthreads();
    }
    if (tid == 0) len[b] = base;
}

// Plain fp32 head: one thread per (b, v), looping over valid positions and the hidden size with
// fp32 FMAs.  Eq. 1 evaluated with the max taken before the activation (Sec. 3).  Not tuned: it
// exists so that small fp32 problems run through the same entry points.
constexpr int F32_THREADS = 128;

template <bool ARG>
__global__ __launch_bounds__(F32_THREADS) void fwd_f32_kernel(const float* __restrict__ H,
                                                              const float* __restrict__ W,
                                                              const float* __restrict__ bias,
                                                              const int* __restrict__ len,
                                                              const int* __restrict__ pos,
                                                              float* __restrict__ Y, int* __restrict__ I,
                                                              int S, int D, int V) {
    const int b = blockIdx.y;
    const int v = blockIdx.x * F32_THREADS + threadIdx.x;
    if (v >= V) return;
    const int n = len[b];
    const float* wrow = W + (size_t)v * D;
    float m = -INFINITY;
    int arg = 0;
    for (int j = 0; j < n; ++j) {
        const int s = pos[(size_t)b * S + j];
        const float* hrow = H + ((size_t)b * S + s) * D;
        float a = 0.f;
        for (int d = 0; d < D; ++d) a = fmaf(hrow[d], wrow[d], a);
        if (a > m) { m = a; arg = s; }
    }
    const size_t o = (size_t)b * V + v;
    Y[o] = n > 0 ? log1pf(fmaxf(m + bias[v], 0.f)) : 0.f;
    if (ARG) I[o] = arg;
}

}  // namespace lsr
