// Measurement aids, not part of the head: reference rates of the device that the benchmark quotes beside
// the backward's gathers.
//   copy_probe_kernel    a plain streaming copy (16 bytes per lane per step): what HBM delivers to the
//                        simplest possible kernel, and the scale reference for profiler byte counters
//   gather_probe_kernel  row pieces of 128 bytes gathered at pseudo-random rows of a window of given
//                        size, eight lanes per piece, four pieces in flight per lane, fp32 FMAs on the
//                        bf16 payload: the access pattern of the sliced dW / dH gathers with the index
//                        lists taken out.  With a window of a few MB it measures the rate of an
//                        L2-resident gather, with tens of MB that of the memory-side cache.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lsr {

constexpr int COPY_THREADS = 256;

__global__ __launch_bounds__(COPY_THREADS) void copy_probe_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                                   size_t n16) {
    const size_t stride = (size_t)gridDim.x * COPY_THREADS;
    for (size_t i = (size_t)blockIdx.x * COPY_THREADS + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

constexpr int GATHER_THREADS = 256;
constexpr int GATHER_NLD = 4;          // pieces in flight per lane

__global__ __launch_bounds__(GATHER_THREADS) void gather_probe_kernel(const uint16_t* __restrict__ table, uint32_t window_rows,
                                                                       int steps, float* __restrict__ out) {
    const int lane8 = threadIdx.x & 7;                                   // 16-byte chunk of the 128-byte piece
    const uint32_t group = (blockIdx.x * GATHER_THREADS + threadIdx.x) >> 3;
    uint32_t state = group * 2654435761u + 12345u;                       // per-group LCG: the eight lanes agree
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    for (int s = 0; s < steps; ++s) {
        uint4 x[GATHER_NLD];
#pragma unroll
        for (int u = 0; u < GATHER_NLD; ++u) {
            state = state * 1664525u + 1013904223u;
            const uint32_t row = (uint32_t)(((uint64_t)(state >> 4) * window_rows) >> 28);   // uniform in [0, window_rows)
            x[u] = *reinterpret_cast<const uint4*>(table + (size_t)row * 64 + lane8 * 8);
        }
#pragma unroll
        for (int u = 0; u < GATHER_NLD; ++u) {
            const uint32_t w[4] = {x[u].x, x[u].y, x[u].z, x[u].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[2 * i] = fmaf(0.5f, __uint_as_float(w[i] << 16), acc[2 * i]);
                acc[2 * i + 1] = fmaf(0.5f, __uint_as_float(w[i] & 0xffff0000u), acc[2 * i + 1]);
            }
        }
    }
    float* o = out + ((size_t)group * 8 + lane8) * 8;
    *reinterpret_cast<float4*>(o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    *reinterpret_cast<float4*>(o + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
}

}  // namespace lsr
