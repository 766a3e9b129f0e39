// Mask compaction (feeds the fused forward) and the plain fp32 forward used for small problems.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fwd_bf16.hpp"

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

// Packing plan for the MFMA forward.  Every sequence takes ceil(len / 32) blocks of 32 rows (one
// block if it has no valid token, so that its zero output is still written); blk0 is the exclusive
// prefix sum of the block counts, and the block list is cut into n_groups contiguous ranges of whole
// sequences with about equal block counts, the cuts nudged so that groups hold whole 8-block tiles
// where a sequence start allows it.  One workgroup; B and n_groups (at most PLAN_MAX_GROUPS) are small
// next to the GEMM.
constexpr int PLAN_THREADS = 256;
constexpr int PLAN_CAND = 5;            // sequence starts proposed per boundary: the even cut and two either side
constexpr int PLAN_MAX_GROUPS = 1024;

__global__ __launch_bounds__(PLAN_THREADS) void fwd_plan_kernel(const int* __restrict__ len, int* blk0,
                                                                 int* __restrict__ grp_blk0, int B,
                                                                 int n_groups, int nudge) {
    __shared__ int s_scan[PLAN_THREADS];
    __shared__ __attribute__((aligned(16))) int s_cand[(PLAN_MAX_GROUPS + 1) * 8];    // PLAN_CAND used of 8 per boundary
    __shared__ int s_cut[PLAN_MAX_GROUPS + 1];          // even cuts, then the chosen boundaries
    const int tid = threadIdx.x;
    int base = 0;
    for (int b0 = 0; b0 < B; b0 += PLAN_THREADS) {
        const int b = b0 + tid;
        int n = 0;
        if (b < B) {
            n = (len[b] + 31) >> 5;
            n = n > 0 ? n : 1;
        }
        s_scan[tid] = n;
        __syncthreads();
        for (int off = 1; off < PLAN_THREADS; off <<= 1) {
            const int add = tid >= off ? s_scan[tid - off] : 0;
            __syncthreads();
            s_scan[tid] += add;
            __syncthreads();
        }
        if (b < B) blk0[b] = base + s_scan[tid] - n;
        base += s_scan[PLAN_THREADS - 1];
        __syncthreads();
    }
    if (tid == 0) blk0[B] = base;
    // the prefix sums are read back below by other threads of this workgroup: make them visible at
    // device scope and read them with device-scope loads (no stale line of the vector L1)
    __threadfence();
    __syncthreads();
    const int total = base;
    auto blk0_at = [&](int b) { return __hip_atomic_load(&blk0[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
    // Every thread proposes, for its boundaries, the sequence starts around the even cut
    // g * total / n_groups; one thread then walks the boundaries in order and takes, among the
    // proposals within half a group of the even cut, the one that leaves the fewest empty block slots
    // in the last 8-block tile of the group it closes (ties: nearest to the even cut).  A group whose
    // block count is a multiple of 8 has no ragged tile; a ragged tile pays the whole vocabulary-tile
    // side of a tile (loads of W, its fragments, barriers, epilogue) for a fraction of the rows.
    // The nudged groups are less even in size, so the host asks for them (`nudge`) only when the grid
    // is many workgroups per CU deep.
    for (int g = tid; g <= n_groups; g += PLAN_THREADS) {
        const int target = (int)(((long long)g * total) / n_groups);
        int lo = 0, hi = B;                       // smallest b in [0, B] with blk0[b] >= target
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (blk0_at(mid) >= target) hi = mid; else lo = mid + 1;
        }
        if (!nudge) {                             // even cuts: no boundary depends on another
            grp_blk0[g] = g == n_groups ? total : blk0_at(lo);
            continue;
        }
        s_cut[g] = target;
#pragma unroll
        for (int k = 0; k < PLAN_CAND; ++k) {
            const int c = lo + k - PLAN_CAND / 2;
            s_cand[g * 8 + k] = (c >= 0 && c <= B) ? blk0_at(c) : -1;
        }
    }
    __syncthreads();
    if (nudge && tid == 0) {
        const int half = total / (2 * n_groups);
        int prev = 0;
        for (int g = 1; g < n_groups; ++g) {
            const int target = s_cut[g];
            // the proposals of this boundary in two 16-byte reads, then branch-free selection
            const int4 c03 = *reinterpret_cast<const int4*>(&s_cand[g * 8]);
            const int c4 = s_cand[g * 8 + 4];
            const int cand[PLAN_CAND] = {c03.x, c03.y, c03.z, c03.w, c4};
            int best = -1, best_key = 0x7fffffff;
#pragma unroll
            for (int k = 0; k < PLAN_CAND; ++k) {
                const int x = cand[k];
                const int dist = x > target ? x - target : target - x;
                const bool ok = x > prev && (dist <= half || k == PLAN_CAND / 2);
                const int waste = (8 - ((x - prev) & 7)) & 7;
                const int key = ok ? (waste << 27) | (dist < (1 << 27) ? dist : (1 << 27) - 1) : 0x7fffffff;
                const bool take = key < best_key;
                best_key = take ? key : best_key;
                best = take ? x : best;
            }
            prev = best < 0 ? prev : best;        // nothing beyond the last boundary: an empty group
            s_cut[g] = prev;
        }
        s_cut[0] = 0;
        s_cut[n_groups] = total;
    }
    __syncthreads();
    if (nudge)
        for (int g = tid; g <= n_groups; g += PLAN_THREADS) grp_blk0[g] = s_cut[g];
}

// Row table of the packed layout, one workgroup per sequence: packed row k of the sequence reads
// token pos[min(k, len-1)] (the tail of the last block repeats the last valid token), and every
// block records its sequence, whether it ends it, and whether the sequence is empty.
constexpr int FWD_ROWS_THREADS = 256;

__global__ __launch_bounds__(FWD_ROWS_THREADS) void fwd_rows_kernel(const int* __restrict__ len,
                                                                     const int* __restrict__ pos,
                                                                     const int* __restrict__ blk0,
                                                                     int2* __restrict__ rows,
                                                                     int* __restrict__ blk_meta, int S) {
    const int b = blockIdx.x;
    const int n = len[b];
    const int g0 = blk0[b];
    const int nblk = blk0[b + 1] - g0;
    const int* prow = pos + (size_t)b * S;
    for (int k = threadIdx.x; k < nblk * 32; k += FWD_ROWS_THREADS) {
        const int s = n > 0 ? prow[k < n ? k : n - 1] : 0;
        rows[(size_t)g0 * 32 + k] = make_int2(b * S + s, s);
    }
    for (int k = threadIdx.x; k < nblk; k += FWD_ROWS_THREADS)
        blk_meta[g0 + k] = b | (k == nblk - 1 ? (1 << 31) : 0) | (n == 0 ? (1 << 30) : 0);
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

// Register-only matrix-core probe: every wave issues `iters` rounds of four independent
// 32x32x16 bf16 MFMAs on operands it never reloads, so the time is the matrix pipes' alone at
// whatever clock the part sustains under that load.  The result is folded into one value per lane
// that is compared with a number it cannot take, so nothing is stored; `sink` only keeps the
// arithmetic alive.  Measurement aid: the denominator "what the matrix cores deliver on this box"
// beside the nominal peak.
constexpr int PROBE_THREADS = 256;
constexpr int PROBE_MFMA_PER_ITER = 4;

__global__ __launch_bounds__(PROBE_THREADS) void mfma_probe_kernel(int iters, float* sink) {
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.001f * (float)((lane + i) & 7));
        b[i] = (__bf16)(0.002f * (float)((lane * 3 + i) & 7));
    }
    floatx16 acc[PROBE_MFMA_PER_ITER];
#pragma unroll
    for (int k = 0; k < PROBE_MFMA_PER_ITER; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < PROBE_MFMA_PER_ITER; ++k)
            acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < PROBE_MFMA_PER_ITER; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[k][r];
    if (sum == -1.2345e30f) *sink = sum;      // sums of non-negative products: never taken
}

}  // namespace lsr
