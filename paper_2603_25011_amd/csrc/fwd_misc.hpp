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

// Packing plan for the MFMA forward.  Every sequence takes ceil(len / seg) segments of seg rows (one
// segment if it has no valid token, so that its zero output is still written; seg = 32, or 8 for batches
// of short sequences); seg0 is the exclusive prefix sum of the segment counts and seg0[B] the length of
// the segment list.  One workgroup; B is small next to the GEMM.
constexpr int PLAN_THREADS = 256;

__global__ __launch_bounds__(PLAN_THREADS) void fwd_plan_kernel(const int* __restrict__ len, int* __restrict__ blk0,
                                                                 int B, int seg) {
    __shared__ int s_scan[PLAN_THREADS];
    const int tid = threadIdx.x;
    int base = 0;
    for (int b0 = 0; b0 < B; b0 += PLAN_THREADS) {
        const int b = b0 + tid;
        int n = 0;
        if (b < B) {
            n = (len[b] + seg - 1) / seg;
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
}

// Row table of the packed layout, one workgroup per sequence: packed row k of the sequence reads
// token pos[min(k, len-1)] (the tail of the last segment repeats the last valid token), and every
// segment records its sequence and whether it begins it, ends it, and whether the sequence is empty.
constexpr int FWD_ROWS_THREADS = 256;

__global__ __launch_bounds__(FWD_ROWS_THREADS) void fwd_rows_kernel(const int* __restrict__ len,
                                                                     const int* __restrict__ pos,
                                                                     const int* __restrict__ blk0,
                                                                     int2* __restrict__ rows,
                                                                     int* __restrict__ blk_meta, int S, int seg) {
    const int b = blockIdx.x;
    const int n = len[b];
    const int g0 = blk0[b];
    const int nblk = blk0[b + 1] - g0;
    const int* prow = pos + (size_t)b * S;
    for (int k = threadIdx.x; k < nblk * seg; k += FWD_ROWS_THREADS) {
        const int s = n > 0 ? prow[k < n ? k : n - 1] : 0;
        rows[(size_t)g0 * seg + k] = make_int2(b * S + s, s);
    }
    for (int k = threadIdx.x; k < nblk; k += FWD_ROWS_THREADS)
        blk_meta[g0 + k] = b | (k == nblk - 1 ? FWD_META_LAST : 0) | (n == 0 ? FWD_META_EMPTY : 0) |
                           (k == 0 ? FWD_META_FIRST : 0);
}

// The three passes above in one launch of one workgroup, for batches of few sequences and tokens (the
// host takes this path up to PACK_MAX_TOKENS mask entries and PACK_MAX_B sequences), where three
// dependent launches cost more than the work in them (B=32 S=256: 15.6 -> 11.6 us, B=16 S=256: 13.5 ->
// 9.8 us; with hundreds of sequences the waves' one-sequence-at-a-time loop loses: B=256 S=32 13.5 ->
// 21.8 us, B=64 S=512 24 -> 37 us).  Wave w serves sequences w, w + 16, ...: it compacts the
// mask row (ballot + popcount), and after the workgroup-wide prefix sum of the block counts writes the
// row table and block records of the same sequences (its own earlier stores, program order).
constexpr int PACK_THREADS = 1024;
constexpr int PACK_MAX_B = 64;
constexpr int PACK_MAX_TOKENS = 16384;

__global__ __launch_bounds__(PACK_THREADS) void fwd_pack_kernel(const uint8_t* __restrict__ mask, int* __restrict__ len,
                                                                 int* __restrict__ pos, int* __restrict__ blk0,
                                                                 int2* __restrict__ rows, int* __restrict__ blk_meta,
                                                                 int B, int S, int seg) {
    __shared__ int s_len[PACK_MAX_B];
    __shared__ int s_blk0[PACK_MAX_B + 1];
    __shared__ int s_part[PACK_THREADS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NW = PACK_THREADS / 64;
    // 1. compaction
    for (int b = wave; b < B; b += NW) {
        const uint8_t* mrow = mask + (size_t)b * S;
        int* prow = pos + (size_t)b * S;
        int base = 0;
        for (int s0 = 0; s0 < S; s0 += 64) {
            const int s = s0 + lane;
            const bool flag = s < S && mrow[s] != 0;
            const unsigned long long bal = __ballot(flag);
            if (flag) prow[base + __popcll(bal & ((1ull << lane) - 1ull))] = s;
            base += __popcll(bal);
        }
        if (lane == 0) { s_len[b] = base; len[b] = base; }
    }
    __syncthreads();
    // 2. exclusive prefix sum of the block counts: consecutive sequences per thread, then the partials
    const int per = (B + PACK_THREADS - 1) / PACK_THREADS;
    const int lo = min(B, tid * per), hi = min(B, lo + per);
    int sum = 0;
    for (int b = lo; b < hi; ++b) sum += max(1, (s_len[b] + seg - 1) / seg);
    s_part[tid] = sum;
    __syncthreads();
    for (int off = 1; off < PACK_THREADS; off <<= 1) {
        const int add = tid >= off ? s_part[tid - off] : 0;
        __syncthreads();
        s_part[tid] += add;
        __syncthreads();
    }
    int run = s_part[tid] - sum;
    for (int b = lo; b < hi; ++b) {
        s_blk0[b] = run;
        blk0[b] = run;
        run += max(1, (s_len[b] + seg - 1) / seg);
    }
    if (tid == PACK_THREADS - 1) { s_blk0[B] = s_part[tid]; blk0[B] = s_part[tid]; }
    __syncthreads();
    // 3. row table and block records
    for (int b = wave; b < B; b += NW) {
        const int n = s_len[b];
        const int g0 = s_blk0[b];
        const int nblk = s_blk0[b + 1] - g0;
        const int* prow = pos + (size_t)b * S;
        for (int k = lane; k < nblk * seg; k += 64) {
            const int s = n > 0 ? prow[k < n ? k : n - 1] : 0;
            rows[(size_t)g0 * seg + k] = make_int2(b * S + s, s);
        }
        for (int k = lane; k < nblk; k += 64)
            blk_meta[g0 + k] = b | (k == nblk - 1 ? FWD_META_LAST : 0) | (n == 0 ? FWD_META_EMPTY : 0) |
                               (k == 0 ? FWD_META_FIRST : 0);
    }
}

// Joins the pieces of the sequences that a chunk boundary of the fused kernel cuts (see fwd_bf16.hpp).
// The workgroups of chunk c leave, for a sequence that runs on into chunk c+1, the raw (max, position)
// of its blocks inside chunk c in Y and I; the workgroups of every later chunk k the sequence reaches
// leave theirs in slot k of part_m / part_s.  One thread per (chunk, vocabulary entry) takes the
// pieces in order (later pieces hold higher positions, so an equal maximum keeps the earlier
// position), applies bias, ReLU and log1p (F4) and overwrites Y and I with the final values.
// grid (ceil(V/256), up to FWD_MERGE_ROWS): a workgroup walks the chunks y, y + gridDim.y, ... (most end
// with a whole sequence and cost one table read).  tpc = most tiles per chunk, spt = segments per tile
// (ChunkSplit); blk0 and blk_meta are the segment tables.
constexpr int FWD_MERGE_THREADS = 256;
constexpr int FWD_MERGE_ROWS = 4;

template <bool ARG>
__global__ __launch_bounds__(FWD_MERGE_THREADS) void fwd_merge_kernel(const int* __restrict__ blk0,
                                                                       const int* __restrict__ blk_meta,
                                                                       const float* __restrict__ part_m,
                                                                       const int* __restrict__ part_s,
                                                                       const float* __restrict__ bias,
                                                                       float* __restrict__ Y, int* __restrict__ I,
                                                                       int B, int V, int tpc, int spt) {
    const int n_blocks = blk0[B];
    const ChunkSplit cs = chunk_split(n_blocks, tpc, spt);
    const int v = blockIdx.x * FWD_MERGE_THREADS + threadIdx.x;
    for (int c = blockIdx.y; c < cs.nc; c += gridDim.y) {
        const int c_lo = cs.first_tile(c) * spt;
        const int c_hi = min(n_blocks, cs.first_tile(c + 1) * spt);        // first segment behind the chunk
        const int meta = blk_meta[c_hi - 1];
        if (meta & FWD_META_LAST) continue;                                // the chunk ends with a sequence
        const int b = meta & FWD_META_SEQ;
        if (blk0[b] < c_lo) continue;                                      // began in an earlier chunk: joined from there
        const int k_end = cs.chunk_of_tile((blk0[b + 1] - 1) / spt);       // chunk that holds the sequence's last segment
        if (v >= V) continue;
        const size_t o = (size_t)b * V + v;
        float m = Y[o];
        int s = ARG ? I[o] : 0;
        for (int k = c + 1; k <= k_end; ++k) {
            const float pm = part_m[(size_t)k * V + v];
            if (pm > m) {
                m = pm;
                if (ARG) s = part_s[(size_t)k * V + v];
            }
        }
        Y[o] = log1pf(fmaxf(m + bias[v], 0.f));
        if (ARG) I[o] = s;
    }
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
