// Backward of the sparse-lexical head (paper Sec. 3 "Backward Pass", Alg. 3).
//
// Per (b,v) the gradient is g = dY * exp(-Y) where Y > 0 (derivative of log(1+ReLU(x)) written
// with the saved output), routed to one hidden state H[b, I[b,v]] and one embedding row W[v]:
//     dW[v,:]   = sum_b g[b,v] * H[b, I[b,v], :]
//     dH[b,s,:] = sum_{v : I[b,v] = s} g[b,v] * W[v,:]
//     db[v]     = sum_b g[b,v]
// The paper accumulates with atomics across blocks.  Here every output row has one owner that
// gathers its contributions in a fixed order (no global atomics, reproducible sums):
//   dW/db : the owner of row v walks b = 0..B-1 and gathers rows of H.
//   dH    : the (b,v) pairs with g != 0 are first bucketed by position s with a stable counting
//           sort (count -> scan -> place); the owner of row (b,s) then walks its bucket in
//           ascending v and gathers rows of W.  Empty buckets write zeros, so dH needs no memset.
// Rows are read as 16-byte chunks: one thread owns chunk c (+128, +256, ...) of the row and keeps
// fp32 accumulators for it.  All of this is bandwidth-bound row gathering; the arithmetic is plain
// fp32 FMA.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lds_dma.hpp"

namespace lsr {

constexpr int ROW_THREADS = 128;     // threads that share one row (16 bytes each per pass)

__device__ __forceinline__ float gate_grad(float dy, float y) { return y > 0.f ? dy * expf(-y) : 0.f; }
__device__ __forceinline__ int clamp_pos(int s, int S) { return s < 0 ? 0 : (s >= S ? S - 1 : s); }

template <typename T> struct RowChunk;
template <> struct RowChunk<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void fma(const uint4& x, float g, float* acc) {
        acc[0] = fmaf(g, __uint_as_float(x.x), acc[0]);
        acc[1] = fmaf(g, __uint_as_float(x.y), acc[1]);
        acc[2] = fmaf(g, __uint_as_float(x.z), acc[2]);
        acc[3] = fmaf(g, __uint_as_float(x.w), acc[3]);
    }
};
template <> struct RowChunk<uint16_t> {       // bfloat16 storage
    static constexpr int N = 8;
    static __device__ __forceinline__ void fma(const uint4& x, float g, float* acc) {
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] = fmaf(g, __uint_as_float(w[i] << 16), acc[2 * i]);
            acc[2 * i + 1] = fmaf(g, __uint_as_float(w[i] & 0xffff0000u), acc[2 * i + 1]);
        }
    }
};

// Gradient outputs are float32 or bfloat16 (OT = float or uint16_t): sums are always formed in float32
// and rounded once, to nearest even, when the final value is stored.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;        // finite inputs
}
template <typename OT> struct OutVec;
template <> struct OutVec<float> {
    // four consecutive elements
    static __device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
    static __device__ __forceinline__ void store4(float* p, float4 x) { *reinterpret_cast<float4*>(p) = x; }
};
template <> struct OutVec<uint16_t> {
    static __device__ __forceinline__ float4 load4(const uint16_t* p) {
        const uint2 u = *reinterpret_cast<const uint2*>(p);
        return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                           __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u));
    }
    static __device__ __forceinline__ void store4(uint16_t* p, float4 x) {
        *reinterpret_cast<uint2*>(p) = make_uint2(f32_to_bf16_bits(x.x) | (f32_to_bf16_bits(x.y) << 16),
                                                  f32_to_bf16_bits(x.z) | (f32_to_bf16_bits(x.w) << 16));
    }
};
__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

// ---------------------------------------------------------------------------------------------
// Stable bucketing of the non-zero (b,v) pairs by position s.
// The vocabulary is cut into n_seg segments of seg_len entries; (b, segment) is the unit of work.
// ---------------------------------------------------------------------------------------------

// cnt[b][seg][s] = number of v in the segment with g != 0 and I[b,v] = s.
__global__ __launch_bounds__(256) void bwd_count_kernel(const float* __restrict__ dY,
                                                        const float* __restrict__ Y,
                                                        const int* __restrict__ I,
                                                        int* __restrict__ cnt,
                                                        int S, int V, int n_seg, int seg_len) {
    extern __shared__ int s_hist[];
    const int seg = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    for (int s = tid; s < S; s += 256) s_hist[s] = 0;
    __syncthreads();
    const int vbeg = seg * seg_len;
    const int vend = min(V, vbeg + seg_len);
    const size_t row = (size_t)b * V;
    for (int v = vbeg + tid; v < vend; v += 256) {
        const float g = gate_grad(dY[row + v], Y[row + v]);
        if (g != 0.f) atomicAdd(&s_hist[clamp_pos(I[row + v], S)], 1);
    }
    __syncthreads();
    int* out = cnt + ((size_t)b * n_seg + seg) * S;
    for (int s = tid; s < S; s += 256) out[s] = s_hist[s];
}

// Per b: cnt[b][seg][s] becomes the number of earlier-segment entries of bucket s, and
// bstart[b][0..S] the exclusive prefix of the bucket sizes (bstart[b][S] = non-zero pairs of row b).
__global__ __launch_bounds__(256) void bwd_scan_kernel(int* __restrict__ cnt, int* __restrict__ bstart,
                                                       int S, int n_seg) {
    extern __shared__ int s_tot[];          // [S] bucket sizes, then [256] partials
    int* s_part = s_tot + S;
    const int b = blockIdx.x, tid = threadIdx.x;
    for (int s = tid; s < S; s += 256) {
        int run = 0;
        // eight segments at a time: the loads of a batch are all issued before the first store,
        // which the compiler cannot do by itself (loads and stores go to the same array)
        for (int seg0 = 0; seg0 < n_seg; seg0 += 8) {
            int c[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                c[u] = seg0 + u < n_seg ? cnt[((size_t)b * n_seg + seg0 + u) * S + s] : 0;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (seg0 + u < n_seg) cnt[((size_t)b * n_seg + seg0 + u) * S + s] = run;
                run += c[u];
            }
        }
        s_tot[s] = run;
    }
    __syncthreads();
    const int per = (S + 255) / 256;
    const int lo = min(S, tid * per), hi = min(S, lo + per);
    int sum = 0;
    for (int s = lo; s < hi; ++s) sum += s_tot[s];
    s_part[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int t = 0; t < 256; ++t) { const int c = s_part[t]; s_part[t] = run; run += c; }
        bstart[(size_t)b * (S + 1) + S] = run;
    }
    __syncthreads();
    int run = s_part[tid];
    int* out = bstart + (size_t)b * (S + 1);
    for (int s = lo; s < hi; ++s) { out[s] = run; run += s_tot[s]; }
}

// One wave per (b, segment) walks its entries in ascending v, 64 at a time.  Lanes holding the
// same position find each other with one ballot per key bit; the rank among them keeps the order
// of v, so every bucket ends up sorted by v (stable) and the later sums have a fixed order.
__global__ __launch_bounds__(64) void bwd_place_kernel(const float* __restrict__ dY,
                                                       const float* __restrict__ Y,
                                                       const int* __restrict__ I,
                                                       const int* __restrict__ cnt,
                                                       const int* __restrict__ bstart,
                                                       uint2* __restrict__ perm,
                                                       int S, int V, int n_seg, int seg_len, int key_bits) {
    extern __shared__ int s_off[];          // [S] next free slot of each bucket
    const int seg = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const int* c0 = cnt + ((size_t)b * n_seg + seg) * S;
    const int* b0 = bstart + (size_t)b * (S + 1);
    for (int s = lane; s < S; s += 64) s_off[s] = b0[s] + c0[s];
    __syncthreads();
    const int vbeg = seg * seg_len;
    const int vend = min(V, vbeg + seg_len);
    const size_t row = (size_t)b * V;
    const unsigned long long lt = (1ull << lane) - 1ull;
    // the next 64 entries are requested before the current ones are ranked (the ranking has two
    // barriers and would otherwise expose a full memory latency per step)
    float n_dy = 0.f, n_y = 0.f;
    int n_i = 0;
    auto request = [&](int base) {
        const int v = base + lane;
        const bool ok = v < vend;
        n_dy = ok ? dY[row + v] : 0.f;
        n_y = ok ? Y[row + v] : 0.f;
        n_i = ok ? I[row + v] : 0;
    };
    request(vbeg);
    for (int base = vbeg; base < vend; base += 64) {
        const int v = base + lane;
        const float g = gate_grad(n_dy, n_y);      // 0 for lanes past the end (dy = 0, y = 0)
        const int key = clamp_pos(n_i, S);
        request(base + 64);
        const bool active = g != 0.f;
        unsigned long long same = __ballot(active);
        for (int bit = 0; bit < key_bits; ++bit) {
            const bool one = (key >> bit) & 1;
            const unsigned long long bm = __ballot(active && one);
            same &= one ? bm : ~bm;
        }
        const int rank = __popcll(same & lt);
        const int group = __popcll(same);
        int dest = 0;
        if (active) {
            dest = s_off[key] + rank;
            perm[row + dest] = make_uint2((unsigned)v, __float_as_uint(g));      // one 8-byte scattered store
        }
        // The workgroup is a single wave: its LDS instructions execute in program order for all lanes,
        // so the read of s_off above precedes this update and the update precedes the next step's
        // read.  wave_barrier only pins that order for the compiler; no hardware barrier is needed.
        __builtin_amdgcn_wave_barrier();
        if (active && rank == group - 1) s_off[key] = dest + 1;
        __builtin_amdgcn_wave_barrier();
    }
}

// Placement through LDS (S <= PLACE_MAX_S, segments of at most PLACE_MAX_SEG entries).
// The kernel above stores every (v, g) pair straight to its bucket: the 64 stores of a step go to some
// fifty buckets, and with thousands of (b, segment) waves in flight every bucket's line leaves L2
// between two stores to it (measured at C5: 0.48 GB written for 0.13 GB of pairs).  Here a workgroup
// of four waves first sorts its whole segment by bucket in LDS and then writes it out in sorted order:
// the pairs a bucket receives from this segment (about a dozen at C5) leave as one contiguous run.
//   1. per bucket, the pairs of this segment (difference of two rows of the scanned count table) and
//      their exclusive prefix = first local slot; s_delta = first global slot - first local slot;
//   2. steps of 256 pairs: ballot ranking inside each wave as above, then the four waves take their
//      slots one after the other (wave order = ascending v, so the order inside a bucket is kept);
//   3. local slot k goes to global slot k + s_delta[bucket of k].
// A staged pair is (v - vbeg) | bucket << 12 and g.   dynamic LDS: 2*S ints + seg_len pairs.
// ---------------------------------------------------------------------------------------------
constexpr int PLACE_MAX_S = 1024;
constexpr int PLACE_MAX_SEG = 4096;

__global__ __launch_bounds__(256) void bwd_place_staged_kernel(const float* __restrict__ dY,
                                                               const float* __restrict__ Y,
                                                               const int* __restrict__ I,
                                                               const int* __restrict__ cnt,
                                                               const int* __restrict__ bstart,
                                                               uint2* __restrict__ perm,
                                                               int S, int V, int n_seg, int seg_len, int key_bits) {
    extern __shared__ int s_place[];
    int* s_next = s_place;                  // [S] next free local slot of each bucket
    int* s_delta = s_place + S;             // [S] global slot - local slot
    uint2* s_stage = reinterpret_cast<uint2*>(s_place + 2 * S);     // [seg_len]
    __shared__ int s_part[256];
    const int seg = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int* c0 = cnt + ((size_t)b * n_seg + seg) * S;
    const int* b0 = bstart + (size_t)b * (S + 1);
    const bool last_seg = seg + 1 == n_seg;

    // 1. counts of this segment, exclusive prefix over the buckets
    const int per = (S + 255) / 256;
    const int lo = min(S, tid * per), hi = min(S, lo + per);
    int sum = 0;
    for (int s = lo; s < hi; ++s) {
        const int earlier = c0[s];
        const int upto = last_seg ? b0[s + 1] - b0[s] : c0[S + s];      // next segment's row, or the bucket size
        s_next[s] = upto - earlier;
        s_delta[s] = b0[s] + earlier;
        sum += upto - earlier;
    }
    s_part[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int t = 0; t < 256; ++t) { const int c = s_part[t]; s_part[t] = run; run += c; }
    }
    __syncthreads();
    int run = s_part[tid];
    for (int s = lo; s < hi; ++s) {
        const int c = s_next[s];
        s_next[s] = run;
        s_delta[s] -= run;
        run += c;
    }
    __shared__ int s_total;
    if (tid == 255) s_total = run;          // the last thread ends on the pairs of the whole segment
    __syncthreads();

    // 2. rank and stage
    const int vbeg = seg * seg_len;
    const int vend = min(V, vbeg + seg_len);
    const size_t row = (size_t)b * V;
    const unsigned long long lt = (1ull << lane) - 1ull;
    float n_dy = 0.f, n_y = 0.f;
    int n_i = 0;
    auto request = [&](int base) {
        const int v = base + tid;
        const bool ok = v < vend;
        n_dy = ok ? dY[row + v] : 0.f;
        n_y = ok ? Y[row + v] : 0.f;
        n_i = ok ? I[row + v] : 0;
    };
    request(vbeg);
    for (int base = vbeg; base < vend; base += 256) {
        const int v = base + tid;
        const float g = gate_grad(n_dy, n_y);      // 0 for threads past the end (dy = 0, y = 0)
        const int key = clamp_pos(n_i, S);
        request(base + 256);
        const bool active = g != 0.f;
        unsigned long long same = __ballot(active);
        for (int bit = 0; bit < key_bits; ++bit) {
            const bool one = (key >> bit) & 1;
            const unsigned long long bm = __ballot(active && one);
            same &= one ? bm : ~bm;
        }
        const int rank = __popcll(same & lt);
        const int group = __popcll(same);
        for (int w = 0; w < 4; ++w) {
            if (wave == w) {
                int slot = 0;
                if (active) {
                    slot = s_next[key] + rank;
                    s_stage[slot] = make_uint2((unsigned)(v - vbeg) | ((unsigned)key << 12), __float_as_uint(g));
                }
                __builtin_amdgcn_wave_barrier();     // LDS operations of one wave execute in program order
                if (active && rank == group - 1) s_next[key] = slot + 1;
            }
            __syncthreads();
        }
    }

    // 3. sorted write-out
    const int total = s_total;
    for (int k = tid; k < total; k += 256) {
        const uint2 e = s_stage[k];
        const int key = (int)(e.x >> 12);
        perm[row + k + s_delta[key]] = make_uint2((unsigned)vbeg + (e.x & 4095u), e.y);
    }
}

// ---------------------------------------------------------------------------------------------
// dH[b,s,:] = sum over the bucket of (b,s), in ascending v, of g * W[v,:].   grid (B, S): b fastest,
// so that the empty buckets behind the ends of the sequences are spread evenly over the chip
// ---------------------------------------------------------------------------------------------
// accumulate: the sums are added to what dH holds
template <typename T, int CPT, typename OT>
__global__ __launch_bounds__(ROW_THREADS) void bwd_dh_kernel(const T* __restrict__ W,
                                                             const int* __restrict__ bstart,
                                                             const uint2* __restrict__ perm,
                                                             OT* __restrict__ dH,
                                                             int S, int D, int V, int accumulate) {
    constexpr int N = RowChunk<T>::N;
    __shared__ int s_v[ROW_THREADS];
    __shared__ float s_g[ROW_THREADS];
    const int b = blockIdx.x, s = blockIdx.y, tid = threadIdx.x;
    const int n_chunks = D / N;
    const int beg = bstart[(size_t)b * (S + 1) + s];
    const int end = bstart[(size_t)b * (S + 1) + s + 1];
    const size_t prow = (size_t)b * V;
    float acc[CPT][N];
#pragma unroll
    for (int cp = 0; cp < CPT; ++cp)
#pragma unroll
        for (int i = 0; i < N; ++i) acc[cp][i] = 0.f;

    for (int base = beg; base < end; base += ROW_THREADS) {
        const int n = min(ROW_THREADS, end - base);
        const uint2 ent = tid < n ? perm[prow + base + tid] : make_uint2(0u, 0u);   // padding: row 0, weight 0
        s_v[tid] = (int)ent.x;
        s_g[tid] = __uint_as_float(ent.y);
        __syncthreads();
        for (int k = 0; k < n; k += 4) {
            uint4 x[4][CPT];
            float g[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                g[u] = s_g[k + u];
                const T* src = W + (size_t)s_v[k + u] * D;
#pragma unroll
                for (int cp = 0; cp < CPT; ++cp) {
                    const int c = tid + cp * ROW_THREADS;
                    x[u][cp] = c < n_chunks ? *reinterpret_cast<const uint4*>(src + c * N) : make_uint4(0, 0, 0, 0);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int cp = 0; cp < CPT; ++cp) RowChunk<T>::fma(x[u][cp], g[u], acc[cp]);
        }
        __syncthreads();
    }
    OT* out = dH + ((size_t)b * S + s) * D;
#pragma unroll
    for (int cp = 0; cp < CPT; ++cp) {
        const int c = tid + cp * ROW_THREADS;
        if (c < n_chunks) {
#pragma unroll
            for (int i = 0; i < N; i += 4) {
                float4 r = make_float4(acc[cp][i], acc[cp][i + 1], acc[cp][i + 2], acc[cp][i + 3]);
                if (accumulate) r = add4(OutVec<OT>::load4(out + c * N + i), r);
                OutVec<OT>::store4(out + c * N + i, r);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// dW[v,:] = sum_b g[b,v] * H[b, I[b,v], :],  db[v] = sum_b g[b,v].
// A workgroup owns VT consecutive vocabulary rows.  It first stages g and I for all B x VT pairs in
// LDS (coalesced along v), then walks the rows one by one, skipping pairs with g = 0.
// dynamic LDS: B*VT floats + B*VT ints.
// ---------------------------------------------------------------------------------------------
// accumulate: the sums are added to what dW and db hold
template <typename T, int CPT, typename OT>
__global__ __launch_bounds__(ROW_THREADS) void bwd_dw_kernel(const T* __restrict__ H,
                                                             const float* __restrict__ dY,
                                                             const float* __restrict__ Y,
                                                             const int* __restrict__ I,
                                                             OT* __restrict__ dW, float* __restrict__ db,
                                                             int B, int S, int D, int V, int VT, int accumulate) {
    constexpr int N = RowChunk<T>::N;
    extern __shared__ int s_dyn[];
    float* s_g = reinterpret_cast<float*>(s_dyn);          // [B][VT]
    int* s_i = s_dyn + (size_t)B * VT;                     // [B][VT]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int v0 = blockIdx.x * VT;
    const int n_chunks = D / N;

    for (int e = tid; e < B * VT; e += ROW_THREADS) {
        const int bb = e / VT, vv = e - bb * VT;
        const int v = v0 + vv;
        float g = 0.f;
        int idx = 0;
        if (v < V) {
            const size_t o = (size_t)bb * V + v;
            g = gate_grad(dY[o], Y[o]);
            idx = clamp_pos(I[o], S);
        }
        s_g[e] = g;
        s_i[e] = idx;
    }
    __syncthreads();

    for (int vv = 0; vv < VT; ++vv) {
        const int v = v0 + vv;
        if (v >= V) break;
        float acc[CPT][N];
#pragma unroll
        for (int cp = 0; cp < CPT; ++cp)
#pragma unroll
            for (int i = 0; i < N; ++i) acc[cp][i] = 0.f;
        float gsum = 0.f;
        for (int bb0 = 0; bb0 < B; bb0 += 64) {
            const int bl = bb0 + lane;
            const float gl = bl < B ? s_g[bl * VT + vv] : 0.f;
            gsum += gl;
            unsigned long long nz = dW ? __ballot(gl != 0.f) : 0ull;       // same in both waves
            while (nz) {
                uint4 x[4][CPT];
                float g[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    // take the next non-zero pair, or repeat a harmless one with weight 0
                    const int bit = nz ? __builtin_ctzll(nz) : 0;
                    const bool have = nz != 0;
                    nz = have ? nz & (nz - 1) : 0;
                    const int bb = bb0 + bit;
                    g[u] = have ? s_g[bb * VT + vv] : 0.f;
                    const int idx = have ? s_i[bb * VT + vv] : 0;
                    const T* src = H + ((size_t)(have ? bb : 0) * S + idx) * D;
#pragma unroll
                    for (int cp = 0; cp < CPT; ++cp) {
                        const int c = tid + cp * ROW_THREADS;
                        x[u][cp] = c < n_chunks ? *reinterpret_cast<const uint4*>(src + c * N) : make_uint4(0, 0, 0, 0);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int cp = 0; cp < CPT; ++cp) RowChunk<T>::fma(x[u][cp], g[u], acc[cp]);
            }
        }
        OT* out = dW + (size_t)v * D;
        if (dW) {
#pragma unroll
            for (int cp = 0; cp < CPT; ++cp) {
                const int c = tid + cp * ROW_THREADS;
                if (c < n_chunks) {
#pragma unroll
                    for (int i = 0; i < N; i += 4) {
                        float4 r = make_float4(acc[cp][i], acc[cp][i + 1], acc[cp][i + 2], acc[cp][i + 3]);
                        if (accumulate) r = add4(OutVec<OT>::load4(out + c * N + i), r);
                        OutVec<OT>::store4(out + c * N + i, r);
                    }
                }
            }
        }
        if (db && tid < 64) {                                    // fixed-order butterfly over b
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) gsum += __shfl_xor(gsum, o);
            if (tid == 0) db[v] = accumulate ? db[v] + gsum : gsum;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// dW/db, column-sliced variant (D a multiple of 64).
// The gathers of the kernel above hit rows of H scattered over all of H (tens of MB), so they are
// served by the memory-side cache at a fraction of the L2 rate.  Here the work is cut into slices of
// 64 hidden-state columns and the grid is ordered slice-major: the workgroups resident at any time
// all gather from the same [tokens x 64] slice of H (a few MB at most), which stays in every XCD's
// L2 (the host sizes a group of NDC consecutive slices to at most 9 MiB of H and a workgroup walks the
// slices of its group, so that the (g, I) staging is not repeated more often than needed).
// A row piece is 64 elements = LPR lanes x 16 bytes; a wave therefore serves 64/LPR vocabulary
// rows at once, walks the sequences that have a gradient for them with eight gathers in flight per
// lane, and writes one 64-column piece of each dW row.  Summation order over b is fixed.
// COMPACT (used for the narrow tiles of large batches, where sequences are short and gradients often
// sparse): after staging, each column of the (g, I) tile is compacted in place to its non-zero
// entries, in ascending b (one wave per column, ballot ranking) and closed by a zero, so that sparse
// gradients cost what they hold; element (b, vv) of the tile then sits at word
// b*VT + (vv ^ (b % VT)), so that staging (lanes along vv), compaction (lanes along b) and the gather
// (eight columns per wave) all spread over the LDS banks.  Without it the tile is plain row-major
// and every b is visited (measured 7 % faster on dense gradients).   VT a power of two.
// When the H slice of the whole batch (B*S rows x 128 bytes) is larger than L2, the host launches
// the kernel once per chunk of consecutive sequences (b_first, B = sequences of the chunk); later
// launches add to dW and db, which keeps the order of the sums fixed.
// Where the partial sums come from and where the result goes is set per launch: `prev` (float32, may
// be null) is added to the sums of this launch, `add_dst` adds what dst already holds (accumulation into
// the caller's gradient), and dst is float32 or bfloat16 (OT).  A float32 result spread over several
// launches passes prev = dst; a bfloat16 result keeps its partial sums in a float32 staging array (dst of
// all launches but the last, prev of all but the first), so that it is rounded once.
// dynamic LDS: B*VT floats + B*VT ints.   grid = ceil(V/VT) * ceil((D/64)/NDC).
// ---------------------------------------------------------------------------------------------
constexpr int DWS_COLS = 64;
constexpr int DH_NLD = 4;                 // gathers in flight per lane of the sliced dH gather
constexpr int PERM_SLACK = 256;           // entries the workspace keeps behind the sorted lists (see bwd_dh_sliced_kernel)

// Slices owned by XCDs.  Workgroup ids go round-robin over the chip's 8 XCDs (id & 7), each with an L2
// of its own.  With n_dc = 8 q + r column slices, XCD x owns slices x, x + 8, ..., x + 8 (q - 1): every
// gather from one of them goes through the same L2, which then holds one copy of the slice's window
// instead of each of the eight L2s fetching its own, and sees all of the window's reuse.  The r slices
// left over are shared: each is dealt out over all XCDs by item (item i goes to XCD i & 7).
// An item is what the kernel iterates within a slice (a group of buckets).  A workgroup of the owned part
// walks up to `walk` of its XCD's slices for one item; of the shared part, one slice.
// Index j = id >> 3 of the workgroup on its XCD: first the owned part, ceil(q / walk) * n_items
// workgroups, item fastest; then the shared part, r * ceil(n_items / 8).  The grid is 8 times the sum;
// ids that fall behind the end of the shared part are not valid.
struct XcdSliceUnit { bool valid, first_of_item; int item, dc_first, dc_step, dc_count; };
__host__ __device__ inline long long xcd_slice_grid(int n_dc, int n_items, int walk) {
    const int q = n_dc >> 3, r = n_dc & 7;
    return 8ll * ((long long)((q + walk - 1) / walk) * n_items + (long long)r * ((n_items + 7) >> 3));
}
__host__ __device__ inline XcdSliceUnit xcd_slice_unit(unsigned id, int n_dc, int n_items, int walk) {
    XcdSliceUnit u;
    const int x = id & 7, j = (int)(id >> 3);
    const int q = n_dc >> 3, r = n_dc & 7;
    const int owned = ((q + walk - 1) / walk) * n_items;
    if (j < owned) {
        const int wg = j / n_items;                         // group of `walk` owned slices
        u.item = j - wg * n_items;
        u.dc_first = wg * walk * 8 + x;
        u.dc_step = 8;
        u.dc_count = (q < (wg + 1) * walk ? q : (wg + 1) * walk) - wg * walk;
        u.first_of_item = x == 0 && wg == 0;
        u.valid = true;
    } else {
        const int per = (n_items + 7) >> 3;
        const int jj = j - owned;
        const int l = jj / per;
        u.item = (jj - l * per) * 8 + x;
        u.dc_first = 8 * q + l;
        u.dc_step = 1;
        u.dc_count = 1;
        u.first_of_item = q == 0 && l == 0;
        u.valid = l < r && u.item < n_items;
    }
    return u;
}

template <typename T, bool COMPACT, typename OT>
__global__ __launch_bounds__(256) void bwd_dw_sliced_kernel(const T* __restrict__ H,
                                                            const float* __restrict__ dY,
                                                            const float* __restrict__ Y,
                                                            const int* __restrict__ I,
                                                            const float* prev, OT* dW, int add_dst,
                                                            float* __restrict__ db, int add_db,
                                                            int b_first, int B, int S, int D, int V, int VT,
                                                            int n_vtiles, int NDC) {
    // b_first, B: the sequences of this launch; prev / add_dst: see above; add_db: db already holds the
    // sums over the sequences before b_first (or the caller's accumulated gradient) and is added to
    constexpr int N = RowChunk<T>::N;          // elements per 16-byte chunk
    constexpr int LPR = DWS_COLS / N;          // lanes per row piece
    constexpr int VPG = 64 / LPR;              // vocabulary rows a wave serves at once
    extern __shared__ int s_dyn[];
    float* s_g = reinterpret_cast<float*>(s_dyn);          // [B][VT]
    int* s_i = s_dyn + (size_t)B * VT;                     // [B][VT]  token row b*S + I[b,v]
    auto at = [VT](int b, int vv) { return COMPACT ? b * VT + (vv ^ (b & (VT - 1))) : b * VT + vv; };
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n_waves = blockDim.x >> 6;
    const int dg = blockIdx.x / n_vtiles;                  // slice-group-major order
    const int v0 = (blockIdx.x - dg * n_vtiles) * VT;
    const int dc_begin = dg * NDC;
    const int dc_end = min(D / DWS_COLS, dc_begin + NDC);

    // staging, four independent (dY, Y, I) triples in flight per thread
    for (int e0 = tid; e0 < B * VT; e0 += 4 * blockDim.x) {
        float dy[4], y[4];
        int ix[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * blockDim.x;
            const int bb = e / VT, vv = e - bb * VT;
            const bool ok = e < B * VT && v0 + vv < V;
            const size_t o = ok ? (size_t)(b_first + bb) * V + v0 + vv : 0;
            dy[u] = ok ? dY[o] : 0.f;
            y[u] = ok ? Y[o] : 0.f;
            ix[u] = ok ? I[o] : 0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * blockDim.x;
            if (e < B * VT) {
                const int bb = e / VT, vv = e - bb * VT;
                s_g[at(bb, vv)] = gate_grad(dy[u], y[u]);
                s_i[at(bb, vv)] = (b_first + bb) * S + clamp_pos(ix[u], S);
            }
        }
    }
    __syncthreads();

    // compaction: column vv keeps its non-zero entries, in ascending b, at rows 0..n-1, and a zero at
    // row n if n < B.  A chunk of 64 rows is read before any of it is written and lands at or below
    // where it was read, so this works in place.
    const unsigned long long lt = (1ull << lane) - 1ull;
    for (int vv = wave; COMPACT && vv < VT; vv += n_waves) {
        int n = 0;
        for (int b0 = 0; b0 < B; b0 += 64) {
            const int b = b0 + lane;
            const float g = b < B ? s_g[at(b, vv)] : 0.f;
            const int r = b < B ? s_i[at(b, vv)] : 0;
            const unsigned long long nz = __ballot(g != 0.f);
            if (g != 0.f) {
                const int k = n + __popcll(nz & lt);
                s_g[at(k, vv)] = g;
                s_i[at(k, vv)] = r;
            }
            n += __popcll(nz);
        }
        if (lane == 0 && n < B) s_g[at(n, vv)] = 0.f;
    }
    if (COMPACT) __syncthreads();

    if (db && dg == 0 && tid < VT && v0 + tid < V) {           // fixed-order sum over b
        float sum = add_db ? db[v0 + tid] : 0.f;
        for (int k = 0; k < B; ++k) {
            const float g = s_g[at(k, tid)];
            if (COMPACT && g == 0.f) break;
            sum += g;
        }
        db[v0 + tid] = sum;
    }
    if (!dW) return;

    for (int dc = dc_begin; dc < dc_end; ++dc) {
        const int col0 = dc * DWS_COLS + (lane % LPR) * N;
        for (int grp = wave; grp * VPG < VT; grp += n_waves) {
            const int vv = grp * VPG + lane / LPR;
            const int v = v0 + vv;
            float acc[N];
#pragma unroll
            for (int i = 0; i < N; ++i) acc[i] = 0.f;
            for (int k0 = 0; k0 < B; k0 += 8) {
                float g[8];
                uint4 x[8];
                bool open = true;                                // false behind the closing zero
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int k = k0 + u;
                    g[u] = (open && k < B) ? s_g[at(k, vv)] : 0.f;
                    if (COMPACT) open = g[u] != 0.f;
                    x[u] = make_uint4(0, 0, 0, 0);
                    if (g[u] != 0.f) x[u] = *reinterpret_cast<const uint4*>(H + (size_t)s_i[at(k, vv)] * D + col0);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) RowChunk<T>::fma(x[u], g[u], acc);
                if (COMPACT && !open) break;
            }
            if (v < V) {
                const size_t o = (size_t)v * D + col0;
#pragma unroll
                for (int i = 0; i < N; i += 4) {
                    float4 r = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
                    if (prev) r = add4(*reinterpret_cast<const float4*>(prev + o + i), r);
                    if (add_dst) r = add4(OutVec<OT>::load4(dW + o + i), r);
                    OutVec<OT>::store4(dW + o + i, r);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// dH, column-sliced variant (D a multiple of 64).
// One sub-group of a wave owns one bucket and one 64-column slice; the grid is ordered slice-major.
// A 64-column piece of a row is LPR lanes x 16 bytes, so a sub-group of G = 64/BPW lanes gathers
// G/LPR bucket entries per load, keeps four loads in flight per lane, and folds the per-entry
// partial sums with a fixed butterfly at the end (reproducible order).
//
// What decides the speed is whether the rows of W being gathered come from L2.  All buckets walk the
// vocabulary in ascending v but not in step, so the working set of one slice pass is the whole slice
// of W: |V| x 128 bytes.  Up to about 4 MB that lives in L2; beyond, the vocabulary is cut into n_vc
// chunks and the pass is launched once per chunk (`vc` = chunk index), each launch gathering only
// the entries of its chunk.  `bounds` then holds, per bucket, the n_vc+1 positions in the sorted
// entry list where the chunks begin (bwd_chunk_bounds_kernel); with n_vc = 1 it is the bucket start
// table itself.  Chunk 0 writes dH (zeros for empty buckets), later chunks add to it: one owner per
// element and launch, launches in stream order, so the sum keeps a fixed order.
// As in the dW gather, `prev` (float32, may be null) is added to the sums of this launch, `add_dst` adds
// what dst already holds, dst is float32 or bfloat16; `write_all` makes every bucket write (the launch
// that produces the final value of a fresh result), otherwise only buckets with entries in this chunk do.
// grid = B * ceil(S / (4*BPW)) * (D/64), 256 threads.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bwd_chunk_bounds_kernel(const int* __restrict__ bstart,
                                                               const uint2* __restrict__ perm,
                                                               int* __restrict__ bounds,
                                                               int n_buckets, int S, int V, int n_vc, int vc_len) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)n_buckets * (n_vc + 1)) return;
    const int bucket = (int)(idx / (n_vc + 1));
    const int c = (int)(idx - (long long)bucket * (n_vc + 1));
    const int b = bucket / S, s = bucket - b * S;
    int lo = bstart[(size_t)b * (S + 1) + s];
    int hi = bstart[(size_t)b * (S + 1) + s + 1];
    if (c == n_vc) lo = hi;
    const unsigned target = (unsigned)c * (unsigned)vc_len;     // first v of chunk c
    const uint2* list = perm + (size_t)b * V;
    while (lo < hi) {                                           // first entry with v >= target
        const int mid = lo + ((hi - lo) >> 1);
        if (list[mid].x < target) lo = mid + 1; else hi = mid;
    }
    bounds[idx] = lo;
}

template <typename T, int BPW, typename OT, bool OFF32>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(8, 8))) void bwd_dh_sliced_kernel(const T* __restrict__ W,
                                                            const int* __restrict__ bounds,
                                                            const uint2* __restrict__ perm,
                                                            const float* prev_sum, OT* dH, int add_dst, int write_all,
                                                            int B, int S, int D, int V, int n_groups,
                                                            int n_vc, int vc, int xcd_own) {
    constexpr int N = RowChunk<T>::N;
    constexpr int LPR = DWS_COLS / N;          // lanes per row piece
    constexpr int G = 64 / BPW;                // lanes per bucket
    constexpr int EPG = G / LPR;               // entries of one bucket gathered per load
    static_assert(EPG >= 1, "a bucket needs at least one row piece worth of lanes");
    constexpr int NLD = DH_NLD;                // gathers in flight per lane (8: more registers, fewer
                                               // waves; C5 2.83 -> 3.71 ms)
    static_assert(2 * G <= PERM_SLACK, "entries read behind the end of a list stay inside the slack");
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    int dc, g;
    if (xcd_own) {                                                 // slices owned by XCDs (see xcd_slice_unit)
        const XcdSliceUnit u = xcd_slice_unit(blockIdx.x, D / DWS_COLS, n_groups, 1);
        if (!u.valid) return;
        dc = u.dc_first;
        g = u.item;
    } else {
        dc = blockIdx.x / n_groups;                                // slice-major order
        g = blockIdx.x - dc * n_groups;
    }
    // Within a slice, consecutive workgroups take the same positions of consecutive sequences
    // (b fastest).  Workgroups are dealt to the chip's shader engines in a fixed rotation; with s
    // fastest, the empty buckets behind the end of each sequence recur with a period that can leave
    // some engines with twice the work of others.
    const int b = g % B;
    const int s = ((g / B) * 4 + wave) * BPW + lane / G;
    const bool live = s < S;
    const int bq = live ? b * S + s : 0;
    const size_t bi = n_vc == 1 ? (size_t)b * (S + 1) + s : (size_t)bq * (n_vc + 1) + vc;
    const int beg = live ? bounds[bi] : 0;
    const int end = live ? bounds[bi + 1] : 0;
    if (!write_all && !__any(beg < end)) return;      // nothing of this chunk in any bucket of the wave
    const int col0 = dc * DWS_COLS + (lane % LPR) * N;
    const int sub = (lane % G) / LPR;
    const bool writer = live && sub == 0 && (write_all || beg < end);
    const size_t o = (size_t)bq * D + col0;
    float acc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.f;
    float4 prev[N / 4];                        // the sum of the earlier chunks, requested early
#pragma unroll
    for (int i = 0; i < N / 4; ++i) prev[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (writer) {
        if (prev_sum) {
#pragma unroll
            for (int i = 0; i < N / 4; ++i) prev[i] = *reinterpret_cast<const float4*>(prev_sum + o + 4 * i);
        }
        if (add_dst) {
#pragma unroll
            for (int i = 0; i < N / 4; ++i) prev[i] = add4(prev[i], OutVec<OT>::load4(dH + o + 4 * i));
        }
    }
    // What limits this loop is the number of vector-memory instructions a CU can issue (counters: one every
    // 20 cycles per CU with an entry load per gather, each holding the address path for about 16), so the
    // (v, g) entries are not fetched per gather slot.  The G lanes of a bucket load G consecutive entries with
    // one coalesced instruction, a block that feeds RPB rounds of NLD gathers per lane; a lane takes the
    // entry of its slot from the lane that loaded it (ds_bpermute, which goes through the LDS crossbar, not
    // the memory path).  The next block is in flight while the current one is used.  Rows are addressed as
    // wave-uniform base + 32-bit byte offset where W allows it.  A slot behind the end of its list
    // contributes through a zero gradient and gathers the row of the block's first entry instead (a row
    // the bucket uses anyway, so nothing that could be non-finite is multiplied by that zero); the entry
    // it read belongs to a later bucket, to the next sequence, or to the PERM_SLACK entries the workspace
    // keeps behind the last list, and is not looked at.
    constexpr int RPB = G / (NLD * EPG);       // rounds per block of entries
    static_assert(RPB * NLD * EPG == G && RPB >= 1, "a block is a whole number of rounds");
    const char* const Wb = reinterpret_cast<const char*>(W);
    const uint2* const pl = perm + (size_t)b * V;                   // b: the same for the whole workgroup
    const uint32_t row_bytes = (uint32_t)D * (uint32_t)sizeof(T);
    const uint32_t col_bytes = (uint32_t)col0 * (uint32_t)sizeof(T);
    const int li = lane % G;                   // lane within its bucket
    const int src0 = (lane - li + sub) * 4;    // bpermute address of the lane holding entry `sub` of the block
    const uint2* pe = pl + beg + li;           // this lane's entry of the current block
    uint2 cur = *pe;
    for (int left = end - beg; left > 0; left -= G) {               // entries from the block's start to the end of the list
        pe += G;
        const uint2 nxt = *pe;
        __builtin_amdgcn_sched_barrier(0);                          // the next block is requested first
        const int v_first = __builtin_amdgcn_ds_bpermute((lane - li) * 4, (int)cur.x);      // the block's first entry: inside the list
        const int rem = left - sub;                                 // slot at block offset c + sub is inside when c < rem
#pragma unroll
        for (int p = 0; p < RPB; ++p) {
            if (p * NLD * EPG < left) {                             // the round has entries; the lanes of a bucket agree
                // three phases, kept apart: the entries of all NLD slots, then all NLD gathers, then the FMAs
                // (left to itself the compiler gathers two rows at a time)
                uint32_t off[NLD];
                float gq[NLD];
                uint4 x[NLD];
#pragma unroll
                for (int u = 0; u < NLD; ++u) {
                    const int c = p * NLD * EPG + u * EPG;          // block offset of the slot of sub-group 0
                    const int from = src0 + c * 4;
                    const int vx = __builtin_amdgcn_ds_bpermute(from, (int)cur.x);
                    const int gy = __builtin_amdgcn_ds_bpermute(from, (int)cur.y);
                    const bool inside = c < rem;
                    const uint32_t v = (uint32_t)(inside ? vx : v_first);
                    gq[u] = inside ? __int_as_float(gy) : 0.f;
                    off[u] = OFF32 ? __umul24(v, row_bytes) + col_bytes : v;
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < NLD; ++u) {
                    if constexpr (OFF32) x[u] = *reinterpret_cast<const uint4*>(Wb + off[u]);
                    else x[u] = *reinterpret_cast<const uint4*>(Wb + ((size_t)off[u] * row_bytes + col_bytes));
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < NLD; ++u) RowChunk<T>::fma(x[u], gq[u], acc);
            }
        }
        cur = nxt;
    }
#pragma unroll
    for (int off = LPR; off < G; off <<= 1)
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] += __shfl_xor(acc[i], off);
    if (writer) {
#pragma unroll
        for (int i = 0; i < N / 4; ++i)
            OutVec<OT>::store4(dH + o + 4 * i, make_float4(prev[i].x + acc[4 * i], prev[i].y + acc[4 * i + 1],
                                                           prev[i].z + acc[4 * i + 2], prev[i].w + acc[4 * i + 3]));
    }
}

// ---------------------------------------------------------------------------------------------
// dW/db, LDS-tile variant (bfloat16 inputs, D a multiple of 64, DWT_MIN_S <= S <= DWT_MAX_S).
// A workgroup of 1024 threads owns 1024 consecutive vocabulary rows and one 64-column slice and walks
// the sequences b = 0 .. B-1 in order.  For each sequence the slice of all S hidden states (S x 128
// bytes, at most 64 KiB) is copied into LDS and every gather of the sequence is an LDS read.  Eight
// lanes share a row piece (16 bytes each) and a thread keeps eight rows (64 float accumulators), so a
// sequence costs one tile copy for 1024 gathers: the traffic out of L2 is the tile (S x 128 bytes)
// instead of the gathers (1024 x 128 bytes), the reads are coalesced, and what is left is the arithmetic
// of the gather itself, one unpack and one FMA per element, with the LDS reads running ahead of it.
// The next sequence's tile travels global -> LDS directly (LDS-DMA, no staging registers) into the other
// buffer while the current one is multiplied; its (dY, Y, I) travel through registers and are turned into
// (g, tile row offset) pairs at the end of the round.  One barrier per sequence, behind a full vmcnt wait.
// Pairs without gradient point at a row of zeros behind the tile (hidden states of padded positions are
// never multiplied, whatever they hold), and a wave skips a pair of rows when none of its sixteen (row,
// row group) entries has a gradient.  The order of the sums over b is the same as in the kernels above.
// Not for sparse gradients (the cost does not fall with the number of non-zero pairs, as it does in the
// compacting kernel above) or for few workgroups: the host takes it for shapes with at least one
// workgroup per CU.
// grid = ceil(V / 1024) * (D / 64), slice-major.  PASSES = ceil(S / 128) copy passes per tile.
// ---------------------------------------------------------------------------------------------
constexpr int DWT_ROWS = 1024;
constexpr int DWT_MAX_S = 512;
constexpr int DWT_MIN_S = 128;

template <typename OT, int PASSES>
__global__ __launch_bounds__(DWT_ROWS) void bwd_dw_tile_kernel(const uint16_t* __restrict__ H,
                                                               const float* __restrict__ dY,
                                                               const float* __restrict__ Y,
                                                               const int* __restrict__ I,
                                                               OT* dW, int add_dst, float* db, int add_db,
                                                               int B, int S, int D, int V, int n_vtiles) {
    constexpr int ROW_B = DWS_COLS * 2;                    // bytes per tile row
    constexpr int RPT = 8;                                 // vocabulary rows per thread
    constexpr int RGS = DWT_ROWS / 8;                      // row groups (eight lanes each) = tile rows per copy pass
    static_assert(PASSES >= 1 && PASSES * RGS <= DWT_MAX_S, "tile rows");      // S <= PASSES * RGS
    // two tiles, each followed by a row of zeros
    __shared__ __attribute__((aligned(1024))) uint8_t s_tile[2][(DWT_MAX_S + 1) * ROW_B];
    __shared__ float2 s_go[2][DWT_ROWS];                   // per pair: g, and (as int bits) the byte offset of its tile row
    const int tid = threadIdx.x;
    const int dc = blockIdx.x / n_vtiles;
    const int v0 = (blockIdx.x - dc * n_vtiles) * DWT_ROWS;
    const int rg = tid >> 3, cc = tid & 7;
    const int vs = v0 + tid;                               // the row this thread stages
    const bool vs_ok = vs < V;
    const int vs_c = vs_ok ? vs : V - 1;

    float acc[RPT][8];
#pragma unroll
    for (int k = 0; k < RPT; ++k)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[k][i] = 0.f;
    float db_acc = (db && dc == 0 && add_db && vs_ok) ? db[vs] : 0.f;

    // The loads of a sequence are straight-line code (clamped addresses instead of predicates) and nothing
    // looks at their results before stage(), so that they stay in flight while the sequence before is
    // multiplied.  Byte offsets within a sequence's hidden states (S * D * 2 bytes is far below 4 GiB) and
    // within a row of dY / Y / I are kept in 32 bits; the sequence's base is wave-uniform.
    float dy_r, y_r;
    int ix_r;
    uint32_t hoff[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) hoff[p] = (uint32_t)((min(p * RGS + rg, S - 1) * D + dc * DWS_COLS + cc * 8) * 2);
    const uint32_t voff = (uint32_t)vs_c * 4u;
    auto gload = [&](int b) {
        const size_t ro = (size_t)b * V * 4;
        dy_r = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(dY) + ro + voff);
        y_r = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(Y) + ro + voff);
        ix_r = *reinterpret_cast<const int*>(reinterpret_cast<const char*>(I) + ro + voff);
    };
    // the eight tile rows a wave copies per pass land in 1024 contiguous LDS bytes, lane l at + 16 l; rows
    // behind S - 1 (when S is not a multiple of 128) receive copies of row S - 1 and are never read
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane((uint32_t)(tid >> 6) * 8u * ROW_B);
    auto tile_load = [&](int b, int buf) {
        const char* hb = reinterpret_cast<const char*>(H) + (size_t)b * S * D * 2;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_addr(&s_tile[buf][0])) + wave_lds;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) dma16_to_lds(hb, hoff[p], dst + p * RGS * ROW_B);
    };
    auto stage = [&](int buf, bool count) {
        const float g = vs_ok ? gate_grad(dy_r, y_r) : 0.f;
        db_acc += count ? g : 0.f;
        s_go[buf][tid] = make_float2(g, __int_as_float((g != 0.f ? clamp_pos(ix_r, S) : DWT_MAX_S) * ROW_B));
    };
    if (tid < 16) *reinterpret_cast<uint4*>(&s_tile[tid >> 3][DWT_MAX_S * ROW_B + (tid & 7) * 16]) = make_uint4(0, 0, 0, 0);
    gload(0);
    tile_load(0, 0);
    stage(0, true);
    wait_vmcnt<0>();
    __syncthreads();
    for (int b = 0; b < B; ++b) {
        const int buf = b & 1;
        // the last round loads and stages the last sequence once more (into the buffer nobody reads again):
        // no branch around the loads
        const bool more = b + 1 < B;
        gload(more ? b + 1 : b);
        tile_load(more ? b + 1 : b, buf ^ 1);
        // all eight (g, offset) pairs first, then the row pieces one pair of rows ahead of the FMAs that
        // use them, so that a wave waits for LDS once per sequence rather than twice per pair of rows
        float2 go[RPT];
#pragma unroll
        for (int k = 0; k < RPT; ++k) go[k] = s_go[buf][rg + RGS * k];
        const uint8_t* tile = &s_tile[buf][cc * 16];
        uint4 xa = *reinterpret_cast<const uint4*>(tile + __float_as_int(go[0].y));
        uint4 xb = *reinterpret_cast<const uint4*>(tile + __float_as_int(go[1].y));
#pragma unroll
        for (int h = 0; h < RPT; h += 2) {
            uint4 na = xa, nb = xb;
            if (h + 2 < RPT) {
                na = *reinterpret_cast<const uint4*>(tile + __float_as_int(go[h + 2].y));
                nb = *reinterpret_cast<const uint4*>(tile + __float_as_int(go[h + 3].y));
            }
            if (__any(go[h].x != 0.f || go[h + 1].x != 0.f)) {
                RowChunk<uint16_t>::fma(xa, go[h].x, acc[h]);
                RowChunk<uint16_t>::fma(xb, go[h + 1].x, acc[h + 1]);
            }
            xa = na;
            xb = nb;
        }
        stage(buf ^ 1, more);
        wait_vmcnt<0>();                               // the tile has landed
        __syncthreads();
    }
    if (db && dc == 0 && vs_ok) db[vs] = db_acc;
    if (!dW) return;
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        const int v = v0 + rg + RGS * k;
        if (v < V) {
            const size_t o = (size_t)v * D + dc * DWS_COLS + cc * 8;
#pragma unroll
            for (int i = 0; i < 8; i += 4) {
                float4 r = make_float4(acc[k][i], acc[k][i + 1], acc[k][i + 2], acc[k][i + 3]);
                if (add_dst) r = add4(OutVec<OT>::load4(dW + o + i), r);
                OutVec<OT>::store4(dW + o + i, r);
            }
        }
    }
}

}  // namespace lsr
