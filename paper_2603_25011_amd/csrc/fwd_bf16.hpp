// Fused forward for bf16 inputs on gfx950: GEMM tile (MFMA, fp32 accumulate) + masked running
// max/argmax over the sequence + bias/ReLU/log1p on the reduced B x V result.
//
// Paper Sec. 3 "Forward Pass": log(1+ReLU(x)) is monotone, so the maximum over the sequence is
// taken on raw logits while they still sit in accumulator registers and the activation is
// applied once afterwards.  The B x S x V logits never leave the chip.
//
// Tiling.  A workgroup of 8 waves owns a 256 (tokens) x 256 (vocabulary) output tile; wave
// (wm, wn) owns rows [128 wm, 128 wm + 128) x columns [64 wn, 64 wn + 64) as 4 x 2 blocks of the
// 32x32x16 bf16 MFMA.  Tokens are the MFMA's row dimension: in the 32x32 accumulator layout a
// lane holds 16 rows of ONE column, so the max over tokens starts as a plain in-lane reduction.
// K (the hidden size D) is walked in slabs of 64 through a double-buffered, XOR-swizzled LDS tile.
//
// Masking.  Only valid tokens are multiplied: a compaction pass lists the valid positions of every
// sequence, and tile rows are gathered through that list.  Rows past the end of a sequence repeat
// its last valid token, which cannot change a maximum or its lowest-index arg-max, so the
// epilogue needs no per-element mask.
//
// Two row layouts, chosen on the host from S alone:
//   long  (S > 128): a workgroup owns one sequence and walks its valid tokens in chunks of 256
//                    rows, keeping a running (max, position) per column in registers.
//   short (S <= 128): every sequence gets a fixed slot of G = 1, 2 or 4 row blocks (32 G >= S);
//                    a tile holds 8/G sequences and each wave reduces its own slots.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lsr {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int FWD_TM = 256;        // tile rows (tokens)
constexpr int FWD_TN = 256;        // tile columns (vocabulary entries)
constexpr int FWD_BK = 64;         // K slab (bf16 elements) = 128 bytes per row
constexpr int FWD_THREADS = 512;
constexpr int FWD_GV = 4;          // vocabulary tiles per L2-sharing group

struct FwdParams {
    const uint16_t* H;
    const uint16_t* W;
    const float* bias;
    const int* len;      // [B]   number of valid tokens per sequence
    const int* pos;      // [B,S] valid positions, ascending, first len[b] entries used
    float* Y;
    int* I;              // may be null
    int B, S, D, V;
    int n_vtiles;        // ceil(V / 256)
    int n_rowgroups;     // long: B; short: ceil(B / (8/G))
    int n_logical;       // ceil(n_vtiles / GV) * GV * n_rowgroups
};

// Byte offset of 16-byte chunk c (0..7) of row r inside a [256 x 128 B] LDS slab.
__device__ __forceinline__ int lds_off(int r, int c) { return r * 128 + (((c ^ r) & 7) << 4); }

// Row (0..127 within the wave's 128 rows) of accumulator element e = 16*block + reg for a lane in
// the given half-wave: MFMA 32x32 output register r of lane l is row 8*(r/4) + 4*(l/32) + r%4.
__device__ __forceinline__ int acc_row(int e, int half) {
    return (e >> 4) * 32 + ((e & 15) >> 2) * 8 + half * 4 + (e & 3);
}

template <bool LONG, int G, bool ARG>
__global__ __launch_bounds__(FWD_THREADS) void fwd_bf16_kernel(FwdParams p) {
    __shared__ __attribute__((aligned(16))) uint8_t s_tile[2][2][FWD_TM * 128];   // [stage][A|B]
    __shared__ int s_rowtok[FWD_TM];     // row of H (b*S+s) feeding each tile row
    __shared__ int s_rowpos[FWD_TM];     // sequence position s of each tile row
    __shared__ float s_xm[4][2][32];
    __shared__ int s_xs[4][2][32];

    // ---- workgroup -> (row group, vocabulary tile); contiguous logical ranges per XCD ----
    const int per_xcd = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= p.n_logical) return;
    const int group_span = p.n_rowgroups * FWD_GV;
    const int vg = logical / group_span;
    const int rem = logical - vg * group_span;
    const int rg = rem / FWD_GV;
    const int vt = vg * FWD_GV + (rem - rg * FWD_GV);
    if (vt >= p.n_vtiles) return;
    const int v0 = vt * FWD_TN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 2;
    const int wn = wave & 3;
    const int half = lane >> 5;
    const int l32 = lane & 31;
    const int D = p.D;
    const int nk = (D + FWD_BK - 1) / FWD_BK;

    // ---- loader geometry: thread -> (row ldr + 64 i, 16-byte chunk ldc) ----
    const int ldc = tid & 7;
    const int ldr = tid >> 3;
    const int st_off = lds_off(ldr, ldc);           // + i * 64 * 128 (row & 7 unchanged)
    const uint16_t* wptr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int v = v0 + ldr + 64 * i;
        v = v < p.V ? v : p.V - 1;
        wptr[i] = p.W + (size_t)v * D + ldc * 8;
    }
    // ---- fragment geometry ----
    const int fa_row = wm * 128 + l32;               // + 32 i
    const int fb_row = wn * 64 + l32;                // + 32 c
    int fsw[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) fsw[ks] = (((ks * 2 + half) ^ l32) & 7) << 4;

    int len_b = 0, b_long = 0, n_chunks = 1;
    if (LONG) {
        b_long = rg;
        len_b = p.len[b_long];
        if (len_b == 0) {                            // no valid token: Y = 0, I = 0
            if (tid < FWD_TN && v0 + tid < p.V) {
                p.Y[(size_t)b_long * p.V + v0 + tid] = 0.f;
                if (ARG) p.I[(size_t)b_long * p.V + v0 + tid] = 0;
            }
            return;
        }
        n_chunks = (len_b + FWD_TM - 1) / FWD_TM;
    }

    float run_m[2] = {-INFINITY, -INFINITY};
    int run_s[2] = {0, 0};

    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        // ---- which token feeds each tile row ----
        if (tid < FWD_TM) {
            int b, j, lb;
            if (LONG) {
                b = b_long; lb = len_b; j = chunk * FWD_TM + tid;
            } else {
                constexpr int SR = 32 * G;
                b = rg * (FWD_TM / SR) + tid / SR;
                b = b < p.B ? b : p.B - 1;
                lb = p.len[b];
                j = tid % SR;
            }
            j = j < lb ? j : lb - 1;
            const int s = lb > 0 ? p.pos[(size_t)b * p.S + j] : 0;
            s_rowtok[tid] = b * p.S + s;
            s_rowpos[tid] = s;
        }
        __syncthreads();
        const uint16_t* hptr[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) hptr[i] = p.H + (size_t)s_rowtok[ldr + 64 * i] * D + ldc * 8;

        floatx16 acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][c][r] = 0.f;

        uint4 ra[4], rb[4];
        // K slabs are full except possibly the last one (D not a multiple of 64): only that one pays
        // for per-chunk predication.
        auto gload = [&](int kt) {
            const int koff = kt * FWD_BK;
            if (koff + FWD_BK <= D) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ra[i] = *reinterpret_cast<const uint4*>(hptr[i] + koff);
                    rb[i] = *reinterpret_cast<const uint4*>(wptr[i] + koff);
                }
            } else {
                const bool kval = koff + ldc * 8 < D;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ra[i] = kval ? *reinterpret_cast<const uint4*>(hptr[i] + koff) : make_uint4(0, 0, 0, 0);
                    rb[i] = kval ? *reinterpret_cast<const uint4*>(wptr[i] + koff) : make_uint4(0, 0, 0, 0);
                }
            }
        };
        auto lstore = [&](int st) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                *reinterpret_cast<uint4*>(&s_tile[st][0][st_off + i * 64 * 128]) = ra[i];
                *reinterpret_cast<uint4*>(&s_tile[st][1][st_off + i * 64 * 128]) = rb[i];
            }
        };

        gload(0);
        lstore(0);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int st = kt & 1;
            if (kt + 1 < nk) gload(kt + 1);
            const uint8_t* sa = &s_tile[st][0][fa_row * 128];
            const uint8_t* sb = &s_tile[st][1][fb_row * 128];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                bf16x8 fa[4], fb[2];
#pragma unroll
                for (int i = 0; i < 4; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * 128 + fsw[ks]);
#pragma unroll
                for (int c = 0; c < 2; ++c) fb[c] = *reinterpret_cast<const bf16x8*>(sb + c * 32 * 128 + fsw[ks]);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int c = 0; c < 2; ++c)
                        acc[i][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[c], acc[i][c], 0, 0, 0);
            }
            if (kt + 1 < nk) lstore(st ^ 1);
            __syncthreads();
        }

        // ---- epilogue: in-lane max/argmax over each slot's rows ----
        constexpr int NSLOT = 4 / G;
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            float m[2];
            int e[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                m[c] = -INFINITY;
                e[c] = 0;
#pragma unroll
                for (int i = q * G; i < q * G + G; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float a = acc[i][c][r];
                        if (ARG) {
                            if (a > m[c]) { m[c] = a; e[c] = i * 16 + r; }
                        } else {
                            m[c] = fmaxf(m[c], a);
                        }
                    }
            }
            if (LONG) {
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const int s = ARG ? s_rowpos[wm * 128 + acc_row(e[c], half)] : 0;
                    if (m[c] > run_m[c]) { run_m[c] = m[c]; run_s[c] = s; }
                }
            } else {
                // a slot lives entirely in this wave: combine the two half-waves and write
                float mm[2];
                int ss[2];
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    int s = ARG ? s_rowpos[wm * 128 + acc_row(e[c], half)] : 0;
                    const float mo = __shfl_xor(m[c], 32);
                    const int so = __shfl_xor(s, 32);
                    float mc = m[c];
                    if (mo > mc || (mo == mc && so < s)) { mc = mo; s = so; }
                    mm[c] = mc;
                    ss[c] = s;
                }
                constexpr int SPT = FWD_TM / (32 * G);            // sequences per tile
                const int b = rg * SPT + wm * NSLOT + q;
                const int v = v0 + wn * 64 + half * 32 + l32;
                if (b < p.B && v < p.V) {
                    const float mv = half ? mm[1] : mm[0];
                    const int sv = half ? ss[1] : ss[0];
                    const bool any = p.len[b] > 0;
                    const float y = any ? log1pf(fmaxf(mv + p.bias[v], 0.f)) : 0.f;
                    p.Y[(size_t)b * p.V + v] = y;
                    if (ARG) p.I[(size_t)b * p.V + v] = any ? sv : 0;
                }
            }
        }
        __syncthreads();     // the next chunk rewrites the row tables
    }

    if (LONG) {
        // combine half-waves, then the two waves that share these columns, then finalise
        float mm[2];
        int ss[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            float mc = run_m[c];
            int s = run_s[c];
            const float mo = __shfl_xor(mc, 32);
            const int so = __shfl_xor(s, 32);
            if (mo > mc || (mo == mc && so < s)) { mc = mo; s = so; }
            mm[c] = mc;
            ss[c] = s;
        }
        if (wm == 1 && half == 0) {
#pragma unroll
            for (int c = 0; c < 2; ++c) { s_xm[wn][c][l32] = mm[c]; s_xs[wn][c][l32] = ss[c]; }
        }
        __syncthreads();
        if (wm == 0) {
            float mv = half ? mm[1] : mm[0];
            int sv = half ? ss[1] : ss[0];
            const float mo = s_xm[wn][half][l32];
            const int so = s_xs[wn][half][l32];
            if (mo > mv || (mo == mv && so < sv)) { mv = mo; sv = so; }
            const int v = v0 + wn * 64 + half * 32 + l32;
            if (v < p.V) {
                p.Y[(size_t)b_long * p.V + v] = log1pf(fmaxf(mv + p.bias[v], 0.f));
                if (ARG) p.I[(size_t)b_long * p.V + v] = sv;
            }
        }
    }
}

}  // namespace lsr
