// Persistent variant of the fused bf16 forward (same tiling, layouts and epilogue as
// fwd_bf16.hpp; needs D % 64 == 0).
//
// One workgroup per CU stays resident and pulls (row group, vocabulary tile) pairs from a per-XCD
// atomic counter, so tiles of unequal length balance dynamically and workgroups of one XCD keep
// working on neighbouring tiles that share operand panels in that XCD's L2.  Work is a stream of
// units (tile, chunk of 256 token rows).  While the last K slab of a unit is being multiplied, the
// first slab of the NEXT unit is already being loaded into the other LDS stage, so the reduction
// epilogue, the accumulator reset and the address set-up of the next unit overlap with loads in
// flight instead of exposing a full memory latency per unit.
//
// Per unit, all discovery work rides on the slab barriers that exist anyway:
//   step 0     : lane 0 takes the next tile index from the counter (if this tile has no more chunks)
//   step 1     : everybody decodes it and writes the next unit's row tables (second table buffer)
//   last step  : row/column pointers are switched to the next unit (this unit's loads have all been
//                issued by then) and the loads interleaved with this step's MFMAs fetch its slab 0.
// Units with fewer than three slabs get phantom steps (barrier only) so the three points stay apart.
#pragma once
#include "fwd_bf16.hpp"

namespace lsr {

struct FwdPersistParams {
    FwdParams f;
    int* ctr;        // [8] tile counters, one per XCD, zeroed before the launch
    int per_xcd;     // ceil(n_tiles / 8): size of each XCD's contiguous range of tile indices
    int n_tiles;     // n_vtiles * n_rowgroups
};

template <bool LONG, int G, bool ARG>
__global__ __launch_bounds__(FWD_THREADS) void fwd_bf16_persistent_kernel(FwdPersistParams pp) {
    constexpr int BK = 64;
    constexpr int RB = BK * 2;
    constexpr int IPW = 4;                   // wave-wide loads per wave, operand and slab
    constexpr int KS = BK / 16;
    constexpr int SLAB = FWD_TM * RB;
    constexpr int LPT = 2 * IPW;
    constexpr int SPREAD = 2;
    const FwdParams& p = pp.f;

    __shared__ __attribute__((aligned(1024))) uint8_t s_tile[2][2][SLAB];   // [stage][A|B]
    __shared__ int s_rowtok[2][FWD_TM];      // [table buffer][tile row] -> row of H (b*S+s)
    __shared__ int s_rowpos[2][FWD_TM];      // [table buffer][tile row] -> sequence position s
    __shared__ float s_xm[4][2][32];
    __shared__ int s_xs[4][2][32];
    __shared__ int s_next;                   // mailbox for the fetched tile index

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const int wm = wave >> 2;
    const int wn = wave & 3;
    const int half = lane >> 5;
    const int l32 = lane & 31;
    const int D = p.D;
    const int nk = D / BK;
    const int n_steps = nk < 3 ? 3 : nk;
    const int xcd = blockIdx.x & 7;

    // loader geometry (see fwd_bf16.hpp): access j of wave w covers tile rows 8 (8 j + w) .. + 8
    const int lrow = wave * 8 + (lane >> 3);
    const int gch = (lane & 7) ^ lds_swz<BK>(lrow);
    const uint32_t lds_dst = __builtin_amdgcn_readfirstlane(lds_addr(&s_tile[0][0][0]) + wave * 1024);
    // fragment geometry
    const int fa_row = (LONG ? wm * 32 : wm * 128) + l32;
    constexpr int A_STRIDE = (LONG ? 64 : 32) * RB;
    constexpr int B_STRIDE = 32 * RB;
    const int fb_row = wn * 64 + l32;
    int fsw[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fsw[ks] = ((ks * 2 + half) ^ lds_swz<BK>(l32)) << 4;

    // k-th tile of this XCD's range -> (row group, vocabulary tile).  Tiles are ordered in groups of
    // FWD_GV vocabulary tiles x all row groups, so that consecutive indices share operand panels.
    auto decode = [&](int k, int& rg, int& vt) -> bool {
        const int t = xcd * pp.per_xcd + k;
        if (k >= pp.per_xcd || t >= pp.n_tiles) return false;
        const int span = p.n_rowgroups * FWD_GV;
        const int vg = t / span;
        const int gsize = min(FWD_GV, p.n_vtiles - vg * FWD_GV);
        const int rem = t - vg * span;
        rg = rem / gsize;
        vt = vg * FWD_GV + (rem - rg * gsize);
        return true;
    };
    auto chunks_of = [&](int len) { return len > FWD_TM ? (len + FWD_TM - 1) / FWD_TM : 1; };
    // live 32-row blocks of a unit (long layout); the short layout multiplies all eight
    auto live_blocks = [&](int len, int chunk) {
        if (!LONG) return FWD_TM / 32;
        const int rows = min(FWD_TM, max(len - chunk * FWD_TM, 0));
        return (rows + 31) >> 5;
    };
    auto build_table = [&](int tb, int rg, int chunk, int len) {
        if (tid < FWD_TM) {
            int b, j, lb;
            if (LONG) {
                b = rg; lb = len; j = chunk * FWD_TM + tid;
            } else {
                constexpr int SR = 32 * G;
                b = rg * (FWD_TM / SR) + tid / SR;
                b = b < p.B ? b : p.B - 1;
                lb = p.len[b];
                j = tid % SR;
            }
            j = j < lb ? j : lb - 1;
            const int s = lb > 0 ? p.pos[(size_t)b * p.S + j] : 0;
            s_rowtok[tb][tid] = b * p.S + s;
            s_rowpos[tb][tid] = s;
        }
    };
    const uint16_t* hptr[IPW];
    const uint16_t* wptr[IPW];
    auto set_pointers = [&](int tb, int vt) {
#pragma unroll
        for (int j = 0; j < IPW; ++j) {
            hptr[j] = p.H + (size_t)s_rowtok[tb][lrow + 64 * j] * D + gch * 8;
            int v = vt * FWD_TN + lrow + 64 * j;
            v = v < p.V ? v : p.V - 1;
            wptr[j] = p.W + (size_t)v * D + gch * 8;
        }
    };
    // load n (0..7) of K slab `slab` into ring stage `stage`: A rows first, then B rows.  A rows of
    // row blocks that hold no token of the target unit are not fetched.
    auto issue_one = [&](int n, int slab, int stage, int live_rows) {
        const uint32_t dst = lds_dst + stage * (2 * SLAB);
        const int koff = slab * BK;
        if (n < IPW) {
            if (wave_s * 8 + 64 * n < live_rows) dma16_to_lds(hptr[n] + koff, dst + n * 8192);
        } else {
            dma16_to_lds(wptr[n - IPW] + koff, dst + SLAB + (n - IPW) * 8192);
        }
    };

    // ---- first unit ----
    if (tid == 0) s_next = atomicAdd(&pp.ctr[xcd], 1);
    __syncthreads();
    int cur_rg = 0, cur_vt = 0;
    if (!decode(s_next, cur_rg, cur_vt)) return;
    int cur_chunk = 0;
    int cur_len = LONG ? p.len[cur_rg] : 0;
    int cur_nch = LONG ? chunks_of(cur_len) : 1;
    build_table(0, cur_rg, 0, cur_len);
    __syncthreads();
    set_pointers(0, cur_vt);
    {
        const int live0 = live_blocks(cur_len, 0) * 32;
#pragma unroll
        for (int n = 0; n < LPT; ++n) issue_one(n, 0, 0, live0);
    }
    int tb = 0;          // table buffer of the current unit
    int parity = 0;      // ring stage that holds the current unit's slab 0
    float run_m[2] = {-INFINITY, -INFINITY};
    int run_s[2] = {0, 0};

    for (;;) {
        const int nrb = live_blocks(cur_len, cur_chunk);
        const int na = LONG ? (nrb + 1 - wm) >> 1 : 4;      // this wave's live row blocks
        const int cur_live = nrb * 32;
        int nxt_rg = cur_rg, nxt_vt = cur_vt, nxt_chunk = cur_chunk + 1, nxt_len = cur_len, nxt_nch = cur_nch;
        bool nxt_valid = LONG && cur_chunk + 1 < cur_nch;
        const bool need_fetch = !nxt_valid;
        int nxt_live = 0;
        int fetched = 0;

        floatx16 acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][c][r] = 0.f;

        auto run_steps = [&](auto na_c) {
            constexpr int NA = decltype(na_c)::value;
            for (int kt = 0; kt < n_steps; ++kt) {
                wait_vmcnt<0>();
                // (the counter value fetched during step 0 is published only now, after a wait that
                // happens anyway, so that its latency never stalls the first slab's MFMAs)
                if (kt == 1 && need_fetch && tid == 0) s_next = fetched;
                __syncthreads();        // slab kt of this unit has landed for every wave
                if (kt == 0 && need_fetch && tid == 0) fetched = atomicAdd(&pp.ctr[xcd], 1);
                if (kt == 1) {
                    if (need_fetch) {
                        nxt_valid = decode(s_next, nxt_rg, nxt_vt);
                        nxt_chunk = 0;
                        if (nxt_valid) {
                            nxt_len = LONG ? p.len[nxt_rg] : 0;
                            nxt_nch = LONG ? chunks_of(nxt_len) : 1;
                        }
                    }
                    if (nxt_valid) {
                        build_table(tb ^ 1, nxt_rg, nxt_chunk, nxt_len);
                        nxt_live = live_blocks(nxt_len, nxt_chunk) * 32;
                    }
                }
                // what the loads interleaved with this step fetch
                int t_slab = kt + 1, t_live = cur_live;
                bool more = kt + 1 < nk;
                if (kt == n_steps - 1) {
                    more = nxt_valid;
                    t_slab = 0;
                    t_live = nxt_live;
                    if (nxt_valid) set_pointers(tb ^ 1, nxt_vt);     // every load of this unit is already issued
                }
                const int t_stage = kt + 1 < nk ? (parity + kt + 1) & 1 : (parity + nk) & 1;
                auto dma = [&](int n) {
                    if (more) issue_one(n, t_slab, t_stage, t_live);
                };
                if (NA == 0 || kt >= nk) {          // nothing to multiply in this step: only the loads
#pragma unroll
                    for (int n = 0; n < LPT; ++n) dma(n);
                } else {
                    const uint8_t* st = &s_tile[(parity + kt) & 1][0][0];
                    if constexpr (NA > 0)
                        mma_slab<NA, KS, true, LPT, SPREAD>(st + fa_row * RB, A_STRIDE, st + SLAB + fb_row * RB, B_STRIDE,
                                                            fsw, acc, dma);
                }
            }
        };
        switch (na) {
            case 4: run_steps(std::integral_constant<int, 4>{}); break;
            case 3: run_steps(std::integral_constant<int, 3>{}); break;
            case 2: run_steps(std::integral_constant<int, 2>{}); break;
            case 1: run_steps(std::integral_constant<int, 1>{}); break;
            default: run_steps(std::integral_constant<int, 0>{}); break;
        }

        // ---- epilogue: in-lane max/argmax over each slot's rows ----
        const int v0 = cur_vt * FWD_TN;
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
                for (int i = q * G; i < q * G + G; ++i) {
                    if (i < na) {
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
                }
            }
            if (LONG) {
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const int s = ARG ? s_rowpos[tb][acc_row<LONG>(e[c], half, wm)] : 0;
                    if (m[c] > run_m[c]) { run_m[c] = m[c]; run_s[c] = s; }
                }
            } else {
                float mm[2];
                int ss[2];
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    int s = ARG ? s_rowpos[tb][acc_row<LONG>(e[c], half, wm)] : 0;
                    const float mo = __shfl_xor(m[c], 32);
                    const int so = __shfl_xor(s, 32);
                    float mc = m[c];
                    if (mo > mc || (mo == mc && so < s)) { mc = mo; s = so; }
                    mm[c] = mc;
                    ss[c] = s;
                }
                constexpr int SPT = FWD_TM / (32 * G);            // sequences per tile
                const int b = cur_rg * SPT + wm * NSLOT + q;
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

        if (LONG && cur_chunk + 1 == cur_nch) {
            // last chunk of the sequence: combine half-waves, then the two waves that share these
            // columns, then bias + ReLU + log1p on the single surviving value per (b, v)
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
                run_m[c] = -INFINITY;
                run_s[c] = 0;
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
                    const bool any = cur_len > 0;
                    p.Y[(size_t)cur_rg * p.V + v] = any ? log1pf(fmaxf(mv + p.bias[v], 0.f)) : 0.f;
                    if (ARG) p.I[(size_t)cur_rg * p.V + v] = any ? sv : 0;
                }
            }
        }

        if (!nxt_valid) break;
        parity = (parity + nk) & 1;
        tb ^= 1;
        cur_rg = nxt_rg; cur_vt = nxt_vt; cur_chunk = nxt_chunk; cur_len = nxt_len; cur_nch = nxt_nch;
    }
}

}  // namespace lsr
