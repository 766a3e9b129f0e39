// Fused forward for bf16 inputs on gfx950: GEMM tile (MFMA, fp32 accumulate) + masked running
// max/argmax over the sequence + bias/ReLU/log1p on the reduced B x V result.
//
// Paper Sec. 3 "Forward Pass": log(1+ReLU(x)) is monotone, so the maximum over the sequence is
// taken on raw logits while they still sit in accumulator registers and the activation is
// applied once afterwards.  The B x S x V logits never leave the chip.
//
// Tiling.  A workgroup of 8 waves (2 per SIMD) owns a 256 (tokens) x 256 (vocabulary) output tile;
// wave (wm, wn) owns four 32-row blocks x columns [64 wn, 64 wn + 64), i.e. 4 x 2 blocks of the
// 32x32x16 bf16 MFMA.  Tokens are the MFMA's row dimension: in the 32x32 accumulator layout a lane
// holds 16 rows of ONE column, so the max over tokens starts as a plain in-lane reduction, is
// finished with one exchange between the two half-waves; what is left per tile is one value per
// (block, column), which goes through LDS to the scan that joins the blocks of a sequence.
//
// Operand staging.  K (the hidden size D) is walked in slabs of BK elements through an NS-stage
// ring of LDS tiles.  Two loaders:
//   DMA = true  : global_load_lds (16 bytes per lane straight into LDS, no staging registers),
//                 slabs issued NS-1 iterations ahead, one barrier per slab.  Needs D % BK == 0.
//   DMA = false : global -> registers -> LDS, one slab ahead (BK = 64, NS = 2).  Handles any D that
//                 is a multiple of 8 (the last slab is zero-filled).
// Rows are XOR-swizzled inside a slab so that the 16-byte fragment reads are bank-conflict free.
//
// Masking and packing.  Only valid tokens are multiplied.  A compaction pass lists the valid
// positions of every sequence; each sequence is then cut into segments of SEG rows, the last segment
// padded with repeats of the sequence's last valid token, which cannot change a maximum or its
// lowest-position arg-max.  The segments of all sequences form one dense list, and a tile is any
// 256 / SEG consecutive segments of it, so tiles are full whatever the length mix; a segment never
// mixes two sequences, which keeps the first reduction step (in-lane over a lane's rows of one
// segment) free of masks.  SEG = 32 is the MFMA's row block (a lane then reduces all 16 of its rows of
// a block); SEG = 8 serves batches of short sequences (S <= 64: a lane reduces its rows in four groups
// of four, one per segment of the block), where 32-row segments would pad 4..32-token sequences by
// 75 % and 8-row segments pad them by 16 %, at the price of four times as many (segment, column) pairs
// through LDS per tile.
//
// Chunks and units.  Tile j is segments j * 256/SEG .. of the list, whatever sequences they belong to, so
// only the very last tile can be short.  The T tiles are split evenly into ceil(T / tpc) chunks of
// consecutive tiles (ChunkSplit below).  A unit of work is (chunk, vocabulary tile): the workgroup that
// takes it walks the chunk's tiles; per tile it reduces every segment to one (max, position) per column,
// and a scan over the tile's segments carries the running pair of the sequence that is still open in
// registers from segment to segment and from tile to tile (the streaming reduction of Sec. 3).  The
// segment that ends a sequence triggers bias + ReLU + log1p and the store of Y and I.  A chunk boundary
// may fall inside a sequence.  The piece in front of the boundary (the sequence began in this chunk)
// leaves its raw pair in Y and I; a piece behind a boundary (the chunk begins inside the sequence)
// leaves its pair in slot `chunk` of the part_m / part_s arrays; a small kernel (fwd_merge_kernel) joins
// the pieces and finalises.  Chunks of whole sequences would need no such pass but end in short tiles
// and need the lengths on the host to size.
// Two launch modes (template parameter RES, chosen by the host from the shape).  Deep problems launch
// one workgroup per unit and let the hardware hand units out in order, which keeps the workgroups of an
// XCD on neighbouring units and their shared rows of H and W in its L2.  Shallow problems (a few short
// units per CU) launch one workgroup per CU that stays resident and walks its share of the units (see
// the schedule at the top of the kernel), the next unit's row table and first slab prefetched like the
// next tile's: there the launch and drain of a workgroup per unit would cost more than the drift.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "lds_dma.hpp"

namespace lsr {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int FWD_TM = 256;        // tile rows (tokens)
// A workgroup has 2 x NWN waves: two wave rows (wm) that split the tile's row blocks, NWN wave
// columns (wn) of 64 vocabulary entries each.
constexpr int fwd_tn(int nwn) { return 64 * nwn; }          // tile columns (vocabulary entries)
constexpr int fwd_threads(int nwn) { return 128 * nwn; }
constexpr int FWD_GV_COLS = 1024;  // vocabulary entries per L2-sharing group of tiles

constexpr int FWD_BLK = 32;                      // rows per MFMA row block
constexpr int FWD_TB = FWD_TM / FWD_BLK;         // blocks per tile
constexpr int FWD_SEG_SHORT = 8;                 // rows per segment for batches of short sequences (else FWD_BLK)
constexpr int FWD_SEG_SHORT_MAX_S = 64;          // sequence lengths up to which the host picks it
constexpr int FWD_META_LAST = 1 << 31;           // block ends its sequence
constexpr int FWD_META_EMPTY = 1 << 30;          // the sequence has no valid token
constexpr int FWD_META_FIRST = 1 << 29;          // block begins its sequence
constexpr int FWD_META_SEQ = 0xffff;             // sequence index b (B <= 65535)

// The T = ceil(n_segs / spt) tiles of the segment list (spt segments per tile) in nc = ceil(T / tpc)
// chunks of as equal size as possible: chunk c holds tiles floor(c T / nc) .. floor((c+1) T / nc) - 1.
struct ChunkSplit {
    int T, nc;
    __device__ __forceinline__ int first_tile(int c) const { return (int)(((long long)c * T) / nc); }
    // largest c with floor(c T / nc) <= t
    __device__ __forceinline__ int chunk_of_tile(int t) const { return (int)((((long long)t + 1) * nc - 1) / T); }
};
__device__ __forceinline__ ChunkSplit chunk_split(int n_segs, int tpc, int spt) {
    ChunkSplit cs;
    cs.T = (n_segs + spt - 1) / spt;
    cs.nc = (cs.T + tpc - 1) / tpc;
    return cs;
}

struct FwdParams {
    const uint16_t* H;
    const uint16_t* W;
    const float* bias;
    const int2* rows;        // [n_segs * SEG] per packed row: (row of H = b*S + s, position s)
    const int* blk_meta;     // [n_segs] sequence index b, ORed with FWD_META_LAST / _EMPTY / _FIRST
    const int* n_blocks;     // n_segs: length of the segment list (written by the planning pass)
    float* Y;
    int* I;                  // may be null
    float* part_m;           // [n_chunks][V] pieces of sequences that begin in an earlier chunk
    int* part_s;             //   "            (positions; unused without I)
    int B, S, D, V;
    int n_vtiles;            // ceil(V / tile columns)
    int n_chunks;            // chunks the grid provides for (from the longest block list the shape allows)
    int tpc;                 // most tiles per chunk
    int gv;                  // vocabulary tiles per L2-sharing group
};

// Swizzle of the 16-byte chunk index inside a tile row.  A fragment read has lanes 0..31 on 32
// consecutive rows of one chunk column and lanes 32..63 on the next column; LDS serves 16 lanes
// (256 bytes, all 64 banks) per cycle.  Measured on gfx950 with 4 waves reading: 128-byte rows
// XORed with row bits 1..3, or 64-byte rows XORed with row bits 2..3, take 4 cycles per wave
// read (conflict free); XOR with the low row bits takes 8; no swizzle 32.
template <int BK>
__device__ __forceinline__ int lds_swz(int r) {
    return BK == 64 ? (r >> 1) & 7 : (r >> 2) & 3;
}

// Tile row of accumulator register r (0..15) of a lane in the given half-wave, in tile block blk:
// MFMA 32x32 output register r of lane l is row 8*(r/4) + 4*(l/32) + r%4 of its block.
__device__ __forceinline__ int acc_row(int blk, int r, int half) {
    return blk * FWD_BLK + (r >> 2) * 8 + half * 4 + (r & 3);
}

// One K slab of MFMAs for the first NA of this wave's four row blocks, fragments read per k-step
// (register-staged loader; the direct-to-LDS pipeline uses mma_rot below).
template <int NA, int KS>
__device__ __forceinline__ void mma_slab(const uint8_t* sa, int a_stride, const uint8_t* sb, int b_stride,
                                         const int (&fsw)[KS], floatx16 (&acc)[4][2]) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        bf16x8 fa[NA], fb[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) fb[c] = *reinterpret_cast<const bf16x8*>(sb + c * b_stride + fsw[ks]);
#pragma unroll
        for (int i = 0; i < NA; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(sa + i * a_stride + fsw[ks]);
#pragma unroll
        for (int i = 0; i < NA; ++i)
#pragma unroll
            for (int c = 0; c < 2; ++c)
                acc[i][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[c], acc[i][c], 0, 0, 0);
    }
}

// The direct-to-LDS pipeline runs its slabs rotated by one k-step against the barriers: the MFMAs
// of a slab's LAST k-step are issued after the barrier that publishes the NEXT slab, from fragments
// that were read before it, and the first fragments of the new slab are read behind them.  No wave
// then waits on LDS right after a barrier, when all eight would do so at once with the matrix pipe
// empty.  Fragment buffers (parity = k-step & 1, KS even) therefore live across calls.
//   MODE 0  first slab of a tile: burst-read k-step 0, then k-steps 0 .. KS-2 (reading 1 .. KS-1)
//   MODE 1  later slabs: k-step KS-1 of the previous slab (reading k-step 0 of this one), then
//           k-steps 0 .. KS-2 (reading 1 .. KS-1)
//   MODE 2  after the last slab of the tile: its k-step KS-1
// The order of the MFMAs on every accumulator is the same as without the rotation.
template <int NA, int KS, int MODE, int NDMA, int SPREAD, typename DmaFn>
__device__ __forceinline__ void mma_rot(const uint8_t* sa, int a_stride, const uint8_t* sb, int b_stride,
                                        const int (&fsw)[KS], bf16x8 (&fa)[2][4], bf16x8 (&fb)[2][2],
                                        floatx16 (&acc)[4][2], DmaFn&& dma) {
    static_assert(KS % 2 == 0 && KS >= 2, "buffer parity must not depend on the slab");
    constexpr int M = NA * 2;
    constexpr int Q = SPREAD > 0 ? NDMA / SPREAD : 0;
    constexpr int GROUPS = MODE == 0 ? KS - 1 : (MODE == 1 ? KS : 1);
    if constexpr (MODE == 0) {
#pragma unroll
        for (int c = 0; c < 2; ++c) fb[0][c] = *reinterpret_cast<const bf16x8*>(sb + c * b_stride + fsw[0]);
#pragma unroll
        for (int i = 0; i < NA; ++i) fa[0][i] = *reinterpret_cast<const bf16x8*>(sa + i * a_stride + fsw[0]);
    }
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        const int mk = MODE == 0 ? g : (MODE == 1 ? (g == 0 ? KS - 1 : g - 1) : KS - 1);   // k-step multiplied
        const int rk = MODE == 0 ? g + 1 : (MODE == 1 ? g : -1);                           // k-step read
        const int cur = mk & 1, nxt = rk & 1;
        auto read_next = [&](int q) {
            if (rk >= 0 && q < NA + 2) {
                if (q == 0 || q == 2) {
                    const int c = q >> 1;
                    fb[nxt][c] = *reinterpret_cast<const bf16x8*>(sb + c * b_stride + fsw[rk < 0 ? 0 : rk]);
                } else {
                    const int i = q == 1 ? 0 : q - 2;
                    fa[nxt][i] = *reinterpret_cast<const bf16x8*>(sa + i * a_stride + fsw[rk < 0 ? 0 : rk]);
                }
            }
        };
#pragma unroll
        for (int m = 0; m < M; ++m) {
            acc[m >> 1][m & 1] =
                __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][m >> 1], fb[cur][m & 1], acc[m >> 1][m & 1], 0, 0, 0);
            if (rk == KS - 1) {
                // the reads before a barrier have to be back when the wave reaches it: two per MFMA,
                // so that the last one still has most of the group to return
                read_next(2 * m);
                read_next(2 * m + 1);
            } else {
                read_next(m);
                if (m == M - 1) {
#pragma unroll
                    for (int q = M; q < NA + 2; ++q) read_next(q);
                }
            }
            if (MODE != 2 && g < SPREAD) {
                const int lo = (m * Q + M - 1) / M, hi = ((m + 1) * Q + M - 1) / M;
#pragma unroll
                for (int t = lo; t < hi; ++t) dma(g * Q + t);
            }
            __builtin_amdgcn_sched_barrier(0);      // keep this interleaving
        }
    }
}

template <int KS>
__device__ __forceinline__ void mma_dispatch(int na, const uint8_t* sa, int a_stride, const uint8_t* sb, int b_stride,
                                             const int (&fsw)[KS], floatx16 (&acc)[4][2]) {
    switch (na) {
        case 4: mma_slab<4, KS>(sa, a_stride, sb, b_stride, fsw, acc); break;
        case 3: mma_slab<3, KS>(sa, a_stride, sb, b_stride, fsw, acc); break;
        case 2: mma_slab<2, KS>(sa, a_stride, sb, b_stride, fsw, acc); break;
        case 1: mma_slab<1, KS>(sa, a_stride, sb, b_stride, fsw, acc); break;
        default: break;                             // no live row block in this wave
    }
}

// One workgroup of 8 waves (2 wave rows x 4 wave columns) per CU on a 256 x 256 tile, K in slabs of 64
// through a ring of two LDS stages.
//   ARG  track the arg-max position (I requested)
//   DMA  operands go global -> LDS directly (D a multiple of 64, H and W below 4 GiB each); otherwise
//        through registers, with 64-bit addresses and a zero-filled last slab
//   SEG  rows per segment of the packed token list: 32 (FWD_BLK) or 8 (FWD_SEG_SHORT)
//   RES  resident workgroups: a workgroup walks several units (see the schedule below); without it the
//        grid has one workgroup per unit and the code that moves on to a next unit is not generated
// (Built and measured slower, and not kept as parameters: two 4-wave workgroups per CU on 256 x 128
//  tiles, which move 1.5x the bytes into LDS, -20 %; 32-deep slabs in four stages, -6 %.)
constexpr int FWD_NWN = 4;               // wave columns
template <bool ARG, bool DMA, int SEG, bool RES>
__global__ __launch_bounds__(fwd_threads(FWD_NWN), 2) void fwd_bf16_kernel(FwdParams p) {
    static_assert(SEG == 32 || SEG == 16 || SEG == 8, "a segment is a whole number of a lane's register quads");
    constexpr int SPB = FWD_BLK / SEG;       // segments per row block
    constexpr int SPT = FWD_TM / SEG;        // segments per tile
    constexpr int RPS = 16 / SPB;            // accumulator registers of a lane per segment
    constexpr int NWN = FWD_NWN;
    constexpr int BK = 64;                   // K elements per slab
    constexpr int NS = 2;                    // ring stages
    constexpr int SPREAD = 2;                // k-steps over which the loads of the next slab are spread
    constexpr int NW = 2 * NWN;              // waves
    constexpr int TN = fwd_tn(NWN);
    constexpr int RB = BK * 2;               // bytes per tile row per slab
    constexpr int CPR = RB / 16;             // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;            // rows covered by one wave-wide 16-byte-per-lane access
    constexpr int IPA = FWD_TM / RPI / NW;   // such accesses per wave and slab, token rows
    constexpr int IPB = TN / RPI / NW;       //                                  vocabulary rows
    constexpr int KS = BK / 16;              // MFMA k-steps per slab
    constexpr int SLAB_A = FWD_TM * RB;      // bytes per stage, token operand
    constexpr int SLAB_B = TN * RB;          //                  vocabulary operand
    constexpr int STAGE = SLAB_A + SLAB_B;
    constexpr int LPT = IPA + IPB;           // loads per thread per slab (A then B)
    constexpr int JSTEP = NW * 1024;         // LDS bytes between a wave's consecutive accesses
    constexpr int PM_BYTES = SPT * TN * 4;   // one float (or int) per (segment, column) of a tile

    // One array per ring stage: distinct objects keep the compiler from serialising a fragment read
    // of one stage against traffic into another.
    __shared__ __attribute__((aligned(1024))) uint8_t s_ring0[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t s_ring1[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t s_pair[2][STAGE];      // register-staged loader only
    auto ring = [&](auto st) -> uint8_t* {
        constexpr int ST = decltype(st)::value;
        if constexpr (ST == 0) return &s_ring0[0];
        else return &s_ring1[0];
    };
    // Row tables of the current and the next tile (double buffered: the next tile's are fetched,
    // straight into LDS, while this one is multiplied).
    __shared__ __attribute__((aligned(1024))) int2 s_rows[2][FWD_TM];   // (row of H = b*S+s, position s) per tile row
    // blk_meta of each tile block, indexed t % 4: the scan of tile t-1 may still be reading its records
    // when the records of tile t+1 arrive
    __shared__ __attribute__((aligned(128))) int s_meta[4][32];
    // per (segment, column): max logit of the segment and its position.  With 32-row segments the table
    // (16 KB) has memory of its own; with shorter segments (up to 64 KB) it lies in ring stage 1, which is
    // free from the last slab's barrier to the first slab barrier of the next tile (see the epilogue).
    __shared__ __attribute__((aligned(16))) uint8_t s_pm_own[SEG == FWD_BLK ? 2 * PM_BYTES : 16];
    static_assert(2 * PM_BYTES <= STAGE, "the pair table must fit a ring stage");

    // ---- schedule.  A unit of work is (chunk, vocabulary tile); units are ordered in groups of gv
    //      vocabulary tiles x all chunks, so that units next to each other share rows of W and of H.
    //      Each XCD takes a contiguous range of the units (its L2 then sees gv tiles of W at a time), and
    //      the n workgroups of an XCD deal that range out round-robin: workgroup j walks units j, j + n,
    //      j + 2n, ... of the range.  With RES the launch has one workgroup per CU, resident for the whole
    //      launch; without it n is at least the length of the range, so every workgroup has at most one
    //      unit and the hardware hands out units in order as CUs come free.  Workgroup ids go round-robin
    //      over the XCDs, so id & 7 is the XCD and id >> 3 the index on it. ----
    const int n_segs = *p.n_blocks;
    const ChunkSplit cs = chunk_split(n_segs, p.tpc, SPT);
    // units per group of vocabulary tiles.  One workgroup per unit: the unit list provides for the chunks
    // of the longest possible token list, as the grid does, and the workgroups of chunks that do not exist
    // return at once, in place (measured 1 % faster at B=64 S=512 than closing the gaps, which moves all
    // idle workgroups to the end of the grid).
    const int span = (RES ? cs.nc : p.n_chunks) * p.gv;
    const long long n_units = (long long)((p.n_vtiles + p.gv - 1) / p.gv) * span;
    const int n_local = gridDim.x >> 3;
    const int u_end = (int)(n_units * ((blockIdx.x & 7) + 1) / 8);
    struct Unit { int u, vt, rc, g0, ns, n_tiles; };
    // the first unit at or behind u (in steps of n_local) that exists: the last group of vocabulary
    // tiles may be short
    auto open_unit = [&](int u, Unit& x) -> bool {
        for (; u < u_end; u += n_local) {
            const int vg = u / span;
            const int rem = u - vg * span;
            const int rc = rem / p.gv;
            const int vt = vg * p.gv + (rem - rc * p.gv);
            if (vt >= p.n_vtiles || rc >= cs.nc) continue;
            x.u = u; x.vt = vt; x.rc = rc;
            x.g0 = cs.first_tile(rc) * SPT;                                              // first segment of the chunk
            x.ns = min(n_segs, cs.first_tile(rc + 1) * SPT) - x.g0;                      // its segments
            x.n_tiles = (x.ns + SPT - 1) / SPT;
            return true;
        }
        return false;
    };
    Unit cur;
    if (!open_unit((int)(n_units * (blockIdx.x & 7) / 8) + (blockIdx.x >> 3), cur)) return;
    int cur_t = 0;                                                       // tile of the unit

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / NWN;
    const int wn = wave % NWN;
    const int half = lane >> 5;
    const int l32 = lane & 31;
    const int D = p.D;
    const int nk = (D + BK - 1) / BK;

    // ---- loader geometry: access j of wave w covers tile rows (NW j + w) RPI .. + RPI, 1024 contiguous
    //      LDS bytes; lane -> (row lrow, LDS chunk slot lp), which holds global chunk lp ^ swizzle(row) ----
    const int lrow = wave * RPI + lane / CPR;                 // + NW RPI j
    const int lp = lane % CPR;
    const int gch = lp ^ lds_swz<BK>(lrow);                   // swizzle bits do not depend on j
    const int st_off = lrow * RB + lp * 16;                   // + JSTEP j   (register-staged loader)
    // Operand rows are addressed as base + byte offset; the direct-to-LDS loader keeps the offsets in
    // 32 bits (the host takes this path only while H and W are each below 4 GiB).
    size_t woff[DMA ? 1 : IPB];
    uint32_t woff32[DMA ? IPB : 1];
    int w_vt = -1;                                            // vocabulary tile the offsets belong to
    auto w_offsets = [&](int vt) {
        if (vt == w_vt) return;
        w_vt = vt;
#pragma unroll
        for (int j = 0; j < IPB; ++j) {
            int v = vt * TN + lrow + NW * RPI * j;
            v = v < p.V ? v : p.V - 1;
            const size_t o = ((size_t)v * D + gch * 8) * 2;
            if constexpr (DMA) woff32[j] = (uint32_t)o;
            else woff[j] = o;
        }
    };
    w_offsets(cur.vt);
    const char* const Hb = reinterpret_cast<const char*>(p.H);
    const char* const Wb = reinterpret_cast<const char*>(p.W);
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(wave * 1024);
    // ---- fragment geometry ----
    // Tile blocks are interleaved between the two wave rows (wave row wm owns tile blocks
    // wm, wm+2, wm+4, wm+6), so that a short last tile splits evenly between them.
    const int fa_row = wm * FWD_BLK + l32;
    constexpr int A_STRIDE = 2 * FWD_BLK * RB;                // bytes between a wave's consecutive row blocks
    constexpr int B_STRIDE = 32 * RB;
    const int fb_row = wn * 64 + l32;
    int fsw[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fsw[ks] = ((ks * 2 + half) ^ lds_swz<BK>(l32)) << 4;

    // ---- row tables of tile t into buffer buf, by direct-to-LDS loads (no registers held while the
    //      tile before it is multiplied): waves 0 and 1 bring 128 rows each (two per lane), wave 2
    //      the segment records.  Rows of dead segments of a short last tile repeat its last live rows. ----
    //      `it` counts the tiles this workgroup has walked: buffer it & 1, record slot it & 3.
    auto fetch_rows = [&](const Unit& x, int t, int it) {
        const int nseg_t = min(SPT, x.ns - SPT * t);
        const size_t g0 = (size_t)x.g0 + (size_t)SPT * t;
        if (wave < 2) {
            const int r = min(2 * (wave * 64 + lane), nseg_t * SEG - 2);
            dma16_to_lds(p.rows + g0 * SEG + r,
                         __builtin_amdgcn_readfirstlane(lds_addr(&s_rows[it & 1][0]) + wave * 1024));
        } else if (wave == 2 && lane < nseg_t) {
            dma4_to_lds(p.blk_meta + g0 + lane, __builtin_amdgcn_readfirstlane(lds_addr(&s_meta[it & 3][0])));
        }
    };
    fetch_rows(cur, 0, 0);
    wait_vmcnt<0>();

    // scan state of thread tid < TN (column of the unit's vocabulary tile): running pair of the sequence
    // still open; output column and bias follow the unit
    float run_m = -INFINITY;
    int run_s = 0;
    int v_out = 0;
    float bias_v = 0.f;
    bool head_open = false;
    __syncthreads();

    size_t hoff[DMA ? 1 : IPA];
    uint32_t hoff32[DMA ? IPA : 1];
    auto row_offsets = [&](int buf) {
#pragma unroll
        for (int j = 0; j < IPA; ++j) {
            const size_t o = ((size_t)s_rows[buf][lrow + NW * RPI * j].x * D + gch * 8) * 2;
            if constexpr (DMA) hoff32[j] = (uint32_t)o;
            else hoff[j] = o;
        }
    };
    bool prefetched = false;      // the first slab of the coming tile is already in flight
    for (int it = 0;; ++it) {
        const int buf = it & 1;
        const int t = cur_t;
        const int rc = cur.rc;
        const int nseg = min(SPT, cur.ns - SPT * t);       // live segments of this tile
        const int nact = (nseg + SPB - 1) / SPB;           // live blocks
        const int na = (nact + 1 - wm) >> 1;               // ... of this wave; the others are not multiplied
        const bool unit_ends = t + 1 == cur.n_tiles;
        // the tile after this one: the next of the unit, or the first of this workgroup's next unit
        Unit nxt = cur;
        int nxt_t = t + 1;
        bool has_next = true;
        if (unit_ends) {
            nxt_t = 0;
            if constexpr (RES) has_next = open_unit(cur.u + n_local, nxt);
            else has_next = false;
        }
        if ((RES ? t == 0 : it == 0) && tid < TN) {
            // a unit begins: its output columns and bias; and whether its chunk begins inside a sequence
            // (until that sequence ends, the running pair is a later piece of it)
            v_out = cur.vt * TN + tid;
            bias_v = v_out < p.V ? p.bias[v_out] : 0.f;
            head_open = !(s_meta[it & 3][0] & FWD_META_FIRST);
        }
        // With two stages and an even slab count a tile ends in stage 1, so the first slab of the next
        // tile can be requested into stage 0 from inside the last slab and flies during the epilogue.
        const bool pf_next = DMA && has_next && nk >= 2 && (nk & 1) == 0;
        if (!prefetched) {
            row_offsets(buf);
            if constexpr (RES) w_offsets(cur.vt);
        }
        // next tile's tables: in flight with the first slab, published by the slab loop's barriers
        if (has_next) fetch_rows(nxt, nxt_t, it + 1);

        floatx16 acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][c][r] = 0.f;

        if constexpr (DMA) {
            // Slab kt goes to ring stage kt % NS.  Each wave-wide load fills 1024 contiguous LDS bytes
            // (lane l lands at +16 l); the wave-uniform base goes through M0.
            // load n (0 .. LPT-1) of a slab into ring stage ST: first the A rows, then the B rows; hb and wb
            // are the operand bases already advanced to the slab's K offset (wave-uniform, in SGPRs)
            auto issue_one = [&](auto st, const char* hb, const char* wb, int n) {
                const uint32_t dst = lds_addr(ring(st)) + wave_lds;
                if (n < IPA) dma16_to_lds(hb, hoff32[n], dst + n * JSTEP);
                else dma16_to_lds(wb, woff32[n - IPA], dst + SLAB_A + (n - IPA) * JSTEP);
            };
            auto issue = [&](auto st, int kt) {
                const char* hb = Hb + (size_t)kt * (BK * 2);
                const char* wb = Wb + (size_t)kt * (BK * 2);
#pragma unroll
                for (int n = 0; n < LPT; ++n) issue_one(st, hb, wb, n);
            };
            // The whole slab loop is instantiated once per count NA of live row blocks and the choice is
            // made per tile, outside the loop, so that each instance is straight-line MFMA code.
            auto run_slabs = [&](auto na_c) {
                constexpr int NA = decltype(na_c)::value;
                bf16x8 fa[2][4], fb[2][2];
                // One pipeline step: barrier that publishes slab kt (stage ST), then a slab's worth of
                // MFMAs (see mma_rot) with the loads of slab kt + 1 riding inside them.
                // (NEXT: this is the last slab of the tile and its loads are the first slab of the next
                //  tile, whose row offsets the caller has already put in place)
                auto step = [&](auto st, auto mode_c, auto next_c, int kt) {
                    constexpr int ST = decltype(st)::value;
                    constexpr int MODE = decltype(mode_c)::value;
                    constexpr bool NEXT = decltype(next_c)::value;
                    // every fragment read of the previous slab has returned (its stage is about to be
                    // reloaded by whoever leaves the barrier first) and slab kt has landed
                    __builtin_amdgcn_s_waitcnt(0xC07F);     // lgkmcnt(0)
                    wait_vmcnt<0>();
                    __syncthreads();
                    // one scalar flag and one pair of advanced bases per slab: what is left per load is
                    // a scalar branch, the M0 write and the load itself
                    const int more = __builtin_amdgcn_readfirstlane((NEXT || kt + 1 < nk) ? 1 : 0);
                    const size_t kbytes = (size_t)(NEXT ? 0 : kt + 1) * (BK * 2);
                    const char* hb = Hb + kbytes;
                    const char* wb = Wb + kbytes;
                    auto dma = [&](int n) {
                        if (more != 0) issue_one(std::integral_constant<int, (ST + 1) % NS>{}, hb, wb, n);
                    };
                    if constexpr (NA == 0) {        // no live row block in this wave: only its loads
#pragma unroll
                        for (int n = 0; n < LPT; ++n) dma(n);
                    } else {
                        const uint8_t* sa = ring(st) + fa_row * RB;
                        const uint8_t* sb = ring(st) + SLAB_A + fb_row * RB;
                        mma_rot<NA, KS, MODE, LPT, SPREAD>(sa, A_STRIDE, sb, B_STRIDE, fsw, fa, fb, acc, dma);
                    }
                };
                constexpr std::false_type no{};
                constexpr std::integral_constant<int, 0> first{};
                constexpr std::integral_constant<int, 1> steady{};
                constexpr std::integral_constant<int, 0> st0{};
                constexpr std::integral_constant<int, 1> st1{};
                if (!prefetched) issue(st0, 0);
                step(st0, first, no, 0);
                const int n_end = pf_next ? nk - 1 : nk;      // steady steps without a successor tile: 1 .. n_end-1
                for (int kt = 1; kt < n_end; kt += 2) {
                    step(st1, steady, no, kt);
                    if (kt + 1 < n_end) step(st0, steady, no, kt + 1);
                }
                if (pf_next) {                                // nk is even: slab nk-1 lives in stage 1
                    row_offsets(buf ^ 1);                     // this tile's are no longer needed
                    if constexpr (RES) w_offsets(nxt.vt);
                    step(st1, steady, std::true_type{}, nk - 1);
                }
                if constexpr (NA > 0) {                       // last k-step of the last slab
                    const uint8_t* dummy = ring(st0);
                    mma_rot<NA, KS, 2, LPT, SPREAD>(dummy, A_STRIDE, dummy, B_STRIDE, fsw, fa, fb, acc, [](int) {});
                }
            };
            switch (na) {
                case 4: run_slabs(std::integral_constant<int, 4>{}); break;
                case 3: run_slabs(std::integral_constant<int, 3>{}); break;
                case 2: run_slabs(std::integral_constant<int, 2>{}); break;
                case 1: run_slabs(std::integral_constant<int, 1>{}); break;
                default: run_slabs(std::integral_constant<int, 0>{}); break;
            }
        } else {
            uint4 ra[IPA], rb[IPB];
            // K slabs are full except possibly the last one (D not a multiple of 64): only that one
            // pays for per-chunk predication.
            auto gload = [&](int kt) {
                const int koff = kt * BK;
                if (koff + BK <= D) {
#pragma unroll
                    for (int j = 0; j < IPA; ++j) ra[j] = *reinterpret_cast<const uint4*>(Hb + hoff[j] + koff * 2);
#pragma unroll
                    for (int j = 0; j < IPB; ++j) rb[j] = *reinterpret_cast<const uint4*>(Wb + woff[j] + koff * 2);
                } else {
                    const bool kval = koff + gch * 8 < D;
#pragma unroll
                    for (int j = 0; j < IPA; ++j)
                        ra[j] = kval ? *reinterpret_cast<const uint4*>(Hb + hoff[j] + koff * 2) : make_uint4(0, 0, 0, 0);
#pragma unroll
                    for (int j = 0; j < IPB; ++j)
                        rb[j] = kval ? *reinterpret_cast<const uint4*>(Wb + woff[j] + koff * 2) : make_uint4(0, 0, 0, 0);
                }
            };
            auto lstore = [&](int st) {
#pragma unroll
                for (int j = 0; j < IPA; ++j) *reinterpret_cast<uint4*>(&s_pair[st][st_off + j * JSTEP]) = ra[j];
#pragma unroll
                for (int j = 0; j < IPB; ++j) *reinterpret_cast<uint4*>(&s_pair[st][SLAB_A + st_off + j * JSTEP]) = rb[j];
            };
            gload(0);
            lstore(0);
            __syncthreads();
            for (int kt = 0; kt < nk; ++kt) {
                const int st = kt & 1;
                if (kt + 1 < nk) gload(kt + 1);
                const uint8_t* sa = &s_pair[st][fa_row * RB];
                const uint8_t* sb = &s_pair[st][SLAB_A + fb_row * RB];
                mma_dispatch<KS>(na, sa, A_STRIDE, sb, B_STRIDE, fsw, acc);
                if (kt + 1 < nk) lstore(st ^ 1);
                __syncthreads();
            }
        }

        // ---- epilogue, part 1: every segment of this wave's live blocks -> one (max, position) per column ----
        uint8_t* pm_base;
        if constexpr (SEG == FWD_BLK) pm_base = &s_pm_own[0];
        else if constexpr (DMA) pm_base = &s_ring1[0];
        else pm_base = &s_pair[1][0];
        if constexpr (SEG != FWD_BLK && DMA) {
            // the table lies in ring stage 1.  With an odd slab count the last slab sat in stage 0 and every
            // read of stage 1 ended before that slab's barrier; with an even count the last slab sat in
            // stage 1 itself, and every wave has to be past its fragment reads first
            if ((nk & 1) == 0) __syncthreads();
        }
        float* s_pm = reinterpret_cast<float*>(pm_base);
        int* s_ps = reinterpret_cast<int*>(s_pm) + SPT * TN;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i < na) {
                const int blk = 2 * i + wm;
                float mm[2][SPB];
                int ss[2][SPB];
#pragma unroll
                for (int c = 0; c < 2; ++c) {
#pragma unroll
                    for (int j = 0; j < SPB; ++j) {
                        // rows grow with the register index, and positions with the rows: the first
                        // register that holds the maximum is the lowest position in this lane
                        // the maximum by a chain of three-way maxima, then the first register equal to it
                        const int r0 = j * RPS;
                        float m = acc[i][c][r0];
#pragma unroll
                        for (int r = 1; r < RPS - 1; r += 2)
                            m = __builtin_fmaxf(__builtin_fmaxf(m, acc[i][c][r0 + r]), acc[i][c][r0 + r + 1]);
                        m = __builtin_fmaxf(m, acc[i][c][r0 + RPS - 1]);
                        // e: row of that register within the block, for half-wave 0 (constants per register)
                        int e = acc_row(0, r0 + RPS - 1, 0);
                        if (ARG) {
#pragma unroll
                            for (int r = RPS - 2; r >= 0; --r) e = acc[i][c][r0 + r] == m ? acc_row(0, r0 + r, 0) : e;
                        }
                        mm[c][j] = m;
                        ss[c][j] = ARG ? s_rows[buf][blk * FWD_BLK + half * 4 + e].y : 0;
                    }
                }
                // Half-wave q stores column 32 q + l32, so it needs the other half-wave's pair for column
                // block q only.  One swap of the upper half of the c = 0 register with the lower half of
                // the c = 1 register leaves, in both half-waves, the two candidates of the column the
                // lane stores (own and partner; which is which does not matter to a symmetric choice).
#pragma unroll
                for (int j = 0; j < SPB; ++j) {
                    const auto pm = __builtin_amdgcn_permlane32_swap(__float_as_int(mm[0][j]), __float_as_int(mm[1][j]), false, false);
                    float m = __int_as_float(pm[0]);
                    const float mo = __int_as_float(pm[1]);
                    int sp = 0;
                    if (ARG) {
                        const auto ps = __builtin_amdgcn_permlane32_swap(ss[0][j], ss[1][j], false, false);
                        sp = ps[0];
                        const int so = ps[1];
                        if (mo > m || (mo == m && so < sp)) sp = so;
                    }
                    m = fmaxf(m, mo);
                    const int col = wn * 64 + half * 32 + l32;
                    s_pm[(blk * SPB + j) * TN + col] = m;
                    if (ARG) s_ps[(blk * SPB + j) * TN + col] = sp;
                }
            }
        }
        if (nk < NS) wait_vmcnt<0>();     // the next tile's tables, if the slab loop was too short to wait for them
        __syncthreads();
        prefetched = pf_next;
        // ---- part 2: join the segments of each sequence; finalise (F4) where a sequence ends.  Only
        //      the first TN threads take part; the others go on to the next tile. ----
        if (tid < TN) {
            // all table reads first (the accumulators are dead here, registers are free): the walk over
            // the segments is a dependent chain, and the other four waves wait for it at the next barrier
            float pm[SPT];
            int ps[SPT], mt[SPT];
#pragma unroll
            for (int k = 0; k < SPT; ++k) {
                const bool live = k < nseg;
                pm[k] = live ? s_pm[k * TN + tid] : -INFINITY;
                ps[k] = (ARG && live) ? s_ps[k * TN + tid] : 0;
                mt[k] = live ? s_meta[it & 3][k] : 0;
            }
#pragma unroll
            for (int k = 0; k < SPT; ++k) {
                if (pm[k] > run_m) {              // later segments hold higher positions: strict
                    run_m = pm[k];
                    run_s = ps[k];
                }
                const int meta = mt[k];
                if (meta & FWD_META_LAST) {
                    if (v_out < p.V) {
                        if (head_open) {                    // the sequence began in an earlier chunk
                            const size_t o = (size_t)rc * p.V + v_out;
                            p.part_m[o] = run_m;
                            if (ARG) p.part_s[o] = run_s;
                        } else {
                            const int b = meta & FWD_META_SEQ;
                            const bool any = !(meta & FWD_META_EMPTY);
                            const size_t o = (size_t)b * p.V + v_out;
                            p.Y[o] = any ? log1pf(fmaxf(run_m + bias_v, 0.f)) : 0.f;
                            if (ARG) p.I[o] = any ? run_s : 0;
                        }
                    }
                    head_open = false;
                    run_m = -INFINITY;
                    run_s = 0;
                }
            }
            if (unit_ends) {
                // the chunk may end inside a sequence: leave the open piece for the merge pass
                const int meta = s_meta[it & 3][nseg - 1];
                if (!(meta & FWD_META_LAST) && v_out < p.V) {
                    if (head_open) {                        // one sequence covers the whole chunk
                        const size_t o = (size_t)rc * p.V + v_out;
                        p.part_m[o] = run_m;
                        if (ARG) p.part_s[o] = run_s;
                    } else {
                        const size_t o = (size_t)(meta & FWD_META_SEQ) * p.V + v_out;
                        p.Y[o] = run_m;
                        if (ARG) p.I[o] = run_s;
                    }
                }
                run_m = -INFINITY;
                run_s = 0;
            }
        }
        if (!has_next) break;
        cur = nxt;
        cur_t = nxt_t;
    }
}

}  // namespace lsr
