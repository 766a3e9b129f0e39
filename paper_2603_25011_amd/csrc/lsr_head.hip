// C ABI of the MI355X sparse-lexical LM head: host-side validation, workspace layout and kernel
// launches.  See include/lsr_head.h for the contract of every entry point.
#include "lsr_head.h"
#include "lsr_head_measure.h"

#include <hip/hip_runtime.h>
#include <string.h>

#include <mutex>

#include "bwd.hpp"
#include "fwd_bf16.hpp"
#include "fwd_misc.hpp"
#include "probes.hpp"

// Scratch of lsr_head_forward_static: device memory that lives in the library's code object, one copy
// per GPU, held until the process ends.  In host code this name is only a stand-in for the symbol; the
// device address comes from hipGetSymbolAddress (static_scratch below) and is what every launch uses.
static __device__ __align__(256) unsigned char scratch[LSR_STATIC_SCRATCH_BYTES];

namespace {

using namespace lsr;

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct Shape {
    int B, S, D, V;
    int dtype;
};

int check_desc(const lsr_head_desc* d, Shape* out) {
    if (!d) return LSR_ERR_NULL;
    if (d->hw_dtype != LSR_F32 && d->hw_dtype != LSR_BF16) return LSR_ERR_DTYPE;
    if (d->B < 1 || d->S < 1 || d->D < 1 || d->V < 1) return LSR_ERR_SHAPE;
    if (d->D % 8 != 0 || d->D > 8192 || d->S > 32768 || d->B > 65535) return LSR_ERR_SHAPE;
    if (d->V >= (int64_t(1) << 31) - 4096) return LSR_ERR_SHAPE;      // every factor is bounded before a product is formed
    if (d->B * d->S >= (int64_t(1) << 31) || d->B * d->V >= (int64_t(1) << 31)) return LSR_ERR_SHAPE;
    out->B = (int)d->B; out->S = (int)d->S; out->D = (int)d->D; out->V = (int)d->V;
    out->dtype = d->hw_dtype;
    return LSR_OK;
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Chunks of the packed forward (see fwd_bf16.hpp).  The host does not know the lengths, so it sizes the
// grid and the workspace for the longest block list the shape allows (every sequence full:
// B * ceil(S/32) blocks, 8 per tile); chunks beyond the real list return at once.
// Chunks and launch mode.  A unit of work is (chunk of tiles, vocabulary tile).
// Deep problems launch one workgroup per unit, with chunks of four tiles: a workgroup that walks several
// tiles hides the start of each behind the one before, the hardware hands the next unit to whichever CU
// comes free (which keeps the CUs of an XCD on neighbouring units), and there are enough units that the
// last, partly filled round costs little.  Chunk lengths 1 / 2 / 4 / 8 measured (forward ms): B=16 S=256
// |V|=250002 0.966 / 0.944 / 0.958 / 1.007; B=64 S=512 D=1024 |V|=250002 8.91 / 8.92 / 8.78 / 8.95.
// Shallow problems (fewer than 24 units of one tile per CU; depth is estimated with sequences taken to
// fill 70 % of S) run one resident workgroup per CU over units of one tile each: no unit pays a workgroup
// launch, the next unit's row table and first slab are prefetched like the next tile's, and the last round
// is as full as the unit count allows (B=32 S=256 |V|=30522 and B=256 S=32: -1.5 to -3 %).  On deep problems
// resident workgroups drift apart and lose L2 locality (B=64 S=512 |V|=250002: L2 hit rate 0.82 -> 0.76,
// 16.1 -> 20.8 GB from the fabric, +1 % time), so they are not used there.
// Never more chunks than sequences: the per-chunk slots for cut sequences (8 bytes per vocabulary entry)
// then stay below the size of the outputs Y and I, whatever the sequence length.
// Rows per segment of the packed token list: the MFMA row block, or 8 for batches of short sequences
// (B=256, S=32, lengths 4..32: 8192 packed rows with 32-row segments, 5 400 with 8-row segments).
int fwd_seg(const Shape& s) { return s.S <= FWD_SEG_SHORT_MAX_S ? FWD_SEG_SHORT : FWD_BLK; }

struct FwdChunks { int tpc, n_chunks; bool cut_possible, resident; };
FwdChunks fwd_chunks(const Shape& s) {
    const int seg = fwd_seg(s);
    const long segs_max = (long)s.B * ((s.S + seg - 1) / seg);
    const long tiles_max = (segs_max * seg + FWD_TM - 1) / FWD_TM;
    FwdChunks c;
    const double units1 = 0.7 * (double)tiles_max * (double)((s.V + 255) / 256) / 256.0;      // per workgroup at one tile per chunk
    c.resident = units1 < 24.0;
    c.tpc = c.resident ? 1 : 4;
    const long per_seq = (tiles_max + s.B - 1) / s.B;
    if (c.tpc < per_seq) c.tpc = (int)per_seq;
    c.n_chunks = (int)((tiles_max + c.tpc - 1) / c.tpc);
    // a sequence of one segment can never lie across a chunk boundary: no pieces, no merge pass
    c.cut_possible = s.S > seg && c.n_chunks > 1;
    return c;
}

// ---- forward workspace: len[B] | pos[B*S] | seg0[B+1] | seg_meta[segs] | rows[segs*seg] |
//      part_m[chunks*V] | part_s[chunks*V]; segs = B * ceil(S/seg) being the most the packed layout can
//      need, the two part arrays only where a chunk boundary can fall inside a sequence ----
struct FwdWs { size_t len_off, pos_off, blk0_off, meta_off, rows_off, pm_off, ps_off, total; };
FwdWs fwd_ws(const Shape& s) {
    FwdWs w;
    const int seg = fwd_seg(s);
    const size_t blocks = (size_t)s.B * ((s.S + seg - 1) / seg);          // segments
    const FwdChunks c = fwd_chunks(s);
    const size_t part = (s.dtype == LSR_BF16 && c.cut_possible) ? align_up(sizeof(float) * (size_t)c.n_chunks * s.V) : 0;
    w.len_off = 0;
    w.pos_off = w.len_off + align_up(sizeof(int) * (size_t)s.B);
    w.blk0_off = w.pos_off + align_up(sizeof(int) * (size_t)s.B * s.S);
    w.meta_off = w.blk0_off + align_up(sizeof(int) * ((size_t)s.B + 1));
    w.rows_off = w.meta_off + align_up(sizeof(int) * blocks);
    w.pm_off = w.rows_off + align_up(sizeof(int2) * blocks * seg);
    w.ps_off = w.pm_off + part;
    w.total = w.ps_off + part;
    return w;
}

// ---- backward workspace: perm[B*V + PERM_SLACK] (v, g) pairs | cnt[B*n_seg*S] | bstart[B*(S+1)] |
//      bounds[B*S*(n_vc+1)] (only when the dH gather is cut into n_vc > 1 vocabulary chunks) ----
struct BwdWs { int n_seg, seg_len, key_bits, n_vc, vc_len; size_t perm_off, cnt_off, bs_off, cb_off, dh_stage_off, dw_stage_off, total; };

// Vocabulary chunks of the sliced dH gather.  A chunk is sized so that one 64-column slice of its
// rows of W is about 4 MB (what stays in L2 while every bucket gathers from it).  Each chunk after
// the first re-reads and re-writes dH once (8*B*S*D bytes), so the count is capped where that
// traffic would pass a quarter of the gather traffic itself (B*|V|*D elements): long sequences
// with few entries per bucket are gathered in one pass.
void dh_chunks(const Shape& s, int* n_vc, int* vc_len) {
    const long esize = s.dtype == LSR_F32 ? 4 : 2;
    const long rows_l2 = (4l << 20) / (DWS_COLS * esize);
    long c = (s.V + rows_l2 - 1) / rows_l2;
    const long cap = (long)s.V * esize / (32l * s.S);
    if (c > cap) c = cap;
    if (c > 64) c = 64;
    if (c < 1 || s.D % DWS_COLS != 0) c = 1;
    *n_vc = (int)c;
    *vc_len = (int)((s.V + c - 1) / c);
}
int dw_batch_chunk(const Shape& s);
int dw_tile_rows(const Shape& s);
// bf16_out: dH and dW are stored as bfloat16.  A result that several launches add up (dH over vocabulary
// chunks, dW over chunks of sequences) then keeps its float32 partial sums in a staging array of the
// workspace and is rounded once, by the last launch.
BwdWs bwd_ws(const Shape& s, bool bf16_out = false) {
    BwdWs w;
    // enough (b, segment) waves to fill the chip, segments of at least 512 entries, and a count
    // table no larger than B*V ints
    long n = 4096 / s.B;
    n = n < s.V / 512 ? n : s.V / 512;
    // short enough segments for the placement that sorts a segment in LDS, where it applies
    if (s.S <= PLACE_MAX_S) {
        const long fit = (s.V + PLACE_MAX_SEG - 129) / (PLACE_MAX_SEG - 128);
        n = n > fit ? n : fit;
    }
    n = n < s.V / s.S ? n : s.V / s.S;
    if (n < 1) n = 1;
    w.n_seg = (int)n;
    w.seg_len = ((s.V + w.n_seg - 1) / w.n_seg + 63) / 64 * 64;
    w.n_seg = (s.V + w.seg_len - 1) / w.seg_len;
    w.key_bits = 0;
    while ((1 << w.key_bits) < s.S) ++w.key_bits;
    const size_t bv = (size_t)s.B * s.V;
    w.perm_off = 0;
    w.cnt_off = w.perm_off + align_up(sizeof(uint2) * (bv + PERM_SLACK));
    w.bs_off = w.cnt_off + align_up(sizeof(int) * (size_t)s.B * w.n_seg * s.S);
    w.cb_off = w.bs_off + align_up(sizeof(int) * (size_t)s.B * (s.S + 1));
    dh_chunks(s, &w.n_vc, &w.vc_len);
    w.dh_stage_off = w.cb_off + (w.n_vc > 1 ? align_up(sizeof(int) * (size_t)s.B * s.S * (w.n_vc + 1)) : 0);
    w.dw_stage_off = w.dh_stage_off + ((bf16_out && w.n_vc > 1) ? align_up(sizeof(float) * (size_t)s.B * s.S * s.D) : 0);
    const bool dw_multi = dw_tile_rows(s) > 0 && dw_batch_chunk(s) < s.B;
    w.total = w.dw_stage_off + ((bf16_out && dw_multi) ? align_up(sizeof(float) * (size_t)s.V * s.D) : 0);
    return w;
}

// Buckets a wave of the sliced dH gather serves.  The lanes of a bucket load its entries in blocks of as many
// entries as the bucket has lanes (64 / k), two rounds of gathers per block.  Several buckets per wave pay
// off when a bucket holds too few entries per chunk to keep a wave busy for several blocks, and cost when
// their lists differ in length.  Lengths are not known on the host: sequences are taken to fill 70 % of S
// and every (b, v) pair to carry a gradient.  Measured (dH ms for k = 1 / 2 / 4 / 8; entries per bucket and
// chunk as estimated here, and as they really were): B=16 S=256 |V|=250002 (174; 217) 0.65 / 0.78 / 1.07 / -;
// B=64 S=512 |V|=250002, lengths 128..512 (87; 98) 2.93 / 2.32 / 2.41 / 3.5; B=256 S=512 |V|=30522, full
// lengths (85; 60) 0.91 / 0.75 / 0.79 / 0.90; B=256 S=512 |V|=250002, full lengths (87; 61) 9.3 / 8.0 / 7.7 /
// 8.6; B=128 S=8192 |V|=30522 (5; 4) 4.4 / 2.4 / 1.55 / 1.37.
int dh_buckets_per_wave(const Shape& s, int n_vc) {
    const double per_bucket = (double)s.V / ((0.7 * s.S > 1.0 ? 0.7 * s.S : 1.0) * n_vc);
    int bpw = per_bucket >= 128.0 ? 1 : (per_bucket >= 48.0 ? 2 : (per_bucket >= 12.0 ? 4 : 8));
    if (s.dtype == LSR_F32 && bpw > 4) bpw = 4;      // a float row piece takes 16 lanes
    return bpw;
}

// Sequences per launch of the sliced dW gather.  The gather is L2-resident while the H slice of the
// sequences in flight (rows x 64 columns) is about 4 MB; larger batches are cut into chunks of
// consecutive sequences, each launch adding to dW (8*|V|*D bytes re-read and re-written per extra
// launch, capped at a quarter of the gather traffic and at 16 launches).  B=256, S=512, |V|=250002:
// dW 14.5 ms in one launch of 16-row tiles (16.8 MB slice).
int dw_batch_chunk(const Shape& s) {
    const long esize = s.dtype == LSR_F32 ? 4 : 2;
    const long per_seq = (long)s.S * DWS_COLS * esize;
    long bc = (4l << 20) / per_seq;
    bc = bc < 1 ? 1 : bc;
    long n = (s.B + bc - 1) / bc;
    const long cap = 1 + (long)s.B * esize / 32;
    n = n > cap ? cap : n;
    n = n > 16 ? 16 : n;
    if ((long)s.V < 16l * s.S) n = 1;      // a row of H is gathered about |V|/S times: too few for L2 to matter
    n = n < 1 ? 1 : n;
    return (int)((s.B + n - 1) / n);
}

// Vocabulary rows of the (g, I) staging tile of the sliced dW gather (at most 48 KiB of LDS for the
// sequences of one launch), or 0 when the whole-row kernel runs instead (D not a multiple of 64, or
// too many sequences per launch for 16 rows).
int dw_tile_rows(const Shape& s) {
    const int nb = dw_batch_chunk(s);
    int VT = 64;
    while (VT > 1 && (size_t)nb * VT * 8 > 48 * 1024) VT /= 2;
    return (s.D % DWS_COLS == 0 && VT >= 16) ? VT : 0;
}

int check_device(int* n_cus) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return LSR_ERR_ARCH; }
    static int ok_dev[64] = {0};     // holds the CU count once a device has been checked
    if (dev >= 0 && dev < 64 && ok_dev[dev]) { *n_cus = ok_dev[dev]; return LSR_OK; }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return LSR_ERR_ARCH; }
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return LSR_ERR_ARCH;
    if (prop.multiProcessorCount < 1) return LSR_ERR_ARCH;
    *n_cus = prop.multiProcessorCount;
    if (dev >= 0 && dev < 64) ok_dev[dev] = prop.multiProcessorCount;
    return LSR_OK;
}

// Device address of `scratch` on the current device, looked up once per device with that device
// current (every GPU holds its own copy at its own address).
int static_scratch(void** out) {
    static std::mutex mu;
    static void* ptr_of[64] = {nullptr};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { (void)hipGetLastError(); return LSR_ERR_ARCH; }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return LSR_ERR_LAUNCH; }
        ptr_of[dev] = p;
    }
    *out = ptr_of[dev];
    return LSR_OK;
}

// Optional per-kernel event timing (the *_profiled entry points).
struct Prof {
    bool on = false;
    hipStream_t stream = nullptr;
    hipEvent_t ev[LSR_PROFILE_SLOTS][2];
    bool used[LSR_PROFILE_SLOTS] = {false};
    bool fail = false;
    void begin(int slot) {
        if (!on) return;
        if (hipEventCreate(&ev[slot][0]) != hipSuccess || hipEventCreate(&ev[slot][1]) != hipSuccess) { fail = true; return; }
        used[slot] = true;
        if (hipEventRecord(ev[slot][0], stream) != hipSuccess) fail = true;
    }
    void end(int slot) {
        if (!on || !used[slot]) return;
        if (hipEventRecord(ev[slot][1], stream) != hipSuccess) fail = true;
    }
    int finish(float* ms) {
        if (!on) return LSR_OK;
        if (hipStreamSynchronize(stream) != hipSuccess) fail = true;
        for (int i = 0; i < LSR_PROFILE_SLOTS; ++i) {
            ms[i] = 0.f;
            if (used[i]) {
                if (!fail && hipEventElapsedTime(&ms[i], ev[i][0], ev[i][1]) != hipSuccess) fail = true;
                (void)hipEventDestroy(ev[i][0]);
                (void)hipEventDestroy(ev[i][1]);
            }
        }
        return fail ? LSR_ERR_LAUNCH : LSR_OK;
    }
};

inline int launch_status() { return hipGetLastError() == hipSuccess ? LSR_OK : LSR_ERR_LAUNCH; }

// Kernel choice: the direct-to-LDS ring when D is a multiple of the 64-wide K slab and H and W are
// each below 4 GiB (32-bit byte offsets per lane), else the register-staged loader (64-bit addresses,
// zero-fills the last slab).
template <bool DMA, int SEG, bool RES>
void launch_fwd_cfg(FwdParams p, int V, bool arg, int n_cus, hipStream_t st) {
    constexpr int TN = fwd_tn(FWD_NWN);
    p.n_vtiles = (V + TN - 1) / TN;
    p.gv = FWD_GV_COLS / TN;
    // RES: one resident workgroup per CU (its LDS leaves room for no second one), a multiple of 8 so that
    // every XCD gets the same number.  Otherwise one workgroup per unit the longest possible token list
    // would need (workgroups beyond the real list return at once).
    const long long n_units = (long long)((p.n_vtiles + p.gv - 1) / p.gv) * p.gv * p.n_chunks;
    const int n_wg = RES ? (n_cus >= 8 ? n_cus / 8 * 8 : 8) : (int)((n_units + 7) / 8 * 8);
    const dim3 grid(n_wg), block(fwd_threads(FWD_NWN));
    if (arg) hipLaunchKernelGGL((fwd_bf16_kernel<true, DMA, SEG, RES>), grid, block, 0, st, p);
    else     hipLaunchKernelGGL((fwd_bf16_kernel<false, DMA, SEG, RES>), grid, block, 0, st, p);
}

void launch_fwd_bf16(const FwdParams& p, int seg, bool resident, bool arg, int n_cus, hipStream_t st) {
    const bool small = (size_t)p.B * p.S * p.D * 2 < ((size_t)1 << 32) && (size_t)p.V * p.D * 2 < ((size_t)1 << 32);
    const bool dma = p.D % 64 == 0 && small;
    if (!dma) {          // the register-staged loader has no prefetch across units to gain from
        if (seg == FWD_BLK) launch_fwd_cfg<false, FWD_BLK, false>(p, p.V, arg, n_cus, st);
        else launch_fwd_cfg<false, FWD_SEG_SHORT, false>(p, p.V, arg, n_cus, st);
    } else if (seg == FWD_BLK) {
        if (resident) launch_fwd_cfg<true, FWD_BLK, true>(p, p.V, arg, n_cus, st);
        else launch_fwd_cfg<true, FWD_BLK, false>(p, p.V, arg, n_cus, st);
    } else {
        if (resident) launch_fwd_cfg<true, FWD_SEG_SHORT, true>(p, p.V, arg, n_cus, st);
        else launch_fwd_cfg<true, FWD_SEG_SHORT, false>(p, p.V, arg, n_cus, st);
    }
}

int forward_impl(const lsr_head_desc* desc, const void* H, const void* W, const float* bias,
                 const uint8_t* mask, float* Y, int32_t* I, void* ws, size_t ws_bytes, hipStream_t st,
                 Prof& prof) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc != LSR_OK) return rc;
    if (!H || !W || !bias || !mask || !Y) return LSR_ERR_NULL;
    if (misaligned(H) || misaligned(W) || misaligned(bias) || misaligned(Y) || (I && misaligned(I)) || misaligned(ws))
        return LSR_ERR_ALIGN;
    const FwdWs w = fwd_ws(s);
    if (!ws || ws_bytes < w.total) return LSR_ERR_WORKSPACE;
    int n_cus = 0;
    rc = check_device(&n_cus);
    if (rc != LSR_OK) return rc;

    prof.stream = st;
    int* len = reinterpret_cast<int*>(static_cast<char*>(ws) + w.len_off);
    int* pos = reinterpret_cast<int*>(static_cast<char*>(ws) + w.pos_off);

    prof.begin(0);
    // batches of few tokens are packed by one workgroup in one launch (bf16 path)
    const bool one_launch = s.dtype == LSR_BF16 && s.B <= PACK_MAX_B && (long)s.B * s.S <= PACK_MAX_TOKENS;
    if (!one_launch) hipLaunchKernelGGL(fwd_prep_kernel, dim3(s.B), dim3(PREP_THREADS), 0, st, mask, len, pos, s.S);
    char* base = static_cast<char*>(ws);
    int* blk0 = reinterpret_cast<int*>(base + w.blk0_off);
    int* blk_meta = reinterpret_cast<int*>(base + w.meta_off);
    int2* rows = reinterpret_cast<int2*>(base + w.rows_off);
    float* part_m = reinterpret_cast<float*>(base + w.pm_off);
    int* part_s = reinterpret_cast<int*>(base + w.ps_off);
    const FwdChunks ck = fwd_chunks(s);
    const int seg = fwd_seg(s);
    if (one_launch) {
        hipLaunchKernelGGL(fwd_pack_kernel, dim3(1), dim3(PACK_THREADS), 0, st, mask, len, pos, blk0, rows, blk_meta, s.B, s.S, seg);
    } else if (s.dtype == LSR_BF16) {
        hipLaunchKernelGGL(fwd_plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, st, len, blk0, s.B, seg);
        hipLaunchKernelGGL(fwd_rows_kernel, dim3(s.B), dim3(FWD_ROWS_THREADS), 0, st, len, pos, blk0, rows, blk_meta, s.S, seg);
    }
    prof.end(0);
    if ((rc = launch_status()) != LSR_OK) return rc;

    prof.begin(1);
    if (s.dtype == LSR_F32) {
        dim3 grid((s.V + F32_THREADS - 1) / F32_THREADS, s.B);
        if (I) hipLaunchKernelGGL((fwd_f32_kernel<true>), grid, dim3(F32_THREADS), 0, st,
                                  static_cast<const float*>(H), static_cast<const float*>(W), bias, len, pos, Y, I, s.S, s.D, s.V);
        else   hipLaunchKernelGGL((fwd_f32_kernel<false>), grid, dim3(F32_THREADS), 0, st,
                                  static_cast<const float*>(H), static_cast<const float*>(W), bias, len, pos, Y, I, s.S, s.D, s.V);
    } else {
        FwdParams p;
        p.H = static_cast<const uint16_t*>(H);
        p.W = static_cast<const uint16_t*>(W);
        p.bias = bias; p.rows = rows; p.blk_meta = blk_meta; p.n_blocks = blk0 + s.B; p.Y = Y; p.I = I;
        p.part_m = part_m; p.part_s = part_s;
        p.B = s.B; p.S = s.S; p.D = s.D; p.V = s.V;
        p.n_chunks = ck.n_chunks; p.tpc = ck.tpc;
        launch_fwd_bf16(p, seg, ck.resident, I != nullptr, n_cus, st);
    }
    prof.end(1);
    if (s.dtype == LSR_BF16 && ck.cut_possible) {
        if ((rc = launch_status()) != LSR_OK) return rc;
        prof.begin(2);
        const dim3 grid((s.V + FWD_MERGE_THREADS - 1) / FWD_MERGE_THREADS, ck.n_chunks < FWD_MERGE_ROWS ? ck.n_chunks : FWD_MERGE_ROWS);
        if (I) hipLaunchKernelGGL((fwd_merge_kernel<true>), grid, dim3(FWD_MERGE_THREADS), 0, st, blk0, blk_meta, part_m, part_s,
                                  bias, Y, I, s.B, s.V, ck.tpc, FWD_TM / seg);
        else   hipLaunchKernelGGL((fwd_merge_kernel<false>), grid, dim3(FWD_MERGE_THREADS), 0, st, blk0, blk_meta, part_m, part_s,
                                  bias, Y, I, s.B, s.V, ck.tpc, FWD_TM / seg);
        prof.end(2);
    }
    return launch_status();
}

template <typename T, typename OT>
void launch_dh(int cpt, dim3 grid, hipStream_t st, const T* W, const int* bstart, const uint2* pm,
               OT* dH, int S, int D, int V, int accumulate) {
    switch (cpt) {
        case 1: hipLaunchKernelGGL((bwd_dh_kernel<T, 1, OT>), grid, dim3(ROW_THREADS), 0, st, W, bstart, pm, dH, S, D, V, accumulate); break;
        case 2: hipLaunchKernelGGL((bwd_dh_kernel<T, 2, OT>), grid, dim3(ROW_THREADS), 0, st, W, bstart, pm, dH, S, D, V, accumulate); break;
        case 4: hipLaunchKernelGGL((bwd_dh_kernel<T, 4, OT>), grid, dim3(ROW_THREADS), 0, st, W, bstart, pm, dH, S, D, V, accumulate); break;
        case 8: hipLaunchKernelGGL((bwd_dh_kernel<T, 8, OT>), grid, dim3(ROW_THREADS), 0, st, W, bstart, pm, dH, S, D, V, accumulate); break;
        default: hipLaunchKernelGGL((bwd_dh_kernel<T, 16, OT>), grid, dim3(ROW_THREADS), 0, st, W, bstart, pm, dH, S, D, V, accumulate); break;
    }
}

template <typename T, typename OT>
void launch_dw(int cpt, dim3 grid, size_t lds, hipStream_t st, const T* H, const float* dY, const float* Y, const int* I,
               OT* dW, float* db, int B, int S, int D, int V, int VT, int accumulate) {
    switch (cpt) {
        case 1: hipLaunchKernelGGL((bwd_dw_kernel<T, 1, OT>), grid, dim3(ROW_THREADS), lds, st, H, dY, Y, I, dW, db, B, S, D, V, VT, accumulate); break;
        case 2: hipLaunchKernelGGL((bwd_dw_kernel<T, 2, OT>), grid, dim3(ROW_THREADS), lds, st, H, dY, Y, I, dW, db, B, S, D, V, VT, accumulate); break;
        case 4: hipLaunchKernelGGL((bwd_dw_kernel<T, 4, OT>), grid, dim3(ROW_THREADS), lds, st, H, dY, Y, I, dW, db, B, S, D, V, VT, accumulate); break;
        case 8: hipLaunchKernelGGL((bwd_dw_kernel<T, 8, OT>), grid, dim3(ROW_THREADS), lds, st, H, dY, Y, I, dW, db, B, S, D, V, VT, accumulate); break;
        default: hipLaunchKernelGGL((bwd_dw_kernel<T, 16, OT>), grid, dim3(ROW_THREADS), lds, st, H, dY, Y, I, dW, db, B, S, D, V, VT, accumulate); break;
    }
}

// One launch of the sliced dH gather (vocabulary chunk vc) / of the sliced dW gather (sequences b0 .. b0+nb-1).
template <typename T, typename OT>
void launch_dh_sliced(int bpw, dim3 grid, hipStream_t st, const T* W, const int* bounds, const uint2* perm, const float* prev,
                      OT* dst, int add_dst, int write_all, const Shape& s, int n_groups, int n_vc, int vc, bool xcd_own) {
    // 32-bit byte offsets into W (one multiply-add of 24-bit factors per gather) where W allows them
    const bool off32 = (size_t)s.V * s.D * sizeof(T) <= 0xffffffffull && s.V <= (1 << 24) && (size_t)s.D * sizeof(T) < (1u << 24);
#define LSR_DH2(BPW, O32) hipLaunchKernelGGL((bwd_dh_sliced_kernel<T, BPW, OT, O32>), grid, dim3(256), 0, st, W, bounds, perm, prev, dst, \
                                             add_dst, write_all, s.B, s.S, s.D, s.V, n_groups, n_vc, vc, xcd_own ? 1 : 0)
#define LSR_DH(BPW) do { if (off32) LSR_DH2(BPW, true); else LSR_DH2(BPW, false); } while (0)
    if (bpw == 1) LSR_DH(1);
    else if (bpw == 2) LSR_DH(2);
    else if (bpw == 4 || sizeof(T) == 4) LSR_DH(4);      // a float row piece takes 16 lanes: at most four buckets per wave
    else if constexpr (sizeof(T) == 2) LSR_DH(8);
#undef LSR_DH
#undef LSR_DH2
}
template <typename T, typename OT>
void launch_dw_sliced(bool compact, dim3 grid, dim3 block, size_t lds, hipStream_t st, const T* H, const float* dY, const float* Y,
                      const int* I, const float* prev, OT* dst, int add_dst, float* db, int add_db, int b0, int nb, const Shape& s,
                      int VT, int n_vtiles, int NDC) {
    if (compact)
        hipLaunchKernelGGL((bwd_dw_sliced_kernel<T, true, OT>), grid, block, lds, st, H, dY, Y, I, prev, dst, add_dst, db, add_db, b0, nb,
                           s.S, s.D, s.V, VT, n_vtiles, NDC);
    else
        hipLaunchKernelGGL((bwd_dw_sliced_kernel<T, false, OT>), grid, block, lds, st, H, dY, Y, I, prev, dst, add_dst, db, add_db, b0, nb,
                           s.S, s.D, s.V, VT, n_vtiles, NDC);
}

// The dW/db gather does not depend on the bucket sort that feeds dH, so the plain (not profiled)
// backward can run it on an auxiliary stream beside the dH chain: fork after the caller's prior
// work, join before returning control of the caller's stream.  Measured: the overlap shortens the
// backward while the gathers are small (B=256 S=32 |V|=30522: 0.42 -> 0.30 ms; B=16 S=256
// |V|=250002: 1.56 -> 1.47 ms) and lengthens it once they stream tens of GB (B=64 S=512
// |V|=250002: 7.2 -> 7.7 ms, the two kernels evict each other's L2-resident slices), so it is used
// up to AUX_MAX_GATHER_BYTES of worst-case gather traffic (2 * B * |V| rows of D elements).
//
// The lane (one stream, one fork and one join event per device, default priority, non-blocking with
// respect to the null stream) is created by the first backward on that device and kept until the
// process ends.  It is shared by every caller on the device, so a call holds the lane's mutex from the
// record of the fork event to the wait on the join event: the three enqueue steps that name the
// shared events (record fork on the caller's stream, wait for it on the lane, ... record join on the
// lane, wait for it on the caller's stream) can then not interleave with another host thread's, and
// a wait always refers to the record made by the same call (a stream wait binds to the event's most
// recent record at the time of the wait call).  Only enqueueing is serialised; the device work of
// two callers still overlaps as their streams allow, except that their dW gathers share one lane.
constexpr double AUX_MAX_GATHER_BYTES = 16e9;
struct AuxLane {
    std::mutex mu;
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool ready = false;
};
AuxLane* aux_lane_of_current_device() {
    static AuxLane lanes[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { (void)hipGetLastError(); return nullptr; }
    return &lanes[dev];
}
// Holds the lane from fork to join.  forked() is false when the lane could not be used; the caller
// then runs everything on its own stream.
class AuxFork {
public:
    AuxFork(AuxLane* lane, hipStream_t main) : main_(main) {
        if (!lane) return;
        lock_ = std::unique_lock<std::mutex>(lane->mu);
        if (!lane->ready) {
            if (hipStreamCreateWithFlags(&lane->stream, hipStreamNonBlocking) != hipSuccess ||
                hipEventCreateWithFlags(&lane->fork, hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&lane->join, hipEventDisableTiming) != hipSuccess) {
                (void)hipGetLastError();
                lock_.unlock();
                return;
            }
            lane->ready = true;
        }
        if (hipEventRecord(lane->fork, main) != hipSuccess || hipStreamWaitEvent(lane->stream, lane->fork, 0) != hipSuccess) {
            (void)hipGetLastError();
            lock_.unlock();
            return;
        }
        lane_ = lane;
    }
    bool forked() const { return lane_ != nullptr; }
    hipStream_t side() const { return lane_ ? lane_->stream : main_; }
    // Joins the lane back into the caller's stream; called on every path once forked, errors included,
    // so that the caller's stream (possibly one that is being captured) is never left with an open fork.
    int join() {
        if (!lane_) return LSR_OK;
        const bool ok = hipEventRecord(lane_->join, lane_->stream) == hipSuccess &&
                        hipStreamWaitEvent(main_, lane_->join, 0) == hipSuccess;
        if (!ok) (void)hipGetLastError();
        lane_ = nullptr;
        lock_.unlock();
        return ok ? LSR_OK : LSR_ERR_LAUNCH;
    }
    ~AuxFork() { (void)join(); }
private:
    hipStream_t main_;
    AuxLane* lane_ = nullptr;
    std::unique_lock<std::mutex> lock_;
};

// Everything the backward launches is decided here, from the shape alone, before anything is enqueued.
struct BwdLaunch {
    int cpt;                 // 16-byte chunks per thread of the whole-row kernels
    bool staged_place;       // the bucket sort places through LDS
    bool dh_sliced;          // column-sliced dH gather (D a multiple of 64)
    int bpw, dh_groups;      // buckets per wave and workgroups per slice of the sliced dH gather
    int dw_vt;               // rows of the dW staging tile: sliced gather if dw_sliced, else whole-row kernel
    bool dw_sliced;
    int dw_bc, dw_ndc, dw_slice_groups, dw_vtiles;
    bool dh_xcd_own;         // sliced dH gather: column slices owned by XCDs
    int dw_tile_passes;      // LDS-tile dW kernel: copy passes per tile (ceil(S / 128)), or 0 when it does not apply
    int dw_tile_vtiles;
};
// The sliced dH gather with its column slices owned by XCDs (xcd_slice_unit).  In the slice-major order every
// XCD fetches the slice's window of W for itself and sees one eighth of its reuse, which is B / 8 gathers
// per row and vocabulary chunk; owned slices pay off while that is small.  Measured (dH, slice-major ->
// owned): B=8 S=512 |V|=30522 0.062 -> 0.047 ms; B=16 S=256 |V|=250002 0.88 -> 0.73; B=32 S=256 |V|=250002
// 1.06 -> 1.01; from B=32 at D=1024 on it loses (B=32 1.45 -> 1.67, B=64 S=512 2.65 -> 3.1: fewer L2 misses
// but a slower kernel; the slice-major order happens to keep every sequence's bucket lists on one XCD).
bool dh_slices_owned(const Shape& s) { return s.B <= 16; }
// The LDS-tile dW kernel (bwd_dw_tile_kernel): bfloat16, D a multiple of 64, S within the tile, and at least
// one workgroup per CU of a 256-CU device.  Measured against the sliced gather (dW): B=64 S=512 D=1024
// |V|=250002 1.98 -> 1.72 ms; B=256 S=512 D=768 |V|=250002 7.84 -> 5.43; B=16 S=256 |V|=250002 0.407 ->
// 0.363; B=256 S=512 |V|=30522 1.02 -> 0.94; B=8 S=512 |V|=30522 0.0445 -> 0.0463; 60 workgroups (D=128,
// |V|=30522) 0.030 -> 0.052.
int dw_tile_passes(const Shape& s) {
    if (s.dtype != LSR_BF16 || s.D % DWS_COLS != 0 || s.S < DWT_MIN_S || s.S > DWT_MAX_S) return 0;
    if (s.V > (1 << 28)) return 0;                       // the kernel keeps byte offsets within a row of dY / Y / I in 32 bits
    const long long units = (long long)((s.V + DWT_ROWS - 1) / DWT_ROWS) * (s.D / DWS_COLS);
    if (units < 256 || units > 0x7fffffffll) return 0;
    return (s.S + 127) / 128;
}
int plan_backward(const Shape& s, const BwdWs& w, BwdLaunch* L) {
    const int chunk_elems = s.dtype == LSR_F32 ? 4 : 8;
    const int n_chunks = s.D / chunk_elems;
    L->cpt = 1;
    while (L->cpt * ROW_THREADS < n_chunks) L->cpt *= 2;
    L->staged_place = s.S <= PLACE_MAX_S && w.seg_len <= PLACE_MAX_SEG;      // plan[3] of lsr_head_plan
    L->dh_sliced = s.D % DWS_COLS == 0;
    L->bpw = L->dh_sliced ? dh_buckets_per_wave(s, w.n_vc) : 0;
    L->dh_groups = L->dh_sliced ? s.B * ((s.S + 4 * L->bpw - 1) / (4 * L->bpw)) : 0;
    if ((long long)L->dh_groups * (s.D / DWS_COLS) > 0x7fffffffll) return LSR_ERR_SHAPE;
    L->dh_xcd_own = L->dh_sliced && dh_slices_owned(s);
    if (L->dh_xcd_own && xcd_slice_grid(s.D / DWS_COLS, L->dh_groups, 1) > 0x7fffffffll) return LSR_ERR_SHAPE;
    L->dw_tile_passes = dw_tile_passes(s);
    L->dw_tile_vtiles = (s.V + DWT_ROWS - 1) / DWT_ROWS;
    // column-sliced dW gathers (L2-resident slices of H) need D % 64 == 0 and a (g, I) staging tile (at
    // most 48 KiB) at least 16 vocabulary rows wide, i.e. at most 384 sequences per launch.  Larger
    // batches keep the whole-row kernel, which also skips zero gradients.
    L->dw_vt = dw_tile_rows(s);
    L->dw_sliced = L->dw_vt > 0;
    L->dw_bc = dw_batch_chunk(s);
    if (L->dw_sliced) {
        // slices per group: a workgroup walks the slices of its group with one staging of (g, I), and
        // the groups run one after the other.  Up to 9 MiB of H rows per group measured best (C5: two
        // 4 MiB slices, dW 2.21 -> 2.02 ms; C3 0.22 -> 0.175; 3 per group at C5 2.11, all 16: 2.48):
        // fewer stagings against a wider window of H in flight.
        const int n_dc = s.D / DWS_COLS;
        const size_t slice_bytes = (size_t)L->dw_bc * s.S * DWS_COLS * (s.dtype == LSR_F32 ? 4 : 2);
        int ndc = (int)((size_t)(9u << 20) / slice_bytes);
        L->dw_ndc = ndc < 1 ? 1 : (ndc > n_dc ? n_dc : ndc);
        L->dw_slice_groups = (n_dc + L->dw_ndc - 1) / L->dw_ndc;
        L->dw_vtiles = (s.V + L->dw_vt - 1) / L->dw_vt;
        if ((long long)L->dw_vtiles * L->dw_slice_groups > 0x7fffffffll) return LSR_ERR_SHAPE;
    } else {
        // whole-row gathers; rows of the (g, I) staging tile: as wide as 48 KiB of LDS allows, at most 32
        int VT = 32;
        while (VT > 1 && (size_t)s.B * VT * 8 > 48 * 1024) VT /= 2;
        L->dw_vt = VT;
        L->dw_ndc = L->dw_slice_groups = 0;
        L->dw_vtiles = (s.V + VT - 1) / VT;
    }
    return LSR_OK;
}

// The whole backward for element types T (H, W) and OT (dH, dW), after every check.
template <typename T, typename OT>
int backward_launches(const Shape& s, const BwdWs& w, const BwdLaunch& L, const T* H, const T* W, const float* dY, const float* Y,
                      const int32_t* I, OT* dH, OT* dW, float* db, int accumulate, char* base, hipStream_t st, hipStream_t st_dw,
                      Prof& prof);

int backward_impl(const lsr_head_desc* desc, const void* H, const void* W, const float* dY, const float* Y,
                  const int32_t* I, void* dH, void* dW, float* db, const lsr_backward_opts* opts, void* ws, size_t ws_bytes,
                  hipStream_t st, Prof& prof) {
    Shape s;
    int rc = check_desc(desc, &s);
    if (rc != LSR_OK) return rc;
    const int grad_dtype = opts ? opts->grad_dtype : LSR_F32;
    const int accumulate = (opts && opts->accumulate) ? 1 : 0;
    if (grad_dtype != LSR_F32 && grad_dtype != LSR_BF16) return LSR_ERR_DTYPE;
    if (grad_dtype == LSR_BF16 && s.dtype != LSR_BF16) return LSR_ERR_DTYPE;      // bfloat16 gradients belong to bfloat16 parameters
    const bool bf16_out = grad_dtype == LSR_BF16;
    if (!H || !W || !dY || !Y || !I) return LSR_ERR_NULL;
    if (misaligned(H) || misaligned(W) || misaligned(dY) || misaligned(Y) || misaligned(I) || misaligned(ws) ||
        (dH && misaligned(dH)) || (dW && misaligned(dW)) || (db && misaligned(db)))
        return LSR_ERR_ALIGN;
    if (s.S > 8192 || s.B > 6144) return LSR_ERR_SHAPE;      // LDS tables of the bucket sort / dW staging
    const BwdWs w = bwd_ws(s, bf16_out);
    if (!ws || ws_bytes < w.total) return LSR_ERR_WORKSPACE;
    BwdLaunch L;
    if ((rc = plan_backward(s, w, &L)) != LSR_OK) return rc;
    int n_cus = 0;
    rc = check_device(&n_cus);
    if (rc != LSR_OK) return rc;
    // ---- nothing has been enqueued up to here; every check is behind us ----

    prof.stream = st;
    char* base = static_cast<char*>(ws);

    // fork: dW/db on the auxiliary stream, the dH chain on the caller's
    const double gather_bytes = 2.0 * s.B * s.V * s.D * (s.dtype == LSR_F32 ? 4 : 2);
    const bool overlap = !prof.on && dH && (dW || db) && gather_bytes <= AUX_MAX_GATHER_BYTES;
    AuxFork lane(overlap ? aux_lane_of_current_device() : nullptr, st);
    const hipStream_t st_dw = lane.side();

    // A failed launch ends the sequence; the join below still runs.
    if (s.dtype == LSR_F32)
        rc = backward_launches<float, float>(s, w, L, static_cast<const float*>(H), static_cast<const float*>(W), dY, Y, I,
                                             static_cast<float*>(dH), static_cast<float*>(dW), db, accumulate, base, st, st_dw, prof);
    else if (!bf16_out)
        rc = backward_launches<uint16_t, float>(s, w, L, static_cast<const uint16_t*>(H), static_cast<const uint16_t*>(W), dY, Y, I,
                                                static_cast<float*>(dH), static_cast<float*>(dW), db, accumulate, base, st, st_dw, prof);
    else
        rc = backward_launches<uint16_t, uint16_t>(s, w, L, static_cast<const uint16_t*>(H), static_cast<const uint16_t*>(W), dY, Y, I,
                                                   static_cast<uint16_t*>(dH), static_cast<uint16_t*>(dW), db, accumulate, base, st,
                                                   st_dw, prof);
    const int rj = lane.join();
    return rc != LSR_OK ? rc : rj;
}

template <typename T, typename OT>
int backward_launches(const Shape& s, const BwdWs& w, const BwdLaunch& L, const T* H, const T* W, const float* dY, const float* Y,
                      const int32_t* I, OT* dH, OT* dW, float* db, int accumulate, char* base, hipStream_t st, hipStream_t st_dw,
                      Prof& prof) {
    constexpr bool OUT_F32 = sizeof(OT) == 4;
    uint2* perm = reinterpret_cast<uint2*>(base + w.perm_off);
    int* cnt = reinterpret_cast<int*>(base + w.cnt_off);
    int* bstart = reinterpret_cast<int*>(base + w.bs_off);
    int r;
    if (dH) {
        const dim3 seg_grid(w.n_seg, s.B);
        prof.begin(0);
        hipLaunchKernelGGL(bwd_count_kernel, seg_grid, dim3(256), sizeof(int) * s.S, st, dY, Y, I, cnt, s.S, s.V, w.n_seg, w.seg_len);
        prof.end(0);
        if ((r = launch_status()) != LSR_OK) return r;
        prof.begin(1);
        hipLaunchKernelGGL(bwd_scan_kernel, dim3(s.B), dim3(256), sizeof(int) * (s.S + 256), st, cnt, bstart, s.S, w.n_seg);
        prof.end(1);
        if ((r = launch_status()) != LSR_OK) return r;
        prof.begin(2);
        if (L.staged_place)
            hipLaunchKernelGGL(bwd_place_staged_kernel, seg_grid, dim3(256), sizeof(int) * 2 * s.S + sizeof(uint2) * w.seg_len, st,
                               dY, Y, I, cnt, bstart, perm, s.S, s.V, w.n_seg, w.seg_len, w.key_bits);
        else
            hipLaunchKernelGGL(bwd_place_kernel, seg_grid, dim3(64), sizeof(int) * s.S, st, dY, Y, I, cnt, bstart, perm,
                               s.S, s.V, w.n_seg, w.seg_len, w.key_bits);
        prof.end(2);
        if ((r = launch_status()) != LSR_OK) return r;
        prof.begin(3);
        if (L.dh_sliced) {
            // column-sliced gathers, one launch per vocabulary chunk: the rows of W in use stay in L2
            const int* bounds = bstart;
            if (w.n_vc > 1) {
                int* cb = reinterpret_cast<int*>(base + w.cb_off);
                const long long n = (long long)s.B * s.S * (w.n_vc + 1);
                hipLaunchKernelGGL(bwd_chunk_bounds_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, bstart, perm, cb,
                                   s.B * s.S, s.S, s.V, w.n_vc, w.vc_len);
                bounds = cb;
            }
            const dim3 grid(L.dh_xcd_own ? (unsigned)xcd_slice_grid(s.D / DWS_COLS, L.dh_groups, 1)
                                         : (unsigned)L.dh_groups * (unsigned)(s.D / DWS_COLS));
            float* stage = reinterpret_cast<float*>(base + w.dh_stage_off);
            for (int vc = 0; vc < w.n_vc; ++vc) {
                const bool last = vc + 1 == w.n_vc;
                if (OUT_F32) {
                    // partial sums live in dH itself; the first chunk of a fresh result writes every bucket
                    float* d = reinterpret_cast<float*>(dH);
                    const bool fresh = vc == 0 && !accumulate;
                    launch_dh_sliced<T, float>(L.bpw, grid, st, W, bounds, perm, fresh ? nullptr : d, d, 0, fresh ? 1 : 0, s, L.dh_groups,
                                               w.n_vc, vc, L.dh_xcd_own);
                } else if (w.n_vc == 1) {
                    launch_dh_sliced<T, OT>(L.bpw, grid, st, W, bounds, perm, nullptr, dH, accumulate, accumulate ? 0 : 1, s, L.dh_groups,
                                            w.n_vc, vc, L.dh_xcd_own);
                } else if (!last) {
                    launch_dh_sliced<T, float>(L.bpw, grid, st, W, bounds, perm, vc > 0 ? stage : nullptr, stage, 0, vc == 0 ? 1 : 0, s,
                                               L.dh_groups, w.n_vc, vc, L.dh_xcd_own);
                } else {
                    launch_dh_sliced<T, OT>(L.bpw, grid, st, W, bounds, perm, stage, dH, accumulate, 1, s, L.dh_groups, w.n_vc, vc, L.dh_xcd_own);
                }
            }
        } else {
            launch_dh<T, OT>(L.cpt, dim3(s.B, s.S), st, W, bstart, perm, dH, s.S, s.D, s.V, accumulate);
        }
        prof.end(3);
        if ((r = launch_status()) != LSR_OK) return r;
    }
    if (dW || db) {
        prof.begin(4);
        const int VT = L.dw_vt;
        if (L.dw_tile_passes > 0 && dW) {
            // one launch for all sequences; the sums start from zero, so bfloat16 results need no staging
            if constexpr (sizeof(T) == 2) {
                const dim3 grid((unsigned)L.dw_tile_vtiles * (unsigned)(s.D / DWS_COLS));
#define LSR_DWT(NP) hipLaunchKernelGGL((bwd_dw_tile_kernel<OT, NP>), grid, dim3(DWT_ROWS), 0, st_dw, H, dY, Y, I, dW, accumulate, db, \
                                       accumulate, s.B, s.S, s.D, s.V, L.dw_tile_vtiles)
                switch (L.dw_tile_passes) {
                    case 1: LSR_DWT(1); break;
                    case 2: LSR_DWT(2); break;
                    case 3: LSR_DWT(3); break;
                    default: LSR_DWT(4); break;
                }
#undef LSR_DWT
            }
        } else if (L.dw_sliced) {
            // four waves also where the tile has fewer row groups than that (16 rows of bf16: two): the
            // others still share the staging and the compaction (C3: dW 0.264 -> 0.222 ms)
            const int waves = 4;
            const int bc = L.dw_bc;                            // sequences per launch
            const size_t lds = (size_t)bc * VT * 8;
            const dim3 grid((unsigned)L.dw_vtiles * (unsigned)L.dw_slice_groups), block(64 * waves);
            float* stage = reinterpret_cast<float*>(base + w.dw_stage_off);
            const bool compact = VT < 32;      // tiles of 16 rows (more than 192 sequences per launch) compact their columns first
            for (int b0 = 0; b0 < s.B; b0 += bc) {
                const int nb = s.B - b0 < bc ? s.B - b0 : bc;
                const bool first = b0 == 0, last = b0 + bc >= s.B;
                const int add_db = (!first || accumulate) ? 1 : 0;
                if (OUT_F32) {
                    float* d = reinterpret_cast<float*>(dW);
                    launch_dw_sliced<T, float>(compact, grid, block, lds, st_dw, H, dY, Y, I, (!first || accumulate) ? d : nullptr, d, 0, db,
                                               add_db, b0, nb, s, VT, L.dw_vtiles, L.dw_ndc);
                } else if (first && last) {
                    launch_dw_sliced<T, OT>(compact, grid, block, lds, st_dw, H, dY, Y, I, nullptr, dW, accumulate, db, add_db, b0, nb, s, VT,
                                            L.dw_vtiles, L.dw_ndc);
                } else if (!last) {
                    launch_dw_sliced<T, float>(compact, grid, block, lds, st_dw, H, dY, Y, I, first ? nullptr : stage, dW ? stage : nullptr, 0,
                                               db, add_db, b0, nb, s, VT, L.dw_vtiles, L.dw_ndc);
                } else {
                    launch_dw_sliced<T, OT>(compact, grid, block, lds, st_dw, H, dY, Y, I, stage, dW, accumulate, db, add_db, b0, nb, s, VT,
                                            L.dw_vtiles, L.dw_ndc);
                }
            }
        } else {
            const size_t lds = (size_t)s.B * VT * 8;
            launch_dw<T, OT>(L.cpt, dim3(L.dw_vtiles), lds, st_dw, H, dY, Y, I, dW, db, s.B, s.S, s.D, s.V, VT, accumulate);
        }
        prof.end(4);
        if ((r = launch_status()) != LSR_OK) return r;
    }
    return LSR_OK;
}

// Runs `launch` `launches` times on st and returns the duration of the last one in ms (< 0 on error).
template <typename F>
float time_last_launch(int launches, hipStream_t st, F&& launch) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) { (void)hipGetLastError(); return -1.f; }
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipGetLastError(); (void)hipEventDestroy(e0); return -1.f; }
    bool ok = true;
    for (int l = 0; l < launches && ok; ++l) {
        const bool timed = l + 1 == launches;
        if (timed) ok = hipEventRecord(e0, st) == hipSuccess;
        launch();
        ok = ok && hipGetLastError() == hipSuccess;
        if (timed) ok = ok && hipEventRecord(e1, st) == hipSuccess;
    }
    float ms = -1.f;
    ok = ok && hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (!ok) { (void)hipGetLastError(); return -1.f; }
    return ms;
}

}  // namespace

extern "C" {

size_t lsr_head_workspace_bytes(const lsr_head_desc* desc, int for_backward) {
    Shape s;
    if (check_desc(desc, &s) != LSR_OK) return 0;
    return for_backward ? bwd_ws(s).total : fwd_ws(s).total;
}

int lsr_head_forward(const lsr_head_desc* desc, const void* H, const void* W, const float* bias, const uint8_t* mask,
                     float* Y, int32_t* I, void* workspace, size_t workspace_bytes, lsr_stream_t stream) {
    Prof prof;
    return forward_impl(desc, H, W, bias, mask, Y, I, workspace, workspace_bytes, stream, prof);
}

int lsr_head_forward_static(const lsr_head_desc* desc, const void* H, const void* W, const float* bias,
                            const uint8_t* mask, float* Y, int32_t* I, lsr_stream_t stream) {
    Shape s;
    const int rc = check_desc(desc, &s);
    if (rc != LSR_OK) return rc;
    if (fwd_ws(s).total > (size_t)LSR_STATIC_SCRATCH_BYTES) return LSR_ERR_STATIC_SCRATCH;
    int n_cus = 0;
    const int rd = check_device(&n_cus);      // a usable gfx950 device is current before its symbol is looked up
    if (rd != LSR_OK) return rd;
    void* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs != LSR_OK) return rs;
    // Every word of the scratch that a kernel reads has been written earlier in the same call (lengths,
    // position lists, block tables), so nothing has to be cleared between calls.
    Prof prof;
    return forward_impl(desc, H, W, bias, mask, Y, I, ws, (size_t)LSR_STATIC_SCRATCH_BYTES, stream, prof);
}

int lsr_head_backward(const lsr_head_desc* desc, const void* H, const void* W, const float* dY, const float* Y,
                      const int32_t* I, float* dH, float* dW, float* db, void* workspace, size_t workspace_bytes,
                      lsr_stream_t stream) {
    Prof prof;
    return backward_impl(desc, H, W, dY, Y, I, dH, dW, db, nullptr, workspace, workspace_bytes, stream, prof);
}

size_t lsr_head_backward_ex_workspace_bytes(const lsr_head_desc* desc, const lsr_backward_opts* opts) {
    Shape s;
    if (check_desc(desc, &s) != LSR_OK) return 0;
    const int grad_dtype = opts ? opts->grad_dtype : LSR_F32;
    if (grad_dtype != LSR_F32 && !(grad_dtype == LSR_BF16 && s.dtype == LSR_BF16)) return 0;
    return bwd_ws(s, grad_dtype == LSR_BF16).total;
}

int lsr_head_backward_ex(const lsr_head_desc* desc, const void* H, const void* W, const float* dY, const float* Y,
                         const int32_t* I, void* dH, void* dW, float* db, const lsr_backward_opts* opts, void* workspace,
                         size_t workspace_bytes, lsr_stream_t stream) {
    Prof prof;
    return backward_impl(desc, H, W, dY, Y, I, dH, dW, db, opts, workspace, workspace_bytes, stream, prof);
}

int lsr_head_forward_profiled(const lsr_head_desc* desc, const void* H, const void* W, const float* bias,
                              const uint8_t* mask, float* Y, int32_t* I, void* workspace, size_t workspace_bytes,
                              lsr_stream_t stream, float* kernel_ms) {
    if (!kernel_ms) return LSR_ERR_NULL;
    Prof prof;
    prof.on = true;
    const int rc = forward_impl(desc, H, W, bias, mask, Y, I, workspace, workspace_bytes, stream, prof);
    const int rc2 = prof.finish(kernel_ms);
    return rc != LSR_OK ? rc : rc2;
}

int lsr_head_backward_profiled(const lsr_head_desc* desc, const void* H, const void* W, const float* dY,
                               const float* Y, const int32_t* I, float* dH, float* dW, float* db, void* workspace,
                               size_t workspace_bytes, lsr_stream_t stream, float* kernel_ms) {
    if (!kernel_ms) return LSR_ERR_NULL;
    Prof prof;
    prof.on = true;
    const int rc = backward_impl(desc, H, W, dY, Y, I, dH, dW, db, nullptr, workspace, workspace_bytes, stream, prof);
    const int rc2 = prof.finish(kernel_ms);
    return rc != LSR_OK ? rc : rc2;
}

int lsr_mfma_peak_probe(int64_t iters, int launches, void* sink, double* tflops, lsr_stream_t stream) {
    if (!sink || !tflops) return LSR_ERR_NULL;
    if (iters < 1 || iters > (1 << 24) || launches < 1 || launches > 64) return LSR_ERR_SHAPE;
    int n_cus = 0;
    int rc = check_device(&n_cus);
    if (rc != LSR_OK) return rc;
    hipStream_t st = stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) { (void)hipGetLastError(); return LSR_ERR_LAUNCH; }
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipGetLastError(); (void)hipEventDestroy(e0); return LSR_ERR_LAUNCH; }
    // two workgroups of four waves per CU: two waves on every SIMD, each with four independent MFMA chains
    const dim3 grid(2 * n_cus);
    float ms = 0.f;
    bool ok = true;
    for (int l = 0; l < launches && ok; ++l) {        // the last launch is the one that is timed
        const bool timed = l + 1 == launches;
        if (timed) ok = hipEventRecord(e0, st) == hipSuccess;
        hipLaunchKernelGGL(mfma_probe_kernel, grid, dim3(PROBE_THREADS), 0, st, (int)iters, static_cast<float*>(sink));
        ok = ok && hipGetLastError() == hipSuccess;
        if (timed) ok = ok && hipEventRecord(e1, st) == hipSuccess;
    }
    ok = ok && hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (!ok || ms <= 0.f) { (void)hipGetLastError(); return LSR_ERR_LAUNCH; }
    const double flops = 2.0 * 32 * 32 * 16 * PROBE_MFMA_PER_ITER * (double)iters * (PROBE_THREADS / 64) * grid.x;
    *tflops = flops / (ms * 1e-3) / 1e12;
    return LSR_OK;
}

int lsr_copy_probe(void* dst, const void* src, size_t bytes, int launches, double* gbytes_per_s, lsr_stream_t stream) {
    if (!dst || !src || !gbytes_per_s) return LSR_ERR_NULL;
    if (misaligned(dst) || misaligned(src)) return LSR_ERR_ALIGN;
    if (bytes < 16 || bytes % 16 != 0 || launches < 1 || launches > 64) return LSR_ERR_SHAPE;
    int n_cus = 0;
    const int rc = check_device(&n_cus);
    if (rc != LSR_OK) return rc;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + COPY_THREADS - 1) / COPY_THREADS;
    const size_t cap = (size_t)n_cus * 32;            // grid-stride loop over a grid that fills the chip a few times
    if (blocks > cap) blocks = cap;
    const float ms = time_last_launch(launches, stream, [&] {
        hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)blocks), dim3(COPY_THREADS), 0, stream, static_cast<uint4*>(dst),
                           static_cast<const uint4*>(src), n16);
    });
    if (ms <= 0.f) return LSR_ERR_LAUNCH;
    *gbytes_per_s = 2.0 * (double)bytes / (ms * 1e-3) / 1e9;      // bytes read + bytes written
    return LSR_OK;
}

int lsr_gather_probe(const void* table, size_t window_bytes, int steps, int launches, void* out, size_t out_bytes,
                     double* gbytes_per_s, lsr_stream_t stream) {
    if (!table || !out || !gbytes_per_s) return LSR_ERR_NULL;
    if (misaligned(table) || misaligned(out)) return LSR_ERR_ALIGN;
    if (window_bytes < 128 || window_bytes % 128 != 0 || window_bytes > ((size_t)1 << 38) || steps < 1 || steps > (1 << 20) ||
        launches < 1 || launches > 64)
        return LSR_ERR_SHAPE;
    int n_cus = 0;
    const int rc = check_device(&n_cus);
    if (rc != LSR_OK) return rc;
    const unsigned blocks = (unsigned)n_cus * 16;                // eight waves resident per SIMD's worth of work in flight
    const size_t groups = (size_t)blocks * GATHER_THREADS / 8;
    if (out_bytes < groups * 8 * 8 * sizeof(float)) return LSR_ERR_WORKSPACE;
    const uint32_t rows = (uint32_t)(window_bytes / 128);
    const float ms = time_last_launch(launches, stream, [&] {
        hipLaunchKernelGGL(gather_probe_kernel, dim3(blocks), dim3(GATHER_THREADS), 0, stream, static_cast<const uint16_t*>(table),
                           rows, steps, static_cast<float*>(out));
    });
    if (ms <= 0.f) return LSR_ERR_LAUNCH;
    *gbytes_per_s = (double)groups * steps * GATHER_NLD * 128.0 / (ms * 1e-3) / 1e9;
    return LSR_OK;
}

int lsr_head_plan(const lsr_head_desc* desc, int32_t* plan) {
    Shape s;
    const int rc = check_desc(desc, &s);
    if (rc != LSR_OK) return rc;
    if (!plan) return LSR_ERR_NULL;
    const BwdWs w = bwd_ws(s);
    plan[0] = fwd_chunks(s).tpc;
    plan[1] = w.n_seg;
    plan[2] = w.seg_len;
    plan[3] = (s.S <= PLACE_MAX_S && w.seg_len <= PLACE_MAX_SEG) ? 1 : 0;
    plan[4] = w.n_vc;
    plan[5] = w.vc_len;
    plan[6] = s.D % DWS_COLS == 0 ? dh_buckets_per_wave(s, w.n_vc) : 0;
    plan[7] = dw_tile_rows(s);
    plan[8] = dw_batch_chunk(s);
    plan[9] = fwd_chunks(s).n_chunks;
    plan[10] = fwd_seg(s);
    plan[11] = fwd_chunks(s).resident ? 1 : 0;
    plan[12] = (s.D % DWS_COLS == 0 && dh_slices_owned(s)) ? 1 : 0;
    plan[13] = dw_tile_passes(s);
    return LSR_OK;
}

const char* lsr_status_string(int status) {
    switch (status) {
        case LSR_OK: return "ok";
        case LSR_ERR_NULL: return "a required pointer is NULL";
        case LSR_ERR_SHAPE: return "shape outside the supported range";
        case LSR_ERR_DTYPE: return "unknown hw_dtype";
        case LSR_ERR_ALIGN: return "pointer not 16-byte aligned";
        case LSR_ERR_WORKSPACE: return "workspace missing or too small";
        case LSR_ERR_ARCH: return "no gfx950 device";
        case LSR_ERR_LAUNCH: return "HIP launch or event error";
        case LSR_ERR_STATIC_SCRATCH: return "shape needs more scratch than the static array of lsr_head_forward_static holds";
        default: return "unknown status";
    }
}

}  // extern "C"
