// Exact attention forward for gfx950 (MI355X): kernels and the C ABI of include/fa.h.
//
// Dataflow (FastAttention appendix A, the FlashAttention2 forward): for each block of
// queries, walk the key/value blocks once; per block compute the logits on the matrix
// cores, exponentiate against a running reference, multiply by V on the matrix cores,
// and carry the reference / row sum.  Mask handling follows section 4.1: blocks that are
// entirely masked are skipped, blocks that are entirely visible take no mask, and only the
// others get a per-element predicate computed from indices -- no mask tensor exists.
//
// What is in this file:
//  * fa_fwd_kernel -- the attention kernel, one source for every variant (template flags):
//    WIDE (256 query rows per workgroup, all eight waves walk the same tiles) or split (128 rows,
//    two groups of four waves on alternate tiles, merged through LDS); CAUSAL; SPLITKV (one run of
//    the key tiles per workgroup, unnormalised result to a workspace); GENMASK (window / prefix /
//    key-count masks from a descriptor).  Entry points fa_fwd, fa_fwd_splitkv, fa_fwd_masked.
//  * fa_combine_kernel -- merges the split-KV runs.
//  * fa_linear_kernel -- the output projection that follows the attention block by block
//    (section 4.2), entry points fa_attn_linear_block / fa_attn_linear.
//  * the host side: argument checks, choice of decomposition, launch shapes, and the
//    host-callable copies of the scheduling logic (fa_fwd_plan, fa_mask_*).
//
// gfx950 mapping common to all variants (this file's own design):
//  * one wavefront owns 32 query rows; a workgroup is 8 wavefronts, two per SIMD.  A wavefront
//    cannot issue vector work while its own matrix instruction runs, so overlap of the matrix
//    and vector units comes from the two wavefronts of a SIMD being in different phases; they
//    run free between the one workgroup barrier per tile.
//  * logits are produced TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16: keys on the
//    M side (A operand, read from LDS with ds_read_b128), queries on the N side (B
//    operand, held in registers for the whole kernel).  A lane then owns ONE query
//    column, so row max / row sum are in-lane reductions plus a single cross-half
//    exchange (v_permlane32_swap), and the exponentiated tile is already in the
//    B-operand register layout of the second product O^T = V^T P^T (no shuffle, no LDS
//    round trip -- the MFMA counterpart of the paper's appendix-B layout converter).
//  * V^T fragments come straight out of the row-major V tile with the transposing LDS
//    read ds_read_b64_tr_b16.
//  * K and V tiles (64 keys) go from global memory straight into LDS (global_load_lds),
//    double-buffered (three-deep for split-KV), bank-swizzled on the global side.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <type_traits>
#include <utility>

#include "../../include/fa.h"

namespace {

typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

struct FaParams {
    const uint16_t *q, *k, *v;
    uint16_t *o;
    float *lse;
    int H, Nq, Nk;
    int q_rows;     // rows between consecutive heads of q, o, lse in memory (>= Nq: the call may cover a row range)
    int kv_rows;    // same for k, v (>= Nk)
    int off;        // causal / window diagonal: row i of this launch sits on key i + off
    int nqt;        // query tiles per (b,h)
    int nwork;      // B*H*nqt
    int per_xcd;    // ceil(nwork / 8)
    float c;        // |scale| * log2(e), or 1 when scale == 0
    int qmode;      // 0: use q as is, 1: negate q (scale < 0), 2: zero q (scale == 0)
    // split-KV only: the keys of every query block are cut into nsplit runs of tiles, one
    // workgroup each (blockIdx.y); a workgroup leaves its unnormalised accumulator, exponent
    // reference and row sum here for the combine kernel
    int nsplit;
    float *part_o;  // [nsplit][B*H*Nq][D]
    float *part_ml; // [nsplit][B*H*Nq][2]: reference (log2 units), row sum relative to it
    // descriptor masks only (see MaskGeom): window limits with "no limit" already replaced by
    // MASK_NO_LIMIT, the prefix clamped to Nk, per-batch key counts or nullptr
    int left, right, prefix;
    const int *kv_len;
};

// ---- masks generated from a descriptor (section 4.1's generator beyond the triangular case).
// Row i of a batch entry with klen valid keys sees key j iff
//     j < pfx  or  ( i + off - left <= j <= min(klen - 1, i + off + right) ),
// with off = Nk - Nq and pfx = min(prefix, klen).  The kernel never evaluates this per element
// unless it has to: per wave (32 rows) and 64-key tile it first classifies the tile, exactly the
// three cases of section 4.1 -- nothing visible: skipped; everything visible: no mask work;
// otherwise: the predicate per element.  Shared by the kernel and the host-side entry points
// that expose it to tests.
constexpr int MASK_NO_LIMIT = 1 << 30;   // window limit standing for "none" (needs Nq + Nk < 2^30)
struct MaskGeom {
    int off, left, right, pfx, klen;
};
enum { TILE_SKIP = 0, TILE_FULL = 1, TILE_PARTIAL = 2 };

// Classification of 64-key tile t for rows r0..r1 (r0 <= r1), reduced to comparisons of t against
// limits that depend on the rows only (computed once per wave): with k0 = 64 t,
//   some key in a window   <=>  k0 <= r1 + off + right  and  k0 + 63 >= r0 + off - left
//   every key in every window <=> k0 >= r1 + off - left  and  k0 + 63 <= r0 + off + right
//   some / every key in the prefix <=> k0 < pfx  /  k0 + 63 < pfx;   every key exists <=> k0 + 63 < klen
// (x >> 6 is the floor of x / 64 for negative x too).  TILE_SKIP and TILE_FULL are only returned
// when they are certain; TILE_PARTIAL may be returned for a tile that is in fact all visible or all
// masked.
struct RowTiles {
    int any_lo, any_hi;     // tiles any_lo..any_hi hold a key of some row's window
    int all_lo, all_hi;     // tiles all_lo..all_hi lie inside every row's window
    int pfx_any, pfx_all;   // tiles below pfx_any hold a prefix key, tiles below pfx_all only prefix keys
    int exist_any, exist_all;   // tiles below exist_any hold an existing key, below exist_all only existing keys
};
__host__ __device__ inline RowTiles row_tiles(const MaskGeom &g, int r0, int r1) {
    RowTiles w;
    w.any_lo = (r0 + g.off - g.left) >> 6;
    w.any_hi = (r1 + g.off + g.right) >> 6;
    if (r0 + g.off - g.left >= g.klen) w.any_hi = w.any_lo - 1;   // every window starts in the padding: none
    w.all_lo = (r1 + g.off - g.left + 63) >> 6;
    w.all_hi = (r0 + g.off + g.right - 63) >> 6;
    w.pfx_any = (g.pfx + 63) >> 6;
    w.pfx_all = g.pfx >> 6;
    w.exist_any = (g.klen + 63) >> 6;
    w.exist_all = g.klen >> 6;
    return w;
}
__host__ __device__ inline int tile_class(const RowTiles &w, int t) {
    if (t >= w.exist_any) return TILE_SKIP;
    if (!(t < w.pfx_any) && !(t >= w.any_lo && t <= w.any_hi)) return TILE_SKIP;
    if (t < w.exist_all && (t < w.pfx_all || (t >= w.all_lo && t <= w.all_hi))) return TILE_FULL;
    return TILE_PARTIAL;
}

// The tiles a workgroup owning rows R0..R1 walks: the prefix tiles 0 .. np-1, then the cw = count - np
// consecutive tiles base .. base+cw-1 that the rows' windows touch; when the two runs touch or overlap
// they are one run from tile 0.  A window run that does not start at tile 0 is walked ROTATED: it starts
// at tile base + rot and wraps around, with rot chosen so that the tile at window position i is
// congruent to i modulo cw.  Neighbouring query blocks' windows are a few tiles apart; walked in
// ascending order they would read the same tile a few iterations apart, and the co-resident
// workgroups of a head would keep that head's whole K/V cycling through the L2; rotated, they read
// the same tile in the same iteration.  (The order of the tiles does not matter to the result.)  Runs
// shorter than 32 tiles are left in order: their footprint is small anyway, and the wrap cuts the
// check-free run in two, of which only the longer is used.
// Position j of the walk is tile (j < np ? j : base + ((j - np + rot) mod cw)).
struct TileSeq {
    int np, base, count, rot;
    __host__ __device__ int tile(int j) const {
        if (j < np) return j;
        int i = j - np + rot;
        const int cw = count - np;
        if (i >= cw) i -= cw;
        return base + i;
    }
};
__host__ __device__ inline TileSeq tile_sequence(const MaskGeom &g, int R0, int R1) {
    constexpr int BNK = 64;
    const int p_t = (g.pfx + BNK - 1) / BNK;
    const int lo_key = max(0, R0 + g.off - g.left);
    const int hi_key = min(g.klen - 1, R1 + g.off + g.right);
    if (hi_key < lo_key) return {p_t, 0, p_t, 0};
    const int w_lo = lo_key / BNK, w_hi = hi_key / BNK;
    if (w_lo <= p_t) return {0, 0, max(p_t, w_hi + 1), 0};
    const int cw = w_hi - w_lo + 1;
    return {p_t, w_lo, p_t + cw, cw >= 32 ? (cw - w_lo % cw) % cw : 0};
}

// Folded row assignment (causal, few rounds of workgroups; kernel variant PAIR).  A head's rows are cut
// into 8 G blocks of 32 rows (G = workgroups per head); block i needs about i/2 + 1 key tiles.
// Workgroup g owns the four blocks 4g .. 4g+3 from the cheap end and their mirror images 8G-1-4g-j
// from the expensive end, so every workgroup carries the same amount of triangular work.  Wave w < 4
// takes cheap block 4g + w, and wave w + 4 -- the wave it shares a SIMD with -- the mirror image of it.
// All four SIMDs of a workgroup then hold the same kind of pair: the waves meet at a barrier per tile,
// so an iteration costs what its busiest SIMD costs, and with like pairs no SIMD is still running two
// waves after the others have dropped to one.  (Dealing one block of every eighth of the sequence to
// each workgroup balances the work just as well but mixes pairs of 4+32 ... 16+20 tiles in one
// workgroup: measured 8% slower, before the finished waves were put to work.)
__host__ __device__ inline int fold_block(int G, int g, int w) {
    return w < 4 ? 4 * g + w : 8 * G - 1 - 4 * g - (w - 4);
}

// The run of positions [first, first + count) of a workgroup's walk that a wave (row limits w) can
// take without any check: every tile of the run is TILE_FULL for the wave, and the tile at the
// next position exists in the walk and lies wholly inside K/V (it is loaded unconditionally).
// `first` and `count` are even (the two tile buffers alternate).  Of the two candidates -- the
// tiles inside every row's window, the tiles made of prefix keys only -- the longer one.
struct Run {
    int first, count;
};
__host__ __device__ inline Run interior_run(const RowTiles &w, const TileSeq &sq, int Nk) {
    const int phys = Nk / 64 - 2;                     // last tile t such that tile t+1 is wholly inside K/V
    const int cw = sq.count - sq.np;                  // tiles of the window part
    // window candidate: tiles f0..f1 inclusive, inside the window part of the walk
    const int f0 = max(w.all_lo, sq.np > 0 ? sq.base : 0);
    const int f1 = min(min(w.all_hi, w.exist_all - 1), min(phys, sq.base + cw - 1));
    int a0 = 0, a1 = 0;                               // their positions [a0, a1)
    if (f1 >= f0) {
        const int ts = sq.base + sq.rot;              // the tile the window part starts with
        // tiles ts .. come first, in order; tiles base .. ts-1 follow after the wrap, in order
        const int hi0 = max(f0, ts), lo1 = min(f1, ts - 1);
        const int len_hi = f1 - hi0 + 1, len_lo = lo1 - f0 + 1;
        const int pos_hi = sq.np + hi0 - ts, pos_lo = sq.np + (cw - sq.rot) + (f0 - sq.base);
        if (len_hi > 0 && len_lo > 0 && f1 == sq.base + cw - 1 && f0 == sq.base) {
            a0 = pos_hi;                              // the two pieces meet at the wrap: one run
            a1 = pos_hi + len_hi + len_lo;
        } else if (len_hi >= len_lo) {
            a0 = pos_hi;
            a1 = pos_hi + max(len_hi, 0);
        } else {
            a0 = pos_lo;
            a1 = pos_lo + len_lo;
        }
    }
    a1 = min(a1, sq.count - 1);
    // prefix candidate: positions = tiles 0 .. p1-1
    int p1 = min(min(w.pfx_all, w.exist_all), phys + 1);
    p1 = min(p1, (sq.np > 0 ? sq.np : sq.count) - 1);
    Run r = {0, 0};
    a0 = (a0 + 1) & ~1;
    if (a1 - a0 >= 2) r = {a0, (a1 - a0) & ~1};
    if (p1 >= 2 && (p1 & ~1) > r.count) r = {0, p1 & ~1};
    return r;
}

constexpr int BN = 64;  // keys per tile

template <int DT>
__device__ __forceinline__ f32x16 mfma32(s16x8 a, s16x8 b, f32x16 c) {
    if constexpr (DT == FA_DTYPE_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// two fp32 -> two 16-bit values of the storage type (round to nearest even), packed in 32 bits
template <int DT>
__device__ __forceinline__ s16x2 pack2(float a, float b) {
    f32x2 x = {a, b};
    if constexpr (DT == FA_DTYPE_F16)
        return __builtin_bit_cast(s16x2, __builtin_convertvector(x, f16x2));
    else
        return __builtin_bit_cast(s16x2, __builtin_convertvector(x, bf16x2));
}

// LDS byte offset of 16-byte chunk c of K-tile row r.  The XOR spreads the 16 rows that
// one quarter-wave reads at the same chunk index over all 64 banks.
template <int D>
__device__ __forceinline__ int k_lds_off(int r, int c) {
    if constexpr (D == 128)
        return r * 256 + ((c ^ (r & 15)) << 4);
    else
        return r * 128 + ((c ^ ((r >> 1) & 7)) << 4);
}

// LDS byte offset of byte b (of the row's D*2) of V-tile row r.  The transposing read
// fetches, per half-wave, 4 consecutive rows x 64 bytes: the XOR puts those four 64-byte
// pieces into four different bank groups.
template <int D>
__device__ __forceinline__ int v_lds_off(int r, int b) {
    if constexpr (D == 128)
        return r * 256 + (b ^ ((r & 3) << 6));
    else
        return r * 128 + (b ^ (((r >> 1) & 1) << 6));
}

// v_permlane32_swap exchanges the upper 32 lanes of its first operand with the lower 32
// lanes of its second: fed the same value twice it returns {lo,lo} and {hi,hi}, i.e. every
// lane sees both halves' values of its column.  (The two results are copied to scalars
// before the bit cast: a bit cast applied directly to an element of the returned vector
// reads element 0 whatever the index.)
__device__ __forceinline__ void xhalf_both(float x, float &lo, float &hi) {
    const unsigned a = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    lo = __builtin_bit_cast(float, r0);
    hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float xhalf_max(float x) {
    float lo, hi;
    xhalf_both(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float xhalf_sum(float x) {
    float lo, hi;
    xhalf_both(x, lo, hi);
    return lo + hi;
}

// 16 bytes per lane from global memory straight into LDS: lane i's data lands at
// lds_addr + IMM + 16*i (the instruction's immediate offset applies to the global address
// and to the LDS address alike).  Issued as inline asm so that the compiler does not put a vmcnt(0) wait
// in front of every later LDS read (it cannot tell the buffers apart); the kernel waits
// for vmcnt(0) itself before the barrier that publishes the tile.
// a pointer that is the same in every lane, moved to scalar registers for the compiler's benefit
__device__ __forceinline__ const unsigned char *uniform_ptr(const unsigned char *p) {
    const uint64_t a = (uint64_t)(uintptr_t)p;
    const uint64_t lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a);
    const uint64_t hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32));
    return (const unsigned char *)(uintptr_t)(lo | (hi << 32));
}

template <int IMM, bool NT = false>
__device__ __forceinline__ void dma16_to_lds(const void *gbase, unsigned voff, unsigned lds_addr) {
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3 nt"
                     :
                     : "s"(lds_addr), "v"(voff), "s"(gbase), "n"(IMM)
                     : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3"
                     :
                     : "s"(lds_addr), "v"(voff), "s"(gbase), "n"(IMM)
                     : "memory", "m0");
}

// WIDE = false: the two groups of four waves work on the SAME 128 query rows and take
//   alternate key tiles (group 0 the even ones, group 1 the odd ones), each group loading its
//   own tiles; their partial results are merged at the end.  Halves the longest chain of
//   tiles per workgroup: the shape for short sequences, where workgroups are few and uneven.
// WIDE = true: the eight waves work on 256 different query rows and all walk the same key
//   tiles, loaded once for the whole workgroup.  Halves the K/V traffic into LDS per unit of
//   work: the shape for long sequences.
// SPLITKV = true (wide only): blockIdx.y picks one of p.nsplit runs of the workgroup's key tiles;
//   the result is left unnormalised in p.part_o / p.part_ml for fa_combine_kernel.  The shape for
//   few queries against a long K/V (decoding, chunked prefill), where batch x heads x query
//   blocks alone cannot fill the chip.
// GENMASK = true (wide only, CAUSAL = false): the mask comes from the descriptor in p (window,
//   prefix, per-batch key count) instead of the causal flag; see MaskGeom.
// PAIR = true (wide, causal only): the folded decomposition for short causal problems, see fold_block.  The
//   two waves of a SIMD hold a cheap block and its expensive mirror image.  Once the cheap blocks are done
//   (phase A, one tile per iteration), their waves store their rows, take over the Q rows of their SIMD
//   partner and the workgroup loads TWO tiles per iteration (phase B): the partner takes the odd ones, the
//   helper the even ones, and the two partial results are merged through LDS at the end.  Without this the
//   long blocks' waves would walk their last tiles alone on their SIMDs, where a lone wave cannot overlap its
//   own matrix and vector work.
template <int DT, int D, bool CAUSAL, bool WIDE, bool SPLITKV = false, bool GENMASK = false, bool PAIR = false>
__global__ __launch_bounds__(512, 2) void fa_fwd_kernel(const FaParams p) {
    static_assert(WIDE || !SPLITKV, "split-KV is built on the wide decomposition");
    static_assert(!PAIR || (WIDE && CAUSAL && !SPLITKV && !GENMASK), "the paired fold is a causal wide decomposition");
    static_assert(!GENMASK || (WIDE && !SPLITKV && !CAUSAL), "descriptor masks are built on the plain wide decomposition");
    constexpr int NWL = WIDE ? 8 : 4;             // waves that load one tile together
    constexpr int BM = WIDE ? 256 : 128;          // query rows per workgroup
    constexpr int TSTEP = WIDE ? 1 : 2;           // a group's consecutive tiles are TSTEP apart
    constexpr int KB = D / 16;                    // k-steps of the first product
    constexpr int DB = D / 32;                    // 32-row blocks of O^T
    constexpr int ROWB = D * 2;
    constexpr int TILEB = BN * ROWB;
    // tile buffers per tensor: tiles are loaded NSTAGE-1 ahead.  Two for the compute-bound shapes (three measured
    // 3-10% slower there); the split-KV shapes are bound by HBM latency x bandwidth and take a third, and
    // issue their loads first thing in an iteration instead of between the two matrix clusters
    constexpr int NSTAGE = SPLITKV ? 3 : 2;
    constexpr bool LOADS_FIRST = SPLITKV;
    // split-KV streams K and V once (few query blocks per head): its loads carry the non-temporal hint, worth
    // 6.6-7.0 instead of 5.6-6.0 TB/s there; on the other kernels, whose workgroups share K/V tiles through L2,
    // the same hint costs 3-15%
    constexpr bool KV_NT = SPLITKV;
    constexpr int GROUPB = 2 * NSTAGE * TILEB;    // one set of buffers: K0 .. K(NSTAGE-1) V0 .. V(NSTAGE-1)
    constexpr int NSETS = (WIDE && !PAIR) ? 1 : 2;   // split mode: one set per group; paired fold: one per tile of an iteration

    __shared__ __attribute__((aligned(16))) unsigned char smem[NSETS * GROUPB];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = WIDE ? 0 : (wave >> 2);       // split mode: 0 = even tiles, 1 = odd tiles
    const int wq = WIDE ? wave : (wave & 3);      // which 32 query rows, and which share of the loads
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // ---- workgroup -> (b*H+h, query tile).  Workgroup ids are dealt round-robin to the 8
    // XCDs; give each XCD one contiguous run of the head-major work list so that the
    // workgroups sharing an L2 walk the same head's K/V.  Causal: heaviest tile first.
    const int wi = (blockIdx.x & 7) * p.per_xcd + (blockIdx.x >> 3);
    if (wi >= p.nwork) return;
    const int bh = wi / p.nqt;
    const int qt = (CAUSAL || GENMASK) ? (p.nqt - 1 - wi % p.nqt) : (wi % p.nqt);

    const int Nq = p.Nq, Nk = p.Nk;
    const int off = p.off;                        // key on the diagonal of query row 0 (Nk - Nq for a whole-q launch)
    int q_wave = qt * BM + wq * 32;               // first query row of this wave
    int last_row_wg = min(qt * BM + BM - 1, Nq - 1);   // last query row of the workgroup
    if constexpr (PAIR) {
        q_wave = fold_block(p.nqt, qt, wq) * 32;
        last_row_wg = -1;
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            const int first = fold_block(p.nqt, qt, w) * 32;
            if (first < Nq) last_row_wg = max(last_row_wg, min(first + 31, Nq - 1));
        }
    }
    int qrow = q_wave + l32;                      // this lane's query row

    int kmax_wg = Nk - 1, kmax_wave = Nk - 1;     // last key index any row may see
    if (CAUSAL) {
        kmax_wg = last_row_wg >= 0 ? min(Nk - 1, last_row_wg + off) : -1;
        kmax_wave = min(Nk - 1, min(q_wave + 31, Nq - 1) + off);
    }
    const int nt_all = kmax_wg >= 0 ? kmax_wg / BN + 1 : 0; // 64-key tiles the query block needs
    // this workgroup walks tiles t_lo .. t_lo + nt - 1 of them (all of them unless split-KV)
    int t_lo = 0, nt = nt_all;
    if constexpr (SPLITKV) {
        t_lo = (int)((long long)blockIdx.y * nt_all / p.nsplit);
        nt = (int)((long long)(blockIdx.y + 1) * nt_all / p.nsplit) - t_lo;
    }
    // group-local tile j is global tile t_lo + TSTEP*j + grp
    int nj_loop = (nt + TSTEP - 1) / TSTEP;                  // tiles of group 0 (>= those of group 1)
    int n_act = 0;                                           // group tiles this wave works on
    if (q_wave < Nq && kmax_wave >= 0 && kmax_wave / BN >= grp) n_act = (kmax_wave / BN - grp) / TSTEP + 1;
    if constexpr (SPLITKV) n_act = max(n_act - t_lo, 0);
    // descriptor masks: the workgroup's walk and this wave's rows
    MaskGeom mg = {off, 0, 0, 0, Nk};
    TileSeq seq = {0, 0, 0, 0};
    RowTiles wt = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (GENMASK) {
        int klen = Nk;
        if (p.kv_len) klen = min(max(p.kv_len[bh / p.H], 0), Nk);
        klen = __builtin_amdgcn_readfirstlane(klen);
        mg = {off, p.left, p.right, min(p.prefix, klen), klen};
        seq = tile_sequence(mg, qt * BM, last_row_wg);
        if (q_wave < Nq) wt = row_tiles(mg, q_wave, min(q_wave + 31, Nq - 1));   // else: exist_any = 0, every tile is skipped
        nt = seq.count;
        nj_loop = nt;
    }
    // position j of this group's walk -> tile index
    // paired fold: the tile this wave works on in the current iteration, and how many tiles its block needs
    int pair_tile = 0, pair_need = 0;
    auto tile_of = [&](int j) __attribute__((always_inline)) -> int {
        if constexpr (GENMASK) return seq.tile(j);
        if constexpr (PAIR) return pair_tile;
        return t_lo + TSTEP * j + grp;
    };
    // ... -> does this wave work on it, and does it need the per-element predicate
    int cls_cur = TILE_PARTIAL;
    auto classify = [&](int j) __attribute__((always_inline)) -> bool {
        if constexpr (GENMASK) {
            cls_cur = tile_class(wt, tile_of(j));
            return cls_cur != TILE_SKIP;
        }
        if constexpr (PAIR) return pair_tile < pair_need;
        return j < n_act;
    };

    const size_t kv_head = (size_t)bh * p.kv_rows * D;
    const unsigned char *kgb = (const unsigned char *)(p.k + kv_head);
    const unsigned char *vgb = (const unsigned char *)(p.v + kv_head);

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds d = 16*kb + 8*h + 0..7 of its row
    s16x8 qf[KB];
    auto load_q = [&]() __attribute__((always_inline)) {
        const uint16_t *qp = p.q + ((size_t)bh * p.q_rows + (qrow < Nq ? qrow : 0)) * D + 8 * h;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            s16x8 x = *(const s16x8 *)(qp + kb * 16);
            if (qrow >= Nq || p.qmode == 2) x = (s16x8)(0);
            if (p.qmode == 1) x ^= (s16x8)((short)0x8000);
            qf[kb] = x;
        }
    };
    load_q();

    // ---- K/V tiles go from global memory straight into LDS (global_load_lds, 16 bytes per
    // lane, no staging registers).  One such instruction fills 1 KiB of LDS contiguously in
    // lane order, so the bank swizzle is applied on the global side: the lane that owns LDS
    // slot (row r, chunk c') fetches the global chunk that the swizzle maps there.  The NWL
    // waves that share a set of buffers load its tiles together.
    constexpr int NINSTR = TILEB / 1024;          // load instructions per tile
    constexpr int NI = (NINSTR + NWL - 1) / NWL;  // ... per wave, at most
    constexpr int RPI = 1024 / ROWB;              // tile rows covered by one load instruction
    // This wave issues instructions wq, wq + NWL, ... (< NINSTR) of a tile; instruction i fills
    // LDS bytes [i*1024, +1024) of the tile, i.e. rows i*RPI + (lane*16)/ROWB.  Stepping i by
    // NWL moves the row by a multiple of 16 (D = 128) or of 16 (D = 64, where the swizzle looks
    // at row/2 mod 8), so the swizzled source chunk is the same for all of a wave's instructions.
    static_assert((NWL * RPI) % 16 == 0, "the swizzle must not depend on the instruction index");
    const int ld_row0 = wq * RPI + (lane * 16) / ROWB;
    const int ld_cs = ((lane * 16) % ROWB) >> 4;
    const int ck = (D == 128) ? (ld_cs ^ (ld_row0 & 15)) : (ld_cs ^ ((ld_row0 >> 1) & 7));
    const int cv = (D == 128) ? (ld_cs ^ ((ld_row0 & 3) << 2)) : (ld_cs ^ (((ld_row0 >> 1) & 1) << 2));
    const int k_voff = ld_row0 * ROWB + ck * 16;  // per-lane byte offset of the K chunk within the tile (first instruction)
    const int v_voff = ld_row0 * ROWB + cv * 16;  // same for V
    unsigned char *gsm = smem + grp * GROUPB;     // this group's buffers
    const unsigned char *rsm = gsm;               // ... as read by the matrix clusters (paired fold: switches sets)
    const unsigned lds_base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)LDS_PTR(unsigned char, gsm));
    // whole tiles take their per-lane offsets as they are (tile start and instruction step go
    // into the scalar base); the ragged last tile clamps its rows to the last key -- those rows
    // are masked, they only have to be readable
    auto load_tile = [&](const unsigned char *gb, int t, int lds_off, auto is_k, auto full_c) __attribute__((always_inline)) {
        constexpr bool IS_K = decltype(is_k)::value;
        const int voff = IS_K ? k_voff : v_voff;
        if (decltype(full_c)::value || t * BN + BN <= Nk) {
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const int i = wq + n * NWL;
                if (NINSTR % NWL == 0 || i < NINSTR)
                    dma16_to_lds<0, KV_NT>(uniform_ptr(gb + (size_t)t * TILEB + n * NWL * 1024), (unsigned)voff,
                                    lds_base + lds_off + i * 1024);
            }
        } else {
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const int i = wq + n * NWL;
                if (NINSTR % NWL == 0 || i < NINSTR) {
                    const int key = min(t * BN + ld_row0 + n * NWL * RPI, Nk - 1);
                    dma16_to_lds<0, KV_NT>(uniform_ptr(gb), (unsigned)(key * ROWB + voff - ld_row0 * ROWB),
                                    lds_base + lds_off + i * 1024);
                }
            }
        }
    };
    // group tile j lives in buffer j % NSTAGE
    // full_c: the caller knows the tile lies wholly inside K/V (no check, no clamped path)
    auto load_k = [&](int j, int st, auto full_c) __attribute__((always_inline)) { load_tile(kgb, tile_of(j), st * TILEB, std::true_type{}, full_c); };
    auto load_v = [&](int j, int st, auto full_c) __attribute__((always_inline)) { load_tile(vgb, tile_of(j), (NSTAGE + st) * TILEB, std::false_type{}, full_c); };

    // ---- operand fragments.  K fragment (mb, kb): rows = keys mb*32 + l32, 8 contiguous d.
    auto k_frag = [&](const unsigned char *ks, int mb, int kb) __attribute__((always_inline)) -> s16x8 {
        return *(const s16x8 *)(ks + k_lds_off<D>(mb * 32 + l32, 2 * kb + h));
    };
    // V^T fragment (j, db): rows = d db*32 + l32, k-slot (h, v) = key 16*j + 8*(v/4) + 4*h + v%4,
    // fetched with two transposing reads of 4 keys x 16 d per 16-lane group.
    const int g2 = (lane >> 4) & 1, li = lane & 15, vi = li >> 2, vc = li & 3;
    auto v_frag = [&](const unsigned char *vs, int j, int db) __attribute__((always_inline)) -> s16x8 {
        const int row = 16 * j + 4 * h + vi;
        const int bcol = db * 64 + g2 * 32 + vc * 8;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, vs + v_lds_off<D>(row, bcol)));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, vs + v_lds_off<D>(row + 8, bcol)));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) oacc[db] = (f32x16)(0.f);
    // Softmax state, in log2 units (logit * c).  m_ref is the reference actually subtracted
    // before exponentiation; it follows the running maximum lazily (only when an exponential
    // could have exceeded RESCALE_LIMIT = 2^8), which keeps P <= 256 (fine for fp16 and for the
    // fp32 sums) and spares the rescale of the accumulator, and the row maximum itself, on
    // almost every tile.  Any reference gives the same quotient O = acc / l.
    constexpr float RESCALE_LIMIT = 256.f;
    float m_ref = -1e30f;
    float l_run = 0.f;         // this half-wave's share of the row sum, relative to m_ref

    f32x16 sreg[2];            // logits of the current tile (two 32-key blocks)
    s16x8 pf[4];               // its exponentials, packed, as B operands of the four 16-key steps

    constexpr int LA = 2;      // operand fragments are read this many matrix instructions ahead (1: 10% slower; 3, 4: no gain)

    // ---- S^T = K(j) Q^T for group tile j (K buffer ST = j % NSTAGE)
    auto qk_cluster = [&](auto st_c) __attribute__((always_inline)) {
        constexpr int ST = decltype(st_c)::value;
        const unsigned char *ks = rsm + ST * TILEB;
        s16x8 fr[2 * KB];
#pragma unroll
        for (int i = 0; i < LA; ++i) fr[i] = k_frag(ks, i & 1, i >> 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2 * KB; ++i) {      // the two key blocks alternate: independent accumulators
            if (i + LA < 2 * KB) fr[i + LA] = k_frag(ks, (i + LA) & 1, (i + LA) >> 1);
            const int mb = i & 1, kb = i >> 1;
            if (kb == 0) sreg[mb] = (f32x16)(0.f);
            sreg[mb] = mfma32<DT>(fr[i], qf[kb], sreg[mb]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // ---- O^T += V(j)^T P(j)^T (V buffer ST = j % NSTAGE)
    auto pv_cluster = [&](auto st_c) __attribute__((always_inline)) {
        constexpr int ST = decltype(st_c)::value;
        const unsigned char *vs = rsm + (NSTAGE + ST) * TILEB;
        s16x8 fr[4 * DB];
#pragma unroll
        for (int i = 0; i < LA; ++i) fr[i] = v_frag(vs, i / DB, i % DB);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4 * DB; ++i) {
            if (i + LA < 4 * DB) fr[i + LA] = v_frag(vs, (i + LA) / DB, (i + LA) % DB);
            oacc[i % DB] = mfma32<DT>(fr[i], pf[i / DB], oacc[i % DB]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- softmax of group tile j: logits in sreg -> packed exponentials in pf, running sums
    auto softmax_cluster = [&](int j, auto maybe_masked_c) __attribute__((always_inline)) {
        {
            const int k0 = tile_of(j) * BN;
            // mask only when the tile straddles the diagonal or the end of K
            const bool need_mask = decltype(maybe_masked_c)::value && !GENMASK &&
                                   ((k0 + BN - 1 >= Nk) || (CAUSAL && (k0 + BN - 1 > q_wave + off)));
            if (GENMASK && decltype(maybe_masked_c)::value && cls_cur == TILE_PARTIAL) {
                // limits relative to this lane's first key of the tile, so that each element compares
                // a constant against them (nothing per element lives across tiles)
                const int kb0 = k0 + 4 * h;
                const int lo = qrow + off - mg.left - kb0;
                const int hi = min(mg.klen - 1, qrow + off + mg.right) - kb0;
                const int pf = mg.pfx - kb0;
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int c = mb * 32 + 8 * (r >> 2) + (r & 3);
                        const bool vis = (c < pf) | ((c >= lo) & (c <= hi));   // no short-circuit: selects, not branches
                        sreg[mb][r] = vis ? sreg[mb][r] : -INFINITY;
                    }
            }
            if (need_mask) {
                int lim = Nk - 1;
                if (CAUSAL) lim = min(lim, qrow + off);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = k0 + mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                        if (key > lim) sreg[mb][r] = -INFINITY;
                    }
            }
            // Exponentials against the current reference, packed as the P^T fragments: 16-key step
            // jj takes logits registers 8*(jj%2)..+7 of block jj/2, i.e. k-slot (h, v) of step jj is
            // key 16*jj + 8*(v/4) + 4*h + v%4.  Returns this lane's sum (its 32 logits all belong to
            // one query).
            auto exponentials = [&]() __attribute__((always_inline)) -> float {
                const float nm = -m_ref;
                float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                    for (int v2 = 0; v2 < 4; ++v2) {
                        const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sreg[jj >> 1][8 * (jj & 1) + 2 * v2], p.c, nm));
                        const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sreg[jj >> 1][8 * (jj & 1) + 2 * v2 + 1], p.c, nm));
                        rs0 += e0;
                        rs1 += e1;
                        const s16x2 pr = pack2<DT>(e0, e1);
                        pf[jj][2 * v2] = pr[0];
                        pf[jj][2 * v2 + 1] = pr[1];
                    }
                return rs0 + rs1;
            };
            float rs = 0.f;
            if constexpr (D == 128) {
                // No row maximum on the common path: the exponentials are non-negative, so a sum of
                // at most RESCALE_LIMIT proves that none of them exceeded it.  Otherwise (the very
                // first tile, where the sum is infinite, or a row whose maximum has risen a lot)
                // take the row maximum, move the reference up to it, rescale what has been
                // accumulated, and redo the exponentials -- a loop of at most two passes, so that
                // the exponentials exist once in the code.
#pragma nounroll
                for (int pass = 0; pass < 2; ++pass) {
                    rs = exponentials();
                    const bool over = !(rs <= RESCALE_LIMIT);   // also true for inf and NaN
                    if (pass == 1 || __builtin_amdgcn_ballot_w64(over) == 0) break;
                    float mx = sreg[0][0];
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sreg[mb][r]);
                    mx = xhalf_max(mx) * p.c;
                    const bool grow = mx > m_ref;
                    const float alpha = grow ? __builtin_amdgcn_exp2f(m_ref - mx) : 1.f;
                    m_ref = grow ? mx : m_ref;
                    l_run *= alpha;
#pragma unroll
                    for (int db = 0; db < DB; ++db) oacc[db] *= alpha;
                }
            } else {
                // D = 64: keeping the logits alive for a possible second pass costs 16 registers and
                // with them the fourth wave per SIMD, which matters more there: take the row
                // maximum up front and move the reference when it has risen by more than 8.
                float mx = sreg[0][0];
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sreg[mb][r]);
                mx = xhalf_max(mx) * p.c;
                const bool grow = mx > m_ref + 8.f;
                if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                    const float alpha = grow ? __builtin_amdgcn_exp2f(m_ref - mx) : 1.f;
                    m_ref = grow ? mx : m_ref;
                    l_run *= alpha;
#pragma unroll
                    for (int db = 0; db < DB; ++db) oacc[db] *= alpha;
                }
                rs = exponentials();
            }
            l_run += rs;
        }
    };

    // ---- result of this wave's rows: combine the two half-wave sums, normalise, store
    auto store_rows = [&]() __attribute__((always_inline)) {
        const float l_tot = xhalf_sum(l_run);
        if (qrow < Nq) {
            const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
            uint16_t *op = p.o + ((size_t)bh * p.q_rows + qrow) * D + 4 * h;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const s16x2 a = pack2<DT>(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv);
                    const s16x2 b = pack2<DT>(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
                    const s16x4 st = {a[0], a[1], b[0], b[1]};
                    *(s16x4 *)(op + db * 32 + 8 * g) = st;
                }
            if (h == 0)
                p.lse[(size_t)bh * p.q_rows + qrow] = l_tot > 0.f ? (m_ref + __log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
        }
    };

    // ---- pipeline.  Tiles are loaded PD = NSTAGE-1 iterations ahead.  Iteration j: each group
    // issues the loads of its tile j+PD (into the buffer tile j-1 used), works on its tile j
    // (logits, softmax, P V), waits until its share of tile j+1 has landed and meets the other
    // waves at the barrier that publishes it.  Between barriers the waves run free.
    constexpr int PD = NSTAGE - 1;
    constexpr int PER_TILE = 2 * NI;              // load instructions a wave issues per tile (K and V)
    static_assert(NINSTR % NWL == 0, "every wave must issue the same number of loads per tile");
    using std::integral_constant;
    if constexpr (PAIR) {
        // ---- paired fold.  helper = the wave that starts on a cheap block (waves 0..3); its SIMD partner
        // (wave + 4) owns the mirror image.  Phase A: iterations 0 .. nA-1, tile j for everybody (set 0).
        // Phase B: iteration nA + i loads tiles nA + 2i (set 0, the helper's) and nA + 2i + 1 (set 1, the
        // owner's).  Tiles are loaded one iteration ahead into stage (iteration & 1) of their set.
        static_assert(NSTAGE == 2, "the paired fold alternates two stages");
        const bool helper = wave < 4;
        auto tiles_of_block = [&](int blk) __attribute__((always_inline)) -> int {
            const int first = blk * 32;
            if (first >= Nq) return 0;
            const int kmax = min(Nk - 1, min(first + 31, Nq - 1) + off);
            return kmax >= 0 ? kmax / BN + 1 : 0;
        };
        const int blk_long = fold_block(p.nqt, qt, (wave & 3) + 4);
        int nA = 0;                                  // tiles the workgroup's cheap blocks need (they grow with the block index)
#pragma unroll
        for (int w = 0; w < 4; ++w) nA = max(nA, tiles_of_block(fold_block(p.nqt, qt, w)));
        const int L = nt;                            // tiles the workgroup walks in all
        const int nB = (max(L - nA, 0) + 1) / 2;
        const int NJ = nA + nB;
        pair_need = tiles_of_block(fold_block(p.nqt, qt, wave));
        // loads of iteration jn (both tensors, every wave its share); nothing to load past the last tile
        auto issue_loads = [&](int jn, int stl) __attribute__((always_inline)) {
            if (jn >= NJ) return;
            if (jn < nA) {
                load_tile(kgb, jn, stl * TILEB, std::true_type{}, std::false_type{});
                load_tile(vgb, jn, (NSTAGE + stl) * TILEB, std::false_type{}, std::false_type{});
            } else {
                const int t0 = nA + 2 * (jn - nA);
                load_tile(kgb, t0, stl * TILEB, std::true_type{}, std::false_type{});
                load_tile(vgb, t0, (NSTAGE + stl) * TILEB, std::false_type{}, std::false_type{});
                if (t0 + 1 < L) {
                    load_tile(kgb, t0 + 1, GROUPB + stl * TILEB, std::true_type{}, std::false_type{});
                    load_tile(vgb, t0 + 1, GROUPB + (NSTAGE + stl) * TILEB, std::false_type{}, std::false_type{});
                }
            }
        };
        auto pair_iteration = [&](auto st_c, int jj) __attribute__((always_inline)) {
            constexpr int ST = decltype(st_c)::value;
            if (jj == nA) {
                // the cheap blocks are done: their waves store them and join their partners' blocks;
                // the partners read their tiles from set 1 from now on
                if (helper) {
                    store_rows();
                    q_wave = blk_long * 32;
                    qrow = q_wave + l32;
                    load_q();
#pragma unroll
                    for (int db = 0; db < DB; ++db) oacc[db] = (f32x16)(0.f);
                    m_ref = -1e30f;
                    l_run = 0.f;
                    pair_need = tiles_of_block(blk_long);
                } else {
                    rsm = smem + GROUPB;
                }
            }
            pair_tile = jj < nA ? jj : nA + 2 * (jj - nA) + (helper ? 0 : 1);
            if (pair_tile < pair_need) {
                qk_cluster(st_c);
                issue_loads(jj + 1, ST ^ 1);
                softmax_cluster(jj, std::true_type{});
                pv_cluster(st_c);
            } else {
                issue_loads(jj + 1, ST ^ 1);
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __builtin_amdgcn_s_barrier();
        };
        // phase-B iteration without checks: this wave's tile is needed, unmasked and wholly inside K/V, and
        // both tiles of the next iteration exist and lie wholly inside K/V
        auto pair_interior = [&](auto st_c, int jj) __attribute__((always_inline)) {
            constexpr int ST = decltype(st_c)::value;
            pair_tile = nA + 2 * (jj - nA) + (helper ? 0 : 1);
            qk_cluster(st_c);
            const int t0 = nA + 2 * (jj + 1 - nA);
            load_tile(kgb, t0, (ST ^ 1) * TILEB, std::true_type{}, std::true_type{});
            load_tile(vgb, t0, (NSTAGE + (ST ^ 1)) * TILEB, std::false_type{}, std::true_type{});
            load_tile(kgb, t0 + 1, GROUPB + (ST ^ 1) * TILEB, std::true_type{}, std::true_type{});
            load_tile(vgb, t0 + 1, GROUPB + (NSTAGE + (ST ^ 1)) * TILEB, std::false_type{}, std::true_type{});
            softmax_cluster(jj, std::false_type{});
            pv_cluster(st_c);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __builtin_amdgcn_s_barrier();
        };
        // iterations nA+1 .. jI-1 are of that kind for this wave (iteration nA holds the switch); slot = which
        // of an iteration's two tiles is this wave's in phase B
        int jI = 0;
        {
            const int slot = helper ? 0 : 1;
            const int free_key = min(Nk - 1, blk_long * 32 + off);            // last key the block's first row sees
            const int t_unmasked = free_key >= BN - 1 ? (free_key - (BN - 1)) / BN : -1;   // last tile without a mask
            const int t_loadable = min(L, Nk / BN) - 1;                            // last tile that is walked and whole
            // i-th phase-B iteration: own tile nA + 2i + slot <= t_unmasked, next iteration's second tile
            // nA + 2i + 3 <= t_loadable
            const int a = t_unmasked - nA - slot, b = t_loadable - nA - 3;
            const int i_last = min(a >= 0 ? a / 2 : -1, b >= 0 ? b / 2 : -1);
            jI = blk_long * 32 < Nq ? nA + i_last + 1 : 0;
        }
        issue_loads(0, 0);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __builtin_amdgcn_s_barrier();
        // general iterations up to the first even one after the switch, check-free ones in whole pairs, general rest
        const int i_first = min((nA + 2) & ~1, NJ);
        const int i_end = jI > i_first ? i_first + ((jI - i_first) & ~1) : i_first;
        int jj = 0;
        if constexpr (D == 128) {   // (D = 64: the extra copies of the loop body would cost the fourth wave per SIMD)
            for (; jj < i_first; jj += 2) {
                pair_iteration(integral_constant<int, 0>{}, jj);
                if (jj + 1 < i_first) pair_iteration(integral_constant<int, 1>{}, jj + 1);
            }
            for (; jj < i_end; jj += 2) {
                pair_interior(integral_constant<int, 0>{}, jj);
                pair_interior(integral_constant<int, 1>{}, jj + 1);
            }
        }
        for (; jj < NJ; jj += 2) {
            pair_iteration(integral_constant<int, 0>{}, jj);
            if (jj + 1 < NJ) pair_iteration(integral_constant<int, 1>{}, jj + 1);
        }
        if (NJ <= nA && helper) {
            // no phase B at all (the expensive blocks need no more tiles than the cheap ones): the switch never ran
            store_rows();
            q_wave = blk_long * 32;
            qrow = q_wave + l32;
#pragma unroll
            for (int db = 0; db < DB; ++db) oacc[db] = (f32x16)(0.f);
            m_ref = -1e30f;
            l_run = 0.f;
        }
        // ---- merge the helper's share of the expensive block into its owner's (all tile buffers are idle now).
        // Lane-major layout: value k of pair w's lane sits at w*XW + k*256 + lane*4.
        constexpr int NV = DB * 16 + 2;               // accumulator + m_ref + l_run
        constexpr int XW = NV * 256;                  // bytes per wave
        static_assert(4 * XW <= NSETS * GROUPB, "exchange area must fit in the tile buffers");
        float *xch = (float *)(smem + (wave & 3) * XW) + lane;
        if (helper) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) xch[(db * 16 + r) * 64] = oacc[db][r];
            xch[(DB * 16) * 64] = m_ref;
            xch[(DB * 16 + 1) * 64] = l_run;
        }
        __syncthreads();
        if (helper) return;
        {
            const float m1 = xch[(DB * 16) * 64];
            const float l1 = xch[(DB * 16 + 1) * 64];
            const float m = fmaxf(m_ref, m1);
            const float a0 = __builtin_amdgcn_exp2f(m_ref - m);
            const float a1 = __builtin_amdgcn_exp2f(m1 - m);
            l_run = l_run * a0 + l1 * a1;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] = oacc[db][r] * a0 + xch[(db * 16 + r) * 64] * a1;
            m_ref = m;
        }
        store_rows();
        return;
    }
#pragma unroll
    for (int j = 0; j < PD; ++j)
        if (TSTEP * j + grp < nt) { load_k(j, j, std::false_type{}); load_v(j, j, std::false_type{}); }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __builtin_amdgcn_s_barrier();
    // general iteration: every condition checked
    auto iteration = [&](auto st_c, int j) __attribute__((always_inline)) {
        constexpr int ST = decltype(st_c)::value;             // j % NSTAGE
        constexpr int ST_LOAD = (ST + PD) % NSTAGE;           // (j + PD) % NSTAGE
        const bool issued = TSTEP * (j + PD) + grp < nt;
        if (classify(j)) {
            // the loads go out between the two matrix clusters (measured 1% better than up front:
            // their LDS writes then land mostly during the softmax, when no wave reads LDS);
            // split-KV waits on HBM, not on LDS: there they go out first
            if (LOADS_FIRST && issued) { load_k(j + PD, ST_LOAD, std::false_type{}); load_v(j + PD, ST_LOAD, std::false_type{}); }
            qk_cluster(st_c);
            if (!LOADS_FIRST && issued) { load_k(j + PD, ST_LOAD, std::false_type{}); load_v(j + PD, ST_LOAD, std::false_type{}); }
            softmax_cluster(j, std::true_type{});
            pv_cluster(st_c);
        } else if (issued) {
            load_k(j + PD, ST_LOAD, std::false_type{});
            load_v(j + PD, ST_LOAD, std::false_type{});
        }
        // loads land in issue order: all but the newest (PD-1) tiles' worth must be done
        if (issued) __builtin_amdgcn_s_waitcnt(0x0F70 | ((PD - 1) * PER_TILE));
        else __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __builtin_amdgcn_s_barrier();
    };
    // interior iteration: this wave's tile j is active and needs no mask, and tile j+1 of its group
    // exists and lies wholly inside K/V -- straight-line code, no checks
    // (written for two buffers; with more the general loop does everything)
    auto interior = [&](auto st_c, int j) __attribute__((always_inline)) {
        constexpr int ST = decltype(st_c)::value;
        if (LOADS_FIRST) { load_k(j + 1, ST ^ 1, std::true_type{}); load_v(j + 1, ST ^ 1, std::true_type{}); }
        qk_cluster(st_c);
        if (!LOADS_FIRST) { load_k(j + 1, ST ^ 1, std::true_type{}); load_v(j + 1, ST ^ 1, std::true_type{}); }
        softmax_cluster(j, std::false_type{});
        pv_cluster(st_c);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __builtin_amdgcn_s_barrier();
    };
    // number of leading iterations that are interior for this wave (every wave runs nj_loop
    // iterations and meets nj_loop barriers, whichever of the two loops each one is in)
    int j_int = 0;
    {
        // tile TSTEP*j+grp is unmasked for this wave while its last key is <= the first row's limit
        const int last_free_key = CAUSAL ? min(Nk - 1, q_wave + off) : Nk - 1;       // may be negative
        const int unmasked = last_free_key >= BN - 1 ? ((last_free_key - (BN - 1)) / BN - grp) / TSTEP + 1 : 0;
        const int full_tiles = Nk / BN;                                              // tiles wholly inside K/V
        const int next_full = (full_tiles - 1 - grp) / TSTEP;                        // j with tile j+1 full: j < next_full
        const int ntg = nt > grp ? (nt - 1 - grp) / TSTEP + 1 : 0;                   // tiles of this wave's group
        j_int = min(min(unmasked, n_act), min(next_full, ntg - 1));
        if (last_free_key < BN - 1 + grp * BN || full_tiles - 1 - grp < 0) j_int = 0;
        if constexpr (SPLITKV)   // the same three limits, counted from this workgroup's first tile
            j_int = last_free_key >= BN - 1 ? min(min(unmasked - t_lo, n_act), min(full_tiles - 1 - t_lo, nt - 1)) : 0;
        j_int = max(j_int, 0) & ~1;                                                  // whole pairs
    }
    int j = 0;
    if constexpr (NSTAGE == 2) {
        if constexpr (GENMASK && D == 64) j_int = 0;   // a third copy of the loop body costs D = 64 its fourth wave per SIMD
        if constexpr (GENMASK && D == 128) {
            // descriptor masks: the check-free run may start anywhere (a window's lower edge comes first)
            const Run run = interior_run(wt, seq, Nk);
            for (; j < run.first; j += 2) {
                iteration(integral_constant<int, 0>{}, j);
                iteration(integral_constant<int, 1>{}, j + 1);
            }
            j_int = run.first + run.count;
        }
        for (; j < j_int; j += 2) {
            interior(integral_constant<int, 0>{}, j);
            interior(integral_constant<int, 1>{}, j + 1);
        }
        for (; j < nj_loop; j += 2) {
            iteration(integral_constant<int, 0>{}, j);
            if (j + 1 < nj_loop) iteration(integral_constant<int, 1>{}, j + 1);
        }
    } else {
        static_assert(NSTAGE == 3, "two or three buffers");
        for (; j < nj_loop; j += 3) {
            iteration(integral_constant<int, 0>{}, j);
            if (j + 1 < nj_loop) iteration(integral_constant<int, 1>{}, j + 1);
            if (j + 2 < nj_loop) iteration(integral_constant<int, 2>{}, j + 2);
        }
    }

    if constexpr (!WIDE) {
        // ---- merge group 1 into group 0 through LDS (all tile buffers are idle now).  Lane-major
        // layout: value k of wave wq's lane sits at wq*XW + k*256 + lane*4.
        constexpr int NV = DB * 16 + 2;               // accumulator + m_ref + l_run
        constexpr int XW = NV * 256;                  // bytes per wave
        static_assert(4 * XW <= NSETS * GROUPB, "exchange area must fit in the tile buffers");
        float *xch = (float *)(smem + wq * XW) + lane;
        if (grp == 1) {
    #pragma unroll
            for (int db = 0; db < DB; ++db)
    #pragma unroll
                for (int r = 0; r < 16; ++r) xch[(db * 16 + r) * 64] = oacc[db][r];
            xch[(DB * 16) * 64] = m_ref;
            xch[(DB * 16 + 1) * 64] = l_run;
        }
        __syncthreads();
        if (grp == 1) return;
        {
            const float m1 = xch[(DB * 16) * 64];
            const float l1 = xch[(DB * 16 + 1) * 64];
            const float m = fmaxf(m_ref, m1);
            const float a0 = __builtin_amdgcn_exp2f(m_ref - m);
            const float a1 = __builtin_amdgcn_exp2f(m1 - m);
            l_run = l_run * a0 + l1 * a1;
    #pragma unroll
            for (int db = 0; db < DB; ++db)
    #pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] = oacc[db][r] * a0 + xch[(db * 16 + r) * 64] * a1;
            m_ref = m;
        }
    }

    // ---- epilogue
    if constexpr (SPLITKV) {
        const float l_tot = xhalf_sum(l_run);
        if (qrow < Nq) {
            const size_t row = (size_t)blockIdx.y * ((size_t)p.nwork / p.nqt) * Nq + (size_t)bh * Nq + qrow;
            float *po = p.part_o + row * D + 4 * h;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 x = {oacc[db][4 * g], oacc[db][4 * g + 1], oacc[db][4 * g + 2], oacc[db][4 * g + 3]};
                    *(float4 *)(po + db * 32 + 8 * g) = x;
                }
            if (h == 0) {
                const float2 ml = {m_ref, l_tot};
                *(float2 *)(p.part_ml + row * 2) = ml;
            }
        }
        return;
    }
    store_rows();
}

// ---- output projection (section 4.2: the Linear that follows the attention, computed block of rows by
// block of rows right after it).  y[b, s, n] = sum_{h, d} o[b, h, s, d] * w[h*D + d, n] for the rows
// s0 <= s < s0 + rows of every batch entry: a GEMM whose A operand is read straight out of the attention
// output layout [B, H, Nq, D] (the heads are never copied side by side), fp32 accumulation, fp32 result.
//
// Workgroup tile 128 tokens x 256 outputs, K step 64, 8 waves as 2 (tokens) x 4 (outputs), wave tile 64 x 64
// = 2 x 2 blocks of v_mfma_f32_32x32x16.  Both operand tiles go from global memory straight into LDS
// (double-buffered, one k-tile ahead) with the bank swizzles of the attention kernel's K and V tiles: the o
// tile (row-major, 128 B rows, k contiguous) is read with ds_read_b128 as the A operand; the w tile (row =
// k, 512 B rows, n contiguous) is read with the transposing ds_read_b64_tr_b16 as the B operand.
struct LinParams {
    const uint16_t *o, *w;
    float *y;
    int H, q_rows, N;      // heads, rows between consecutive heads of o, outputs per token
    int s0, rows;          // the block of rows
    int mt_per_b;          // 128-row tiles per batch entry
    int n_tiles;           // 256-wide tiles of N
    int ntile_total, per_xcd;
    int panel;             // row tiles per panel of the tile order
};

template <int DT, int D, int BM>
__global__ __launch_bounds__(512, 1) void fa_linear_kernel(const LinParams p) {
    static_assert(BM == 128 || BM == 256, "token rows per workgroup tile");
    constexpr int BNO = 256, BK = 64;
    constexpr int MB = BM / 64;                   // 32-row blocks per wave (wave tile BM/2 x 64)
    constexpr int A_TILE = BM * BK * 2;           // 16 / 32 KiB
    constexpr int W_TILE = BK * BNO * 2;          // 32 KiB
    constexpr int STAGE = A_TILE + W_TILE;
    // tile buffers: the small tile runs its loads two k-tiles ahead (3 x 48 KiB), the large one, whose
    // iterations are twice as long, one ahead (2 x 64 KiB)
    constexpr int NST = BM == 128 ? 3 : 2;
    constexpr int NA = BM / 64;                   // o-tile load instructions per wave and k-tile
    constexpr int PER_TILE = NA + 4;              // ... all load instructions per wave and k-tile
    __shared__ __attribute__((aligned(16))) unsigned char smem[NST * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int l32 = lane & 31, h = lane >> 5;

    // workgroup ids are dealt round-robin to the 8 XCDs; each XCD gets a contiguous run of the tile list.
    // The list goes panel of `panel` row tiles by panel, within a panel column slice by column slice, so
    // that the workgroups sharing an L2 cover a block of about as many bytes of o rows as of w columns
    // (every L2 has to fetch the rows and the columns of its block once)
    const int wi = (blockIdx.x & 7) * p.per_xcd + (blockIdx.x >> 3);
    if (wi >= p.ntile_total) return;
    const int m_tiles = p.ntile_total / p.n_tiles;
    const int panel_tiles = p.panel * p.n_tiles;
    const int pn = wi / panel_tiles, rem = wi - pn * panel_tiles;
    const int panel_rows = min(p.panel, m_tiles - pn * p.panel);
    const int nt = rem / panel_rows, mt = pn * p.panel + rem % panel_rows;
    const int b = mt / p.mt_per_b;
    const int r0 = (mt % p.mt_per_b) * BM;        // first row of the tile within the block
    const int n0 = nt * BNO;
    const int KT = p.H * D / BK;                  // k-tiles

    const unsigned lds_base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)LDS_PTR(unsigned char, smem));

    // ---- loads.  o tile: instruction i (1 KiB) fills rows 8i..8i+7; this wave issues i = wave + 8n.
    // The lane that owns LDS slot (row r, chunk c') fetches global chunk c' ^ ((r >> 1) & 7).  Rows past the
    // end of the block are clamped to its last row (computed, never stored).
    const int a_r = lane >> 3, a_c = lane & 7;
    unsigned a_voff[NA];
#pragma unroll
    for (int n = 0; n < NA; ++n) {
        const int r = (wave + 8 * n) * 8 + a_r;
        const int s = p.s0 + min(r0 + r, p.rows - 1);
        a_voff[n] = (unsigned)(s * (D * 2) + ((a_c ^ ((r >> 1) & 7)) << 4));
    }
    // w tile: instruction i fills k-rows 2i, 2i+1 (512 B each); this wave issues i = wave + 8n, n = 0..3.
    // The lane that owns slot (row r, byte b') fetches global byte b' ^ ((r & 3) << 6).
    const int w_r = lane >> 5;
    unsigned w_voff[4];
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int r = (wave + 8 * n) * 2 + w_r;
        w_voff[n] = (unsigned)(r * (p.N * 2) + (((lane & 31) << 4) ^ ((r & 3) << 6)));
    }
    const unsigned char *ob = (const unsigned char *)p.o;
    const unsigned char *wb = (const unsigned char *)p.w + (size_t)n0 * 2;
    auto load_tiles = [&](int kt, int st) __attribute__((always_inline)) {
        const int k0 = kt * BK;
        const int hh = k0 / D, d0 = k0 % D;
        const unsigned char *ag = ob + ((size_t)(b * p.H + hh) * p.q_rows * D + d0) * 2;
        const unsigned char *wg = wb + (size_t)k0 * p.N * 2;
#pragma unroll
        for (int n = 0; n < NA; ++n)
            dma16_to_lds<0>(uniform_ptr(ag), a_voff[n], lds_base + st * STAGE + (wave + 8 * n) * 1024);
#pragma unroll
        for (int n = 0; n < 4; ++n)
            dma16_to_lds<0>(uniform_ptr(wg), w_voff[n], lds_base + st * STAGE + A_TILE + (wave + 8 * n) * 1024);
    };

    // ---- operand fragments
    auto a_frag = [&](const unsigned char *as, int mb, int ks) __attribute__((always_inline)) -> s16x8 {
        return *(const s16x8 *)(as + k_lds_off<64>(wm * (BM / 2) + mb * 32 + l32, 2 * ks + h));
    };
    // k-slot (h, v) of 16-step ks is k = 16 ks + 8 h + v: two transposing reads of 4 k-rows x 16 outputs
    const int g2 = (lane >> 4) & 1, li = lane & 15, vi = li >> 2, vc = li & 3;
    auto w_frag = [&](const unsigned char *ws, int ks, int nb) __attribute__((always_inline)) -> s16x8 {
        const int row = 16 * ks + 8 * h + vi;
        const int bcol = (wn * 64 + nb * 32) * 2 + g2 * 32 + vc * 8;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ws + row * 512 + (bcol ^ ((row & 3) << 6))));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ws + (row + 4) * 512 + (bcol ^ (((row + 4) & 3) << 6))));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    f32x16 acc[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) acc[mb][nb] = (f32x16)(0.f);

    // k-tile kt lives in buffer kt % NST and is loaded NST - 1 iterations ahead.  Iteration kt issues the loads
    // of tile kt + NST - 1 (into the buffer tile kt - 1 used: every wave has passed the barrier that ended
    // iteration kt - 1), works on tile kt, then waits until its own share of tile kt + 1 has landed (loads
    // complete in order: all but the newest NST - 2 tiles' worth) and meets the other waves.
    constexpr int PD = NST - 1;
#pragma unroll
    for (int t = 0; t < PD; ++t)
        if (t < KT) load_tiles(t, t);
    if (PD == 2 && KT > 1) __builtin_amdgcn_s_waitcnt(0x0F70 | PER_TILE);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    int st = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + PD < KT;
        if (more) load_tiles(kt + PD, st >= 1 ? st - 1 : NST - 1);
        const unsigned char *as = smem + st * STAGE;
        const unsigned char *ws = as + A_TILE;
        s16x8 af[2][MB], wf[2][2];          // [ks parity][block]
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) af[0][mb] = a_frag(as, mb, 0);
        wf[0][0] = w_frag(ws, 0, 0);
        wf[0][1] = w_frag(ws, 0, 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks + 1 < 4) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) af[nxt][mb] = a_frag(as, mb, ks + 1);
                wf[nxt][0] = w_frag(ws, ks + 1, 0);
                wf[nxt][1] = w_frag(ws, ks + 1, 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) acc[mb][nb] = mfma32<DT>(af[cur][mb], wf[cur][nb], acc[mb][nb]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more && PD == 2) __builtin_amdgcn_s_waitcnt(0x0F70 | PER_TILE);
        else __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __builtin_amdgcn_s_barrier();
        st = st == NST - 1 ? 0 : st + 1;
    }

    // ---- store: register r of block (mb, nb) is token row 8 (r/4) + 4 h + r%4, output column l32
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = r0 + wm * (BM / 2) + mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            if (row < p.rows) {
                float *yp = p.y + ((size_t)b * p.q_rows + p.s0 + row) * p.N + n0 + wn * 64 + l32;
#pragma unroll
                // written once, 128 contiguous bytes per half-wave, the largest tensor of the call: the
                // non-temporal hint keeps it from displacing o and w in L2 (1-2%)
                for (int nb = 0; nb < 2; ++nb) __builtin_nontemporal_store(acc[mb][nb][r], yp + nb * 32);
            }
        }
}

// ---- ceiling probe: nothing but independent matrix instructions, two waves per SIMD on every compute unit.
// What this reaches is what the chip sustains under its power limit with the matrix pipes saturated and nothing
// else going on -- the practical ceiling beside the nominal peak.  Four accumulators per wave keep the pipe fed.
// RANDOM = false: one pair of operands with a few low bits set, the same for every instruction (hardly any
// switching in the multipliers: the friendliest case for the power limit).  RANDOM = true: four pairs of
// operands with pseudo-random signs and mantissas, magnitudes in [0.5, 2) (fp16) or [2^-15, 2) (bf16),
// taken in turn, so that consecutive instructions toggle the multiplier inputs the way real data does.
template <int DT, bool RANDOM>
__global__ __launch_bounds__(512, 1) void fa_mfma_probe_kernel(float *out, int iters) {
    s16x8 a[4], b[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (RANDOM) {
                unsigned x = (threadIdx.x * 8u + i) * 4u + n + 1u + blockIdx.x * 16384u;
                x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;   // integer hash
                a[n][i] = (short)(0x3800 | (x & 0x87ff));            // sign, 11 random low bits
                b[n][i] = (short)(0x3800 | ((x >> 16) & 0x87ff));
            } else {
                a[n][i] = (short)(0x3c00 + ((threadIdx.x + i) & 7));   // small finite values in either format
                b[n][i] = (short)(0x3800 + ((threadIdx.x + 3 * i) & 7));
            }
        }
    f32x16 c0 = (f32x16)(0.f), c1 = c0, c2 = c0, c3 = c0;
    for (int it = 0; it < iters; ++it) {
        c0 = mfma32<DT>(a[0], b[0], c0);
        c1 = mfma32<DT>(a[1], b[1], c1);
        c2 = mfma32<DT>(a[2], b[2], c2);
        c3 = mfma32<DT>(a[3], b[3], c3);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    if (s == 12345.678f) out[0] = s;                        // never true: keeps the loop alive
}

// ---- decoding step (appendix C's decoding equations: one query row per head against the whole cache).
// With a single query there is nothing for the matrix cores to reuse: every byte of K and V meets one
// multiply-add, the bound is HBM, and the tile machinery of fa_fwd_kernel (LDS staging, barriers, 31 idle
// rows of every matrix instruction) only stands between the memory system and the arithmetic.  This kernel
// streams K and V through registers instead.  blockIdx.x = (batch, head), blockIdx.y = one of p.nsplit runs
// of keys (the same runs of 64-key tiles as the split-KV kernel's); four waves take the run's blocks of KB
// keys in turn.  A load instruction fetches 64 x 16 bytes = RPI whole rows, LPR = D/8 lanes per row; the LPR
// lanes of a row each multiply their 8 channels by the matching channels of q (held in registers, scale
// folded in) and add up across the row with DPP moves; each of the RPI lane groups keeps its own running
// reference, sum and 8-channel slice of the output for the rows it sees, in fp32 throughout (the
// probabilities are never rounded to 16 bits here).  The 4 x RPI partial states of the workgroup are merged
// through LDS and written to the split-KV workspace in the layout fa_combine_kernel reads.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}
// sum over the LPR (8 or 16) consecutive lanes that share a row; every one of them gets the total
template <int LPR>
__device__ __forceinline__ float row_lanes_sum(float x) {
    x += dpp_move<0xB1>(x);              // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);              // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);             // row_half_mirror: lane i <-> 7 - i of each 8
    if constexpr (LPR == 16) x += dpp_move<0x140>(x);   // row_mirror: lane i <-> 15 - i of each 16
    return x;
}
// two 16-bit values of the storage type packed in 32 bits -> two fp32 (exact)
template <int DT>
__device__ __forceinline__ f32x2 unpack2(unsigned u) {
    if constexpr (DT == FA_DTYPE_F16) {
        const f16x2 hh = __builtin_bit_cast(f16x2, u);
        return f32x2{(float)hh[0], (float)hh[1]};
    } else {
        return f32x2{__builtin_bit_cast(float, u << 16), __builtin_bit_cast(float, u & 0xffff0000u)};
    }
}

// 16 bytes that no other workgroup will ask for again: loaded with the non-temporal hint, so that the
// stream does not displace anything in L2 or the Infinity Cache (measured: 6.7-7.0 TB/s instead of 5.9-6.0)
__device__ __forceinline__ uint4 load16_streaming(const uint16_t *p) {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 x = __builtin_nontemporal_load((const u32x4 *)p);
    return uint4{x[0], x[1], x[2], x[3]};
}
constexpr int DECODE_WAVES = 4;
template <int DT, int D>
__global__ __launch_bounds__(DECODE_WAVES * 64) void fa_decode_kernel(const FaParams p) {
    constexpr int LPR = D / 8;                    // lanes per K/V row (16 bytes each)
    constexpr int RPI = 64 / LPR;                 // rows per load instruction
    constexpr int NLD = 8;                        // load instructions per block and tensor
    constexpr int KB = NLD * RPI;                 // keys per block
    constexpr int NW = DECODE_WAVES;              // waves
    constexpr int NG = NW * RPI;                  // lane groups, each with a partial state
    __shared__ float sm_o[NG][D];
    __shared__ float sm_ml[NG][2];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane / LPR, c = lane % LPR;
    const int bh = blockIdx.x, sp = blockIdx.y;
    const int Nk = p.Nk;
    const int nt_all = (Nk + BN - 1) / BN;
    const int k_lo = (int)((long long)sp * nt_all / p.nsplit) * BN;
    const int k_hi = min(Nk, (int)((long long)(sp + 1) * nt_all / p.nsplit) * BN);

    // this lane's 8 channels of q, times scale * log2(e): logits in base-2 units as in fa_fwd_kernel
    const float cs = p.qmode == 0 ? p.c : (p.qmode == 1 ? -p.c : 0.f);
    float qf[8];
    {
        const uint4 qq = *(const uint4 *)(p.q + (size_t)bh * D + c * 8);
        const unsigned qw[4] = {qq.x, qq.y, qq.z, qq.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const f32x2 f = unpack2<DT>(qw[j]);
            qf[2 * j] = f[0] * cs;
            qf[2 * j + 1] = f[1] * cs;
        }
    }
    const uint16_t *kbase = p.k + (size_t)bh * Nk * D + c * 8;
    const uint16_t *vbase = p.v + (size_t)bh * Nk * D + c * 8;

    float m = -1e30f, l = 0.f, o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = 0.f;

    // rows past the end of the run are fetched as its last row (and masked below)
    auto load_block = [&](int key0, uint4 *kk, uint4 *vv) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < NLD; ++n) {
            const int row = min(key0 + n * RPI + g, k_hi - 1);
            kk[n] = load16_streaming(kbase + (size_t)row * D);
        }
#pragma unroll
        for (int n = 0; n < NLD; ++n) {
            const int row = min(key0 + n * RPI + g, k_hi - 1);
            vv[n] = load16_streaming(vbase + (size_t)row * D);
        }
    };
    auto compute_block = [&](int key0, const uint4 *kk, const uint4 *vv) __attribute__((always_inline)) {
        float t[NLD];
        float mx = -INFINITY;
#pragma unroll
        for (int n = 0; n < NLD; ++n) {
            const unsigned kw[4] = {kk[n].x, kk[n].y, kk[n].z, kk[n].w};
            float a = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const f32x2 f = unpack2<DT>(kw[j]);
                a = __builtin_fmaf(qf[2 * j], f[0], a);
                a = __builtin_fmaf(qf[2 * j + 1], f[1], a);
            }
            a = row_lanes_sum<LPR>(a);
            t[n] = key0 + n * RPI + g < k_hi ? a : -INFINITY;
            mx = fmaxf(mx, t[n]);
        }
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        l *= alpha;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] *= alpha;
#pragma unroll
        for (int n = 0; n < NLD; ++n) {
            const float pn = __builtin_amdgcn_exp2f(t[n] - m_new);
            l += pn;
            const unsigned vw[4] = {vv[n].x, vv[n].y, vv[n].z, vv[n].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const f32x2 f = unpack2<DT>(vw[j]);
                o[2 * j] = __builtin_fmaf(pn, f[0], o[2 * j]);
                o[2 * j + 1] = __builtin_fmaf(pn, f[1], o[2 * j + 1]);
            }
        }
        m = m_new;
    };

    // this wave's blocks: wave, wave + NW, ...; the next block's loads are in flight while one is worked on
    const int nb = k_hi > k_lo ? (k_hi - k_lo + KB - 1) / KB : 0;
    uint4 kb0[NLD], vb0[NLD], kb1[NLD], vb1[NLD];
    if (wave < nb) load_block(k_lo + wave * KB, kb0, vb0);
    for (int i = wave; i < nb; i += 2 * NW) {
        const bool second = i + NW < nb;
        if (second) load_block(k_lo + (i + NW) * KB, kb1, vb1);
        compute_block(k_lo + i * KB, kb0, vb0);
        if (second) {
            if (i + 2 * NW < nb) load_block(k_lo + (i + 2 * NW) * KB, kb0, vb0);
            compute_block(k_lo + (i + NW) * KB, kb1, vb1);
        }
    }

    // ---- merge the workgroup's NG partial states
    const int grp = wave * RPI + g;
#pragma unroll
    for (int j = 0; j < 8; ++j) sm_o[grp][c * 8 + j] = o[j];
    if (c == 0) {
        sm_ml[grp][0] = m;
        sm_ml[grp][1] = l;
    }
    __syncthreads();
    if (tid < D) {
        float M = -1e30f;
#pragma unroll
        for (int q = 0; q < NG; ++q) M = fmaxf(M, sm_ml[q][0]);
        float L = 0.f, O = 0.f;
#pragma unroll
        for (int q = 0; q < NG; ++q) {
            const float w = __builtin_amdgcn_exp2f(sm_ml[q][0] - M);
            L += sm_ml[q][1] * w;
            O += sm_o[q][tid] * w;
        }
        if (p.nsplit == 1) {
            // a single run is the whole result: normalise and store it here, no merge kernel follows
            const float inv = L > 0.f ? 1.f / L : 0.f;
            p.o[(size_t)bh * D + tid] = (uint16_t)pack2<DT>(O * inv, 0.f)[0];
            if (tid == 0) p.lse[bh] = L > 0.f ? (M + __log2f(L)) * 0.6931471805599453f : -INFINITY;
        } else {
            const size_t row = (size_t)sp * gridDim.x + bh;
            p.part_o[row * D + tid] = O;
            if (tid == 0) {
                const float2 ml = {M, L};
                *(float2 *)(p.part_ml + row * 2) = ml;
            }
        }
    }
}

// Merge of the split-KV partial results (the same merge the split mode does between its two
// wave groups): with M = max_s m_s, L = sum_s l_s 2^(m_s - M), the row is
// o = sum_s acc_s 2^(m_s - M) / L and lse = (M + log2 L) ln 2.  A run that saw no visible key
// left m = -1e30, l = 0, acc = 0 and drops out; a row with no visible key at all gets o = 0,
// lse = -inf.  One thread per (row, 4 consecutive d).
template <int DT, int D>
__global__ __launch_bounds__(256) void fa_combine_kernel(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                                         uint16_t *__restrict__ o, float *__restrict__ lse, long long rows,
                                                         int nsplit) {
    constexpr int TPR = D / 4;                    // threads per row
    const long long row = (long long)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
    const int d4 = threadIdx.x % TPR;
    if (row >= rows) return;
    float M = -1e30f;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, part_ml[((size_t)s * rows + row) * 2]);
    float L = 0.f;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < nsplit; ++s) {
        const float2 ml = *(const float2 *)(part_ml + ((size_t)s * rows + row) * 2);
        const float w = __builtin_amdgcn_exp2f(ml.x - M);
        const float4 x = *(const float4 *)(part_o + ((size_t)s * rows + row) * D + 4 * d4);
        L += ml.y * w;
        acc.x += x.x * w;
        acc.y += x.y * w;
        acc.z += x.z * w;
        acc.w += x.w * w;
    }
    const float inv = L > 0.f ? 1.f / L : 0.f;
    const s16x2 a = pack2<DT>(acc.x * inv, acc.y * inv);
    const s16x2 b = pack2<DT>(acc.z * inv, acc.w * inv);
    const s16x4 st = {a[0], a[1], b[0], b[1]};
    *(s16x4 *)(o + (size_t)row * D + 4 * d4) = st;
    if (d4 == 0) lse[row] = L > 0.f ? (M + __log2f(L)) * 0.6931471805599453f : -INFINITY;
}

template <int DT, int D, bool CAUSAL, bool WIDE>
hipError_t launch(const FaParams &p, int nwork_padded, hipStream_t stream) {
    hipLaunchKernelGGL((fa_fwd_kernel<DT, D, CAUSAL, WIDE>), dim3(nwork_padded), dim3(512), 0, stream, p);
    return hipGetLastError();
}

template <int DT, int D>
hipError_t launch_masked(const FaParams &p, int nwork_padded, hipStream_t stream) {
    hipLaunchKernelGGL((fa_fwd_kernel<DT, D, false, true, false, true>), dim3(nwork_padded), dim3(512), 0, stream, p);
    return hipGetLastError();
}

template <int DT, int D, bool CAUSAL>
hipError_t launch_splitkv(const FaParams &p, int nwork_padded, long long rows, hipStream_t stream) {
    hipLaunchKernelGGL((fa_fwd_kernel<DT, D, CAUSAL, true, true>), dim3(nwork_padded, p.nsplit), dim3(512), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    constexpr int RPB = 256 / (D / 4);            // rows per combine block
    hipLaunchKernelGGL((fa_combine_kernel<DT, D>), dim3((unsigned)((rows + RPB - 1) / RPB)), dim3(256), 0, stream,
                       p.part_o, p.part_ml, p.o, p.lse, rows, p.nsplit);
    return hipGetLastError();
}

template <int DT, int D>
hipError_t launch_decode(const FaParams &p, int heads, long long rows, hipStream_t stream) {
    hipLaunchKernelGGL((fa_decode_kernel<DT, D>), dim3(heads, p.nsplit), dim3(DECODE_WAVES * 64), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.nsplit == 1) return e;   // a single run stores o and lse itself
    constexpr int RPB = 256 / (D / 4);
    hipLaunchKernelGGL((fa_combine_kernel<DT, D>), dim3((unsigned)((rows + RPB - 1) / RPB)), dim3(256), 0, stream,
                       p.part_o, p.part_ml, p.o, p.lse, rows, p.nsplit);
    return hipGetLastError();
}

thread_local int g_last_hip_error = 0;



// Shape checks shared by fa_fwd and fa_fwd_plan; everything here runs before any HIP call.
int check_shape(int B, int H, int Nq, int Nk, int D, int dtype) {
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0) return FA_ERR_SHAPE;
    if (D != 64 && D != 128) return FA_ERR_HEADDIM;
    if (dtype != FA_DTYPE_F16 && dtype != FA_DTYPE_BF16) return FA_ERR_DTYPE;
    if ((long long)B * H > 0x7fffffffLL) return FA_ERR_SHAPE;
    if ((long long)B * H * (((long long)Nq + 127) / 128) > 0x7ffffff0LL) return FA_ERR_SHAPE;   // grid size
    if ((long long)Nq + Nk > 0x7fffff00LL) return FA_ERR_SHAPE;                                   // int index arithmetic
    if ((long long)Nk * D * 2 > 0x7fffffffLL) return FA_ERR_SHAPE;                                // 32-bit offsets inside one head of K/V
    return FA_OK;
}

// Work decomposition for a problem, W = B * H * ceil(Nq / 256) being the number of 256-row workgroups
// (the chip has 256 compute units and a D = 128 workgroup fills one).  From a sweep of forced modes
// over 19 causal shapes:
//  * fewer workgroups than compute units: FA_MODE_SPLIT doubles their number and halves their chains;
//  * causal, 1024 <= Nq <= 4096, up to four rounds of workgroups that fill their last round to 85%:
//    FA_MODE_WIDE_FOLD -- every workgroup carries the same triangular work, so whole rounds take
//    equal time, and the waves of finished cheap blocks help with the expensive ones (5-25% faster
//    than the others there; with a poorly filled last round it loses to the split mode, whose
//    workgroups are half the size);
//  * causal, few rounds of long chains otherwise (W < 640 up to Nq = 4096, W < 384 beyond):
//    FA_MODE_SPLIT, whose shorter chains matter more than its extra K/V traffic;
//  * otherwise FA_MODE_WIDE: with many rounds the heavy-first dynamic dispatch evens out the triangle.
// The environment variable FA_FWD_MODE ("split" / "wide" / "fold") overrides.
int choose_mode(int B, int H, int Nq, int causal) {
    const char *env = getenv("FA_FWD_MODE");
    if (env && !strcmp(env, "split")) return FA_MODE_SPLIT;
    if (env && !strcmp(env, "wide")) return FA_MODE_WIDE;
    if (env && !strcmp(env, "fold")) return causal ? FA_MODE_WIDE_FOLD : FA_MODE_WIDE;
    const long long nqt = ((long long)Nq + 255) / 256;
    const long long W = (long long)B * H * nqt;
    if (W < 256) return FA_MODE_SPLIT;
    if (causal && nqt >= 4) {
        const long long rounds = (W + 255) / 256;
        const bool fills_last_round = rounds * 256 * 100 <= W * 115;
        if (Nq <= 4096 && W <= 1024 && fills_last_round) return FA_MODE_WIDE_FOLD;
        if (Nq <= 4096 ? W < 640 : W < 384) return FA_MODE_SPLIT;
    }
    return FA_MODE_WIDE;
}

// 64-key tiles the workgroup of query block qt walks (mirrors the kernel's kmax_wg)
long long tiles_walked(int mode, long long nqt, long long qt, int Nq, int Nk, int causal) {
    const int BM = mode == FA_MODE_SPLIT ? 128 : 256;
    long long kmax = (long long)Nk - 1;
    if (causal) {
        long long last_row = qt * BM + BM - 1;
        if (last_row > (long long)Nq - 1) last_row = (long long)Nq - 1;
        if (mode == FA_MODE_WIDE_FOLD) {
            last_row = -1;
            for (int w = 0; w < 8; ++w) {
                const long long first = (long long)fold_block((int)nqt, (int)qt, w) * 32;
                if (first < Nq) {
                    const long long l = first + 31 < (long long)Nq - 1 ? first + 31 : (long long)Nq - 1;
                    if (l > last_row) last_row = l;
                }
            }
            if (last_row < 0) return 0;
        }
        const long long lim = last_row + ((long long)Nk - Nq);
        if (lim < kmax) kmax = lim;
    }
    return kmax >= 0 ? kmax / BN + 1 : 0;
}

// Split-KV launch shape.  nsplit_in > 0 is taken as given (clamped to the number of key
// tiles); otherwise pick enough runs for one workgroup per compute unit at D = 128 and two at
// D = 64, whose tiles are half the bytes (measured best: the path is bound by HBM, which that
// many workgroups' loads in flight saturate, and every further run only adds its fixed cost
// and its share of the merge), each run at least four tiles long.
// The streaming kernel of the single-query case (fa_decode_kernel) does best with one four-wave workgroup
// per compute unit as well (each wave keeps 32 KiB of loads in flight): more of them only shorten the
// contiguous runs and add partial results to merge (measured: 512 workgroups 1-3% slower, 1024 5-10%).
constexpr int SPLITKV_MAX = 1024;
constexpr long long DECODE_WORKGROUPS = 256;
int choose_nsplit(long long nwork, long long tiles_k, int D, int nsplit_in, bool streaming) {
    long long n = nsplit_in;
    if (n <= 0) {
        long long target = streaming ? DECODE_WORKGROUPS : (D == 128 ? 256 : 512);
        if (streaming)
            if (const char *env = getenv("FA_DECODE_WORKGROUPS")) { const long long v = atoll(env); if (v >= 1) target = v; }
        n = (target + nwork - 1) / nwork;
        if (n > tiles_k / 4) n = tiles_k / 4;
    }
    if (n > tiles_k) n = tiles_k;
    if (n > SPLITKV_MAX) n = SPLITKV_MAX;
    if (n < 1) n = 1;
    return (int)n;
}

// One query row per head goes through the streaming kernel (FA_DECODE=mfma keeps the tile kernel: tests, tuning)
bool use_streaming_decode(int Nq) {
    if (Nq != 1) return false;
    const char *env = getenv("FA_DECODE");
    return !(env && !strcmp(env, "mfma"));
}

template <int DT, int D>
hipError_t launch_pair(const FaParams &p, int nwork_padded, hipStream_t stream) {
    hipLaunchKernelGGL((fa_fwd_kernel<DT, D, true, true, false, false, true>), dim3(nwork_padded), dim3(512), 0, stream, p);
    return hipGetLastError();
}

// the plain instantiations: (split | wide) x dtype x head dimension x causal, and the paired fold (causal only)
hipError_t launch_attention(const FaParams &p, int mode, int D, int causal, int dtype, int grid, hipStream_t st) {
    hipError_t e;
    if (mode == FA_MODE_WIDE_FOLD && causal) {
        switch ((dtype << 1) | (D == 128)) {
            case 0: return launch_pair<0, 64>(p, grid, st);
            case 1: return launch_pair<0, 128>(p, grid, st);
            case 2: return launch_pair<1, 64>(p, grid, st);
            default: return launch_pair<1, 128>(p, grid, st);
        }
    }
    const int key = ((mode != FA_MODE_SPLIT) << 3) | (dtype << 2) | ((D == 128) << 1) | (causal ? 1 : 0);
    switch (key) {
        case 0: e = launch<0, 64, false, false>(p, grid, st); break;
        case 1: e = launch<0, 64, true, false>(p, grid, st); break;
        case 2: e = launch<0, 128, false, false>(p, grid, st); break;
        case 3: e = launch<0, 128, true, false>(p, grid, st); break;
        case 4: e = launch<1, 64, false, false>(p, grid, st); break;
        case 5: e = launch<1, 64, true, false>(p, grid, st); break;
        case 6: e = launch<1, 128, false, false>(p, grid, st); break;
        case 7: e = launch<1, 128, true, false>(p, grid, st); break;
        case 8: e = launch<0, 64, false, true>(p, grid, st); break;
        case 9: e = launch<0, 64, true, true>(p, grid, st); break;
        case 10: e = launch<0, 128, false, true>(p, grid, st); break;
        case 11: e = launch<0, 128, true, true>(p, grid, st); break;
        case 12: e = launch<1, 64, false, true>(p, grid, st); break;
        case 13: e = launch<1, 64, true, true>(p, grid, st); break;
        case 14: e = launch<1, 128, false, true>(p, grid, st); break;
        case 15: e = launch<1, 128, true, true>(p, grid, st); break;
        default: e = hipErrorInvalidValue; break;
    }
    return e;
}

template <int DT, int D>
hipError_t launch_linear(const LinParams &p, int BM, hipStream_t stream) {
    if (BM == 256) hipLaunchKernelGGL((fa_linear_kernel<DT, D, 256>), dim3(p.per_xcd * 8), dim3(512), 0, stream, p);
    else hipLaunchKernelGGL((fa_linear_kernel<DT, D, 128>), dim3(p.per_xcd * 8), dim3(512), 0, stream, p);
    return hipGetLastError();
}

// Row tiles per panel of the projection's tile order.  The c = min(per_xcd, 32) workgroups an XCD runs at a
// time (one per compute unit) are consecutive tiles of its run: R row tiles by c / R column slices, for which
// its L2 fetches R * BM rows of o and (c / R) * 256 columns of w, each K elements long: least for
// R = sqrt(c * 256 / BM).  Measured: 4% on launches of several rounds, nothing on single-round ones.
int linear_panel(int per_xcd, int BM, int m_tiles) {
    const int c = per_xcd < 32 ? per_xcd : 32;
    int R = 1;
    while ((R + 1) * (R + 1) * BM <= c * 256) ++R;
    if (R > m_tiles) R = m_tiles;
    return R < 1 ? 1 : R;
}

// The parameter block every entry point starts from: one launch over the whole of q (no row range,
// no split, no descriptor mask).
FaParams base_params(const void *q, const void *k, const void *v, void *o, float *lse, int H, int Nq, int Nk,
                     long long nqt, long long nwork, float scale) {
    FaParams p;
    p.q = (const uint16_t *)q;
    p.k = (const uint16_t *)k;
    p.v = (const uint16_t *)v;
    p.o = (uint16_t *)o;
    p.lse = lse;
    p.H = H;
    p.Nq = Nq;
    p.Nk = Nk;
    p.q_rows = Nq;
    p.kv_rows = Nk;
    p.off = Nk - Nq;
    p.nqt = (int)nqt;
    p.nwork = (int)nwork;
    p.per_xcd = (int)((nwork + 7) / 8);
    const float LOG2E = 1.4426950408889634f;
    p.qmode = scale > 0.f ? 0 : (scale < 0.f ? 1 : 2);
    p.c = scale == 0.f ? 1.f : fabsf(scale) * LOG2E;
    p.nsplit = 1;
    p.part_o = nullptr;
    p.part_ml = nullptr;
    p.left = p.right = p.prefix = 0;
    p.kv_len = nullptr;
    return p;
}

// Descriptor checks shared by the masked entry points; fills the geometry for `klen` valid keys.
int mask_geometry(const fa_mask_t *mask, int klen, int Nq, int Nk, MaskGeom *g) {
    if (!mask) return FA_ERR_NULL;
    if (Nq <= 0 || Nk <= 0) return FA_ERR_SHAPE;
    if ((long long)Nq + Nk >= MASK_NO_LIMIT) return FA_ERR_SHAPE;   // window arithmetic stays inside int
    if (mask->prefix < 0) return FA_ERR_MASK;
    if (klen < 0 || klen > Nk) return FA_ERR_MASK;
    g->off = Nk - Nq;
    g->left = mask->window_left < 0 || mask->window_left > MASK_NO_LIMIT ? MASK_NO_LIMIT : mask->window_left;
    g->right = mask->window_right < 0 || mask->window_right > MASK_NO_LIMIT ? MASK_NO_LIMIT : mask->window_right;
    g->pfx = mask->prefix < klen ? mask->prefix : klen;
    g->klen = klen;
    return FA_OK;
}

}  // namespace

extern "C" {

int fa_fwd_plan(int B, int H, int Nq, int Nk, int D, int causal, int dtype, fa_plan_t *plan) {
    if (!plan) return FA_ERR_NULL;
    const int rc = check_shape(B, H, Nq, Nk, D, dtype);
    if (rc != FA_OK) return rc;
    const int mode = choose_mode(B, H, Nq, causal);
    const int BM = mode == FA_MODE_SPLIT ? 128 : 256;
    const long long nqt = ((long long)Nq + BM - 1) / BM;
    const long long nwork = (long long)B * H * nqt;
    const long long tiles_k = ((long long)Nk + BN - 1) / BN;
    long long visited = 0;
    for (long long qt = 0; qt < nqt; ++qt) visited += tiles_walked(mode, nqt, qt, Nq, Nk, causal);
    plan->mode = mode;
    plan->block_m = BM;
    plan->block_n = BN;
    plan->threads = 512;
    plan->grid = (int)(((nwork + 7) / 8) * 8);
    plan->work_items = nwork;
    plan->tiles_visited = visited * B * H;
    plan->tiles_total = nwork * tiles_k;
    plan->lds_bytes = (mode == FA_MODE_WIDE ? 1 : 2) * 4 * BN * D * 2;    // sets of 2+2 tiles
    return FA_OK;
}

int fa_fwd(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int Nq, int Nk,
           int D, float scale, int causal, int dtype, void *stream) {
    if (!q || !k || !v || !o || !lse) return FA_ERR_NULL;
    const int rc = check_shape(B, H, Nq, Nk, D, dtype);
    if (rc != FA_OK) return rc;
    if (!isfinite(scale)) return FA_ERR_SCALE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return FA_ERR_ALIGN;
    if ((uintptr_t)lse & 3) return FA_ERR_ALIGN;

    const int mode = choose_mode(B, H, Nq, causal);
    const int BM = mode == FA_MODE_SPLIT ? 128 : 256;   // query rows per workgroup
    const long long nqt = ((long long)Nq + BM - 1) / BM;
    const long long nwork = (long long)B * H * nqt;

    FaParams p = base_params(q, k, v, o, lse, H, Nq, Nk, nqt, nwork, scale);
    const int grid = p.per_xcd * 8;
    hipStream_t st = (hipStream_t)stream;

    const hipError_t e = launch_attention(p, mode, D, causal, dtype, grid, st);
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return FA_ERR_LAUNCH;
    }
    return FA_OK;
}

int fa_fwd_splitkv_plan(int B, int H, int Nq, int Nk, int D, int causal, int dtype, int nsplit,
                        fa_splitkv_plan_t *plan) {
    (void)causal;
    if (!plan) return FA_ERR_NULL;
    const int rc = check_shape(B, H, Nq, Nk, D, dtype);
    if (rc != FA_OK) return rc;
    if (nsplit > SPLITKV_MAX) return FA_ERR_NSPLIT;
    const long long nqt = ((long long)Nq + 255) / 256;
    const long long nwork = (long long)B * H * nqt;
    const long long tiles_k = ((long long)Nk + BN - 1) / BN;
    const bool streaming = use_streaming_decode(Nq);
    const int ns = choose_nsplit(nwork, tiles_k, D, nsplit, streaming);
    const long long rows = (long long)B * H * Nq;
    plan->nsplit = ns;
    plan->streaming = streaming ? 1 : 0;
    plan->grid_x = streaming ? (int)nwork : (int)(((nwork + 7) / 8) * 8);
    plan->grid_y = ns;
    plan->combine_grid = streaming && ns == 1 ? 0 : (int)((rows + (1024 / D) - 1) / (1024 / D));
    plan->work_items = nwork;
    plan->workspace_bytes = (long long)ns * rows * (D + 2) * 4;
    return FA_OK;
}

int fa_fwd_splitkv(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int Nq, int Nk,
                   int D, float scale, int causal, int dtype, int nsplit, void *workspace, long long workspace_bytes,
                   void *stream) {
    if (!q || !k || !v || !o || !lse) return FA_ERR_NULL;
    fa_splitkv_plan_t pl;
    const int rc = fa_fwd_splitkv_plan(B, H, Nq, Nk, D, causal, dtype, nsplit, &pl);
    if (rc != FA_OK) return rc;
    if (!isfinite(scale)) return FA_ERR_SCALE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return FA_ERR_ALIGN;
    if ((uintptr_t)lse & 3) return FA_ERR_ALIGN;
    if (!workspace || workspace_bytes < pl.workspace_bytes) return FA_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 15) return FA_ERR_ALIGN;
    const long long rows = (long long)B * H * Nq;
    if (rows > 0x7fffffffLL * 8) return FA_ERR_SHAPE;   // combine grid

    FaParams p = base_params(q, k, v, o, lse, H, Nq, Nk, ((long long)Nq + 255) / 256, pl.work_items, scale);
    p.nsplit = pl.nsplit;
    p.part_o = (float *)workspace;
    p.part_ml = p.part_o + (size_t)pl.nsplit * rows * D;
    hipStream_t st = (hipStream_t)stream;

    hipError_t e;
    if (pl.streaming) {
        // one query sees every key under the bottom-right-aligned causal mask: causal or not is the same
        switch ((dtype << 1) | (D == 128)) {
            case 0: e = launch_decode<0, 64>(p, pl.grid_x, rows, st); break;
            case 1: e = launch_decode<0, 128>(p, pl.grid_x, rows, st); break;
            case 2: e = launch_decode<1, 64>(p, pl.grid_x, rows, st); break;
            default: e = launch_decode<1, 128>(p, pl.grid_x, rows, st); break;
        }
        if (e != hipSuccess) {
            g_last_hip_error = (int)e;
            return FA_ERR_LAUNCH;
        }
        return FA_OK;
    }
    const int key = (dtype << 2) | ((D == 128) << 1) | (causal ? 1 : 0);
    switch (key) {
        case 0: e = launch_splitkv<0, 64, false>(p, pl.grid_x, rows, st); break;
        case 1: e = launch_splitkv<0, 64, true>(p, pl.grid_x, rows, st); break;
        case 2: e = launch_splitkv<0, 128, false>(p, pl.grid_x, rows, st); break;
        case 3: e = launch_splitkv<0, 128, true>(p, pl.grid_x, rows, st); break;
        case 4: e = launch_splitkv<1, 64, false>(p, pl.grid_x, rows, st); break;
        case 5: e = launch_splitkv<1, 64, true>(p, pl.grid_x, rows, st); break;
        case 6: e = launch_splitkv<1, 128, false>(p, pl.grid_x, rows, st); break;
        case 7: e = launch_splitkv<1, 128, true>(p, pl.grid_x, rows, st); break;
        default: return FA_ERR_SHAPE;
    }
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return FA_ERR_LAUNCH;
    }
    return FA_OK;
}

int fa_fwd_masked(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int Nq, int Nk,
                  int D, float scale, const fa_mask_t *mask, int dtype, void *stream) {
    if (!q || !k || !v || !o || !lse || !mask) return FA_ERR_NULL;
    const int rc = check_shape(B, H, Nq, Nk, D, dtype);
    if (rc != FA_OK) return rc;
    if (!isfinite(scale)) return FA_ERR_SCALE;
    MaskGeom g;
    const int mrc = mask_geometry(mask, Nk, Nq, Nk, &g);
    if (mrc != FA_OK) return mrc;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return FA_ERR_ALIGN;
    if (((uintptr_t)lse | (uintptr_t)mask->kv_len) & 3) return FA_ERR_ALIGN;

    const long long nqt = ((long long)Nq + 255) / 256;
    const long long nwork = (long long)B * H * nqt;
    FaParams p = base_params(q, k, v, o, lse, H, Nq, Nk, nqt, nwork, scale);
    p.left = g.left;
    p.right = g.right;
    p.prefix = mask->prefix < Nk ? mask->prefix : Nk;
    p.kv_len = mask->kv_len;
    const int grid = p.per_xcd * 8;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    switch ((dtype << 1) | (D == 128)) {
        case 0: e = launch_masked<0, 64>(p, grid, st); break;
        case 1: e = launch_masked<0, 128>(p, grid, st); break;
        case 2: e = launch_masked<1, 64>(p, grid, st); break;
        case 3: e = launch_masked<1, 128>(p, grid, st); break;
        default: return FA_ERR_SHAPE;
    }
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return FA_ERR_LAUNCH;
    }
    return FA_OK;
}

int fa_attn_linear_block(const void *q, const void *k, const void *v, const void *w, void *o, float *lse, float *y,
                         int B, int H, int Nq, int Nk, int D, int N, float scale, int causal, int dtype,
                         int row_first, int row_count, void *stream) {
    if (!q || !k || !v || !w || !o || !lse || !y) return FA_ERR_NULL;
    const int rc = check_shape(B, H, Nq, Nk, D, dtype);
    if (rc != FA_OK) return rc;
    if (N <= 0 || N % 256 != 0 || (long long)N * H * D * 2 > 0x7fffffffLL) return FA_ERR_SHAPE;
    if ((long long)Nq * D * 2 > 0x7fffffffLL) return FA_ERR_SHAPE;          // 32-bit offsets inside one head of o
    if (row_first < 0 || row_count <= 0 || (long long)row_first + row_count > Nq) return FA_ERR_SHAPE;
    if (!isfinite(scale)) return FA_ERR_SCALE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o | (uintptr_t)w) & 15) return FA_ERR_ALIGN;
    if (((uintptr_t)lse | (uintptr_t)y) & 3) return FA_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;

    // 1. attention of the block's rows, every head: a launch over row_count rows whose diagonal is shifted
    //    by row_first; q, o, lse keep the full tensors' head pitch
    {
        const int mode = choose_mode(B, H, row_count, causal);
        const int BM = mode == FA_MODE_SPLIT ? 128 : 256;
        const long long nqt = ((long long)row_count + BM - 1) / BM;
        const long long nwork = (long long)B * H * nqt;
        FaParams p = base_params((const uint16_t *)q + (size_t)row_first * D, k, v, (uint16_t *)o + (size_t)row_first * D,
                                 lse + row_first, H, row_count, Nk, nqt, nwork, scale);
        p.q_rows = Nq;
        p.off = Nk - Nq + row_first;
        const hipError_t e = launch_attention(p, mode, D, causal, dtype, p.per_xcd * 8, st);
        if (e != hipSuccess) {
            g_last_hip_error = (int)e;
            return FA_ERR_LAUNCH;
        }
    }
    // 2. the block's rows of y = (heads side by side) x w
    {
        LinParams lp;
        lp.o = (const uint16_t *)o;
        lp.w = (const uint16_t *)w;
        lp.y = y;
        lp.H = H;
        lp.q_rows = Nq;
        lp.N = N;
        lp.s0 = row_first;
        lp.rows = row_count;
        lp.n_tiles = N / 256;
        // 256-row tiles (less LDS traffic per matrix instruction, twice the work per barrier) when they still
        // give every compute unit a workgroup; FA_LINEAR_TILE=128|256 overrides (tests, tuning)
        int BM = (long long)B * ((row_count + 255) / 256) * lp.n_tiles >= 256 ? 256 : 128;
        if (const char *env = getenv("FA_LINEAR_TILE")) BM = !strcmp(env, "256") ? 256 : (!strcmp(env, "128") ? 128 : BM);
        lp.mt_per_b = (row_count + BM - 1) / BM;
        const long long tiles = (long long)B * lp.mt_per_b * lp.n_tiles;
        if (tiles > 0x7ffffff0LL) return FA_ERR_SHAPE;
        lp.ntile_total = (int)tiles;
        lp.per_xcd = (int)((tiles + 7) / 8);
        lp.panel = linear_panel(lp.per_xcd, BM, B * lp.mt_per_b);
        if (const char *env = getenv("FA_LINEAR_PANEL")) {   // tests, tuning
            const int v = atoi(env);
            if (v >= 1) lp.panel = v < B * lp.mt_per_b ? v : B * lp.mt_per_b;
        }
        hipError_t e;
        switch ((dtype << 1) | (D == 128)) {
            case 0: e = launch_linear<0, 64>(lp, BM, st); break;
            case 1: e = launch_linear<0, 128>(lp, BM, st); break;
            case 2: e = launch_linear<1, 64>(lp, BM, st); break;
            default: e = launch_linear<1, 128>(lp, BM, st); break;
        }
        if (e != hipSuccess) {
            g_last_hip_error = (int)e;
            return FA_ERR_LAUNCH;
        }
    }
    return FA_OK;
}

int fa_attn_linear(const void *q, const void *k, const void *v, const void *w, void *o, float *lse, float *y, int B,
                   int H, int Nq, int Nk, int D, int N, float scale, int causal, int dtype, int rows_per_block,
                   void *stream) {
    if (rows_per_block <= 0 || rows_per_block >= Nq)
        return fa_attn_linear_block(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, scale, causal, dtype, 0, Nq, stream);
    // the first block is half size (section 4.2: nothing overlaps with the first block's computation)
    int first = rows_per_block / 2 > 0 ? rows_per_block / 2 : rows_per_block;
    for (int r = 0; r < Nq;) {
        const int n = r == 0 ? first : (Nq - r < rows_per_block ? Nq - r : rows_per_block);
        const int rc = fa_attn_linear_block(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, scale, causal, dtype, r, n, stream);
        if (rc != FA_OK) return rc;
        r += n;
    }
    return FA_OK;
}

int fa_mask_tile_class(const fa_mask_t *mask, int kv_len, int Nq, int Nk, int row_first, int row_last, int key_first) {
    MaskGeom g;
    const int rc = mask_geometry(mask, kv_len, Nq, Nk, &g);
    if (rc != FA_OK) return rc;
    if (row_first < 0 || row_last < row_first || row_last >= Nq || key_first < 0 || key_first >= Nk) return FA_ERR_SHAPE;
    if (key_first % BN) return FA_ERR_SHAPE;
    return tile_class(row_tiles(g, row_first, row_last), key_first / BN);
}

int fa_mask_tile_walk(const fa_mask_t *mask, int kv_len, int Nq, int Nk, int row_first, int row_last,
                      int *prefix_tiles, int *window_first_tile, int *count, int *window_rotation) {
    if (!prefix_tiles || !window_first_tile || !count || !window_rotation) return FA_ERR_NULL;
    MaskGeom g;
    const int rc = mask_geometry(mask, kv_len, Nq, Nk, &g);
    if (rc != FA_OK) return rc;
    if (row_first < 0 || row_last < row_first || row_last >= Nq) return FA_ERR_SHAPE;
    const TileSeq sq = tile_sequence(g, row_first, row_last);
    *prefix_tiles = sq.np;
    *window_first_tile = sq.base;
    *count = sq.count;
    *window_rotation = sq.rot;
    return FA_OK;
}

int fa_mask_interior_run(const fa_mask_t *mask, int kv_len, int Nq, int Nk, int wg_row_first, int wg_row_last,
                         int row_first, int row_last, int *first, int *count) {
    if (!first || !count) return FA_ERR_NULL;
    MaskGeom g;
    const int rc = mask_geometry(mask, kv_len, Nq, Nk, &g);
    if (rc != FA_OK) return rc;
    if (wg_row_first < 0 || wg_row_last < wg_row_first || wg_row_last >= Nq) return FA_ERR_SHAPE;
    if (row_first < wg_row_first || row_last < row_first || row_last > wg_row_last) return FA_ERR_SHAPE;
    const Run r = interior_run(row_tiles(g, row_first, row_last), tile_sequence(g, wg_row_first, wg_row_last), Nk);
    *first = r.first;
    *count = r.count;
    return FA_OK;
}

int fa_mfma_probe(int dtype, int operands, int iters, float *scratch, long long *flops, void *stream) {
    if (!scratch || !flops) return FA_ERR_NULL;
    if (dtype != FA_DTYPE_F16 && dtype != FA_DTYPE_BF16) return FA_ERR_DTYPE;
    if (operands != 0 && operands != 1) return FA_ERR_SHAPE;
    if (iters <= 0 || iters > (1 << 24)) return FA_ERR_SHAPE;
    if ((uintptr_t)scratch & 3) return FA_ERR_ALIGN;
    const int grid = 256;                                   // one workgroup of 8 waves per compute unit
    hipStream_t st = (hipStream_t)stream;
    switch ((dtype << 1) | operands) {
        case 0: hipLaunchKernelGGL((fa_mfma_probe_kernel<0, false>), dim3(grid), dim3(512), 0, st, scratch, iters); break;
        case 1: hipLaunchKernelGGL((fa_mfma_probe_kernel<0, true>), dim3(grid), dim3(512), 0, st, scratch, iters); break;
        case 2: hipLaunchKernelGGL((fa_mfma_probe_kernel<1, false>), dim3(grid), dim3(512), 0, st, scratch, iters); break;
        default: hipLaunchKernelGGL((fa_mfma_probe_kernel<1, true>), dim3(grid), dim3(512), 0, st, scratch, iters); break;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return FA_ERR_LAUNCH;
    }
    *flops = (long long)grid * 8 * iters * 4 * (2LL * 32 * 32 * 16);
    return FA_OK;
}

const char *fa_strerror(int code) {
    switch (code) {
        case FA_OK: return "success";
        case FA_ERR_NULL: return "a required pointer is NULL";
        case FA_ERR_SHAPE: return "B, H, Nq, Nk must be positive and the problem must be indexable";
        case FA_ERR_HEADDIM: return "head dimension D must be 64 or 128";
        case FA_ERR_DTYPE: return "dtype must be 0 (fp16) or 1 (bf16)";
        case FA_ERR_SCALE: return "scale must be finite";
        case FA_ERR_ALIGN: return "q, k, v, o must be 16-byte aligned and lse 4-byte aligned";
        case FA_ERR_LAUNCH: return "the HIP runtime rejected the kernel launch";
        case FA_ERR_WORKSPACE: return "workspace is NULL or smaller than fa_fwd_splitkv_plan reports";
        case FA_ERR_NSPLIT: return "nsplit exceeds 1024";
        case FA_ERR_MASK: return "mask descriptor: prefix must be >= 0 and a key count within 0..Nk";
        default: return "unknown error code";
    }
}

int fa_version(void) { return 200; }

int fa_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
