// Exact attention forward for gfx950 (MI355X): kernels and the C ABI of include/fa.h.
//
// Dataflow (FastAttention appendix A, the FlashAttention2 forward): for each block of
// queries, walk the key/value blocks once; per block compute the logits on the matrix
// cores, exponentiate against a running reference, multiply by V on the matrix cores,
// and carry the reference / row sum.  Mask handling follows section 4.1: blocks that are
// entirely masked are skipped, blocks that are entirely visible take no mask, and only the
// others get a per-element predicate computed from indices -- no mask tensor exists.
//
// Where things are (the .inc files are fragments of this one translation unit, included below):
//  * fa_attention_kernel.inc -- fa_fwd_kernel, the attention kernel, one source for every variant (template
//    flags): WIDE (256 query rows per workgroup, all eight waves walk the same tiles) or split (128 rows, two
//    groups of four waves on alternate tiles, merged through LDS); CAUSAL; PAIR (folded rows for short causal
//    problems); SPLITKV (one run of the key tiles per workgroup, unnormalised result to a workspace); GENMASK
//    (window / prefix / key-count masks from a descriptor).  Entry points fa_fwd, fa_fwd_splitkv, fa_fwd_masked.
//  * fa_decode_kernels.inc -- fa_decode_kernel, the single-query decoding step with K/V streamed through
//    registers, and fa_combine_kernel, which merges the split-KV runs.
//  * fa_linear_kernel.inc -- the output projection that follows the attention block by block (section 4.2),
//    entry points fa_attn_linear_block / fa_attn_linear.
//  * fa_mask.inc -- descriptor masks: tile classification and walk, shared by the kernel and the host entry
//    points fa_mask_*.
//  * fa_types.inc, fa_device.inc -- vector types and parameter block; device helpers (LDS swizzles,
//    global-to-LDS load, cross-half exchange).
//  * this file -- the host side: argument checks, choice of decomposition, launch shapes, the C ABI.
//
// gfx950 mapping common to all variants of the attention kernel (this library's own design):
//  * one wavefront owns 32 query rows; a workgroup is 8 wavefronts, two per SIMD.  Each wavefront
//    runs a tile as three clusters (logits, softmax, second product); overlap of the matrix and
//    vector units comes mostly from the two wavefronts of a SIMD being in different clusters; they
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

#include <atomic>
#include <mutex>
#include <type_traits>
#include <utility>

#include "../../include/fa.h"

// Workspace of fa_fwd_splitkv_static: the split-KV partial results of callers that cannot pass a workspace of their
// own.  Every GPU the library's code object is loaded on holds its own copy at its own address, until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress, never a device address.
#define FA_STATIC_WORKSPACE_BYTES (64ll << 20)
static __device__ __align__(256) unsigned char scratch[FA_STATIC_WORKSPACE_BYTES];

namespace {

#include "fa_types.inc"
#include "fa_mask.inc"
#include "fa_device.inc"
#include "fa_attention_kernel.inc"
#include "fa_attention_wide64_kernel.inc"
#include "fa_linear_kernel.inc"
#include "fa_decode_kernels.inc"

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
hipError_t launch_splitkv(const FaParams &p, int nwork_padded, long long rows, bool long_runs, hipStream_t stream) {
    // long runs of a compute-bound shape (several query blocks per head) at D = 128: the 64-row waves with the
    // pipelined loop; everything else the tile kernel's split-KV instantiation, which is tuned for streaming K/V
    if constexpr (D == 128) {
        if (long_runs)
            hipLaunchKernelGGL((fa_fwd_wide64_kernel<DT, CAUSAL, true>), dim3(nwork_padded, p.nsplit), dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL((fa_fwd_kernel<DT, D, CAUSAL, true, true>), dim3(nwork_padded, p.nsplit), dim3(512), 0, stream, p);
    } else {
        hipLaunchKernelGGL((fa_fwd_kernel<DT, D, CAUSAL, true, true>), dim3(nwork_padded, p.nsplit), dim3(512), 0, stream, p);
    }
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

// single query under a mask descriptor: p.nsplit workgroups per (batch, head); a single one stores o and lse itself
template <int DT, int D>
hipError_t launch_decode_masked(const FaParams &p, int heads, hipStream_t stream) {
    hipLaunchKernelGGL((fa_decode_kernel<DT, D, true>), dim3(heads, p.nsplit), dim3(DECODE_WAVES * 64), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.nsplit == 1) return e;
    constexpr int RPB = 256 / (D / 4);
    hipLaunchKernelGGL((fa_combine_kernel<DT, D>), dim3((unsigned)((heads + RPB - 1) / RPB)), dim3(256), 0, stream,
                       p.part_o, p.part_ml, p.o, p.lse, (long long)heads, p.nsplit);
    return hipGetLastError();
}

thread_local int g_last_hip_error = 0;

// fa_set_option's values (FA_AUTO: the library chooses).  Every entry point reads each of them at most once per call.
std::atomic<int> g_options[5] = {{FA_AUTO}, {FA_AUTO}, {FA_AUTO}, {FA_AUTO}, {FA_AUTO}};
int option(int which) { return g_options[which].load(std::memory_order_relaxed); }

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

// One query row per head goes through the streaming kernel (FA_OPT_DECODE_KERNEL = 1 keeps the tile kernel:
// tests, tuning)
bool use_streaming_decode(int Nq) { return Nq == 1 && option(FA_OPT_DECODE_KERNEL) != 1; }

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
// fa_set_option(FA_OPT_FWD_MODE, ...) overrides.
int choose_mode(int B, int H, int Nq, int Nk, int D, int causal) {
    const int forced = option(FA_OPT_FWD_MODE);
    if (forced == FA_MODE_SPLIT || forced == FA_MODE_WIDE) return forced;
    if (forced == FA_MODE_WIDE64) return D == 128 ? FA_MODE_WIDE64 : FA_MODE_WIDE;
    if (forced == FA_MODE_WIDE_FOLD) return causal ? FA_MODE_WIDE_FOLD : FA_MODE_WIDE;
    const long long nqt = ((long long)Nq + 255) / 256;
    const long long W = (long long)B * H * nqt;
    if (W < 256) return FA_MODE_SPLIT;
    if (causal && nqt >= 4) {
        const long long rounds = (W + 255) / 256;
        const bool fills_last_round = rounds * 256 * 100 <= W * 115;
        if (Nq <= 4096 && W <= 1024 && fills_last_round) return FA_MODE_WIDE_FOLD;
        if (Nq <= 4096 ? W < 640 : W < 384) return FA_MODE_SPLIT;
    }
    // long walks at D = 128: the 64-row waves with the pipelined loop (the loop takes whole unmasked tiles two at
    // a time, so it needs walks long enough to consist mostly of those: measured faster from about 64 tiles per
    // workgroup on average -- 1-2% -- and 2-14% slower at 32 tiles and below)
    const long long avg_keys = causal ? (long long)Nk - Nq / 2 : (long long)Nk;
    if (D == 128 && avg_keys >= 4096) return FA_MODE_WIDE64;
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
        const long long target = streaming ? DECODE_WORKGROUPS : (D == 128 ? 256 : 512);
        n = (target + nwork - 1) / nwork;
        if (n > tiles_k / 4) n = tiles_k / 4;
    }
    if (n > tiles_k) n = tiles_k;
    if (n > SPLITKV_MAX) n = SPLITKV_MAX;
    if (n < 1) n = 1;
    return (int)n;
}

template <int DT, int D>
hipError_t launch_pair(const FaParams &p, int nwork_padded, hipStream_t stream) {
    hipLaunchKernelGGL((fa_fwd_kernel<DT, D, true, true, false, false, true>), dim3(nwork_padded), dim3(512), 0, stream, p);
    return hipGetLastError();
}

// the plain instantiations: (split | wide) x dtype x head dimension x causal, and the paired fold (causal only)
hipError_t launch_attention(const FaParams &p, int mode, int D, int causal, int dtype, int grid, hipStream_t st) {
    hipError_t e;
    if (mode == FA_MODE_WIDE64) {
        if (D != 128) return hipErrorInvalidValue;
        if (dtype == 0 && causal) hipLaunchKernelGGL((fa_fwd_wide64_kernel<0, true>), dim3(grid), dim3(256), 0, st, p);
        else if (dtype == 0) hipLaunchKernelGGL((fa_fwd_wide64_kernel<0, false>), dim3(grid), dim3(256), 0, st, p);
        else if (causal) hipLaunchKernelGGL((fa_fwd_wide64_kernel<1, true>), dim3(grid), dim3(256), 0, st, p);
        else hipLaunchKernelGGL((fa_fwd_wide64_kernel<1, false>), dim3(grid), dim3(256), 0, st, p);
        return hipGetLastError();
    }
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
    p.kv_stream = 0;
    p.part_o = nullptr;
    p.part_ml = nullptr;
    p.left = p.right = p.prefix = 0;
    p.anchor = 0;
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
    if (mask->diag_from_kv_len != 0 && mask->diag_from_kv_len != 1) return FA_ERR_MASK;
    g->off = (mask->diag_from_kv_len ? klen : Nk) - Nq;
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
    const long long tiles_k = ((long long)Nk + BN - 1) / BN;
    if (use_streaming_decode(Nq)) {
        // one query per head (it sees every key, causal or not): fa_decode_kernel, one workgroup per (batch, head)
        plan->mode = FA_MODE_STREAM;
        plan->block_m = 1;
        plan->block_n = BN;
        plan->threads = DECODE_WAVES * 64;
        plan->grid = B * H;
        plan->work_items = (long long)B * H;
        plan->tiles_visited = plan->tiles_total = (long long)B * H * tiles_k;
        plan->lds_bytes = DECODE_WAVES * (512 / D) * (D + 2) * 4;     // one partial state per lane group
        return FA_OK;
    }
    const int mode = choose_mode(B, H, Nq, Nk, D, causal);
    const int BM = mode == FA_MODE_SPLIT ? 128 : 256;
    const long long nqt = ((long long)Nq + BM - 1) / BM;
    const long long nwork = (long long)B * H * nqt;
    long long visited = 0;
    for (long long qt = 0; qt < nqt; ++qt) visited += tiles_walked(mode, nqt, qt, Nq, Nk, causal);
    plan->mode = mode;
    plan->block_m = BM;
    plan->block_n = BN;
    plan->threads = mode == FA_MODE_WIDE64 ? 256 : 512;
    plan->grid = (int)(((nwork + 7) / 8) * 8);
    plan->work_items = nwork;
    plan->tiles_visited = visited * B * H;
    plan->tiles_total = nwork * tiles_k;
    plan->lds_bytes = (mode == FA_MODE_WIDE ? 1 : 2) * 4 * BN * D * 2;    // sets of 2+2 tiles
    if (mode == FA_MODE_WIDE64) plan->lds_bytes = 4 * (16 * 1088 + BN * D * 2);   // ring of four (padded K tile, V tile)
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

    const int mode = use_streaming_decode(Nq) ? FA_MODE_STREAM : choose_mode(B, H, Nq, Nk, D, causal);
    const int BM = mode == FA_MODE_SPLIT ? 128 : 256;   // query rows per workgroup
    const long long nqt = ((long long)Nq + BM - 1) / BM;
    const long long nwork = (long long)B * H * nqt;

    FaParams p = base_params(q, k, v, o, lse, H, Nq, Nk, nqt, nwork, scale);
    const int grid = p.per_xcd * 8;
    hipStream_t st = (hipStream_t)stream;

    hipError_t e;
    if (mode == FA_MODE_STREAM) {
        // a single query per head: the streaming kernel, one run per (batch, head), which stores o and lse itself
        switch ((dtype << 1) | (D == 128)) {
            case 0: e = launch_decode<0, 64>(p, (int)nwork, nwork, st); break;
            case 1: e = launch_decode<0, 128>(p, (int)nwork, nwork, st); break;
            case 2: e = launch_decode<1, 64>(p, (int)nwork, nwork, st); break;
            default: e = launch_decode<1, 128>(p, (int)nwork, nwork, st); break;
        }
    } else {
        e = launch_attention(p, mode, D, causal, dtype, grid, st);
    }
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
    plan->combine_grid = ns == 1 ? 0 : (int)((rows + (1024 / D) - 1) / (1024 / D));   // a single run is fa_fwd's launch
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
    // a single run has nothing to merge: it is fa_fwd's launch (whose decompositions beat a one-run walk of
    // the split-KV kernel by about 5% when there are enough query blocks to fill the chip without splitting)
    if (pl.nsplit == 1) return fa_fwd(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, stream);

    FaParams p = base_params(q, k, v, o, lse, H, Nq, Nk, ((long long)Nq + 255) / 256, pl.work_items, scale);
    p.nsplit = pl.nsplit;
    p.kv_stream = Nq <= 256;
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
    // keys a query sees per run, on average (as in choose_mode): from 4096 the wide64 kernel is the faster one
    const long long avg_keys = causal ? (long long)Nk - Nq / 2 : (long long)Nk;
    const bool long_runs = D == 128 && !p.kv_stream && option(FA_OPT_FWD_MODE) != FA_MODE_WIDE &&
                           avg_keys / pl.nsplit >= 4096;
    const int key = (dtype << 2) | ((D == 128) << 1) | (causal ? 1 : 0);
    switch (key) {
        case 0: e = launch_splitkv<0, 64, false>(p, pl.grid_x, rows, long_runs, st); break;
        case 1: e = launch_splitkv<0, 64, true>(p, pl.grid_x, rows, long_runs, st); break;
        case 2: e = launch_splitkv<0, 128, false>(p, pl.grid_x, rows, long_runs, st); break;
        case 3: e = launch_splitkv<0, 128, true>(p, pl.grid_x, rows, long_runs, st); break;
        case 4: e = launch_splitkv<1, 64, false>(p, pl.grid_x, rows, long_runs, st); break;
        case 5: e = launch_splitkv<1, 64, true>(p, pl.grid_x, rows, long_runs, st); break;
        case 6: e = launch_splitkv<1, 128, false>(p, pl.grid_x, rows, long_runs, st); break;
        case 7: e = launch_splitkv<1, 128, true>(p, pl.grid_x, rows, long_runs, st); break;
        default: return FA_ERR_SHAPE;
    }
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return FA_ERR_LAUNCH;
    }
    return FA_OK;
}

int fa_fwd_splitkv_static(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int Nq,
                          int Nk, int D, float scale, int causal, int dtype, int nsplit, void *stream) {
    // every argument check first (no HIP call before them), the size limit among them
    if (!q || !k || !v || !o || !lse) return FA_ERR_NULL;
    fa_splitkv_plan_t pl;
    const int rc = fa_fwd_splitkv_plan(B, H, Nq, Nk, D, causal, dtype, nsplit, &pl);
    if (rc != FA_OK) return rc;
    if (!isfinite(scale)) return FA_ERR_SCALE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return FA_ERR_ALIGN;
    if ((uintptr_t)lse & 3) return FA_ERR_ALIGN;
    if (pl.nsplit == 1) return fa_fwd(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, stream);   // nothing to merge
    if (pl.workspace_bytes > FA_STATIC_WORKSPACE_BYTES) return FA_ERR_WORKSPACE;
    void *ws = nullptr;
    {
        // the array's device address on the current GPU, asked for once per device and kept
        constexpr int MAX_DEVICES = 64;
        static std::mutex lock;
        static void *address[MAX_DEVICES] = {};
        int dev = -1;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess && (dev < 0 || dev >= MAX_DEVICES)) e = hipErrorInvalidDevice;
        if (e == hipSuccess) {
            std::lock_guard<std::mutex> guard(lock);
            if (!address[dev]) {
                void *ptr = nullptr;
                e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
                if (e == hipSuccess && !ptr) e = hipErrorInvalidSymbol;
                if (e == hipSuccess) address[dev] = ptr;
            }
            ws = address[dev];
        }
        if (e != hipSuccess) {
            g_last_hip_error = (int)e;
            return FA_ERR_LAUNCH;
        }
    }
    return fa_fwd_splitkv(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, nsplit, ws, FA_STATIC_WORKSPACE_BYTES,
                          stream);
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
    p.anchor = mask->diag_from_kv_len;
    const int grid = p.per_xcd * 8;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (use_streaming_decode(Nq)) {
        // one query per head: the streaming kernel walks the prefix and the window as runs of consecutive keys
        switch ((dtype << 1) | (D == 128)) {
            case 0: e = launch_decode_masked<0, 64>(p, (int)nwork, st); break;
            case 1: e = launch_decode_masked<0, 128>(p, (int)nwork, st); break;
            case 2: e = launch_decode_masked<1, 64>(p, (int)nwork, st); break;
            default: e = launch_decode_masked<1, 128>(p, (int)nwork, st); break;
        }
        if (e != hipSuccess) {
            g_last_hip_error = (int)e;
            return FA_ERR_LAUNCH;
        }
        return FA_OK;
    }
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

int fa_decode_masked(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int Nk, int D,
                     float scale, const fa_mask_t *mask, int dtype, int nsplit, void *workspace,
                     long long workspace_bytes, void *stream) {
    if (!q || !k || !v || !o || !lse || !mask) return FA_ERR_NULL;
    fa_splitkv_plan_t pl;
    const int rc = fa_fwd_splitkv_plan(B, H, 1, Nk, D, 0, dtype, nsplit, &pl);
    if (rc != FA_OK) return rc;
    if (!isfinite(scale)) return FA_ERR_SCALE;
    MaskGeom g;
    const int mrc = mask_geometry(mask, Nk, 1, Nk, &g);
    if (mrc != FA_OK) return mrc;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return FA_ERR_ALIGN;
    if (((uintptr_t)lse | (uintptr_t)mask->kv_len) & 3) return FA_ERR_ALIGN;
    if (pl.nsplit > 1) {
        if (!workspace || workspace_bytes < pl.workspace_bytes) return FA_ERR_WORKSPACE;
        if ((uintptr_t)workspace & 15) return FA_ERR_ALIGN;
    }
    const long long heads = (long long)B * H;
    FaParams p = base_params(q, k, v, o, lse, H, 1, Nk, 1, heads, scale);
    p.left = g.left;
    p.right = g.right;
    p.prefix = mask->prefix < Nk ? mask->prefix : Nk;
    p.kv_len = mask->kv_len;
    p.anchor = mask->diag_from_kv_len;
    p.nsplit = pl.nsplit;
    p.part_o = (float *)workspace;
    p.part_ml = p.part_o + (size_t)pl.nsplit * heads * D;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    switch ((dtype << 1) | (D == 128)) {
        case 0: e = launch_decode_masked<0, 64>(p, (int)heads, st); break;
        case 1: e = launch_decode_masked<0, 128>(p, (int)heads, st); break;
        case 2: e = launch_decode_masked<1, 64>(p, (int)heads, st); break;
        default: e = launch_decode_masked<1, 128>(p, (int)heads, st); break;
    }
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return FA_ERR_LAUNCH;
    }
    return FA_OK;
}

namespace {

int check_attn_linear(const void *q, const void *k, const void *v, const void *w, void *o, float *lse, float *y,
                      int B, int H, int Nq, int Nk, int D, int N, float scale, int dtype, int row_first, int row_count) {
    if (!q || !k || !v || !w || !o || !lse || !y) return FA_ERR_NULL;
    const int rc = check_shape(B, H, Nq, Nk, D, dtype);
    if (rc != FA_OK) return rc;
    if (N <= 0 || N % 256 != 0 || (long long)N * H * D * 2 > 0x7fffffffLL) return FA_ERR_SHAPE;
    if ((long long)Nq * D * 2 > 0x7fffffffLL) return FA_ERR_SHAPE;          // 32-bit offsets inside one head of o
    if (row_first < 0 || row_count <= 0 || (long long)row_first + row_count > Nq) return FA_ERR_SHAPE;
    if (!isfinite(scale)) return FA_ERR_SCALE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o | (uintptr_t)w) & 15) return FA_ERR_ALIGN;
    if (((uintptr_t)lse | (uintptr_t)y) & 3) return FA_ERR_ALIGN;
    return FA_OK;
}

// attention of one block of rows, every head: a launch over row_count rows whose diagonal is shifted by
// row_first; q, o, lse keep the full tensors' head pitch.  Arguments already checked.
int block_attention(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int Nq, int Nk,
                    int D, float scale, int causal, int dtype, int row_first, int row_count, hipStream_t st) {
    {
        // (the keys the block's rows can see end at its last row's diagonal)
        const int nk_seen = causal ? Nk - (Nq - row_first - row_count) : Nk;
        const int mode = choose_mode(B, H, row_count, nk_seen > 0 ? nk_seen : 1, D, causal);
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
    return FA_OK;
}

// the block's rows of y = (heads side by side) x w.  Arguments already checked.
int block_projection(const void *w, const void *o, float *y, int B, int H, int Nq, int D, int N, int dtype,
                     int row_first, int row_count, hipStream_t st) {
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
        // give every compute unit a workgroup; FA_OPT_LINEAR_TILE overrides (tests, tuning)
        int BM = (long long)B * ((row_count + 255) / 256) * lp.n_tiles >= 256 ? 256 : 128;
        if (const int forced = option(FA_OPT_LINEAR_TILE); forced == 128 || forced == 256) BM = forced;
        lp.mt_per_b = (row_count + BM - 1) / BM;
        const long long tiles = (long long)B * lp.mt_per_b * lp.n_tiles;
        if (tiles > 0x7ffffff0LL) return FA_ERR_SHAPE;
        lp.ntile_total = (int)tiles;
        lp.per_xcd = (int)((tiles + 7) / 8);
        lp.panel = linear_panel(lp.per_xcd, BM, B * lp.mt_per_b);
        if (const int v = option(FA_OPT_LINEAR_PANEL); v >= 1)   // tests, tuning
            lp.panel = v < B * lp.mt_per_b ? v : B * lp.mt_per_b;
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

// fa_attn_linear's second stream (default priority) and the two events that tie it to the caller's stream, one
// set per device, created on the first call that may create them (not under stream capture) and kept until the
// process ends.  `busy` serialises the enqueueing of calls that share them.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t attn_done = nullptr, joined = nullptr;
    bool ready = false;
    std::mutex busy;
};
SideStream g_side[64];

}  // namespace

int fa_attn_linear_block(const void *q, const void *k, const void *v, const void *w, void *o, float *lse, float *y,
                         int B, int H, int Nq, int Nk, int D, int N, float scale, int causal, int dtype,
                         int row_first, int row_count, void *stream) {
    int rc = check_attn_linear(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, scale, dtype, row_first, row_count);
    if (rc != FA_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    rc = block_attention(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, row_first, row_count, st);
    if (rc != FA_OK) return rc;
    return block_projection(w, o, y, B, H, Nq, D, N, dtype, row_first, row_count, st);
}

int fa_attn_linear(const void *q, const void *k, const void *v, const void *w, void *o, float *lse, float *y, int B,
                   int H, int Nq, int Nk, int D, int N, float scale, int causal, int dtype, int rows_per_block,
                   void *stream) {
    if (rows_per_block <= 0 || rows_per_block >= Nq)
        return fa_attn_linear_block(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, scale, causal, dtype, 0, Nq, stream);
    int rc = check_attn_linear(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, scale, dtype, 0, Nq);
    if (rc != FA_OK) return rc;
    hipStream_t st = (hipStream_t)stream;

    // The projection of block i and the attention of block i + 1 touch different rows, so the projections go to
    // a second stream behind an event recorded after each attention launch: the tail of one kernel (its last
    // workgroups, its stores) then overlaps the head of the next instead of leaving compute units idle between
    // ten short launches.  The caller's stream waits for the second stream at the end, so to the caller the call
    // behaves as if everything had been enqueued on `stream`.
    SideStream *side = nullptr;
    std::unique_lock<std::mutex> hold;
    if (option(FA_OPT_LINEAR_OVERLAP) != 0) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess || dev < 0 || dev >= 64) {
            g_last_hip_error = (int)e;
            return FA_ERR_LAUNCH;
        }
        hold = std::unique_lock<std::mutex>(g_side[dev].busy);
        if (!g_side[dev].ready) {
            hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
            e = hipStreamIsCapturing(st, &cap);
            if (e != hipSuccess) {
                g_last_hip_error = (int)e;
                return FA_ERR_LAUNCH;
            }
            if (cap == hipStreamCaptureStatusNone) {     // nothing is created while a capture is in progress
                SideStream &n = g_side[dev];
                e = hipStreamCreateWithFlags(&n.stream, hipStreamNonBlocking);
                if (e == hipSuccess) e = hipEventCreateWithFlags(&n.attn_done, hipEventDisableTiming);
                if (e == hipSuccess) e = hipEventCreateWithFlags(&n.joined, hipEventDisableTiming);
                if (e != hipSuccess) {
                    g_last_hip_error = (int)e;
                    return FA_ERR_LAUNCH;
                }
                n.ready = true;
            }
        }
        if (g_side[dev].ready) side = &g_side[dev];
        else hold.unlock();
    }

    // the first block is half size (section 4.2: nothing overlaps with the first block's computation)
    const int first = rows_per_block / 2 > 0 ? rows_per_block / 2 : rows_per_block;
    bool forked = false;
    for (int r = 0; r < Nq && rc == FA_OK;) {
        const int n = r == 0 ? first : (Nq - r < rows_per_block ? Nq - r : rows_per_block);
        rc = block_attention(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, r, n, st);
        if (rc != FA_OK) break;
        hipStream_t lin_stream = st;
        if (side) {
            hipError_t e = hipEventRecord(side->attn_done, st);
            if (e == hipSuccess) e = hipStreamWaitEvent(side->stream, side->attn_done, 0);
            if (e != hipSuccess) {
                g_last_hip_error = (int)e;
                rc = FA_ERR_LAUNCH;
                break;
            }
            forked = true;
            lin_stream = side->stream;
        }
        rc = block_projection(w, o, y, B, H, Nq, D, N, dtype, r, n, lin_stream);
        r += n;
    }
    if (forked) {      // also after an error: the second stream must rejoin (a capture could not end otherwise)
        hipError_t e = hipEventRecord(side->joined, side->stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(st, side->joined, 0);
        if (e != hipSuccess && rc == FA_OK) {
            g_last_hip_error = (int)e;
            rc = FA_ERR_LAUNCH;
        }
    }
    return rc;
}

int fa_mask_tile_class(const fa_mask_t *mask, int kv_len, int Nq, int Nk, int row_first, int row_last, int key_first) {
    MaskGeom g;
    const int rc = mask_geometry(mask, kv_len, Nq, Nk, &g);
    if (rc != FA_OK) return rc;
    if (row_first < 0 || row_last < row_first || row_last >= Nq || key_first < 0 || key_first >= Nk) return FA_ERR_SHAPE;
    if (key_first % BN) return FA_ERR_SHAPE;
    return tile_class(row_tiles(g, row_first, row_last), key_first / BN);
}

int fa_mask_tile_walk(const fa_mask_t *mask, int kv_len, int Nq, int Nk, int row_first, int row_last, int *tiles,
                      int capacity, int *count) {
    if (!count || (capacity > 0 && !tiles)) return FA_ERR_NULL;
    MaskGeom g;
    const int rc = mask_geometry(mask, kv_len, Nq, Nk, &g);
    if (rc != FA_OK) return rc;
    if (row_first < 0 || row_last < row_first || row_last >= Nq || capacity < 0) return FA_ERR_SHAPE;
    const TileSeq sq = tile_sequence(g, row_first, row_last);
    *count = sq.count;
    for (int j = 0; j < sq.count && j < capacity; ++j) tiles[j] = sq.tile(j);   // the kernel's own position -> tile map
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

int fa_set_option(int opt, int value) {
    bool ok = value == FA_AUTO;
    switch (opt) {
        case FA_OPT_FWD_MODE:
            ok = ok || value == FA_MODE_SPLIT || value == FA_MODE_WIDE || value == FA_MODE_WIDE_FOLD || value == FA_MODE_WIDE64;
            break;
        case FA_OPT_DECODE_KERNEL: ok = ok || value == 0 || value == 1; break;
        case FA_OPT_LINEAR_TILE: ok = ok || value == 128 || value == 256; break;
        case FA_OPT_LINEAR_PANEL: ok = ok || value >= 1; break;
        case FA_OPT_LINEAR_OVERLAP: ok = ok || value == 0 || value == 1; break;
        default: return FA_ERR_OPTION;
    }
    if (!ok) return FA_ERR_OPTION;
    return g_options[opt].exchange(value, std::memory_order_relaxed);
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
        case FA_ERR_WORKSPACE:
            return "workspace is NULL or smaller than fa_fwd_splitkv_plan reports (fa_fwd_splitkv_static: the problem needs "
                   "more than the library's 64 MiB)";
        case FA_ERR_NSPLIT: return "nsplit exceeds 1024";
        case FA_ERR_MASK: return "mask descriptor: prefix must be >= 0 and a key count within 0..Nk";
        case FA_ERR_OPTION: return "fa_set_option: unknown option, or a value it does not take";
        default: return "unknown error code";
    }
}

int fa_version(void) { return 300; }

int fa_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
