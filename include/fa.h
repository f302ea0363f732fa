/*
 * fa.h -- C ABI of the MI355X (gfx950) exact attention forward library.
 *
 * The operation is the attention of FastAttention section 5.1 / appendix C
 * (prefill and decoding equations), O = softmax(scale * Q K^T + mask) V, with the
 * lower-triangular mask of section 4.1 generated from indices per tile (no mask
 * tensor exists), evaluated tile by tile with the online-softmax dataflow of
 * appendix A (Q K^T, exp, exp * V, running row max / row sum).
 *
 * All entry points are plain C: device pointers and sizes, no C++ or torch types.
 */
#ifndef FA_H
#define FA_H

#ifdef __cplusplus
extern "C" {
#endif

/* error codes (0 = success); every argument error is detected on the host before any HIP call */
#define FA_OK            0
#define FA_ERR_NULL     -1 /* a required pointer is NULL */
#define FA_ERR_SHAPE    -2 /* B, H, Nq or Nk <= 0, or a tensor/grid too large to index (one head of K/V must stay under 2 GiB) */
#define FA_ERR_HEADDIM  -3 /* D is not 64 or 128 */
#define FA_ERR_DTYPE    -4 /* dtype is not FA_DTYPE_F16 or FA_DTYPE_BF16 */
#define FA_ERR_SCALE    -5 /* scale is NaN or infinite */
#define FA_ERR_ALIGN    -6 /* q, k, v or o not 16-byte aligned, or lse not 4-byte aligned */
#define FA_ERR_LAUNCH   -7 /* the HIP runtime rejected the launch (see fa_last_hip_error) */
#define FA_ERR_WORKSPACE -8 /* fa_fwd_splitkv: workspace NULL or smaller than fa_fwd_splitkv_plan reports */
#define FA_ERR_NSPLIT   -9 /* fa_fwd_splitkv: nsplit > 1024 */
#define FA_ERR_MASK     -10 /* fa_fwd_masked: prefix < 0, or a key count outside 0..Nk */
#define FA_ERR_OPTION   -11 /* fa_set_option: unknown option, or a value it does not take */

#define FA_DTYPE_F16  0 /* IEEE binary16 */
#define FA_DTYPE_BF16 1 /* bfloat16 */

/*
 * fa_fwd -- exact attention forward (appendix A dataflow; section 4.1 mask handling:
 * tiles entirely above the diagonal are skipped, tiles entirely below it take no
 * mask, only tiles that straddle it get a per-element predicate).
 *
 * For every batch b, head h and query row i:
 *     J_i    = all keys                    (causal == 0)
 *            = { j : j <= i + (Nk - Nq) }  (causal != 0; bottom-right aligned, so a
 *              single decode query attends to the whole cache, appendix C)
 *     s_ij   = scale * sum_d q[b,h,i,d] * k[b,h,j,d]
 *     o[b,h,i,:] = sum_{j in J_i} softmax_j(s_ij) * v[b,h,j,:]    rounded to dtype
 *     lse[b,h,i] = ln sum_{j in J_i} exp(s_ij)                     (natural log, fp32)
 *     rows with empty J_i (causal, Nq > Nk): o = 0, lse = -inf.
 *
 * Arguments
 *   q, o   : DEVICE pointers, [B, H, Nq, D] contiguous, D fastest, 16-bit elements of `dtype`
 *   k, v   : DEVICE pointers, [B, H, Nk, D] contiguous
 *   lse    : DEVICE pointer,  [B, H, Nq] fp32
 *   D      : 64 or 128
 *   scale  : any finite float (1/sqrt(D) in the paper)
 *   dtype  : FA_DTYPE_F16 or FA_DTYPE_BF16; both products accumulate in fp32 on MFMA,
 *            the probabilities are rounded to `dtype` before the second product
 *   stream : hipStream_t (as void*); NULL is the default stream
 *
 * Ownership: the caller owns every buffer; the library allocates nothing, keeps no
 * state between calls, needs no workspace and enqueues exactly one kernel on `stream`
 * without synchronising.  o and lse must not alias the inputs.  q, k, v, o must be
 * 16-byte aligned.  Nq and Nk need not be multiples of any tile size.
 *
 * Returns FA_OK or a negative FA_ERR_* code; on an argument error nothing is launched.
 */
int fa_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
           int B, int H, int Nq, int Nk, int D, float scale, int causal, int dtype,
           void *stream);

/*
 * Work decomposition fa_fwd uses for a problem (section 4.1: tiles above the diagonal are
 * skipped; appendix A: the work is split over the sequence as well as over batch and heads).
 * FA_MODE_SPLIT: a workgroup owns 128 query rows and its two wave groups take alternate
 * 64-key tiles; FA_MODE_WIDE: a workgroup owns 256 query rows and all its waves walk the same
 * tiles; FA_MODE_WIDE_FOLD (causal only): WIDE with each workgroup's eight 32-row blocks taken
 * four from the cheap end of the sequence and four, mirrored, from the expensive end; once the
 * cheap blocks are done their waves take every other tile of the expensive ones.
 * FA_MODE_WIDE64 (D = 128 only): 256 query rows per workgroup as in WIDE, but as four waves of 64
 * rows, one per SIMD, so that every K and V fragment read from LDS feeds two matrix instructions,
 * with a software-pipelined main loop (the softmax of one 32-key unit issued between the matrix
 * instructions of its neighbours).
 * With W = B*H*ceil(Nq/256), fa_fwd picks SPLIT when W < 256; for causal problems with
 * Nq > 768: WIDE_FOLD when Nq <= 4096, W <= 1024 and the last round of 256 workgroups is at
 * least 85% full, else SPLIT when W < 640 (Nq <= 4096) or W < 384 (longer); otherwise WIDE64 when
 * D = 128 and a query sees 4096 keys or more on average (Nk, or Nk - Nq/2 when causal), else WIDE.
 * fa_set_option(FA_OPT_FWD_MODE, ...) overrides the choice (tests, tuning).
 * Nq = 1 (one decoding step) takes none of these: FA_MODE_STREAM, the register-streaming kernel
 * described at fa_fwd_splitkv, one workgroup per (batch, head) -- full speed when B*H fills the
 * chip; with fewer heads fa_fwd_splitkv, which has a workspace to split the cache over, is the
 * call to make.  fa_set_option(FA_OPT_DECODE_KERNEL, 1) keeps Nq = 1 on the tile kernels.
 */
#define FA_MODE_SPLIT 0
#define FA_MODE_WIDE  1
#define FA_MODE_WIDE_FOLD 2
#define FA_MODE_STREAM 3   /* Nq = 1: the register-streaming kernel of fa_fwd_splitkv, one run per (batch, head) */
#define FA_MODE_WIDE64 4   /* D = 128: four waves of 64 rows, software-pipelined main loop */

typedef struct fa_plan {
    int mode;                 /* FA_MODE_SPLIT, FA_MODE_WIDE, FA_MODE_WIDE_FOLD, FA_MODE_STREAM or FA_MODE_WIDE64 */
    int block_m;              /* query rows per workgroup */
    int block_n;              /* keys per tile */
    int threads;              /* threads per workgroup */
    int grid;                 /* workgroups launched (work items rounded up to a multiple of 8) */
    int lds_bytes;            /* LDS per workgroup */
    long long work_items;     /* B * H * ceil(Nq / block_m) */
    long long tiles_visited;  /* (query block, key tile) pairs the kernel walks: masked-out tiles are skipped */
    long long tiles_total;    /* the same count without skipping */
} fa_plan_t;

/*
 * fa_fwd_plan -- host-only: fills *plan (caller-owned, HOST pointer) for the given problem
 * without touching the GPU.  Same shape checks and error codes as fa_fwd.
 */
int fa_fwd_plan(int B, int H, int Nq, int Nk, int D, int causal, int dtype, fa_plan_t *plan);

/*
 * fa_fwd_splitkv -- the same operation as fa_fwd (same formula, same arguments, same
 * results up to fp32 rounding order) for the decoding shape of appendix C: one or a few
 * query rows per head against a long K/V cache, where B * H * ceil(Nq/256) workgroups cannot
 * fill the chip.  The key tiles of every 256-row query block are cut into `nsplit` runs, one
 * workgroup each; every run leaves an unnormalised partial result (accumulator, exponent
 * reference, row sum -- the running quantities of appendix A) in `workspace`, and a second
 * kernel merges them: lse = logsumexp over runs, o = sum_runs exp(lse_run - lse) o_run.
 * Bound by reading K and V once from HBM.  Nq = 1, the decoding step proper, runs a kernel of its
 * own that streams K and V through registers (one multiply-add per element leaves the matrix
 * cores nothing to reuse) and keeps the probabilities in fp32; fa_set_option(FA_OPT_DECODE_KERNEL, 1)
 * sends it through the tile kernel instead (tests, tuning).  With several query blocks per head (a chunk
 * of a chunked prefill: Nq > 256) the call is bound by the matrix cores instead, and at D = 128 runs of 4096
 * keys or more go to the kernel of FA_MODE_WIDE64.
 *
 *   nsplit          : > 0: number of runs (clamped to the number of 64-key tiles, at most 1024);
 *                     <= 0: the library picks (256 workgroups at D = 128 and for a single query,
 *                     512 at D = 64 otherwise; runs of >= 4 tiles)
 *   workspace       : DEVICE pointer, 16-byte aligned, caller-owned scratch of at least
 *                     fa_fwd_splitkv_plan(...).workspace_bytes; contents on entry are ignored,
 *                     contents on return are unspecified; must not alias any other argument
 *   workspace_bytes : size of `workspace`
 *   everything else : as for fa_fwd
 *
 * Enqueues two kernels on `stream` (with a single run, chosen or asked for, there is nothing
 * to merge and the call enqueues exactly what fa_fwd would), allocates nothing, does not
 * synchronise.  Calls that share a workspace must be ordered (same
 * stream).  Returns FA_OK or a negative FA_ERR_* code; on an
 * argument error nothing is launched.
 */
int fa_fwd_splitkv(const void *q, const void *k, const void *v, void *o, float *lse,
                   int B, int H, int Nq, int Nk, int D, float scale, int causal, int dtype,
                   int nsplit, void *workspace, long long workspace_bytes, void *stream);

/*
 * fa_fwd_splitkv_static -- fa_fwd_splitkv for callers that cannot allocate or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results (bit for
 * bit) and error codes as fa_fwd_splitkv without `workspace` / `workspace_bytes`: the partial results go to a
 * 64 MiB array that is part of the library's device code (each GPU the library runs on holds its own copy
 * until the process ends).  The call allocates and frees nothing, on the host or on the device.
 *
 *   limit   : fa_fwd_splitkv_plan(...).workspace_bytes = nsplit * B * H * Nq * (D + 2) * 4 must not exceed
 *             64 MiB (67108864 bytes), else FA_ERR_WORKSPACE and nothing is launched; with a single run
 *             (chosen or asked for) no workspace is needed and the limit does not apply
 *   sharing : every call on one GPU uses that GPU's one array.  Nothing in it needs clearing (every partial
 *             result is written before it is read), but calls that may overlap on one GPU -- different
 *             streams, different threads -- race on it: keep them ordered (one stream, or events).
 *   first call on a device: looks the array's device address up (hipGetSymbolAddress, once per device, the
 *             device being current); make that call outside of a graph capture.
 */
int fa_fwd_splitkv_static(const void *q, const void *k, const void *v, void *o, float *lse,
                          int B, int H, int Nq, int Nk, int D, float scale, int causal, int dtype,
                          int nsplit, void *stream);

typedef struct fa_splitkv_plan {
    int nsplit;                 /* runs actually used */
    int grid_x, grid_y;         /* first kernel: work items (tile kernel: rounded up to a multiple of 8) x runs */
    int combine_grid;           /* second kernel: blocks of 256 threads (0: none -- with a single run the call is fa_fwd's launch) */
    long long work_items;       /* B * H * ceil(Nq / 256) */
    long long workspace_bytes;  /* nsplit * B * H * Nq * (D + 2) * 4 */
    int streaming;              /* 1: the register-streaming kernel of the single-query case, 0: the tile kernel */
} fa_splitkv_plan_t;

/*
 * fa_fwd_splitkv_plan -- host-only: the launch shape and workspace size fa_fwd_splitkv uses for
 * the given problem and `nsplit` argument.  *plan is a caller-owned HOST pointer.
 */
int fa_fwd_splitkv_plan(int B, int H, int Nq, int Nk, int D, int causal, int dtype, int nsplit,
                        fa_splitkv_plan_t *plan);

/*
 * fa_attn_linear_block -- attention followed by the output projection for ONE block of query rows
 * (section 4.2: the attention and the Linear after it are computed together, block of rows by
 * block of rows, so that the AllReduce of a finished block can run while the next block is
 * computed).  For the rows row_first <= i < row_first + row_count of every batch entry:
 *     o[b,h,i,:]  and lse[b,h,i]   exactly as fa_fwd gives them for the whole problem
 *     y[b,i,n] = sum_{h,d} o[b,h,i,d] * w[h*D + d, n]       n = 0 .. N-1, fp32
 * i.e. the heads' attention rows laid side by side times w (appendix C: Softmax(...) X_V W_O); with
 * the heads of one device, y is that device's partial sum of the projection.
 *
 *   q, k, v, o, lse : as for fa_fwd (the FULL tensors; only the block's rows of o, lse are written)
 *   w   : DEVICE pointer, [H*D, N] contiguous, N fastest, 16-bit elements of `dtype`, 16-byte aligned
 *   y   : DEVICE pointer, [B, Nq, N] fp32; only the block's rows are written
 *   N   : outputs per token, a positive multiple of 256
 *   row_first, row_count : the block; 0 <= row_first, 1 <= row_count, row_first + row_count <= Nq
 *
 * Enqueues two kernels on `stream` (the attention of the block, then a GEMM that reads the
 * attention output in its own [B,H,Nq,D] layout; o is rounded to `dtype` in between, products
 * accumulate in fp32).  No allocation, no workspace, no synchronisation: a caller overlaps
 * communication by enqueueing it on another stream behind an event recorded after this call.
 * Calls for different blocks are independent.  Error behaviour as for fa_fwd.  The GEMM's
 * workgroup tile is 256 tokens x 256 outputs when that still gives each of the 256 compute units
 * a workgroup (B * ceil(row_count/256) * N/256 >= 256), else 128 x 256; fa_set_option(FA_OPT_LINEAR_TILE,
 * 128 | 256) overrides (tests, tuning).  The tiles are dealt to the XCDs in panels of
 * a few row tiles so that each L2 fetches about as many bytes of o as of w; fa_set_option(
 * FA_OPT_LINEAR_PANEL, row tiles per panel) overrides that too (the order changes no result).
 *
 * fa_attn_linear -- every block in order: blocks of rows_per_block rows, the first one half that size
 * (nothing can overlap with the first block); rows_per_block <= 0: one block.  With more than one block
 * the projection of a block and the attention of the next touch different rows, so the projections are
 * enqueued on a second stream of the library's own (default priority, one per device, created by the first
 * such call on that device that is not under stream capture and kept until the process ends), each behind
 * an event recorded on `stream` after its block's attention, and `stream` is made to wait for the second
 * stream before the call returns: all of the call's work is ordered after what `stream` held before and
 * before what is enqueued on it afterwards, as if it had all gone to `stream`, and a capture of `stream`
 * records it as a fork and a join.  Calls on one device share that second stream: their enqueueing is
 * serialised by a lock, their projections run in enqueue order.  Results are identical either way
 * (fa_set_option(FA_OPT_LINEAR_OVERLAP, 0) keeps everything on `stream`).
 */
int fa_attn_linear_block(const void *q, const void *k, const void *v, const void *w, void *o, float *lse,
                         float *y, int B, int H, int Nq, int Nk, int D, int N, float scale, int causal,
                         int dtype, int row_first, int row_count, void *stream);
int fa_attn_linear(const void *q, const void *k, const void *v, const void *w, void *o, float *lse,
                   float *y, int B, int H, int Nq, int Nk, int D, int N, float scale, int causal,
                   int dtype, int rows_per_block, void *stream);

/*
 * Masks generated from a descriptor.  Section 4.1 replaces the stored S x S lower-triangular
 * mask by a generator that yields any tile's mask on demand, and treats tiles that are
 * entirely masked (skipped) or entirely visible (no mask applied) specially.  The same scheme,
 * with an index predicate as the generator, covers the other masks inference uses:
 *
 *   row i of batch entry b sees key j  iff   j < klen_b  and
 *       ( j < prefix   or   diag_i - window_left <= j <= diag_i + window_right ),
 *   diag_i = i + (Nk - Nq)   (the key on the bottom-right-aligned diagonal),
 *   klen_b = kv_len[b], or Nk when kv_len is NULL.
 *
 *   window_left  : keys before diag_i a row still sees;  < 0: no limit
 *   window_right : keys after diag_i a row still sees;   < 0: no limit
 *                  (-1, 0) is the causal mask, (-1, -1) no mask, (W-1, 0) a causal sliding
 *                  window of W keys, (W, W) a symmetric local window
 *   prefix       : >= 0; the first `prefix` keys are visible to every row whatever the window
 *                  (prefix-LM: a bidirectional prompt followed by causal text)
 *   diag_from_kv_len : 0: diag_i as above.  1: diag_i = i + (klen_b - Nq) -- the Nq queries of entry b are
 *                  the LAST Nq positions of its own klen_b keys, wherever those end inside the Nk
 *                  allocated rows: appendix C's decoding step (or a chunk of a chunked prefill) for a
 *                  batch of caches of different lengths, where a causal limit or a sliding window must
 *                  hang on each sequence's own last token.  Any other value: FA_ERR_MASK.  Set every
 *                  member (or zero the struct first): the member occupies what used to be padding
 *   kv_len       : DEVICE pointer to B int32 (4-byte aligned) or NULL: keys at and after
 *                  kv_len[b] are padding; values are clamped to 0..Nk on the device
 */
typedef struct fa_mask {
    int window_left;
    int window_right;
    int prefix;
    int diag_from_kv_len;
    const int *kv_len;
} fa_mask_t;

/*
 * fa_fwd_masked -- fa_fwd under a descriptor mask.  Arguments, layouts, ownership, results
 * (rows that see no key: o = 0, lse = -inf) and error behaviour as for fa_fwd; `mask` is a HOST
 * pointer, read during the call only.  Needs Nq + Nk < 2^30.  One kernel, no workspace.  Per
 * wave (32 query rows) and 64-key tile the kernel classifies the tile from the descriptor:
 * nothing visible -> not computed; everything visible -> no mask work; otherwise the predicate
 * is evaluated per element.  A workgroup (256 rows) only walks the prefix tiles and the tiles its
 * rows' windows touch.  Nq = 1 (a decoding step over caches of different lengths, or with a
 * sliding window) runs the register-streaming kernel of fa_fwd_splitkv instead, one workgroup
 * per (batch, head), which walks the prefix and the window as runs of consecutive keys
 * (fa_set_option(FA_OPT_DECODE_KERNEL, 1) keeps the tile kernel).
 */
int fa_fwd_masked(const void *q, const void *k, const void *v, void *o, float *lse,
                  int B, int H, int Nq, int Nk, int D, float scale, const fa_mask_t *mask, int dtype,
                  void *stream);

/*
 * fa_decode_masked -- one decoding step (Nq = 1: q, o [B,H,1,D], lse [B,H]) under a descriptor mask, with the
 * visible keys of every (batch, head) cut into `nsplit` equal shares as in fa_fwd_splitkv: the call for small
 * batches of caches of different lengths (appendix C's decoding equations with section 4.1's generated mask),
 * where B * H workgroups alone cannot fill the chip.  The query sits on the last key (diag = Nk - 1), so
 * (-1, 0) lets it see kv_len[b] keys, (W - 1, 0) the last W of the Nk; with diag_from_kv_len = 1 it sits on
 * key kv_len[b] - 1 and (W - 1, 0) is the last W keys of each cache.  Each share is counted along the
 * prefix and the window laid end to end, so entries with few keys are split as evenly as entries with many.
 *
 *   nsplit, workspace, workspace_bytes : as for fa_fwd_splitkv with Nq = 1; fa_fwd_splitkv_plan(B, H, 1, Nk, D,
 *                     0, dtype, nsplit) reports the number of shares and the bytes (a single share needs no
 *                     workspace: NULL is accepted then)
 *   everything else : as for fa_fwd_masked
 *
 * Enqueues the streaming kernel and, with more than one share, the merge kernel on `stream`; allocates
 * nothing; does not synchronise.  Same error codes as fa_fwd_masked and fa_fwd_splitkv.
 */
int fa_decode_masked(const void *q, const void *k, const void *v, void *o, float *lse,
                     int B, int H, int Nk, int D, float scale, const fa_mask_t *mask, int dtype,
                     int nsplit, void *workspace, long long workspace_bytes, void *stream);

/*
 * The tile classification and the workgroup's walk, callable on the host (the kernel runs the
 * same code): for tests and for callers that want to know the work a mask leaves.
 * kv_len here is ONE batch entry's key count (host int, 0..Nk); mask->kv_len is not read (mask->diag_from_kv_len is).
 *
 * fa_mask_tile_class: rows row_first..row_last against keys key_first..key_first+63 (key_first a
 *   multiple of 64).  Returns
 *   FA_TILE_SKIP (certainly nothing visible), FA_TILE_FULL (certainly everything visible, and all
 *   64 keys exist), FA_TILE_PARTIAL (anything else), or a negative FA_ERR_* code.
 * fa_mask_tile_walk: the 64-key tiles a workgroup owning rows row_first..row_last visits, in the
 *   order the kernel visits them (position j -> tile index, by the kernel's own mapping): the tiles
 *   holding prefix keys, then the consecutive tiles the rows' windows touch, a long window run
 *   starting somewhere in its middle and wrapping around (so that co-resident workgroups with
 *   shifted windows read the same tile at the same time).  *count (HOST pointer) receives the
 *   length of the walk; the first min(*count, capacity) tile indices are written to `tiles` (HOST
 *   array of `capacity` ints; NULL with capacity 0 just asks for the length).  Every tile holding a
 *   key visible to one of the rows is among them.
 * fa_mask_interior_run: within the walk of the workgroup owning rows wg_row_first..wg_row_last, the
 *   positions [*first, *first + *count) that the wave owning rows row_first..row_last processes
 *   without any check: each of those tiles is FA_TILE_FULL for the wave and the tile at the next
 *   position exists and lies wholly inside K/V.  *first and *count are even; *count may be 0.
 */
#define FA_TILE_SKIP    0
#define FA_TILE_FULL    1
#define FA_TILE_PARTIAL 2
int fa_mask_tile_class(const fa_mask_t *mask, int kv_len, int Nq, int Nk,
                       int row_first, int row_last, int key_first);
int fa_mask_tile_walk(const fa_mask_t *mask, int kv_len, int Nq, int Nk, int row_first, int row_last,
                      int *tiles, int capacity, int *count);
int fa_mask_interior_run(const fa_mask_t *mask, int kv_len, int Nq, int Nk, int wg_row_first, int wg_row_last,
                         int row_first, int row_last, int *first, int *count);

/*
 * fa_set_option -- test and tuning hook: overrides a choice the library otherwise makes from the
 * problem's shape (the work decompositions described at fa_plan_t, fa_fwd_splitkv and
 * fa_attn_linear_block).  Process-wide; every entry point reads each option once per call, so a
 * change made while another thread is inside a call applies to that thread's next call.  No
 * environment variable is read anywhere in the library.
 *
 *   FA_OPT_FWD_MODE      : FA_MODE_SPLIT, FA_MODE_WIDE, FA_MODE_WIDE_FOLD (causal problems only; WIDE
 *                          otherwise), FA_MODE_WIDE64 (D = 128 only; WIDE otherwise) or FA_AUTO.
 *                          FA_MODE_WIDE also keeps fa_fwd_splitkv's long runs on the tile kernel
 *   FA_OPT_DECODE_KERNEL : 0 or FA_AUTO: Nq = 1 runs the register-streaming kernel; 1: the tile kernels
 *   FA_OPT_LINEAR_TILE   : 128, 256 or FA_AUTO: token rows per workgroup tile of the projection
 *   FA_OPT_LINEAR_PANEL  : >= 1 or FA_AUTO: row tiles per panel of the projection's tile order
 *   FA_OPT_LINEAR_OVERLAP: 1 or FA_AUTO: fa_attn_linear runs the projections on its second stream; 0: everything
 *                          on the caller's stream
 *
 * Returns the option's previous value (FA_AUTO = -1 if it was never set), or FA_ERR_OPTION for an
 * unknown option or a value outside the list above (nothing is changed then).
 */
#define FA_AUTO (-1)
#define FA_OPT_FWD_MODE      0
#define FA_OPT_DECODE_KERNEL 1
#define FA_OPT_LINEAR_TILE   2
#define FA_OPT_LINEAR_PANEL  3
#define FA_OPT_LINEAR_OVERLAP 4
int fa_set_option(int option, int value);

/* static, never-freed description of an FA_ERR_* code */
const char *fa_strerror(int code);

/* library version, major * 10000 + minor * 100 + patch */
int fa_version(void);

/* hipError_t value of the last launch failure seen by this thread (0 if none) */
int fa_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FA_H */
