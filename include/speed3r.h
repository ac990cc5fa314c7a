/*
 * speed3r.h -- C ABI of the MI355X (gfx950) implementation of Speed3R's Global
 * Sparse Attention (GSA), Sec. 3.2 of the paper, forward pass, one scene
 * (batch omitted as in the paper), one GPU.
 *
 * The path (Sec. 3.2, eqs. 3-8; supplementary Alg. 1 and Alg. 2):
 *   1. pool      Q, K, V are mean-pooled over blocks of `block` tokens: runs of
 *                consecutive tokens (the last block may be short and is averaged
 *                over its valid tokens) or, on request, the paper's s x s spatial
 *                windows of every view's patch grid.
 *   2. scores    S_guide[h,i,j] = Qc[h,i] . Kc[h,j]                  (eq. 4)
 *   3. compress  Oc'[h,i] = softmax_j(scale * S_guide[h,i,:]) Vc[h]  (eq. 3)
 *   4. topk      per (h,i): the k = min(topk, n_blk) key blocks with the
 *                largest S_guide[h,i,:] ("Selection Branch"); all queries of a
 *                block share the set; stored ascending.
 *   5. select    O_sel[t,h] = softmax over the valid tokens of the selected
 *                blocks of (scale * q[t,h] . k[u,h]), times v      (eq. 6, Alg. 2)
 *   6. merge     out = g * Oc'[h, t / block] + (1 - g) * O_sel,
 *                g = sigmoid(gate_logits) or 1/2                   (eqs. 5, 7, 8)
 * and, as the comparison point, plain dense softmax attention (eq. 2 form).
 * Optional parts of the layer (fields of s3r_params): special tokens, which get
 * dense attention over all tokens (eqs. 1-2), a fixed set of key blocks every
 * query block attends besides its TopK (Sec. 3.3), spatial pooling windows,
 * unpooled queries in the compression branch.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer unless stated otherwise; the
 *     caller owns all of them; the library never frees caller memory.
 *   - q, k, v, out, gate_logits, o_sel: layout [n_tok][heads][head_dim],
 *     contiguous, element type given by `dtype`, 16-byte aligned (q, k, v of
 *     speed3r_sparse_global_attn_ex may instead be strided, see stride_tok).
 *     Inputs are read-only and must not alias outputs.
 *   - n_blk = ceil(n_tok / block).  head_dim must be 64, block one of
 *     16, 32, 64, 128 (else S3R_ERR_UNSUPPORTED).  topk > n_blk is clamped.
 *     n_tok need not be a multiple of block.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream); no call synchronises the host except where noted.
 *   - Every function returns a status code; speed3r_last_error() gives a
 *     message for the last failure on the calling thread.  Nothing is thrown.
 *   - Entry points that say "library-held scratch" keep one grow-only device
 *     buffer per process (allocated with hipMalloc on first use or growth;
 *     growth synchronises the device); calls using it must not overlap.
 */
#ifndef SPEED3R_H
#define SPEED3R_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    S3R_OK = 0,
    S3R_ERR_INVALID_ARG = 1, /* null / misaligned pointer, non-positive size ...   */
    S3R_ERR_UNSUPPORTED = 2, /* head_dim != 64, block not in {16,32,64,128}, dtype */
    S3R_ERR_WORKSPACE = 3,   /* caller workspace too small / allocation failed     */
    S3R_ERR_HIP = 4          /* a HIP runtime call or kernel launch failed         */
} s3r_status;

typedef enum { S3R_F32 = 0, S3R_BF16 = 1 } s3r_dtype;

/* Bits of the device status word (s3r_params.status). */
enum { S3R_DIAG_FORCED_RANGE = 1, S3R_DIAG_FORCED_ORDER = 2 };

/* Stages of the path, for speed3r_get_stage_ms(). */
enum {
    S3R_STAGE_POOL = 0,     /* block pooling (+ K/V tile re-layout for the MFMA path) */
    S3R_STAGE_SPLIT = 1,    /* pooled fp32 -> operand tiles (+ their per-head statistics) */
    S3R_STAGE_COMPRESS = 2, /* S_guide + compressed attention                         */
    S3R_STAGE_TOPK = 3,     /* per-query-block TopK (incl. its filter sweep)          */
    S3R_STAGE_SELECT = 4,   /* block-sparse attention + merge                         */
    S3R_STAGE_DENSE = 5,    /* dense attention                                        */
    S3R_N_STAGES = 6
};

typedef struct s3r_params {
    const void *q, *k, *v;   /* in   [n_tok][heads][head_dim] (or stride_tok, stride_head below)  */
    void *out;               /* out  [n_tok][heads][head_dim], merged result (eq. 8)            */
    const void *gate_logits; /* in, optional (NULL: g = 1/2), same layout and dtype as q        */
    /* Forced blocks (Sec. 3.3: the fixed global context of the VGGT variant, e.g. all blocks of the
     * reference view): n_forced block indices in DEVICE memory that every query block attends in
     * addition to its TopK, which then runs over the other blocks only.  The list must be strictly
     * ascending and within [0, n_blk).  The library cannot look at device memory without a host
     * synchronisation, which it never does: a list that breaks this is reported through `status`
     * below; the call itself then runs on the list with its entries clamped into range (memory-safe;
     * a block listed twice is attended twice, so the result is not the paper's). */
    const int32_t *forced_blocks; /* in, optional (NULL: none)                                   */
    int n_forced;            /* 0 when forced_blocks is NULL                                    */
    /* out, optional: one device word, written by the call (stream-ordered like every output): 0, or
     * S3R_DIAG_FORCED_RANGE | S3R_DIAG_FORCED_ORDER for a forced_blocks list with an entry outside
     * [0, n_blk) / not strictly ascending.  4-byte aligned. */
    int32_t *status;
    /* Special tokens (Sec. 3.2 eqs. 1-2 and "Final Output"): the n_tok rows come in views of
     * tokens_per_view rows, the first special_per_view of each being special (camera / register)
     * tokens.  Those rows get plain softmax attention over ALL n_tok rows; the remaining image rows,
     * taken in order, form the sequence the sparse path works on (blocks, TopK, forced blocks and the
     * optional block-level outputs all refer to that image-only sequence); every result is written to
     * the row it belongs to.  Both 0: no special tokens.  tokens_per_view = n_tok with the special
     * tokens first is the paper's own [X_spec; X_img] arrangement. */
    int tokens_per_view;     /* 0, or a divisor of n_tok                                        */
    int special_per_view;    /* 0 <= special_per_view < tokens_per_view                         */
    /* Spatial pooling windows (Sec. 3.2: non-overlapping s x s average pooling on each image's patch
     * grid).  The tokens_per_view - special_per_view image rows of a view are a row-major grid_h x
     * grid_w grid; blocks are its window x window windows (block must equal window * window), taken in
     * row-major order over the grid, views one after another: n_blk = views * ceil(grid_h / window) *
     * ceil(grid_w / window).  Windows on the right and bottom edges are cut where the grid ends and hold
     * fewer tokens.  All 0: blocks are runs of `block` consecutive image rows. */
    int grid_h, grid_w, window;
    /* Queries of the compression branch.  0: pooled like the keys (Q_comp, eq. 3; the paper's form): one
     * compressed output per block, upsampled to its tokens (eq. 5).  1: every image row's own query
     * attends the pooled keys, O_comp[t] = softmax_j(scale * q[t] . Kc[j]) Vc, and that row's result is
     * merged (eq. 8); block scores and TopK remain those of the pooled queries, and the optional
     * output o_comp remains the per-block result.  bf16 data: Kc and Vc enter this product rounded to
     * bf16.  Costs n_tok x n_blk attention (at 1000 views several times the rest of the path). */
    int compress_queries;
    int64_t n_tok;
    /* Layout of q, k and v (all three alike; Sec. 3.2 takes Q, K, V as given, e.g. as three views of one
     * packed projection output): elements between consecutive rows and between heads; the head_dim
     * channels of a head are contiguous.  0: the packed default (stride_tok = heads * head_dim,
     * stride_head = head_dim).  Multiples of 8 elements.  out, gate_logits and o_sel are always packed. */
    int64_t stride_tok, stride_head;
    int heads, head_dim, block, topk;
    s3r_dtype dtype;
    float softmax_scale;     /* <= 0: 1/sqrt(head_dim).  Used by both branches.                 */
    /* w = speed3r_selected_per_row(n_tok, block, topk, n_forced) blocks per row: */
    int32_t *topk_idx;       /* out, optional: [heads][n_blk][w] ascending block indices        */
    float *lse_sel;          /* out, optional: [heads][n_tok], Alg. 2's L (natural log); special
                                rows are left untouched, and so are theirs in o_sel               */
    float *o_comp;           /* out, optional: [heads][n_blk][head_dim] fp32, Oc' of eq. 3      */
    void *o_sel;             /* out, optional: [n_tok][heads][head_dim], O_sel of eq. 6         */
    void *workspace;         /* caller-owned device scratch, 256-byte aligned                   */
    size_t workspace_bytes;  /* >= speed3r_workspace_bytes(...) for the same problem            */
    void *stream;            /* hipStream_t                                                     */
} s3r_params;

/* Bytes of device scratch speed3r_sparse_global_attn_ex needs (0 on invalid arguments) for
 * the given n_forced (0 without forced blocks). */
size_t speed3r_workspace_bytes(int64_t n_tok, int heads, int head_dim, int block, int topk, int n_forced,
                               s3r_dtype dtype);

/* The same from a filled-in parameter block (only its shape fields are read: n_tok, heads, head_dim,
 * block, topk, dtype, n_forced, tokens_per_view, special_per_view); needed with special tokens. */
size_t speed3r_workspace_bytes_ex(const s3r_params *p);

/* Number of blocks n_blk of the sequence the sparse path works on, for a filled-in parameter block
 * (shape fields only); -1 on invalid arguments. */
int64_t speed3r_num_blocks(const s3r_params *p);

/* Key blocks each query block attends: n_forced + min(topk, n_blk - n_forced) (Sec. 3.3), or
 * min(topk, n_blk) without forced blocks; -1 on invalid arguments. */
int speed3r_selected_per_row(int64_t n_tok, int block, int topk, int n_forced);

/* The whole GSA path (steps 1-6 above; Sec. 3.2, eqs. 3-8).  Re-entrant across streams when each
 * call has its own workspace.  Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
s3r_status speed3r_sparse_global_attn_ex(const s3r_params *params);

/* Short form of the above: bf16, scale 1/sqrt(head_dim), no gate (g = 1/2), library-held scratch.
 * Returns an s3r_status as int. */
int speed3r_sparse_global_attn(const void *q, const void *k, const void *v, void *out,
                               int64_t n_tok, int heads, int head_dim, int block, int topk,
                               void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the short form above with its scratch in a fixed device array of
 * S3R_STATIC_SCRATCH_BYTES that is part of the library's code object, so the call performs no hipMalloc,
 * hipFree, event creation or any other allocating call; every GPU the library runs on holds its own copy of
 * that array until the process ends.  Same arguments, same kernels and bit-identical results as
 * speed3r_sparse_global_attn.  Problems whose speed3r_workspace_bytes(..., n_forced = 0, S3R_BF16) exceeds
 * S3R_STATIC_SCRATCH_BYTES are refused with S3R_ERR_WORKSPACE before anything is enqueued (8 views x 1374
 * tokens x 16 heads, block 64, top-16 needs 57 MiB and fits).  All calls on one GPU share that GPU's array:
 * calls that overlap in time on one GPU (different streams or threads) race; calls ordered on one stream are
 * fine, and no call depends on what an earlier one left in the array. */
#define S3R_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int speed3r_sparse_global_attn_noalloc(const void *q, const void *k, const void *v, void *out,
                                       int64_t n_tok, int heads, int head_dim, int block, int topk,
                                       void *stream);

/* Dense softmax attention over all n_tok keys (eq. 2 form): out[t,h] = softmax_u(scale q.k) v.
 * The speed-up denominator.  lse (optional) is [heads][n_tok].  Library-held scratch. */
s3r_status speed3r_dense_attn(const void *q, const void *k, const void *v, void *out, float *lse,
                              int64_t n_tok, int heads, int head_dim, s3r_dtype dtype,
                              float softmax_scale, void *stream);

/* ---- stage entry points (per-kernel parity tests and profiling) ---------------------------- */

/* Step 1 (Sec. 3.2 "Compression Branch"): block means of q, k, v.
 * qc, kc, vc: out, fp32 [heads][n_blk][head_dim]. */
s3r_status speed3r_pool_blocks(const void *q, const void *k, const void *v, float *qc, float *kc,
                               float *vc, int64_t n_tok, int heads, int head_dim, int block,
                               s3r_dtype dtype, void *stream);

/* Steps 2-3 (eqs. 3-4; Alg. 1 without its TopK part) on pooled fp32 tensors.
 *   qc, kc, vc : in  fp32 [heads][n_blk][head_dim]
 *   s_guide    : out fp32 [heads][n_blk][ld_s], unscaled scores; ld_s >= n_blk, ld_s % 4 == 0;
 *                columns n_blk..ld_s-1 of a row are scratch (unspecified values)
 *   o_comp     : out fp32 [heads][n_blk][head_dim]
 *   accurate_pv: nonzero computes P.Vc with bf16 hi+lo operand pairs (fp32-level accuracy,
 *                used for S3R_F32 problems); zero uses single bf16 operands.
 * Library-held scratch. */
s3r_status speed3r_compress_attn_scores(const float *qc, const float *kc, const float *vc,
                                        float *s_guide, int64_t ld_s, float *o_comp, int64_t n_blk,
                                        int heads, int head_dim, float softmax_scale,
                                        int accurate_pv, void *stream);

/* Steps 2-4 in one go, without S_guide in memory (Sec. 3.2 "Efficient Kernel Implementation",
 * supplementary Sec. 1): compressed attention and, for every query block, the ascending indices of the
 * k = min(topk, n_blk) pooled keys with the largest scores; equal scores go to the smaller index.
 *   qc, kc, vc : in  fp32 [heads][n_blk][head_dim]
 *   o_comp     : out fp32 [heads][n_blk][head_dim]
 *   idx        : out int32 [heads][n_blk][k]
 *   accurate_pv: nonzero keeps the logits of the compressed softmax and the P.Vc product at fp32
 *                accuracy (bf16 hi+lo operand pairs; used for S3R_F32 problems); zero computes them
 *                from single fp16 / bf16 operands (logits good to 2^-10 |q||k|).  The index sets do
 *                not depend on it: they are decided by fp32 dot products either way.
 * Requires k <= 64 (S3R_ERR_UNSUPPORTED otherwise: use the two entry points around this one).
 * Should the scores of a row tie so massively that its candidate lists run over, the call falls back,
 * on the device, to scores written to library scratch; the result is the same.  Library-held scratch. */
s3r_status speed3r_compress_attn_topk(const float *qc, const float *kc, const float *vc, float *o_comp,
                                      int32_t *idx, int64_t n_blk, int heads, int head_dim, int topk,
                                      float softmax_scale, int accurate_pv, void *stream);

/* Step 4 (TopKSelect): idx[h][i][0..k) = ascending indices of the k = min(topk, n_blk) largest
 * entries of s_guide[h][i][0..n_blk); equal scores go to the smaller index.  Deterministic.
 * s_guide must hold no NaN. */
s3r_status speed3r_topk_blocks(const float *s_guide, int64_t ld_s, int32_t *idx, int64_t n_blk,
                               int heads, int topk, void *stream);

/* Steps 5-6 (eq. 6 / Alg. 2, then eqs. 5, 7, 8) with a given index tensor.
 *   idx     : in  [heads][n_blk][kk] block indices in [0, n_blk), distinct per row; 1 <= kk <= n_blk
 *             (entries outside the range are held into it, so that a broken list stays memory-safe; a
 *             block listed twice is attended twice)
 *   o_comp  : in, optional fp32 [heads][n_blk][head_dim]; NULL: `out` receives O_sel unmerged
 *   gate_logits, o_sel, lse: as in s3r_params (all optional)
 * Library-held scratch. */
s3r_status speed3r_select_attn(const void *q, const void *k, const void *v, const int32_t *idx,
                               const float *o_comp, const void *gate_logits, void *out, void *o_sel,
                               float *lse, int64_t n_tok, int heads, int head_dim, int block, int kk,
                               s3r_dtype dtype, float softmax_scale, void *stream);

/* ---- utilities ------------------------------------------------------------------------------ */

/* Measurement of what the data movement of the selection stage (eq. 6 / Alg. 2) costs by itself: the
 * selection kernel for bf16 blocks of 64 or 128 tokens with its arithmetic taken out.  It walks idx
 * ([heads][n_blk][kk], as in speed3r_select_attn) with the same work mapping, brings every selected K/V
 * unit into LDS through the same ring with the same waits and barriers, reads Q and writes `out` (which
 * receives a copy of q).  Time it with speed3r_set_profiling / speed3r_get_stage_ms (stage SELECT): the
 * real kernel cannot be faster than this on the same index lists.
 *   ring_stages: 0 or 2 = the real kernels' two-stage LDS ring; 3, 4 = deeper rings (more units on their
 *                way per workgroup);
 *   wg_per_cu  : 0 = as many workgroups per CU as fit (the real kernels' five); 1..5 = at most that many
 *                (fewer query blocks in progress per XCD: more of the units neighbouring query blocks share
 *                are still in that XCD's L2 when the second one asks).
 * Library-held scratch. */
s3r_status speed3r_probe_select_loads(const void *q, const void *k, const void *v, const int32_t *idx,
                                      void *out, int64_t n_tok, int heads, int head_dim, int block, int kk,
                                      int ring_stages, int wg_per_cu, void *stream);

/* When enabled, every entry point brackets each kernel launch with HIP events on the call's own
 * stream and keeps them until speed3r_get_stage_ms reads them (process-wide switch; default off). */
s3r_status speed3r_set_profiling(int enable);

/* Host arrays of S3R_N_STAGES entries: summed kernel milliseconds and number of launches per
 * stage over all profiled calls since the previous speed3r_get_stage_ms (or since profiling was
 * switched on); the record is cleared.  Waits for the recorded events, so call it after the work. */
s3r_status speed3r_get_stage_ms(float *ms, int *launches);

/* Selects kernel families, process-wide.  0 = automatic: MFMA attention kernels (fp32 problems in bf16
 * operand parts), and for up to 64 TopK blocks per row the TopK that runs
 * inside the compression sweep without writing S_guide to memory (supplementary Sec. 1).  1 = always
 * the generic attention kernel.  2 = like 0 but TopK always from S_guide written to memory. */
s3r_status speed3r_set_kernel_choice(int choice);

/* Frees the library-held scratch (synchronises the device). */
s3r_status speed3r_release_scratch(void);

/* Message for the last non-OK status on this thread (static storage, never NULL). */
const char *speed3r_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SPEED3R_H */
