// Host-side launchers of the gfx950 kernels.  Each returns the hipError_t of its launch.
// All pointers are device pointers; shapes are checked by the callers in speed3r_api.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s3r {

// Number of 32-row operand tiles that cover n_blk pooled rows, padded to a multiple of 4 so that
// a 4-wave workgroup and a 64-key staging step never run past the allocation.
inline int64_t pooled_tiles_padded(int64_t n_blk) { return ((n_blk + 31) / 32 + 3) / 4 * 4; }

// Where the tokens of a sub-sequence sit in the caller's [rows][heads][64] tensors.  The rows come
// in periods (views) of `period` rows; the sub-sequence takes the `count` consecutive rows that
// start at row `first` of every period (image tokens: first = special tokens per view; special
// tokens: first = 0).  period == 0 is the identity.  Sub-sequence indices must stay below 2^31.
//
// With win > 0 the `count` = grid_h * grid_w rows of a period are a row-major patch grid and the
// sub-sequence is laid out in spatial windows of win x win cells (Sec. 3.2): block b of win * win
// slots is window (b % nw) of view b / nw, windows in row-major order over the grid, the cells of
// a window in row-major order; windows on the right and bottom edges are cut at the grid border
// and fill only the first block_len slots of their block.
struct TokenMap {
    int period = 0, first = 0, count = 0;
    int win = 0, grid_h = 0, grid_w = 0, nwx = 0, nw = 0;
    __host__ __device__ int64_t row(int64_t t) const
    {
        if (period == 0) return t;
        const unsigned tt = static_cast<unsigned>(t);
        if (win == 0) {
            const unsigned view = tt / static_cast<unsigned>(count);
            return static_cast<int64_t>(view) * period + first + (tt - view * static_cast<unsigned>(count));
        }
        const unsigned slots = static_cast<unsigned>(win * win);
        const unsigned blk = tt / slots, p = tt - blk * slots;
        const unsigned view = blk / static_cast<unsigned>(nw), wid = blk - view * static_cast<unsigned>(nw);
        const unsigned wy = wid / static_cast<unsigned>(nwx), wx = wid - wy * static_cast<unsigned>(nwx);
        const unsigned left = static_cast<unsigned>(grid_w) - wx * win;
        const unsigned cw = left < static_cast<unsigned>(win) ? left : static_cast<unsigned>(win);
        const unsigned y = wy * win + p / cw, x = wx * win + p % cw;
        return static_cast<int64_t>(view) * period + first + y * static_cast<unsigned>(grid_w) + x;
    }
    // Tokens of block `blk` of `block` slots in a sub-sequence of n_tok slots.
    __host__ __device__ int block_len(int64_t blk, int block, int64_t n_tok) const
    {
        if (win == 0) {
            const int64_t left = n_tok - blk * block;
            return static_cast<int>(left < block ? left : block);
        }
        const unsigned wid = static_cast<unsigned>(blk) % static_cast<unsigned>(nw);
        const unsigned wy = wid / static_cast<unsigned>(nwx), wx = wid - wy * static_cast<unsigned>(nwx);
        const int ch = grid_h - static_cast<int>(wy) * win < win ? grid_h - static_cast<int>(wy) * win : win;
        const int cw = grid_w - static_cast<int>(wx) * win < win ? grid_w - static_cast<int>(wx) * win : win;
        return ch * cw;
    }
};

// Where row r, head h of the caller's q, k, v starts: element strides between consecutive rows and between
// heads (the 64 channels of a head are contiguous).  {0, 0}: the packed [rows][heads][64] layout.
struct InStride {
    int64_t tok = 0, head = 0;
    __host__ __device__ int64_t at(int64_t row, int h, int heads) const
    {
        return tok != 0 ? row * tok + h * head : (row * heads + h) * 64;
    }
};

// blk_len[j] = map.block_len(j, block, n_tok) for every block (the table the attention kernels read
// when blocks are spatial windows).
hipError_t launch_block_lens(TokenMap map, int block, int64_t n_tok, int64_t n_blk, int32_t *blk_len,
                             hipStream_t stream);

// Block means of q, k, v (fp32 [heads][n_blk][64]; any of qc/kc/vc may be null together) and,
// when kb/vb are given (bf16 input), the per-(head, block) K and V tiles in MFMA operand order:
// kb, vb are bf16 [heads][n_blk][block * 64] (blocks of 16 rows: half tiles, see pool.hip).  fp32 input (blocks of
// 64 and 128 tokens only): kb, vb are [2][heads][n_blk][block * 64], the bf16 hi parts followed by the lo parts
// (x - hi rounded to bf16).  n_tok counts the tokens of the
// sub-sequence `map` picks out of q, k, v; blocks are runs of that sub-sequence.
hipError_t launch_pool(const void *q, const void *k, const void *v, float *qc, float *kc, float *vc,
                       void *kb, void *vb, int64_t n_tok, int heads, int block, bool is_bf16,
                       TokenMap map, InStride in, hipStream_t stream);

// Per-head figures the TopK sweeps need: power-of-two factors that bring the largest |component| of the
// head's pooled queries (sq) and keys (sk) into [0.5, 1), their product and its inverse, and the largest
// L2 norm of a scaled pooled key (rounded up).
struct HeadStats { float sq, sk, sqsk, inv_sqsk, kn; };
constexpr int kStatSlots = 64;
// slots: scratch of heads * 3 * kStatSlots words; stats: [heads].
hipError_t launch_pooled_stats(const float *qc, const float *kc, int64_t n_blk, int heads, void *slots,
                               HeadStats *stats, hipStream_t stream);

// Pooled fp32 -> bf16 hi/lo operand tiles ([heads][tiles_padded][32 * 64] each, zero padded).
// vt_lo may be null.  q_f16, k_f16 (optional, need stats): Qc and Kc as fp16 tiles of the same
// shape, scaled by the head's sq and sk.
hipError_t launch_split(const float *qc, const float *kc, const float *vc, void *qs_hi, void *qs_lo,
                        void *ks_hi, void *ks_lo, void *vt_hi, void *vt_lo, void *q_f16, void *k_f16,
                        const HeadStats *stats, int64_t n_blk, int heads, hipStream_t stream);

// S_guide rows + compressed attention for `heads` heads (operand tiles as written by launch_split).
// forced_words (optional): bit b of word kt set = pooled key 64 kt + b is a forced block; its
// score is written as -inf so that TopK never picks it (it still takes part in the softmax).
// Launches that take a run flag use a grid of at most this many workgroups, which walk over the work.
constexpr unsigned kFlaggedGrid = 1024;

// run_flag (optional, device): when given and 0 at run time the launch does nothing.
hipError_t launch_compress(const void *qs_hi, const void *qs_lo, const void *ks_hi,
                           const void *ks_lo, const void *vt_hi, const void *vt_lo, float *s_guide,
                           int64_t ld_s, float *o_comp, int64_t n_blk, int heads, float scale,
                           const unsigned long long *forced_words, const int *run_flag, hipStream_t stream);

// TopK without S_guide in memory, k <= kFusedTopkMaxK, in three launches:
//  threshold: the compression sweep (writes o_comp) that also leaves, per query row, thr [heads][n_blk]:
//             a lower bound of its k-th largest non-forced score, in the scaled units of the fp16
//             tiles, less the margin by which fp16 scores may differ from the fp32-grade ones, and
//             clears *overflow.  bf16 problems (vt_lo null) sweep over the fp16 tiles, fp32 problems
//             over the bf16 hi/lo tiles;
//  filter:    recomputes the scores from the fp16 tiles and appends the index of every one >= thr to
//             cand [heads][n_blk][2][cap] (counts in cand_count [heads][n_blk][2], which may exceed
//             cap: the list is then cut and *overflow set);
//  candidates (launch_topk_candidates): exact TopK among the candidates from fp32 dot products.
constexpr int kFusedTopkMaxK = 64;
hipError_t launch_compress_threshold(const void *qs_hi, const void *qs_lo, const void *ks_hi, const void *ks_lo,
                                     const void *vt_hi, const void *vt_lo, const void *q_f16, const void *k_f16,
                                     float *o_comp, int64_t n_blk, int heads, float scale,
                                     const unsigned long long *forced_words, int k, const HeadStats *stats,
                                     float *thr, int *overflow, hipStream_t stream);
hipError_t launch_compress_filter(const void *q_f16, const void *k_f16,
                                  int64_t n_blk, int heads, const unsigned long long *forced_words,
                                  const float *thr, int32_t *cand, int *cand_count, int cap, int *overflow,
                                  hipStream_t stream);
// qc, kc: fp32 [heads][n_blk][64] of the same heads; idx [heads * n_blk][k].
hipError_t launch_topk_candidates(const float *qc, const float *kc, const int32_t *cand, const int *cand_count,
                                  int cap, int32_t *idx, int64_t n_blk, int heads, int k, hipStream_t stream);

// Forced (always attended) blocks: clamp the caller's list into `forced_clean` and build the
// 64-key bit words for the compression kernel.  status (optional, device): receives 0, or bit 0 = an entry
// out of range, bit 1 = list not strictly ascending.  With n_forced == 0 only *status is written.
hipError_t launch_forced_prepare(const int32_t *forced, int n_forced, int64_t n_blk, int32_t *forced_clean,
                                 unsigned long long *forced_words, int32_t *status, hipStream_t stream);

// out[r][0 .. k_dyn + n_forced) = ascending merge of dyn[r][0 .. k_dyn) and forced_clean[0 .. n_forced).
hipError_t launch_merge_forced(const int32_t *dyn, int k_dyn, const int32_t *forced_clean, int n_forced,
                               int32_t *out, int64_t n_rows, hipStream_t stream);

// TopK of each of n_rows rows of s_guide (row r at s_guide + r * ld_s, n_blk valid entries).
// run_flag (optional, device): when given and 0 at run time the launch does nothing.
hipError_t launch_topk(const float *s_guide, int64_t ld_s, int32_t *idx, int64_t n_blk,
                       int64_t n_rows, int k, const int *run_flag, hipStream_t stream);

// Rarely used arguments of the selection / dense kernels (all optional).
struct SelectExtras {
    const float *o_comp_tok = nullptr;  // selection: compressed outputs per query slot [n_tok][heads][64], merged
                                        // instead of the per-block o_comp (unpooled-query compression branch)
    float *out_f32 = nullptr;           // dense: fp32 result per query slot [n_tok][heads][64] instead of `out`
    int64_t kv_head_stride = 0;         // dense, MFMA: elements between the heads' tile arrays (0: n_blk * block * 64)
    const int32_t *q_blk_len = nullptr; // dense: the query slots come in blocks of q_block slots of which only
    int q_block = 0;                    //        the first q_blk_len[j] exist (spatial windows)
    int64_t k_row_stride = 0;           // dense, generic: elements between consecutive keys of one head in k and v,
    int64_t k_head_stride = 0;          //        and between heads (0, 0: as q, see `in`)
    InStride in;                        // layout of q (generic kernels: of k and v too)
    // dense, MFMA, blocks of 64 or 128 tokens: the key units are cut into n_split equal shares, each worked on
    // by workgroups of its own; share i leaves its normalised result at out_f32 [i][n_tok][heads][64] and the
    // base-2 logarithm of its sum of exponentials at part_lse [i][n_tok][heads] (launch_dense_combine adds
    // the shares up).  For few query rows: more, shorter workgroups spread evenly over the CUs.
    int n_split = 0;
    float *part_lse = nullptr;
};

struct SelectArgs {
    const void *q, *k, *v;     // the caller's layout: [rows][heads][64], or the strides x.in
    const void *kb, *vb;       // operand-order tiles of the keys (MFMA path only)
    const void *kb2 = nullptr, *vb2 = nullptr;  // MFMA dense only: a second key segment, 64-key tiles
    int64_t lo_off = 0, lo_off2 = 0;  // fp32 problems on the MFMA path: kb, vb (kb2, vb2) hold [hi tiles | lo tiles],
                                      // the lo tiles this many elements after the hi ones
    const int32_t *idx;        // [heads][n_blk][kk]; null = every key (dense attention)
    const float *o_comp;       // [heads][n_blk][64] or null (no merge)
    const void *gate;          // [rows][heads][64] or null
    void *out;                 // [rows][heads][64]
    void *o_sel;               // optional, like out
    float *lse;                // optional [heads][lse_stride], indexed by the caller's row
    int64_t n_tok;             // query tokens (sub-sequence qmap picks)
    int64_t n_keys;            // key tokens (tiles kb/vb; for the generic kernels the sub-sequence kmap picks)
    int64_t n_keys2 = 0;       // keys of the second segment
    int64_t n_blk;             // key blocks = ceil(n_keys / block); also the query blocks when idx is given
    int64_t lse_stride;        // rows of the caller's tensors
    TokenMap qmap, kmap;
    const int32_t *blk_len = nullptr;  // tokens per block of the kb/vb (or kmap) sequence; null: full blocks and a short last one
    int heads, block, kk;
    int n_common = 0;          // selection: entries of every index row known to be the same in all rows (forced blocks)
    float scale;
    bool is_bf16;
    bool loads_only = false;   // MFMA selection, blocks of 64 / 128 tokens: move the K/V units, skip the arithmetic
                               // (a measurement of the stage's data movement; `out` receives the Q rows)
    int probe_stages = 0;      // loads_only: LDS ring stages, 2 (the real kernels', also 0), 3 or 4
    int probe_wg_per_cu = 0;   // loads_only: at most this many workgroups per CU (0: as many as fit)
    SelectExtras x;
};

// out[qmap.row(t)][h][:] = sum_i w_i part_o[i][t][h][:], w_i = 2^(part_lse[i][t][h]) / sum_j 2^(part_lse[j][t][h]):
// the softmax over all keys from its shares (out: bf16 [rows][heads][64]).
hipError_t launch_dense_combine(const float *part_o, const float *part_lse, int n_split, int64_t n_tok, int heads,
                                TokenMap qmap, void *out, bool is_bf16, hipStream_t stream);

// One thread per query row, fp32 FMA; any dtype, any supported block size.
hipError_t launch_select_generic(const SelectArgs &a, hipStream_t stream);

// bf16 MFMA kernels (any supported block size).
hipError_t launch_select_mfma(const SelectArgs &a, hipStream_t stream);

// bf16 MFMA selection for plain index rows (at most 128 blocks of 64 tokens each, packed q, per-block compressed
// outputs): few workgroups per CU, each wave software-pipelined (launch_select_mfma routes here).
hipError_t launch_select_pipe(const SelectArgs &a, hipStream_t stream);


}  // namespace s3r
