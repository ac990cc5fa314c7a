// Host-side launchers of the gfx950 kernels.  Each returns the hipError_t of its launch.
// All pointers are device pointers; shapes are checked by the callers in speed3r_api.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s3r {

// Number of 32-row operand tiles that cover n_blk pooled rows, padded to a multiple of 4 so that
// a 4-wave workgroup and a 64-key staging step never run past the allocation.
inline int64_t pooled_tiles_padded(int64_t n_blk) { return ((n_blk + 31) / 32 + 3) / 4 * 4; }

// Block means of q, k, v (fp32 [heads][n_blk][64]; any of qc/kc/vc may be null together) and,
// when kb/vb are given (bf16 input, block 64 or 128), the per-(head, block) K and V tiles in
// MFMA operand order: kb, vb are bf16 [heads][n_blk][block * 64].
hipError_t launch_pool(const void *q, const void *k, const void *v, float *qc, float *kc, float *vc,
                       void *kb, void *vb, int64_t n_tok, int heads, int block, bool is_bf16,
                       hipStream_t stream);

// Pooled fp32 -> bf16 hi/lo operand tiles ([heads][tiles_padded][32 * 64] each, zero padded).
// vt_lo may be null.
hipError_t launch_split(const float *qc, const float *kc, const float *vc, void *qs_hi, void *qs_lo,
                        void *ks_hi, void *ks_lo, void *vt_hi, void *vt_lo, int64_t n_blk,
                        int heads, hipStream_t stream);

// S_guide rows + compressed attention for `heads` heads (operand tiles as written by launch_split).
// forced_words (optional): bit b of word kt set = pooled key 64 kt + b is a forced block; its
// score is written as -inf so that TopK never picks it (it still takes part in the softmax).
hipError_t launch_compress(const void *qs_hi, const void *qs_lo, const void *ks_hi,
                           const void *ks_lo, const void *vt_hi, const void *vt_lo, float *s_guide,
                           int64_t ld_s, float *o_comp, int64_t n_blk, int heads, float scale,
                           const unsigned long long *forced_words, hipStream_t stream);

// Forced (always attended) blocks: clamp the caller's list into `forced_clean` and build the
// 64-key bit words for the compression kernel.
hipError_t launch_forced_prepare(const int32_t *forced, int n_forced, int64_t n_blk, int32_t *forced_clean,
                                 unsigned long long *forced_words, hipStream_t stream);

// out[r][0 .. k_dyn + n_forced) = ascending merge of dyn[r][0 .. k_dyn) and forced_clean[0 .. n_forced).
hipError_t launch_merge_forced(const int32_t *dyn, int k_dyn, const int32_t *forced_clean, int n_forced,
                               int32_t *out, int64_t n_rows, hipStream_t stream);

// TopK of each of n_rows rows of s_guide (row r at s_guide + r * ld_s, n_blk valid entries).
hipError_t launch_topk(const float *s_guide, int64_t ld_s, int32_t *idx, int64_t n_blk,
                       int64_t n_rows, int k, hipStream_t stream);

struct SelectArgs {
    const void *q, *k, *v;     // [n_tok][heads][64], original layout
    const void *kb, *vb;       // operand-order tiles (MFMA path only)
    const int32_t *idx;        // [heads][n_blk][kk]; null = every block (dense attention)
    const float *o_comp;       // [heads][n_blk][64] or null (no merge)
    const void *gate;          // [n_tok][heads][64] or null
    void *out;                 // [n_tok][heads][64]
    void *o_sel;               // optional
    float *lse;                // optional [heads][n_tok]
    int64_t n_tok;
    int64_t n_blk;
    int heads, block, kk;
    float scale;
    bool is_bf16;
};

// One thread per query row, fp32 FMA; any dtype, any supported block size.
hipError_t launch_select_generic(const SelectArgs &a, hipStream_t stream);

// bf16 MFMA kernels (block 64 or 128).
hipError_t launch_select_mfma(const SelectArgs &a, hipStream_t stream);

}  // namespace s3r
