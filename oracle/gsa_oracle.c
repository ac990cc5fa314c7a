/*
 * gsa_oracle.c -- slow, plain fp64 CPU oracle for Speed3R's Global Sparse
 * Attention (GSA), Sec. 3.2 of the paper (eqs. 2-8) and the two forward
 * listings of the supplementary (Alg. 1 "Compression Branch Forward Pass",
 * Alg. 2 "Selection Attention Forward Pass").
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the HIP library; it is not
 * a product path and nothing in the product may call it.  It shares no code,
 * header, table or helper with the HIP sources.
 *
 * Conventions
 *   - q, k, v, gate logits: float32, layout [n_tok][heads][d], contiguous.
 *     (bf16 inputs are widened exactly to float32 by the caller; every
 *     arithmetic step below is done in double.)
 *   - "block" = `block` consecutive tokens of the flat sequence; the paper's
 *     s x s pooling window (Sec. 3.2 "Compression Branch") read as a 1-D run
 *     of tokens.  n_blk = ceil(n_tok / block); the last block may be short and
 *     is averaged over its valid tokens only.
 *   - pooled tensors: double, layout [heads][n_blk][d].
 *   - `rows` = the query blocks to evaluate (any subset, any order), so that
 *     large problems can be checked on a sample.
 *   - softmax is the two-pass textbook form (max, then exp / sum).  The online
 *     recurrences of Alg. 1 / Alg. 2 are algebraically the same thing.
 *
 * Pins (tests/test_oracle_*.py): block = 1 reduces pooling to the identity and
 * the compression branch to dense attention; topk = n_blk reduces the selection
 * branch to dense attention (checked against torch's CPU SDPA in fp64); a
 * separately written numpy masked-dense brute force; closed forms on 2-3 token
 * cases; softmax-row-sum invariants; planted TopK sets.
 * End-to-end numbers: parity unpinned by the paper (it prints no worked
 * example); pinned only through the reductions above.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int gsa_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int64_t n_blocks(int64_t n_tok, int block) { return (n_tok + block - 1) / block; }

/* Sec. 3.2 "Compression Branch": non-overlapping average pooling.
 * xc[h][j][c] = mean over the valid tokens t of block j of x[t][h][c]. */
void gsa_oracle_pool(const float *x, int64_t n_tok, int heads, int d, int block, double *xc)
{
    const int64_t nb = n_blocks(n_tok, block);
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < heads; ++h) {
        for (int64_t j = 0; j < nb; ++j) {
            const int64_t t0 = j * block;
            const int64_t t1 = (t0 + block < n_tok) ? t0 + block : n_tok;
            double *dst = xc + ((int64_t)h * nb + j) * d;
            for (int c = 0; c < d; ++c) {
                double acc = 0.0;
                for (int64_t t = t0; t < t1; ++t) acc += (double)x[(t * heads + h) * d + c];
                dst[c] = acc / (double)(t1 - t0);
            }
        }
    }
}

/* Eq. 4: S_guide = Q_comp K_comp^T, unscaled, for the requested query blocks.
 * s[h][r][j] = qc[h][rows[r]] . kc[h][j]        (layout [heads][n_rows][n_blk]) */
void gsa_oracle_scores(const double *qc, const double *kc, int64_t n_blk, int heads, int d,
                       const int64_t *rows, int64_t n_rows, double *s)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < heads; ++h) {
        for (int64_t r = 0; r < n_rows; ++r) {
            const double *qi = qc + ((int64_t)h * n_blk + rows[r]) * d;
            double *srow = s + ((int64_t)h * n_rows + r) * n_blk;
            for (int64_t j = 0; j < n_blk; ++j) {
                const double *kj = kc + ((int64_t)h * n_blk + j) * d;
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += qi[c] * kj[c];
                srow[j] = acc;
            }
        }
    }
}

/* Eq. 3: O'_comp = softmax(scale * S_guide) V_comp, over all n_blk pooled keys.
 * oc[h][r][c]  (layout [heads][n_rows][d]) */
void gsa_oracle_compressed_attn(const double *s, const double *vc, int64_t n_blk, int heads, int d,
                                int64_t n_rows, double scale, double *oc)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < heads; ++h) {
        for (int64_t r = 0; r < n_rows; ++r) {
            const double *srow = s + ((int64_t)h * n_rows + r) * n_blk;
            double *dst = oc + ((int64_t)h * n_rows + r) * d;
            double mx = -INFINITY;
            for (int64_t j = 0; j < n_blk; ++j)
                if (scale * srow[j] > mx) mx = scale * srow[j];
            double den = 0.0;
            for (int c = 0; c < d; ++c) dst[c] = 0.0;
            for (int64_t j = 0; j < n_blk; ++j) {
                const double p = exp(scale * srow[j] - mx);
                den += p;
                const double *vj = vc + ((int64_t)h * n_blk + j) * d;
                for (int c = 0; c < d; ++c) dst[c] += p * vj[c];
            }
            for (int c = 0; c < d; ++c) dst[c] /= den;
        }
    }
}

typedef struct { double s; int32_t j; } scored_t;

static int by_score_desc_then_index(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

static int by_int32(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Sec. 3.2 "Selection Branch", TopKSelect on the raw rows of S_guide: the kk
 * largest entries of each row, equal scores resolved towards the smaller block
 * index; the chosen indices are stored in ascending order.  Blocks j with
 * excluded[j] != 0 never compete (Sec. 3.3: the fixed global-context blocks of
 * the VGGT variant are always attended, so the dynamic TopK runs over the rest;
 * the supplementary's "mask the first frame token").  excluded == NULL: none.
 * idx[h][r][0..kk)  (layout [heads][n_rows][kk]);
 * requires 1 <= kk <= number of blocks that are not excluded. */
void gsa_oracle_topk_excluding(const double *s, int64_t n_blk, int heads, int64_t n_rows, int kk,
                               const uint8_t *excluded, int32_t *idx)
{
#pragma omp parallel
    {
        scored_t *tmp = (scored_t *)malloc((size_t)n_blk * sizeof(scored_t));
#pragma omp for collapse(2) schedule(static)
        for (int h = 0; h < heads; ++h) {
            for (int64_t r = 0; r < n_rows; ++r) {
                const double *srow = s + ((int64_t)h * n_rows + r) * n_blk;
                int64_t n = 0;
                for (int64_t j = 0; j < n_blk; ++j) {
                    if (excluded && excluded[j]) continue;
                    tmp[n].s = srow[j];
                    tmp[n].j = (int32_t)j;
                    ++n;
                }
                qsort(tmp, (size_t)n, sizeof(scored_t), by_score_desc_then_index);
                int32_t *dst = idx + ((int64_t)h * n_rows + r) * kk;
                for (int a = 0; a < kk; ++a) dst[a] = tmp[a].j;
                qsort(dst, (size_t)kk, sizeof(int32_t), by_int32);
            }
        }
        free(tmp);
    }
}

void gsa_oracle_topk(const double *s, int64_t n_blk, int heads, int64_t n_rows, int kk,
                     int32_t *idx)
{
    gsa_oracle_topk_excluding(s, n_blk, heads, n_rows, kk, NULL, idx);
}

/* Eq. 6 / Alg. 2: for every query token t of query block rows[r] and head h,
 * softmax attention over exactly the valid tokens of the kk key blocks
 * idx[h][r][.], logits scale * q_t . k_u.
 *   o_sel[r][p][h][c]  (layout [n_rows][block][heads][d]; rows p >= len are 0)
 *   lse  [h][r][p]     (layout [heads][n_rows][block]; natural log of the sum
 *                       of exp(logit): Alg. 2's L = m + log l)
 * The index set is an argument so that either resolution of a near-tie can be
 * evaluated. */
void gsa_oracle_select_attn(const float *q, const float *k, const float *v, int64_t n_tok,
                            int heads, int d, int block, const int64_t *rows, int64_t n_rows,
                            const int32_t *idx, int kk, double scale, double *o_sel, double *lse)
{
#pragma omp parallel
    {
        double *logit = (double *)malloc((size_t)kk * block * sizeof(double));
        int64_t *tok = (int64_t *)malloc((size_t)kk * block * sizeof(int64_t));
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int64_t r = 0; r < n_rows; ++r) {
            for (int h = 0; h < heads; ++h) {
                const int32_t *sel = idx + ((int64_t)h * n_rows + r) * kk;
                /* the union U of the valid tokens of the selected blocks */
                int64_t nu = 0;
                for (int a = 0; a < kk; ++a) {
                    const int64_t u0 = (int64_t)sel[a] * block;
                    const int64_t u1 = (u0 + block < n_tok) ? u0 + block : n_tok;
                    for (int64_t u = u0; u < u1; ++u) tok[nu++] = u;
                }
                for (int p = 0; p < block; ++p) {
                    const int64_t t = rows[r] * block + p;
                    double *dst = o_sel + (((int64_t)r * block + p) * heads + h) * d;
                    double *ldst = lse + ((int64_t)h * n_rows + r) * block + p;
                    for (int c = 0; c < d; ++c) dst[c] = 0.0;
                    *ldst = 0.0;
                    if (t >= n_tok) continue;
                    const float *qt = q + (t * heads + h) * d;
                    double mx = -INFINITY;
                    for (int64_t a = 0; a < nu; ++a) {
                        const float *ku = k + (tok[a] * heads + h) * d;
                        double acc = 0.0;
                        for (int c = 0; c < d; ++c) acc += (double)qt[c] * (double)ku[c];
                        logit[a] = scale * acc;
                        if (logit[a] > mx) mx = logit[a];
                    }
                    double den = 0.0;
                    for (int64_t a = 0; a < nu; ++a) {
                        const double p_u = exp(logit[a] - mx);
                        den += p_u;
                        const float *vu = v + (tok[a] * heads + h) * d;
                        for (int c = 0; c < d; ++c) dst[c] += p_u * (double)vu[c];
                    }
                    for (int c = 0; c < d; ++c) dst[c] /= den;
                    *ldst = mx + log(den);
                }
            }
        }
        free(logit);
        free(tok);
    }
}

/* Eqs. 5, 7, 8: nearest-neighbour upsampling of O'_comp (every token of a block
 * gets its block's row) and the gated sum
 *   out = g * O_comp + (1 - g) * O_sel,  g = sigmoid(gate_logit)  (elementwise);
 * gate == NULL means g = 1/2 everywhere (W_g = 0).
 *   oc    [heads][n_rows][d], o_sel [n_rows][block][heads][d],
 *   gate  [n_tok][heads][d] (float32, full sequence, may be NULL),
 *   out   [n_rows][block][heads][d]  (rows beyond n_tok are 0). */
void gsa_oracle_merge(const double *oc, const double *o_sel, const float *gate, int64_t n_tok,
                      int heads, int d, int block, const int64_t *rows, int64_t n_rows, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        for (int p = 0; p < block; ++p) {
            const int64_t t = rows[r] * block + p;
            for (int h = 0; h < heads; ++h) {
                const int64_t o = (((int64_t)r * block + p) * heads + h) * d;
                for (int c = 0; c < d; ++c) {
                    if (t >= n_tok) { out[o + c] = 0.0; continue; }
                    double g = 0.5;
                    if (gate) g = 1.0 / (1.0 + exp(-(double)gate[(t * heads + h) * d + c]));
                    out[o + c] = g * oc[((int64_t)h * n_rows + r) * d + c] + (1.0 - g) * o_sel[o + c];
                }
            }
        }
    }
}

/* Eq. 2 form: plain softmax attention of the listed query tokens over all
 * n_tok keys.  out[i][h][c] for i < n_q  (layout [n_q][heads][d]);
 * lse[h][i] may be NULL. */
void gsa_oracle_dense_attn(const float *q, const float *k, const float *v, int64_t n_tok, int heads,
                           int d, const int64_t *q_tok, int64_t n_q, double scale, double *out,
                           double *lse)
{
#pragma omp parallel
    {
        double *logit = (double *)malloc((size_t)n_tok * sizeof(double));
#pragma omp for collapse(2) schedule(dynamic, 4)
        for (int64_t i = 0; i < n_q; ++i) {
            for (int h = 0; h < heads; ++h) {
                const float *qt = q + (q_tok[i] * heads + h) * d;
                double *dst = out + ((int64_t)i * heads + h) * d;
                double mx = -INFINITY;
                for (int64_t u = 0; u < n_tok; ++u) {
                    const float *ku = k + (u * heads + h) * d;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += (double)qt[c] * (double)ku[c];
                    logit[u] = scale * acc;
                    if (logit[u] > mx) mx = logit[u];
                }
                double den = 0.0;
                for (int c = 0; c < d; ++c) dst[c] = 0.0;
                for (int64_t u = 0; u < n_tok; ++u) {
                    const double p_u = exp(logit[u] - mx);
                    den += p_u;
                    const float *vu = v + (u * heads + h) * d;
                    for (int c = 0; c < d; ++c) dst[c] += p_u * (double)vu[c];
                }
                for (int c = 0; c < d; ++c) dst[c] /= den;
                if (lse) lse[(int64_t)h * n_q + i] = mx + log(den);
            }
        }
        free(logit);
    }
}
