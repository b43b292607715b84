/*
 * CPU oracle for mesh-aligned block-sparse attention (BSA).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and nothing in the product path may call it: only the
 * tests, the smoke check and the benchmark's CPU-baseline leg load it.
 *
 * What is computed follows the paper's "Block-Sparse Attention" subsection:
 *   - tokens are partitioned into m non-overlapping blocks (Compression
 *     paragraph); here a block is a bh x bw tile of the row-major H x W
 *     lat-lon grid, its tokens enumerated row-major inside the tile;
 *   - block representations are mean-pooled queries and keys (the pooling
 *     equation, phi = mean);
 *   - block-level scores are the pooled dot products of the block-level
 *     attention equation.  Its softmax and 1/sqrt(d_k) are strictly
 *     increasing per row, so ranking by the raw dot product selects the same
 *     blocks as ranking by the coarse attention weight;
 *   - each query block keeps the top-n key blocks (Selection paragraph),
 *     never counting itself, ordered by (score descending, index ascending);
 *   - every token of query block i attends, in ONE softmax, to all tokens of
 *     block i (Local Attention paragraph) and of the selected blocks (the
 *     fine-grained attention equation, with its normaliser Z_l);
 *   - backward holds the selection fixed (Appendix, kernel design paragraph).
 *
 * Arithmetic:
 *   pooling   fp32, sequential adds in in-tile row-major order, then one
 *             multiply by 1/b;
 *   scores    fp32, acc = fmaf(qbar[d], kbar[d], acc) for d = 0..D-1 from +0;
 *   attention double precision throughout, no tiling, no online softmax.
 * All inputs are fp32 arrays [B, heads, N, D] (bf16 inputs are widened exactly
 * by the caller).  OpenMP, when enabled, only distributes independent
 * (batch*head, block) work items; it never changes a summation order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t batch, heads;
    int32_t grid_h, grid_w;
    int32_t block_h, block_w;
    int32_t head_dim;
    int32_t n_select;
} oracle_shape;

static int64_t n_tokens(const oracle_shape *s) { return (int64_t)s->grid_h * s->grid_w; }
static int block_tokens(const oracle_shape *s) { return s->block_h * s->block_w; }
static int n_blocks(const oracle_shape *s) { return (int)(n_tokens(s) / block_tokens(s)); }

/* Token index of position tau (row-major inside the tile) of block beta. */
static int64_t token_of(const oracle_shape *s, int beta, int tau)
{
    int blocks_per_row = s->grid_w / s->block_w;
    int br = beta / blocks_per_row, bc = beta % blocks_per_row;
    int r = br * s->block_h + tau / s->block_w;
    int c = bc * s->block_w + tau % s->block_w;
    return (int64_t)r * s->grid_w + c;
}

/* Exported so that tests can pin the partition itself. */
int64_t oracle_token_of(const oracle_shape *s, int beta, int tau)
{
    return token_of(s, beta, tau);
}

int oracle_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- pooling equation: xbar_i = mean over the tokens of block i ---------- */
void oracle_pool(const oracle_shape *s, const float *x, float *pooled /* [B*h, m, D] */)
{
    const int D = s->head_dim, b = block_tokens(s), m = n_blocks(s);
    const int64_t N = n_tokens(s);
    const int64_t BH = (int64_t)s->batch * s->heads;
    const float inv_b = 1.0f / (float)b;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t g = 0; g < BH; ++g)
        for (int i = 0; i < m; ++i)
            for (int d = 0; d < D; ++d) {
                float sum = 0.0f;
                for (int tau = 0; tau < b; ++tau)
                    sum = sum + x[(g * N + token_of(s, i, tau)) * D + d];
                pooled[(g * m + i) * D + d] = sum * inv_b;
            }
}

/* ---- block-level scores (ranking form of the block attention equation) --- */
static float block_score(const float *qb, const float *kb, int D)
{
    float acc = 0.0f;
    for (int d = 0; d < D; ++d)
        acc = fmaf(qb[d], kb[d], acc);
    return acc;
}

void oracle_scores(const oracle_shape *s, const float *qbar, const float *kbar,
                   float *scores /* [B*h, m, m] */)
{
    const int D = s->head_dim, m = n_blocks(s);
    const int64_t BH = (int64_t)s->batch * s->heads;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t g = 0; g < BH; ++g)
        for (int i = 0; i < m; ++i)
            for (int j = 0; j < m; ++j)
                scores[(g * m + i) * m + j] =
                    block_score(qbar + (g * m + i) * D, kbar + (g * m + j) * D, D);
}

/* ---- selection: top-n of row i over j != i ------------------------------- */
typedef struct { float score; int32_t index; } cand;

static int cand_before(const void *pa, const void *pb)
{
    const cand *a = (const cand *)pa, *b = (const cand *)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    return (a->index > b->index) - (a->index < b->index);
}

void oracle_select_from_pooled(const oracle_shape *s, const float *qbar, const float *kbar,
                               int32_t *sel_idx /* [B*h, m, n] */)
{
    const int D = s->head_dim, m = n_blocks(s), n = s->n_select;
    const int64_t BH = (int64_t)s->batch * s->heads;
#pragma omp parallel
    {
        cand *row = (cand *)malloc(sizeof(cand) * (size_t)(m > 0 ? m : 1));
#pragma omp for collapse(2) schedule(static)
        for (int64_t g = 0; g < BH; ++g)
            for (int i = 0; i < m; ++i) {
                int cnt = 0;
                for (int j = 0; j < m; ++j) {
                    if (j == i) continue;
                    row[cnt].score = block_score(qbar + (g * m + i) * D,
                                                 kbar + (g * m + j) * D, D);
                    row[cnt].index = j;
                    ++cnt;
                }
                qsort(row, (size_t)cnt, sizeof(cand), cand_before);
                for (int r = 0; r < n; ++r)
                    sel_idx[(g * m + i) * n + r] = row[r].index;
            }
        free(row);
    }
}

void oracle_select(const oracle_shape *s, const float *q, const float *k, int32_t *sel_idx)
{
    const int64_t cnt = (int64_t)s->batch * s->heads * n_blocks(s) * s->head_dim;
    float *qbar = (float *)malloc(sizeof(float) * (size_t)cnt);
    float *kbar = (float *)malloc(sizeof(float) * (size_t)cnt);
    oracle_pool(s, q, qbar);
    oracle_pool(s, k, kbar);
    oracle_select_from_pooled(s, qbar, kbar, sel_idx);
    free(qbar);
    free(kbar);
}

/* ---- attention of one query block over {own block} U selected blocks ----- */
/* P (optional, [b, (n+1)*b]) receives the attention weights of the block's
 * rows; column c*b + tau is token tau of the c-th attended block, c = 0 being
 * the block itself and c >= 1 the selected blocks in sel_idx order. */
static void attend_block(const oracle_shape *s, const float *q, const float *k, const float *v,
                         const int32_t *sel_row, int64_t g, int i, double scale,
                         double *out_g /* [N, D] of this batch*head */,
                         double *lse_g /* [N] of this batch*head, or NULL */,
                         double *P, double *z /* scratch (n+1)*b */)
{
    const int D = s->head_dim, b = block_tokens(s), n = s->n_select;
    const int64_t N = n_tokens(s);
    const int nk = (n + 1) * b;
    for (int tq = 0; tq < b; ++tq) {
        const int64_t l = token_of(s, i, tq);
        const float *ql = q + (g * N + l) * D;
        double M = -INFINITY;
        for (int c = 0; c <= n; ++c) {
            const int beta = (c == 0) ? i : sel_row[c - 1];
            for (int tau = 0; tau < b; ++tau) {
                const float *kt = k + (g * N + token_of(s, beta, tau)) * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d)
                    dot += (double)ql[d] * (double)kt[d];
                z[c * b + tau] = scale * dot;
                if (z[c * b + tau] > M) M = z[c * b + tau];
            }
        }
        double Z = 0.0;
        for (int t = 0; t < nk; ++t) {
            z[t] = exp(z[t] - M);
            Z += z[t];
        }
        double *ol = out_g + l * D;
        for (int d = 0; d < D; ++d) ol[d] = 0.0;
        for (int c = 0; c <= n; ++c) {
            const int beta = (c == 0) ? i : sel_row[c - 1];
            for (int tau = 0; tau < b; ++tau) {
                const double p = z[c * b + tau] / Z;
                const float *vt = v + (g * N + token_of(s, beta, tau)) * D;
                for (int d = 0; d < D; ++d)
                    ol[d] += p * (double)vt[d];
                if (P) P[(int64_t)tq * nk + c * b + tau] = p;
            }
        }
        if (lse_g) lse_g[l] = M + log(Z);
    }
}

/* Forward over every (batch*head, block). scale <= 0 means 1/sqrt(D). */
void oracle_fwd(const oracle_shape *s, const float *q, const float *k, const float *v,
                const int32_t *sel_idx, double scale, double *out, double *lse)
{
    const int m = n_blocks(s), n = s->n_select, b = block_tokens(s), D = s->head_dim;
    const int64_t BH = (int64_t)s->batch * s->heads, N = n_tokens(s);
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)s->head_dim);
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)(n + 1) * b);
#pragma omp for collapse(2) schedule(dynamic, 4)
        for (int64_t g = 0; g < BH; ++g)
            for (int i = 0; i < m; ++i)
                attend_block(s, q, k, v, sel_idx + (g * m + i) * n, g, i, scale,
                             out + g * N * D, lse ? lse + g * N : NULL, NULL, z);
        free(z);
    }
}

/* Forward for a list of (batch*head, block) pairs only; rows of the other
 * blocks of out/lse are left untouched.  Used for sampled checks at sizes the
 * full oracle cannot finish, and for the bounded CPU-baseline timing. */
void oracle_fwd_blocks(const oracle_shape *s, const float *q, const float *k, const float *v,
                       const int32_t *sel_idx, double scale, const int64_t *pairs /* [cnt,2] */,
                       int64_t cnt, double *out, double *lse)
{
    const int m = n_blocks(s), n = s->n_select, b = block_tokens(s), D = s->head_dim;
    const int64_t N = n_tokens(s);
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)s->head_dim);
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)(n + 1) * b);
#pragma omp for schedule(dynamic, 1)
        for (int64_t w = 0; w < cnt; ++w) {
            const int64_t g = pairs[2 * w];
            const int i = (int)pairs[2 * w + 1];
            attend_block(s, q, k, v, sel_idx + (g * m + i) * n, g, i, scale,
                         out + g * N * D, lse ? lse + g * N : NULL, NULL, z);
        }
        free(z);
    }
}

/* ---- backward on sampled blocks ------------------------------------------
 * The same closed forms as oracle_bwd, written for one block at a time so that
 * problems too large for a full pass can be checked on samples.  For sample w =
 * (slice g, block x):
 *   dq[w]         rows of dQ of the tokens of block x as a QUERY block;
 *   dk[w], dv[w]  rows of dK, dV of the tokens of block x as a KEY block: sums
 *                 over every query block i of the slice that attends to x (i == x
 *                 or x in sel_idx[i]), query blocks and their tokens ascending.
 * Each [b, D], in-tile row-major token order.  One key/value head per query
 * head.  Every query row's weights are recomputed in full (all its (n+1) b
 * keys): nothing is shared with or taken from another routine's results. */
static void bwd_row(const oracle_shape *s, const float *q, const float *k, const float *v,
                    const float *dout, const int32_t *sel_row, int64_t g, int i, int tq,
                    double scale, double *z /* (n+1) b: P of the row on return */,
                    double *delta_out)
{
    const int D = s->head_dim, n = s->n_select, b = block_tokens(s);
    const int64_t N = n_tokens(s);
    const int nk = (n + 1) * b;
    const int64_t l = token_of(s, i, tq);
    const float *ql = q + (g * N + l) * D;
    const float *dol = dout + (g * N + l) * D;
    double M = -INFINITY;
    for (int c = 0; c <= n; ++c) {
        const int beta = (c == 0) ? i : sel_row[c - 1];
        for (int tau = 0; tau < b; ++tau) {
            const float *kt = k + (g * N + token_of(s, beta, tau)) * D;
            double dot = 0.0;
            for (int d = 0; d < D; ++d) dot += (double)ql[d] * (double)kt[d];
            z[c * b + tau] = scale * dot;
            if (z[c * b + tau] > M) M = z[c * b + tau];
        }
    }
    double Z = 0.0;
    for (int t = 0; t < nk; ++t) { z[t] = exp(z[t] - M); Z += z[t]; }
    for (int t = 0; t < nk; ++t) z[t] /= Z;
    double delta = 0.0;                               /* dO_l . O_l, O_l = sum_t P_lt v_t */
    for (int d = 0; d < D; ++d) {
        double o = 0.0;
        for (int c = 0; c <= n; ++c) {
            const int beta = (c == 0) ? i : sel_row[c - 1];
            for (int tau = 0; tau < b; ++tau)
                o += z[c * b + tau] * (double)v[(g * N + token_of(s, beta, tau)) * D + d];
        }
        delta += (double)dol[d] * o;
    }
    *delta_out = delta;
}

void oracle_bwd_blocks(const oracle_shape *s, const float *q, const float *k, const float *v,
                       const float *dout, const int32_t *sel_idx, double scale,
                       const int64_t *pairs /* [cnt, 2] = (slice, block) */, int64_t cnt,
                       double *dq, double *dk, double *dv /* [cnt, b, D] each */)
{
    const int D = s->head_dim, m = n_blocks(s), n = s->n_select, b = block_tokens(s);
    const int64_t N = n_tokens(s);
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)s->head_dim);
    memset(dq, 0, sizeof(double) * (size_t)(cnt * b * D));
    memset(dk, 0, sizeof(double) * (size_t)(cnt * b * D));
    memset(dv, 0, sizeof(double) * (size_t)(cnt * b * D));
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)(n + 1) * b);
#pragma omp for schedule(dynamic, 1)
        for (int64_t w = 0; w < cnt; ++w) {
            const int64_t g = pairs[2 * w];
            const int x = (int)pairs[2 * w + 1];
            /* dQ of block x as a query block: dQ_l = scale sum_t dS_lt k_t */
            {
                const int32_t *sel_row = sel_idx + (g * m + x) * n;
                for (int tq = 0; tq < b; ++tq) {
                    double delta;
                    bwd_row(s, q, k, v, dout, sel_row, g, x, tq, scale, z, &delta);
                    const float *dol = dout + (g * N + token_of(s, x, tq)) * D;
                    for (int c = 0; c <= n; ++c) {
                        const int beta = (c == 0) ? x : sel_row[c - 1];
                        for (int tau = 0; tau < b; ++tau) {
                            const int64_t t = token_of(s, beta, tau);
                            const float *kt = k + (g * N + t) * D;
                            const float *vt = v + (g * N + t) * D;
                            double dp = 0.0;
                            for (int d = 0; d < D; ++d) dp += (double)dol[d] * (double)vt[d];
                            const double ds = z[c * b + tau] * (dp - delta);
                            for (int d = 0; d < D; ++d)
                                dq[(w * b + tq) * D + d] += scale * ds * (double)kt[d];
                        }
                    }
                }
            }
            /* dK, dV of block x as a key block */
            for (int i = 0; i < m; ++i) {
                const int32_t *sel_row = sel_idx + (g * m + i) * n;
                int c_of_x = (i == x) ? 0 : -1;
                for (int r = 0; r < n && c_of_x < 0; ++r)
                    if (sel_row[r] == x) c_of_x = r + 1;
                if (c_of_x < 0) continue;
                for (int tq = 0; tq < b; ++tq) {
                    double delta;
                    bwd_row(s, q, k, v, dout, sel_row, g, i, tq, scale, z, &delta);
                    const int64_t l = token_of(s, i, tq);
                    const float *ql = q + (g * N + l) * D;
                    const float *dol = dout + (g * N + l) * D;
                    for (int tau = 0; tau < b; ++tau) {
                        const float *vt = v + (g * N + token_of(s, x, tau)) * D;
                        const double p = z[c_of_x * b + tau];
                        double dp = 0.0;
                        for (int d = 0; d < D; ++d) dp += (double)dol[d] * (double)vt[d];
                        const double ds = p * (dp - delta);
                        for (int d = 0; d < D; ++d) {
                            dv[(w * b + tau) * D + d] += p * (double)dol[d];
                            dk[(w * b + tau) * D + d] += scale * ds * (double)ql[d];
                        }
                    }
                }
            }
        }
        free(z);
    }
}

/* Attention weights of one query block: P [b, (n+1)*b] (see attend_block). */
void oracle_block_weights(const oracle_shape *s, const float *q, const float *k, const float *v,
                          const int32_t *sel_idx, double scale, int64_t g, int i, double *P)
{
    const int m = n_blocks(s), n = s->n_select, b = block_tokens(s);
    const int64_t N = n_tokens(s);
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)s->head_dim);
    double *z = (double *)malloc(sizeof(double) * (size_t)(n + 1) * b);
    double *out = (double *)malloc(sizeof(double) * (size_t)(N * s->head_dim));
    attend_block(s, q, k, v, sel_idx + (g * m + i) * n, g, i, scale, out, NULL, P, z);
    free(out);
    free(z);
}

/* ---- the paper's three branches (Block-Sparse Attention subsection) -------
 * The single-softmax path above is one reading; the subsection itself keeps
 * three branches with a softmax each, summed with gates (the aggregation
 * equation of the Native Sparse Attention subsection).  The two C routines
 * below are their building blocks; oracle/bsa_oracle.py composes them.
 */

/* Selection paragraph, taken literally: the top-n entries of row i of the
 * block-level attention over ALL m key blocks (the block itself is a
 * candidate), ordered by (score descending, index ascending); 1 <= n <= m. */
void oracle_select_all_from_pooled(const oracle_shape *s, const float *qbar, const float *kbar,
                                   int32_t *sel_idx /* [B*h, m, n] */)
{
    const int D = s->head_dim, m = n_blocks(s), n = s->n_select;
    const int64_t BH = (int64_t)s->batch * s->heads;
#pragma omp parallel
    {
        cand *row = (cand *)malloc(sizeof(cand) * (size_t)(m > 0 ? m : 1));
#pragma omp for collapse(2) schedule(static)
        for (int64_t g = 0; g < BH; ++g)
            for (int i = 0; i < m; ++i) {
                for (int j = 0; j < m; ++j) {
                    row[j].score = block_score(qbar + (g * m + i) * D, kbar + (g * m + j) * D, D);
                    row[j].index = j;
                }
                qsort(row, (size_t)m, sizeof(cand), cand_before);
                for (int r = 0; r < n; ++r)
                    sel_idx[(g * m + i) * n + r] = row[r].index;
            }
        free(row);
    }
}

/* Fine-grained attention equation with an explicit block list: every token l
 * of query block i attends, in one softmax with normaliser Z_l, to exactly
 * the tokens of the cnt blocks lists[g, i, 0..cnt-1] (nothing is added to the
 * list).  With the selected blocks this is the selection branch; with the
 * blocks of a large local block it is the local branch. */
void oracle_attend_lists(const oracle_shape *s, const float *q, const float *k, const float *v,
                         const int32_t *lists /* [B*h, m, cnt] */, int cnt, double scale,
                         double *out /* [B*h, N, D] */, double *lse /* [B*h, N] or NULL */)
{
    const int m = n_blocks(s), b = block_tokens(s), D = s->head_dim;
    const int64_t BH = (int64_t)s->batch * s->heads, N = n_tokens(s);
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)s->head_dim);
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)cnt * b);
#pragma omp for collapse(2) schedule(dynamic, 4)
        for (int64_t g = 0; g < BH; ++g)
            for (int i = 0; i < m; ++i) {
                const int32_t *list = lists + (g * m + i) * cnt;
                for (int tq = 0; tq < b; ++tq) {
                    const int64_t l = token_of(s, i, tq);
                    const float *ql = q + (g * N + l) * D;
                    double M = -INFINITY, Z = 0.0;
                    for (int c = 0; c < cnt; ++c)
                        for (int tau = 0; tau < b; ++tau) {
                            const float *kt = k + (g * N + token_of(s, list[c], tau)) * D;
                            double dot = 0.0;
                            for (int d = 0; d < D; ++d) dot += (double)ql[d] * (double)kt[d];
                            z[c * b + tau] = scale * dot;
                            if (z[c * b + tau] > M) M = z[c * b + tau];
                        }
                    for (int t = 0; t < cnt * b; ++t) {
                        z[t] = exp(z[t] - M);
                        Z += z[t];
                    }
                    double *ol = out + (g * N + l) * D;
                    for (int d = 0; d < D; ++d) ol[d] = 0.0;
                    for (int c = 0; c < cnt; ++c)
                        for (int tau = 0; tau < b; ++tau) {
                            const float *vt = v + (g * N + token_of(s, list[c], tau)) * D;
                            const double p = z[c * b + tau] / Z;
                            for (int d = 0; d < D; ++d) ol[d] += p * (double)vt[d];
                        }
                    if (lse) lse[g * N + l] = M + log(Z);
                }
            }
        free(z);
    }
}

/* ---- backward with the selection held fixed -------------------------------
 * With P the attention weights of the forward pass:
 *   delta_l = sum_d dO_l[d] O_l[d]
 *   dV_t   += P_lt dO_l
 *   dP_lt   = dO_l . v_t
 *   dS_lt   = P_lt (dP_lt - delta_l)
 *   dQ_l   += scale dS_lt k_t
 *   dK_t   += scale dS_lt q_l
 * summed over every (l, t) pair that the forward pass connects.  No gradient
 * flows through the top-n choice.  Serial over query blocks inside one
 * (batch, head) because several query blocks add into the same dK/dV rows. */
void oracle_bwd(const oracle_shape *s, const float *q, const float *k, const float *v,
                const float *dout, const int32_t *sel_idx, double scale,
                double *dq, double *dk, double *dv)
{
    const int D = s->head_dim, m = n_blocks(s), n = s->n_select, b = block_tokens(s);
    const int64_t N = n_tokens(s);
    const int64_t BH = (int64_t)s->batch * s->heads;
    const int nk = (n + 1) * b;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)s->head_dim);
    memset(dq, 0, sizeof(double) * (size_t)(BH * N * D));
    memset(dk, 0, sizeof(double) * (size_t)(BH * N * D));
    memset(dv, 0, sizeof(double) * (size_t)(BH * N * D));
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t g = 0; g < BH; ++g) {
        double *z = (double *)malloc(sizeof(double) * (size_t)nk);
        double *o = (double *)malloc(sizeof(double) * (size_t)D);
        for (int i = 0; i < m; ++i) {
            const int32_t *sel_row = sel_idx + (g * m + i) * n;
            for (int tq = 0; tq < b; ++tq) {
                const int64_t l = token_of(s, i, tq);
                const float *ql = q + (g * N + l) * D;
                const float *dol = dout + (g * N + l) * D;
                /* recompute this row's weights and output */
                double M = -INFINITY;
                for (int c = 0; c <= n; ++c) {
                    const int beta = (c == 0) ? i : sel_row[c - 1];
                    for (int tau = 0; tau < b; ++tau) {
                        const float *kt = k + (g * N + token_of(s, beta, tau)) * D;
                        double dot = 0.0;
                        for (int d = 0; d < D; ++d) dot += (double)ql[d] * (double)kt[d];
                        z[c * b + tau] = scale * dot;
                        if (z[c * b + tau] > M) M = z[c * b + tau];
                    }
                }
                double Z = 0.0;
                for (int t = 0; t < nk; ++t) { z[t] = exp(z[t] - M); Z += z[t]; }
                for (int t = 0; t < nk; ++t) z[t] /= Z;        /* P_lt */
                for (int d = 0; d < D; ++d) o[d] = 0.0;        /* O_l */
                for (int c = 0; c <= n; ++c) {
                    const int beta = (c == 0) ? i : sel_row[c - 1];
                    for (int tau = 0; tau < b; ++tau) {
                        const float *vt = v + (g * N + token_of(s, beta, tau)) * D;
                        for (int d = 0; d < D; ++d) o[d] += z[c * b + tau] * (double)vt[d];
                    }
                }
                double delta = 0.0;                            /* dO_l . O_l */
                for (int d = 0; d < D; ++d) delta += (double)dol[d] * o[d];
                for (int c = 0; c <= n; ++c) {
                    const int beta = (c == 0) ? i : sel_row[c - 1];
                    for (int tau = 0; tau < b; ++tau) {
                        const int64_t t = token_of(s, beta, tau);
                        const float *kt = k + (g * N + t) * D;
                        const float *vt = v + (g * N + t) * D;
                        const double p = z[c * b + tau];
                        double dp = 0.0;
                        for (int d = 0; d < D; ++d) dp += (double)dol[d] * (double)vt[d];
                        const double ds = p * (dp - delta);
                        for (int d = 0; d < D; ++d) {
                            dv[(g * N + t) * D + d] += p * (double)dol[d];
                            dq[(g * N + l) * D + d] += scale * ds * (double)kt[d];
                            dk[(g * N + t) * D + d] += scale * ds * (double)ql[d];
                        }
                    }
                }
            }
        }
        free(z);
        free(o);
    }
}
