/*
 * lvx_oracle.c -- fp64 CPU oracle for the LV-XAttn single-worker compute path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is
 * checked against.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product (the HIP library and its Python
 * binding) never links, imports or executes anything in this directory, and
 * this file shares no code, header, table or helper with the HIP path.
 *
 * What is computed, and from where in the paper:
 *   - forward: the definition of cross-attention, O = softmax(Q K^T / sqrt(d)) V
 *     (Section 2, the unnumbered attention equation), evaluated row by row with
 *     every score of a row held at once -- no tiling, no running maximum.  The
 *     per-row softmax statistic L (Section 2, the block-wise decomposition; the
 *     "+ S_Q/n" term of Eq. 1 fixes it to one scalar per query row) is taken
 *     as the natural-log-sum-exp of the scaled scores.
 *   - merge: the Rescale step of Algorithm 1.  The paper never prints its
 *     formula; the only combination of normalised partial outputs that makes
 *     the block-wise decomposition of Section 2 exact is the log-sum-exp
 *     weighted sum written out in lvx_oracle_merge.
 *   - backward: the paper gives only its FLOP count (Table 1) and the saved
 *     set {x, O, L} (Section 3.2).  The oracle is the plain derivative of the
 *     forward definition through the explicit softmax Jacobian.
 *   - block backward: the step one worker takes for its own K/V block when
 *     only the final O and L are available (Section 3.2 saves nothing else):
 *     p = exp(s - L), delta = rowsum(dO * O).
 *   - projection: the products of Section 2 that make the operands of the
 *     attention, Q = x W_Q and K, V = y W_K, y W_V, which Section 3.2 has the
 *     backward pass compute again instead of keeping Q, K and V.  Written
 *     out as the definition of a matrix product, one dot product per output
 *     element, with the d columns of the result cut into heads.
 *   - projection gradients: the paper prints no formula for them either; they
 *     are the chain rule through those same linear maps (what the recomputed
 *     K and V of Section 3.2 are for: carrying dK, dV back to the visual
 *     tokens and to W_K, W_V), one sum per element of dW and of dx.
 *
 * Conventions:
 *   Q, dO      [B, Hq,  Sq,  D]  float32, contiguous, values already rounded
 *   K, V       [B, Hkv, Skv, D]  to the workload's storage type by the caller
 *   O, L, dQ, dK, dV  float64 outputs, contiguous, same index order
 *   GQA: query head hq reads K/V head hq / (Hq / Hkv)   (contiguous groups)
 *   mask (optional, NULL = dense): allow[b * mask_sb + (i / q_chunk) * n_kv_blocks
 *        + (j / kv_block)] != 0  means query row i may attend key row j.
 *   A masked score is -infinity.  A row with no visible key has O = 0,
 *   L = -infinity and zero gradients.
 *   All arithmetic is double precision; exp/log are libm's.
 *
 * Pinned by tests/test_oracle_*.py (closed forms, brute force in numpy on tiny
 * inputs, finite differences, invariants).  The paper prints no worked
 * numerical example, so there are no paper-printed values to pin against.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int B, Hq, Hkv, Sq, Skv, D;
    double scale;                 /* multiplies Q K^T; 1/sqrt(D) in the paper */
    const uint8_t *allow;         /* NULL = dense */
    int q_chunk, kv_block, n_q_chunks, n_kv_blocks;
    long mask_sb;                 /* batch stride of allow, 0 = shared */
} lvx_oracle_problem;

int lvx_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline int visible(const lvx_oracle_problem *p, int b, int i, int j)
{
    if (!p->allow) return 1;
    return p->allow[(long)b * p->mask_sb + (long)(i / p->q_chunk) * p->n_kv_blocks
                    + (j / p->kv_block)] != 0;
}

static inline const float *q_row(const lvx_oracle_problem *p, const float *q, int b, int hq, int i)
{
    return q + (((long)b * p->Hq + hq) * p->Sq + i) * p->D;
}

static inline const float *kv_row(const lvx_oracle_problem *p, const float *k, int b, int hkv, int j)
{
    return k + (((long)b * p->Hkv + hkv) * p->Skv + j) * p->D;
}

static inline int kv_head(const lvx_oracle_problem *p, int hq)
{
    return hq / (p->Hq / p->Hkv);
}

static inline double dot_fd(const float *a, const float *b, int D)
{
    double s = 0.0;
#pragma omp simd reduction(+ : s)
    for (int d = 0; d < D; ++d) s += (double)a[d] * (double)b[d];
    return s;
}

/* Scaled, masked scores of query row (b,hq,i) against keys [j0,j1):
 * s[j-j0] = scale * <Q_i, K_j>, or -inf where the mask forbids the pair. */
static void row_scores(const lvx_oracle_problem *p, const float *q, const float *k,
                       int b, int hq, int i, int j0, int j1, double *s)
{
    const float *qi = q_row(p, q, b, hq, i);
    const int hk = kv_head(p, hq);
    for (int j = j0; j < j1; ++j) {
        if (!visible(p, b, i, j)) { s[j - j0] = -INFINITY; continue; }
        s[j - j0] = p->scale * dot_fd(qi, kv_row(p, k, b, hk, j), p->D);
    }
}

/* softmax of one row: prob[j] = exp(s_j - m) / sum_j exp(s_j - m); returns the
 * log-sum-exp m + ln(sum).  All -inf -> prob = 0, returns -inf. */
static double row_softmax(const double *s, int n, double *prob)
{
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) if (s[j] > m) m = s[j];
    if (m == -INFINITY) { for (int j = 0; j < n; ++j) prob[j] = 0.0; return -INFINITY; }
    double l = 0.0;
    for (int j = 0; j < n; ++j) { prob[j] = exp(s[j] - m); l += prob[j]; }
    for (int j = 0; j < n; ++j) prob[j] /= l;
    return m + log(l);
}

/* One output row of the attention definition. */
static void fwd_row(const lvx_oracle_problem *p, const float *q, const float *k, const float *v,
                    int b, int hq, int i, double *work /* Skv */, double *o_row, double *lse)
{
    const int hk = kv_head(p, hq);
    row_scores(p, q, k, b, hq, i, 0, p->Skv, work);
    *lse = row_softmax(work, p->Skv, work);
    for (int d = 0; d < p->D; ++d) o_row[d] = 0.0;
    for (int j = 0; j < p->Skv; ++j) {
        const double pj = work[j];
        if (pj == 0.0) continue;
        const float *vj = kv_row(p, v, b, hk, j);
        for (int d = 0; d < p->D; ++d) o_row[d] += pj * (double)vj[d];
    }
}

/* Attention probabilities of one query row (for the "rows of P sum to one" pin). */
void lvx_oracle_prob_row(const lvx_oracle_problem *p, const float *q, const float *k,
                         int b, int hq, int i, double *prob /* Skv */)
{
    row_scores(p, q, k, b, hq, i, 0, p->Skv, prob);
    (void)row_softmax(prob, p->Skv, prob);
}

/* Forward for every row.  O [B,Hq,Sq,D], L [B,Hq,Sq]. */
void lvx_oracle_fwd(const lvx_oracle_problem *p, const float *q, const float *k, const float *v,
                    double *O, double *L)
{
    const long rows = (long)p->B * p->Hq * p->Sq;
#pragma omp parallel
    {
        double *work = (double *)malloc(sizeof(double) * (size_t)p->Skv);
#pragma omp for schedule(dynamic, 4)
        for (long r = 0; r < rows; ++r) {
            const int i = (int)(r % p->Sq);
            const int hq = (int)((r / p->Sq) % p->Hq);
            const int b = (int)(r / ((long)p->Sq * p->Hq));
            fwd_row(p, q, k, v, b, hq, i, work, O + r * p->D, L + r);
        }
        free(work);
    }
}

/* Forward for a list of rows: rows[3*n] = (b, hq, i).  O_rows [n,D], L_rows [n]. */
void lvx_oracle_fwd_rows(const lvx_oracle_problem *p, const float *q, const float *k, const float *v,
                         int n, const int *rows, double *O_rows, double *L_rows)
{
#pragma omp parallel
    {
        double *work = (double *)malloc(sizeof(double) * (size_t)p->Skv);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n; ++r)
            fwd_row(p, q, k, v, rows[3 * r], rows[3 * r + 1], rows[3 * r + 2], work,
                    O_rows + (long)r * p->D, L_rows + r);
        free(work);
    }
}

/* Rescale / merge (Algorithm 1's Rescale, generalised to n parts).
 * O_parts [n_parts, rows, D], L_parts [n_parts, rows] ->
 *   L = ln sum_k exp(L_k),   O = sum_k exp(L_k - L) O_k.
 * All parts empty (L_k = -inf) -> O = 0, L = -inf: the identity element of
 * the merge is (O, L) = (0, -inf). */
void lvx_oracle_merge(int n_parts, long rows, int D, const double *O_parts, const double *L_parts,
                      double *O, double *L)
{
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        double M = -INFINITY;
        for (int k = 0; k < n_parts; ++k) {
            const double lk = L_parts[(long)k * rows + r];
            if (lk > M) M = lk;
        }
        for (int d = 0; d < D; ++d) O[r * D + d] = 0.0;
        if (M == -INFINITY) { L[r] = -INFINITY; continue; }
        double z = 0.0;
        for (int k = 0; k < n_parts; ++k) z += exp(L_parts[(long)k * rows + r] - M);
        const double Lr = M + log(z);
        L[r] = Lr;
        for (int k = 0; k < n_parts; ++k) {
            const double lk = L_parts[(long)k * rows + r];
            if (lk == -INFINITY) continue;
            const double w = exp(lk - Lr);
            const double *ok = O_parts + ((long)k * rows + r) * D;
            for (int d = 0; d < D; ++d) O[r * D + d] += w * ok[d];
        }
    }
}

/* Per-row quantities of the naive backward for query row (b,hq,i):
 *   prob[j] = p_ij,  dP_ij = <dO_i, V_j>,  rowdot = sum_j p_ij dP_ij,
 *   ds[j] = p_ij (dP_ij - rowdot)      (softmax Jacobian applied to dP)
 * Returns rowdot; *m_out, *l_out give max and sum so that
 * p_ij = exp(s_ij - m) / l can be re-formed elsewhere. */
static double bwd_row(const lvx_oracle_problem *p, const float *q, const float *k, const float *v,
                      const float *dO, int b, int hq, int i,
                      double *prob, double *ds, double *m_out, double *l_out)
{
    const int hk = kv_head(p, hq);
    const int n = p->Skv;
    row_scores(p, q, k, b, hq, i, 0, n, prob);
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) if (prob[j] > m) m = prob[j];
    *m_out = m;
    if (m == -INFINITY) {
        for (int j = 0; j < n; ++j) { prob[j] = 0.0; ds[j] = 0.0; }
        *l_out = 0.0;
        return 0.0;
    }
    double l = 0.0;
    for (int j = 0; j < n; ++j) { prob[j] = exp(prob[j] - m); l += prob[j]; }
    for (int j = 0; j < n; ++j) prob[j] /= l;
    *l_out = l;
    const float *doi = q_row(p, dO, b, hq, i);
    double rowdot = 0.0;
    for (int j = 0; j < n; ++j) {
        if (prob[j] == 0.0) { ds[j] = 0.0; continue; }
        ds[j] = dot_fd(doi, kv_row(p, v, b, hk, j), p->D);   /* dP_ij for now */
        rowdot += prob[j] * ds[j];
    }
    for (int j = 0; j < n; ++j) ds[j] = prob[j] * (ds[j] - rowdot);
    return rowdot;
}

static void dq_from_ds(const lvx_oracle_problem *p, const float *k, int b, int hq,
                       const double *ds, double *dq_row)
{
    const int hk = kv_head(p, hq);
    for (int d = 0; d < p->D; ++d) dq_row[d] = 0.0;
    for (int j = 0; j < p->Skv; ++j) {
        if (ds[j] == 0.0) continue;
        const float *kj = kv_row(p, k, b, hk, j);
        for (int d = 0; d < p->D; ++d) dq_row[d] += ds[j] * (double)kj[d];
    }
    for (int d = 0; d < p->D; ++d) dq_row[d] *= p->scale;
}

/* dK and dV of one key row (b,hk,j): the sum, over every query row of the
 * heads sharing this K/V head, of that row's contribution, with p_ij re-formed
 * from the row's stored max m, sum l and rowdot. */
static void dkv_row(const lvx_oracle_problem *p, const float *q, const float *k, const float *v,
                    const float *dO, int b, int hk, int j,
                    const double *m, const double *l, const double *rowdot, /* [B,Hq,Sq] */
                    double *dk_row, double *dv_row)
{
    const int G = p->Hq / p->Hkv;
    const float *kj = kv_row(p, k, b, hk, j);
    const float *vj = kv_row(p, v, b, hk, j);
    for (int d = 0; d < p->D; ++d) { dk_row[d] = 0.0; dv_row[d] = 0.0; }
    for (int hq = hk * G; hq < (hk + 1) * G; ++hq) {
        for (int i = 0; i < p->Sq; ++i) {
            if (!visible(p, b, i, j)) continue;
            const long r = ((long)b * p->Hq + hq) * p->Sq + i;
            if (m[r] == -INFINITY) continue;
            const float *qi = q_row(p, q, b, hq, i);
            const float *doi = q_row(p, dO, b, hq, i);
            const double s = p->scale * dot_fd(qi, kj, p->D);
            const double pij = exp(s - m[r]) / l[r];
            const double dP = dot_fd(doi, vj, p->D);
            const double dS = pij * (dP - rowdot[r]);
            for (int d = 0; d < p->D; ++d) {
                dv_row[d] += pij * (double)doi[d];
                dk_row[d] += dS * (double)qi[d];
            }
        }
    }
    for (int d = 0; d < p->D; ++d) dk_row[d] *= p->scale;
}

/* Row statistics (m, l, rowdot) for every query row; also dQ when non-NULL. */
static void bwd_pass_rows(const lvx_oracle_problem *p, const float *q, const float *k,
                          const float *v, const float *dO, const uint8_t *need /* [B,Hkv] or NULL */,
                          double *m, double *l, double *rowdot, double *dQ)
{
    const long rows = (long)p->B * p->Hq * p->Sq;
#pragma omp parallel
    {
        double *prob = (double *)malloc(sizeof(double) * (size_t)p->Skv);
        double *ds = (double *)malloc(sizeof(double) * (size_t)p->Skv);
#pragma omp for schedule(dynamic, 4)
        for (long r = 0; r < rows; ++r) {
            const int i = (int)(r % p->Sq);
            const int hq = (int)((r / p->Sq) % p->Hq);
            const int b = (int)(r / ((long)p->Sq * p->Hq));
            if (need && !need[b * p->Hkv + kv_head(p, hq)]) continue;
            rowdot[r] = bwd_row(p, q, k, v, dO, b, hq, i, prob, ds, m + r, l + r);
            if (dQ) dq_from_ds(p, k, b, hq, ds, dQ + r * p->D);
        }
        free(prob);
        free(ds);
    }
}

/* Naive backward of  loss = sum(O * dO)  with respect to Q, K, V.
 * dQ [B,Hq,Sq,D], dK, dV [B,Hkv,Skv,D].  No gradient flows through L. */
void lvx_oracle_bwd(const lvx_oracle_problem *p, const float *q, const float *k, const float *v,
                    const float *dO, double *dQ, double *dK, double *dV)
{
    const long rows = (long)p->B * p->Hq * p->Sq;
    double *m = (double *)malloc(sizeof(double) * (size_t)rows);
    double *l = (double *)malloc(sizeof(double) * (size_t)rows);
    double *rowdot = (double *)malloc(sizeof(double) * (size_t)rows);
    bwd_pass_rows(p, q, k, v, dO, NULL, m, l, rowdot, dQ);
    const long kvrows = (long)p->B * p->Hkv * p->Skv;
#pragma omp parallel for schedule(dynamic, 16)
    for (long r = 0; r < kvrows; ++r) {
        const int j = (int)(r % p->Skv);
        const int hk = (int)((r / p->Skv) % p->Hkv);
        const int b = (int)(r / ((long)p->Skv * p->Hkv));
        dkv_row(p, q, k, v, dO, b, hk, j, m, l, rowdot, dK + r * p->D, dV + r * p->D);
    }
    free(m); free(l); free(rowdot);
}

/* dQ for a list of query rows: rows[3*n] = (b, hq, i); dQ_rows [n, D]. */
void lvx_oracle_bwd_q_rows(const lvx_oracle_problem *p, const float *q, const float *k,
                           const float *v, const float *dO, int n, const int *rows, double *dQ_rows)
{
#pragma omp parallel
    {
        double *prob = (double *)malloc(sizeof(double) * (size_t)p->Skv);
        double *ds = (double *)malloc(sizeof(double) * (size_t)p->Skv);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n; ++r) {
            double m, l;
            (void)bwd_row(p, q, k, v, dO, rows[3 * r], rows[3 * r + 1], rows[3 * r + 2],
                          prob, ds, &m, &l);
            dq_from_ds(p, k, rows[3 * r], rows[3 * r + 1], ds, dQ_rows + (long)r * p->D);
        }
        free(prob);
        free(ds);
    }
}

/* dK, dV for a list of key rows: rows[3*n] = (b, hkv, j); outputs [n, D].
 * Needs the row statistics of every query row of the heads that share the
 * sampled K/V heads, i.e. a full pass over those heads' Q. */
void lvx_oracle_bwd_kv_rows(const lvx_oracle_problem *p, const float *q, const float *k,
                            const float *v, const float *dO, int n, const int *rows,
                            double *dK_rows, double *dV_rows)
{
    const long nr = (long)p->B * p->Hq * p->Sq;
    double *m = (double *)malloc(sizeof(double) * (size_t)nr);
    double *l = (double *)malloc(sizeof(double) * (size_t)nr);
    double *rowdot = (double *)malloc(sizeof(double) * (size_t)nr);
    uint8_t *need = (uint8_t *)calloc((size_t)p->B * p->Hkv, 1);
    for (int r = 0; r < n; ++r) need[rows[3 * r] * p->Hkv + rows[3 * r + 1]] = 1;
    bwd_pass_rows(p, q, k, v, dO, need, m, l, rowdot, NULL);
    free(need);
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n; ++r)
        dkv_row(p, q, k, v, dO, rows[3 * r], rows[3 * r + 1], rows[3 * r + 2], m, l, rowdot,
                dK_rows + (long)r * p->D, dV_rows + (long)r * p->D);
    free(m); free(l); free(rowdot);
}

/* Backward step of one worker for its own K/V block [kv0, kv1), given the
 * FINAL output O and statistic L of the whole key range (all that is saved,
 * Section 3.2).  K, V are still passed whole; only rows kv0..kv1-1 are read.
 *   p_ij   = exp(s_ij - L_i)
 *   delta_i = sum_d dO_id O_id
 *   dV_j  = sum_i p_ij dO_i,   dS_ij = p_ij (<dO_i, V_j> - delta_i)
 *   dK_j  = scale sum_i dS_ij Q_i,   dQ_i(block) = scale sum_{j in block} dS_ij K_j
 * Outputs: dQ_part [B,Hq,Sq,D] (this block's addend), dK_blk, dV_blk
 * [B,Hkv,kv1-kv0,D].  Summed over a partition of the keys this must equal
 * lvx_oracle_bwd (checked in the tests). */
void lvx_oracle_bwd_block(const lvx_oracle_problem *p, const float *q, const float *k,
                          const float *v, const float *dO, const double *O, const double *L,
                          int kv0, int kv1, double *dQ_part, double *dK_blk, double *dV_blk)
{
    const long rows = (long)p->B * p->Hq * p->Sq;
    const int nb = kv1 - kv0;
    const int G = p->Hq / p->Hkv;
    double *delta = (double *)malloc(sizeof(double) * (size_t)rows);
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        double s = 0.0;
        for (int d = 0; d < p->D; ++d) s += (double)dO[r * p->D + d] * O[r * p->D + d];
        delta[r] = s;
    }
#pragma omp parallel for schedule(dynamic, 4)
    for (long r = 0; r < rows; ++r) {
        const int i = (int)(r % p->Sq);
        const int hq = (int)((r / p->Sq) % p->Hq);
        const int b = (int)(r / ((long)p->Sq * p->Hq));
        const int hk = kv_head(p, hq);
        double *dq = dQ_part + r * p->D;
        for (int d = 0; d < p->D; ++d) dq[d] = 0.0;
        if (L[r] == -INFINITY) continue;
        const float *qi = q_row(p, q, b, hq, i);
        const float *doi = q_row(p, dO, b, hq, i);
        for (int j = kv0; j < kv1; ++j) {
            if (!visible(p, b, i, j)) continue;
            const float *kj = kv_row(p, k, b, hk, j);
            const double pij = exp(p->scale * dot_fd(qi, kj, p->D) - L[r]);
            const double dS = pij * (dot_fd(doi, kv_row(p, v, b, hk, j), p->D) - delta[r]);
            for (int d = 0; d < p->D; ++d) dq[d] += dS * (double)kj[d];
        }
        for (int d = 0; d < p->D; ++d) dq[d] *= p->scale;
    }
    const long kvrows = (long)p->B * p->Hkv * nb;
#pragma omp parallel for schedule(dynamic, 16)
    for (long r = 0; r < kvrows; ++r) {
        const int j = kv0 + (int)(r % nb);
        const int hk = (int)((r / nb) % p->Hkv);
        const int b = (int)(r / ((long)nb * p->Hkv));
        const float *kj = kv_row(p, k, b, hk, j);
        const float *vj = kv_row(p, v, b, hk, j);
        double *dk = dK_blk + r * p->D, *dv = dV_blk + r * p->D;
        for (int d = 0; d < p->D; ++d) { dk[d] = 0.0; dv[d] = 0.0; }
        for (int hq = hk * G; hq < (hk + 1) * G; ++hq) {
            for (int i = 0; i < p->Sq; ++i) {
                if (!visible(p, b, i, j)) continue;
                const long qr = ((long)b * p->Hq + hq) * p->Sq + i;
                if (L[qr] == -INFINITY) continue;
                const float *qi = q_row(p, q, b, hq, i);
                const float *doi = q_row(p, dO, b, hq, i);
                const double pij = exp(p->scale * dot_fd(qi, kj, p->D) - L[qr]);
                const double dS = pij * (dot_fd(doi, vj, p->D) - delta[qr]);
                for (int d = 0; d < p->D; ++d) {
                    dv[d] += pij * (double)doi[d];
                    dk[d] += dS * (double)qi[d];
                }
            }
        }
        for (int d = 0; d < p->D; ++d) dk[d] *= p->scale;
    }
    free(delta);
}

/* ---------------------------------------------------------------------------
 * Projection (Section 2: Q = x W_Q, K = y W_K, V = y W_V; Section 3.2: done
 * again in the backward pass).  x is [B, S, E]; w holds W TRANSPOSED, one row
 * of E weights per output column, [H * D, E] (the way a linear layer stores
 * it); column h * D + c of the product is element c of head h:
 *     out[b, h, s, c] = sum_e x[b, s, e] * w[h * D + c, e].
 * rows == NULL: every token, out is [B, H, S, D].  Otherwise rows holds n_rows
 * pairs (b, s) and out is [n_rows, H, D].
 * ------------------------------------------------------------------------- */
void lvx_oracle_project(int B, int S, int E, int H, int D, const float *x, const float *w,
                        int n_rows, const int32_t *rows, double *out)
{
    const long n = rows ? n_rows : (long)B * S;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < n; ++r) {
        const int b = rows ? rows[2 * r] : (int)(r / S);
        const int s = rows ? rows[2 * r + 1] : (int)(r % S);
        const float *xr = x + ((long)b * S + s) * E;
        for (int h = 0; h < H; ++h)
            for (int c = 0; c < D; ++c) {
                const float *wr = w + ((long)h * D + c) * E;
                double acc = 0.0;
                for (int e = 0; e < E; ++e)
                    acc += (double)xr[e] * (double)wr[e];
                if (rows)
                    out[(r * H + h) * D + c] = acc;
                else
                    out[(((long)b * H + h) * S + s) * D + c] = acc;
            }
    }
}

/* ---------------------------------------------------------------------------
 * Gradients of the projection.  Section 3.2 has the backward pass form K and V
 * again from the saved visual tokens; what it then owes the rest of the network
 * is the chain rule through out = project(x, w) (Section 2's linear maps):
 * with g = d loss / d out, [B, H, S, D] like out,
 *     dw[h * D + c, e] = sum_{b, s} g[b, h, s, c] * x[b, s, e]
 *     dx[b, s, e]      = sum_{h, c} g[b, h, s, c] * w[h * D + c, e].
 * One double-precision sum per element, in the order written.
 * cols == NULL: every row of dw, [H * D, E]; otherwise cols lists n_cols output
 * columns n = h * D + c and dw is [n_cols, E].
 * rows == NULL: every token, dx is [B, S, E]; otherwise rows holds n_rows pairs
 * (b, s) and dx is [n_rows, E].
 * ------------------------------------------------------------------------- */
void lvx_oracle_project_bwd_w(int B, int S, int E, int H, int D, const float *x, const float *g,
                              int n_cols, const int32_t *cols, double *dw)
{
    const long n = cols ? n_cols : (long)H * D;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < n; ++r) {
        const int col = cols ? cols[r] : (int)r;
        const int h = col / D, c = col % D;
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int b = 0; b < B; ++b)
                for (int s = 0; s < S; ++s)
                    acc += (double)g[(((long)b * H + h) * S + s) * D + c] *
                           (double)x[((long)b * S + s) * E + e];
            dw[r * E + e] = acc;
        }
    }
}

void lvx_oracle_project_bwd_x(int B, int S, int E, int H, int D, const float *w, const float *g,
                              int n_rows, const int32_t *rows, double *dx)
{
    const long n = rows ? n_rows : (long)B * S;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < n; ++r) {
        const int b = rows ? rows[2 * r] : (int)(r / S);
        const int s = rows ? rows[2 * r + 1] : (int)(r % S);
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                for (int c = 0; c < D; ++c)
                    acc += (double)g[(((long)b * H + h) * S + s) * D + c] *
                           (double)w[((long)h * D + c) * E + e];
            dx[r * E + e] = acc;
        }
    }
}
