/*
 * CPU oracle for the SVG2 per-layer sparse-attention path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision implementation of what the path computes,
 * written from the paper's definitions, one head at a time.  It shares no code
 * with the HIP library and must never be called from the product path: only
 * tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 *   dense attention            Section 3.1 (O = softmax(Q K^T / sqrt(d)) V)
 *   k-means (Lloyd)            Section 4.1 (independent per head, Q and K)
 *   permutation                Section 4.1 (pi_q, pi_k make clusters contiguous)
 *   centroid scores + top-p    Section 4.2, Eq. 1 and Eq. 2, top-p rule
 *   block-sparse attention     Section 4.3 with the equivalence of Section 4.1
 *   density                    Section 5.1 "Metrics"
 *   attention recall           Section 3.1 (attention mass the selected keys capture)
 *   k-means++ seeding          Section 4.3 / 5.3 (the initialisation the paper starts from)
 *   FP8 E4M3 quantisation      Table 1, "+ FP8" rows (per-head scaling: a reading, the paper gives no recipe)
 *   rounded-weights budget     error bound of a weighted mean whose weights are rounded (tests of the FP8 path)
 *
 * Inputs are float arrays (bf16 workloads pass bf16-representable floats, so
 * reading them is exact); every sum is accumulated in double.  OpenMP is used
 * only over independent rows / tokens; there is no blocking or fusion.
 *
 * Readings of the paper where it is silent (kept in step with the HIP path's
 * header): squared Euclidean distance, one iteration = assign then update,
 * empty cluster keeps its centroid, argmin ties go to the lowest index, stable
 * order inside a cluster, top-p keeps the element that crosses p, ties in P'
 * go to the lower index, zero-size key clusters are never selected, softmax is
 * renormalised over the selected keys only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- bfloat16 rounding of a double (round to nearest, ties to even) ---- */
static double round_bf16(double v)
{
    if (v == 0.0 || !isfinite(v)) return v;
    int e;
    double m = frexp(v, &e);            /* v = m * 2^e, 0.5 <= |m| < 1 */
    /* bf16 keeps 8 significant bits: scale so that one ulp is 1.0 */
    double scaled = ldexp(m, 8);        /* 128 <= |scaled| < 256 */
    double r = nearbyint(scaled);       /* default rounding mode: ties to even */
    return ldexp(r, e - 8);
}

/* ------------------------------------------------------------------------
 * Dense attention, Section 3.1.  Q [Nq,d], K [Nk,d], V [Nk,d] -> O [Nq,d],
 * lse [Nq] (natural-log sum of exp of the scaled scores), either may be NULL.
 * ------------------------------------------------------------------------ */
void svg2o_dense_attention(const float *Q, const float *K, const float *V,
                           int Nq, int Nk, int d, double scale,
                           double *O, double *lse)
{
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(Nk > 0 ? Nk : 1));
#pragma omp for schedule(dynamic, 16)
        for (int n = 0; n < Nq; ++n) {
            const float *q = Q + (size_t)n * d;
            double mx = -INFINITY;
            for (int m = 0; m < Nk; ++m) {
                const float *k = K + (size_t)m * d;
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += (double)q[c] * (double)k[c];
                s[m] = acc * scale;
                if (s[m] > mx) mx = s[m];
            }
            double den = 0.0;
            for (int m = 0; m < Nk; ++m) { s[m] = exp(s[m] - mx); den += s[m]; }
            if (O) {
                double *o = O + (size_t)n * d;
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int m = 0; m < Nk; ++m) {
                    const float *v = V + (size_t)m * d;
                    double p = s[m] / den;
                    for (int c = 0; c < d; ++c) o[c] += p * (double)v[c];
                }
            }
            if (lse) lse[n] = (Nk > 0) ? mx + log(den) : -INFINITY;
        }
        free(s);
    }
}

/* ------------------------------------------------------------------------
 * k-means, Section 4.1.  X [N,d]; init [C,d]; T >= 1 iterations of
 * (assign, update).  round_bf16_centroids != 0: the assign step sees the
 * centroids rounded to bfloat16 (the storage type of X), the update step and
 * the returned centroids stay unrounded means.
 * Outputs: centroids [C,d] (means of the returned labels; an empty cluster
 * keeps its previous centroid), labels [N], counts [C], and if non-NULL
 * objective [2*T]: objective[2t] = sum of squared distances right after
 * assign t (to the centroids that assign used), objective[2t+1] = the same
 * sum right after update t (to the new means).
 * ------------------------------------------------------------------------ */
void svg2o_kmeans(const float *X, int N, int d, int C, int T,
                  int round_bf16_centroids, const double *init,
                  double *centroids, int32_t *labels, int32_t *counts,
                  double *objective)
{
    double *c = centroids;
    if (c != init) memcpy(c, init, sizeof(double) * (size_t)C * d);
    double *cr = (double *)malloc(sizeof(double) * (size_t)C * d);
    double *cn = (double *)malloc(sizeof(double) * (size_t)C);
    double *sum = (double *)malloc(sizeof(double) * (size_t)C * d);

    for (int t = 0; t < T; ++t) {
        /* centroids as the assign step sees them, and their squared norms */
        for (size_t i = 0; i < (size_t)C * d; ++i)
            cr[i] = round_bf16_centroids ? round_bf16(c[i]) : c[i];
        for (int j = 0; j < C; ++j) {
            double a = 0.0;
            for (int k = 0; k < d; ++k) a += cr[(size_t)j * d + k] * cr[(size_t)j * d + k];
            cn[j] = a;
        }
        /* assign: argmin_j ||c_j||^2 - 2 x.c_j  (||x||^2 is common to all j) */
        double J = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : J)
        for (int n = 0; n < N; ++n) {
            const float *x = X + (size_t)n * d;
            double best = INFINITY;
            int bj = 0;
            for (int j = 0; j < C; ++j) {
                const double *cj = cr + (size_t)j * d;
                double dot = 0.0;
                for (int k = 0; k < d; ++k) dot += (double)x[k] * cj[k];
                double dist = cn[j] - 2.0 * dot;
                if (dist < best) { best = dist; bj = j; }
            }
            labels[n] = bj;
            double xx = 0.0;
            for (int k = 0; k < d; ++k) xx += (double)x[k] * (double)x[k];
            J += xx + best;
        }
        if (objective) objective[2 * t] = J;

        /* update: mean of each cluster's members, in token order */
        memset(sum, 0, sizeof(double) * (size_t)C * d);
        memset(counts, 0, sizeof(int32_t) * (size_t)C);
        for (int n = 0; n < N; ++n) {
            const float *x = X + (size_t)n * d;
            double *s = sum + (size_t)labels[n] * d;
            for (int k = 0; k < d; ++k) s[k] += (double)x[k];
            counts[labels[n]] += 1;
        }
        for (int j = 0; j < C; ++j) {
            if (counts[j] == 0) continue;            /* empty: keep previous centroid */
            for (int k = 0; k < d; ++k)
                c[(size_t)j * d + k] = sum[(size_t)j * d + k] / (double)counts[j];
        }
        if (objective) {
            double J2 = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : J2)
            for (int n = 0; n < N; ++n) {
                const float *x = X + (size_t)n * d;
                const double *cj = c + (size_t)labels[n] * d;
                double a = 0.0;
                for (int k = 0; k < d; ++k) { double e = (double)x[k] - cj[k]; a += e * e; }
                J2 += a;
            }
            objective[2 * t + 1] = J2;
        }
    }
    free(cr); free(cn); free(sum);
}

/* Relative gap between the two smallest full squared distances of each token
 * to the given centroids (as the assign step would see them): used by tests to
 * decide whether a label disagreement is a near-tie.  gap [N]. */
void svg2o_top2_gap(const float *X, int N, int d, int C, int round_bf16_centroids,
                    const double *centroids, double *gap)
{
    double *cr = (double *)malloc(sizeof(double) * (size_t)C * d);
    for (size_t i = 0; i < (size_t)C * d; ++i)
        cr[i] = round_bf16_centroids ? round_bf16(centroids[i]) : centroids[i];
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const float *x = X + (size_t)n * d;
        double d1 = INFINITY, d2 = INFINITY;
        for (int j = 0; j < C; ++j) {
            const double *cj = cr + (size_t)j * d;
            double a = 0.0;
            for (int k = 0; k < d; ++k) { double e = (double)x[k] - cj[k]; a += e * e; }
            if (a < d1) { d2 = d1; d1 = a; } else if (a < d2) { d2 = a; }
        }
        gap[n] = (C > 1) ? (d2 - d1) / fmax(fabs(d2), 1e-12) : INFINITY;
    }
    free(cr);
}

/* ------------------------------------------------------------------------
 * Permutation, Section 4.1.  labels [N] in [0,C) -> counts [C], offsets [C+1]
 * (exclusive scan), perm [N] (sorted position r holds original token perm[r];
 * clusters ascending, original order kept inside a cluster), inv_perm [N].
 * ------------------------------------------------------------------------ */
void svg2o_permute(const int32_t *labels, int N, int C,
                   int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm)
{
    memset(counts, 0, sizeof(int32_t) * (size_t)C);
    for (int n = 0; n < N; ++n) counts[labels[n]] += 1;
    offsets[0] = 0;
    for (int j = 0; j < C; ++j) offsets[j + 1] = offsets[j] + counts[j];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(C > 0 ? C : 1));
    memcpy(cursor, offsets, sizeof(int32_t) * (size_t)C);
    for (int n = 0; n < N; ++n) {
        int r = cursor[labels[n]]++;
        perm[r] = n;
        if (inv_perm) inv_perm[n] = r;
    }
    free(cursor);
}

/* X' [r] = X [perm[r]] : the product pi X of Section 4.1 for a row-index permutation. */
void svg2o_gather_rows(const float *X, const int32_t *perm, int N, int d, float *Xp)
{
    for (int r = 0; r < N; ++r)
        memcpy(Xp + (size_t)r * d, X + (size_t)perm[r] * d, sizeof(float) * (size_t)d);
}

/* ------------------------------------------------------------------------
 * Centroid scores and top-p selection, Section 4.2.
 *   S_ij  = cq_i . ck_j / sqrt(d)                                   (Eq. 1)
 *   P'_ij = |K_j| exp(S_ij) / sum_k |K_k| exp(S_ik)                 (Eq. 2)
 * For every query cluster i: key clusters in descending P' (ties: lower j
 * first); the element at sorted position t is kept iff the sum of the
 * elements before it is < p, so the one that crosses p is included.  p >= 1
 * keeps every non-empty key cluster.  Key clusters of size 0 are never kept;
 * a query cluster of size 0 (when counts_q is given) gets an empty row.
 * Outputs: row_ptr [Cq+1], col_idx [capacity Cq*Ck] ascending inside a row,
 * p_est [Cq,Ck] or NULL, margin [Cq] or NULL (how far the stopping decision
 * of the row is from flipping: min of |sum before last kept - p|, |sum
 * including last kept - p| and the relative P' gap between last kept and
 * first dropped), density (Section 5.1; needs counts_q, else NaN).
 * ------------------------------------------------------------------------ */
typedef struct { double p; int j; } svg2o_pj;

static int cmp_desc(const void *a, const void *b)
{
    const svg2o_pj *x = (const svg2o_pj *)a, *y = (const svg2o_pj *)b;
    if (x->p > y->p) return -1;
    if (x->p < y->p) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

void svg2o_select_topp(const double *cq, const double *ck,
                       const int32_t *counts_q, const int32_t *counts_k,
                       int Cq, int Ck, int d, double top_p,
                       int32_t *row_ptr, int32_t *col_idx,
                       double *p_est, double *margin, double *density)
{
    double *P = (double *)malloc(sizeof(double) * (size_t)Ck);
    svg2o_pj *ord = (svg2o_pj *)malloc(sizeof(svg2o_pj) * (size_t)Ck);
    char *keep = (char *)malloc((size_t)Ck);
    double inv_sqrt_d = 1.0 / sqrt((double)d);
    long long nq_total = 0, nk_total = 0;
    double work = 0.0;
    for (int j = 0; j < Ck; ++j) nk_total += counts_k[j];
    row_ptr[0] = 0;
    for (int i = 0; i < Cq; ++i) {
        /* Eq. 1 */
        double mx = -INFINITY;
        for (int j = 0; j < Ck; ++j) {
            double a = 0.0;
            for (int k = 0; k < d; ++k) a += cq[(size_t)i * d + k] * ck[(size_t)j * d + k];
            P[j] = a * inv_sqrt_d;
            if (counts_k[j] > 0 && P[j] > mx) mx = P[j];
        }
        /* Eq. 2, with the row maximum subtracted from S (cancels in the ratio) */
        double den = 0.0;
        for (int j = 0; j < Ck; ++j) {
            P[j] = (counts_k[j] > 0) ? (double)counts_k[j] * exp(P[j] - mx) : 0.0;
            den += P[j];
        }
        for (int j = 0; j < Ck; ++j) {
            P[j] = (den > 0.0) ? P[j] / den : 0.0;
            if (p_est) p_est[(size_t)i * Ck + j] = P[j];
        }
        /* top-p */
        memset(keep, 0, (size_t)Ck);
        double mg = INFINITY;
        int empty_row = (counts_q && counts_q[i] == 0);
        if (!empty_row) {
            if (top_p >= 1.0) {
                for (int j = 0; j < Ck; ++j) keep[j] = counts_k[j] > 0;
            } else {
                for (int j = 0; j < Ck; ++j) { ord[j].p = P[j]; ord[j].j = j; }
                qsort(ord, (size_t)Ck, sizeof(svg2o_pj), cmp_desc);
                double cum = 0.0, last = 0.0, first_dropped = -1.0;
                int n_kept = 0;
                for (int t = 0; t < Ck; ++t) {
                    int j = ord[t].j;
                    if (counts_k[j] == 0) continue;          /* never kept */
                    if (!(cum < top_p)) { first_dropped = ord[t].p; break; }
                    keep[j] = 1;
                    last = ord[t].p;
                    cum += last;
                    n_kept += 1;
                }
                if (n_kept > 0) {
                    double before = cum - last;
                    mg = fmin(fabs(before - top_p), fabs(cum - top_p));
                    if (first_dropped >= 0.0 && last > 0.0) mg = fmin(mg, (last - first_dropped) / last);
                }
            }
        }
        if (margin) margin[i] = mg;
        int nnz = row_ptr[i];
        long long keys = 0;
        for (int j = 0; j < Ck; ++j)
            if (keep[j]) { col_idx[nnz++] = j; keys += counts_k[j]; }
        row_ptr[i + 1] = nnz;
        if (counts_q) { nq_total += counts_q[i]; work += (double)counts_q[i] * (double)keys; }
    }
    if (density)
        *density = (counts_q && nq_total > 0 && nk_total > 0)
                       ? work / ((double)nq_total * (double)nk_total) : NAN;
    free(P); free(ord); free(keep);
}

/* ------------------------------------------------------------------------
 * Block-sparse attention over variable-size clusters, Section 4.3.
 * Qp, Kp, Vp are the permuted tensors (clusters contiguous; cluster i of Q is
 * rows offsets_q[i]..offsets_q[i+1]).  Every row of query cluster i attends,
 * with an ordinary softmax, over exactly the keys of its selected key
 * clusters.  perm_q != NULL: the result of permuted row r is written to
 * original row perm_q[r] (pi_q^T of Section 4.1); else it stays at r.
 * rows != NULL: only the n_rows permuted rows listed are computed (the rest
 * of O is left untouched) -- rows are independent, so a sample is exact.
 * A row with no selected key gets O = 0, lse = -inf.
 * ------------------------------------------------------------------------ */
void svg2o_sparse_attention(const float *Qp, const float *Kp, const float *Vp,
                            int N, int d, int Cq, int Ck,
                            const int32_t *offsets_q, const int32_t *offsets_k,
                            const int32_t *row_ptr, const int32_t *col_idx,
                            const int32_t *perm_q, double scale,
                            const int32_t *rows, int n_rows,
                            double *O, double *lse)
{
    (void)Ck;
    int total = rows ? n_rows : N;
    /* cluster of every permuted query row */
    int32_t *cl = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    for (int i = 0; i < Cq; ++i)
        for (int r = offsets_q[i]; r < offsets_q[i + 1]; ++r) cl[r] = i;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        double *acc = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 8)
        for (int t = 0; t < total; ++t) {
            int r = rows ? rows[t] : t;
            int i = cl[r];
            const float *q = Qp + (size_t)r * d;
            int cnt = 0;
            double mx = -INFINITY;
            for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
                int j = col_idx[e];
                for (int m = offsets_k[j]; m < offsets_k[j + 1]; ++m) {
                    const float *k = Kp + (size_t)m * d;
                    double a = 0.0;
                    for (int c = 0; c < d; ++c) a += (double)q[c] * (double)k[c];
                    a *= scale;
                    s[cnt++] = a;
                    if (a > mx) mx = a;
                }
            }
            double den = 0.0;
            for (int u = 0; u < cnt; ++u) { s[u] = exp(s[u] - mx); den += s[u]; }
            for (int c = 0; c < d; ++c) acc[c] = 0.0;
            cnt = 0;
            for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
                int j = col_idx[e];
                for (int m = offsets_k[j]; m < offsets_k[j + 1]; ++m) {
                    const float *v = Vp + (size_t)m * d;
                    double p = s[cnt++] / den;
                    for (int c = 0; c < d; ++c) acc[c] += p * (double)v[c];
                }
            }
            size_t dst = (size_t)(perm_q ? perm_q[r] : r);
            if (O) for (int c = 0; c < d; ++c) O[dst * d + c] = (cnt > 0) ? acc[c] : 0.0;
            if (lse) lse[dst] = (cnt > 0) ? mx + log(den) : -INFINITY;
        }
        free(s); free(acc);
    }
    free(cl);
}

/* ------------------------------------------------------------------------
 * Error budget of block-sparse attention whose probabilities are ROUNDED
 * before they multiply V (the "+ FP8" rows of Table 1 under this build's
 * reading: probabilities enter the second product as E4M3).  This is a bound
 * calculator for tests, derived from the mathematics of a weighted mean, not a
 * model of any kernel's blocking or order.
 *
 * For one query row with exact probabilities pi_j (softmax over the selected
 * keys, Section 4.3), values v_jc and exact output O_c = sum_j pi_j v_jc:
 * if every weight is replaced by w_j = pi_j (1 + e_j) and the result is
 * renormalised by sum_j w_j (the row sum is taken over the rounded weights),
 *     O'_c - O_c = sum_j pi_j e_j (v_jc - O_c) / (1 + sum_j pi_j e_j).
 * Hence, with |e_j| <= eps for every key,
 *     |O'_c - O_c| <= eps / (1 - eps) * dev1[c],  dev1[c] = sum_j pi_j |v_jc - O_c|,
 * and if the e_j are independent and uniform in [-eps, eps] the error has
 * standard deviation  eps / sqrt(3) * sqrt(dev2[c]),  dev2[c] = sum_j pi_j^2 (v_jc - O_c)^2.
 * Weights far below the row maximum may be rounded with an ABSOLUTE rather
 * than a relative error (subnormal range of the 8-bit format, flush to zero):
 * for a key with pi_j < tail_ratio * pi_max (pi_max = max_j pi_j) the weight
 * error is at most a_j = min(pi_j, tail_abs * pi_max) on top of the relative
 * one -- min(pi_j, .) because a weight cannot lose more than itself.  For those
 *     tail1[c] = sum_tail a_j |v_jc - O_c|,  tail2[c] = sum_tail a_j^2 (v_jc - O_c)^2,
 *     tailw    = sum_tail a_j   (what the row sum can be off by, relative to itself),
 * and the bound becomes (eps dev1[c] + tail1[c]) / (1 - eps - tailw).
 *
 * Same arguments as svg2o_sparse_attention; rows != NULL restricts the rows.
 * Outputs, indexed like O (original row if perm_q is given), untouched for
 * rows not computed: dev1, dev2, tail1, tail2 [N,d] and tailw [N].
 * ------------------------------------------------------------------------ */
void svg2o_rounded_weights_budget(const float *Qp, const float *Kp, const float *Vp,
                                  int N, int d, int Cq, int Ck,
                                  const int32_t *offsets_q, const int32_t *offsets_k,
                                  const int32_t *row_ptr, const int32_t *col_idx,
                                  const int32_t *perm_q, double scale, double tail_ratio, double tail_abs,
                                  const int32_t *rows, int n_rows,
                                  double *dev1, double *dev2, double *tail1, double *tail2, double *tailw)
{
    (void)Ck;
    int total = rows ? n_rows : N;
    int32_t *cl = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    for (int i = 0; i < Cq; ++i)
        for (int r = offsets_q[i]; r < offsets_q[i + 1]; ++r) cl[r] = i;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 8)
        for (int t = 0; t < total; ++t) {
            int r = rows ? rows[t] : t;
            int i = cl[r];
            const float *q = Qp + (size_t)r * d;
            int cnt = 0;
            double mx = -INFINITY;
            for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
                int j = col_idx[e];
                for (int m = offsets_k[j]; m < offsets_k[j + 1]; ++m) {
                    const float *k = Kp + (size_t)m * d;
                    double a = 0.0;
                    for (int c = 0; c < d; ++c) a += (double)q[c] * (double)k[c];
                    a *= scale;
                    s[cnt++] = a;
                    if (a > mx) mx = a;
                }
            }
            /* exact probabilities and exact output */
            double den = 0.0;
            for (int u = 0; u < cnt; ++u) { s[u] = exp(s[u] - mx); den += s[u]; }
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            cnt = 0;
            for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
                int j = col_idx[e];
                for (int m = offsets_k[j]; m < offsets_k[j + 1]; ++m) {
                    const float *v = Vp + (size_t)m * d;
                    s[cnt] /= den;                       /* pi_j; the largest is 1 / den */
                    for (int c = 0; c < d; ++c) o[c] += s[cnt] * (double)v[c];
                    cnt += 1;
                }
            }
            size_t dst = (size_t)(perm_q ? perm_q[r] : r);
            double *a1 = dev1 + dst * d, *a2 = dev2 + dst * d, *b1 = tail1 + dst * d, *b2 = tail2 + dst * d;
            for (int c = 0; c < d; ++c) a1[c] = a2[c] = b1[c] = b2[c] = 0.0;
            double pmax = (cnt > 0) ? 1.0 / den : 0.0;      /* the largest exp(s - mx) is 1 */
            double tw = 0.0;
            cnt = 0;
            for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
                int j = col_idx[e];
                for (int m = offsets_k[j]; m < offsets_k[j + 1]; ++m) {
                    const float *v = Vp + (size_t)m * d;
                    double p = s[cnt++];
                    int in_tail = p < tail_ratio * pmax;
                    double a = fmin(p, tail_abs * pmax);
                    if (in_tail) tw += a;
                    for (int c = 0; c < d; ++c) {
                        double dv = fabs((double)v[c] - o[c]);
                        a1[c] += p * dv;
                        a2[c] += p * p * dv * dv;
                        if (in_tail) { b1[c] += a * dv; b2[c] += a * a * dv * dv; }
                    }
                }
            }
            tailw[dst] = tw;
        }
        free(s); free(o);
    }
    free(cl);
}

/* Accounting helper for the paper's padding example (Section 4.3): the share
 * of a fixed bm x bn tile that is padding when it holds a rows x cols block. */
double svg2o_padding_waste(int rows, int cols, int bm, int bn)
{
    long long tiles_r = (rows + bm - 1) / bm, tiles_c = (cols + bn - 1) / bn;
    double padded = (double)(tiles_r * bm) * (double)(tiles_c * bn);
    return padded > 0.0 ? 1.0 - ((double)rows * (double)cols) / padded : 0.0;
}

/* ------------------------------------------------------------------------
 * Attention recall, Section 3.1: for a query, the sum of the true attention
 * scores (the softmax over ALL keys) of the keys that are computed.  Here the
 * computed keys of query n are the keys whose cluster is selected for the
 * cluster of n (Section 4.2).  Q, K [N,d] in ORIGINAL token order, labels_q,
 * labels_k [N]; row_ptr / col_idx the CSR list of selected key clusters per
 * query cluster.  rows != NULL: only those n_rows tokens are filled.
 * ------------------------------------------------------------------------ */
void svg2o_attention_recall(const float *Q, const float *K, int N, int d,
                            const int32_t *labels_q, const int32_t *labels_k, int Cq, int Ck,
                            const int32_t *row_ptr, const int32_t *col_idx, double scale,
                            const int32_t *rows, int n_rows, double *recall)
{
    int total = rows ? n_rows : N;
    /* selected[i * Ck + j] = 1 if key cluster j is selected for query cluster i */
    unsigned char *selected = (unsigned char *)calloc((size_t)Cq * (size_t)Ck, 1);
    for (int i = 0; i < Cq; ++i)
        for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) selected[(size_t)i * Ck + col_idx[e]] = 1;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
#pragma omp for schedule(dynamic, 8)
        for (int t = 0; t < total; ++t) {
            int n = rows ? rows[t] : t;
            const float *q = Q + (size_t)n * d;
            double mx = -INFINITY;
            for (int m = 0; m < N; ++m) {
                const float *k = K + (size_t)m * d;
                double a = 0.0;
                for (int c = 0; c < d; ++c) a += (double)q[c] * (double)k[c];
                s[m] = a * scale;
                if (s[m] > mx) mx = s[m];
            }
            double den = 0.0, kept = 0.0;
            const unsigned char *sel_row = selected + (size_t)labels_q[n] * Ck;
            for (int m = 0; m < N; ++m) {
                double p = exp(s[m] - mx);
                den += p;
                if (sel_row[labels_k[m]]) kept += p;
            }
            recall[n] = kept / den;
        }
        free(s);
    }
    free(selected);
}

/* ------------------------------------------------------------------------
 * k-means++ seeding (the initialisation the paper's un-cached k-means starts
 * from, Section 4.3; Arthur & Vassilvitskii's D^2 sampling).  The random
 * numbers are inputs: u[C] uniform in [0,1).
 *   centre 0      token floor(u[0] * N)
 *   centre k >= 1 with D2[n] = min over the centres chosen so far of
 *                 ||x_n - c||^2: the first token whose running sum of D2
 *                 exceeds u[k] * sum(D2) (so a token is drawn with probability
 *                 D2[n] / sum(D2)); if every D2 is zero, token floor(u[k] * N).
 * picked[C] receives the token indices; the centres are those rows of X.
 * ------------------------------------------------------------------------ */
void svg2o_kmeans_pp(const float *X, int N, int d, int C, const double *u, int32_t *picked)
{
    double *d2 = (double *)malloc(sizeof(double) * (size_t)N);
    for (int n = 0; n < N; ++n) d2[n] = INFINITY;
    for (int k = 0; k < C; ++k) {
        int pick;
        if (k == 0) {
            pick = (int)floor(u[0] * (double)N);
        } else {
            double total = 0.0;
            for (int n = 0; n < N; ++n) total += d2[n];
            if (total > 0.0) {
                double target = u[k] * total, run = 0.0;
                pick = -1;
                for (int n = 0; n < N; ++n) {
                    run += d2[n];
                    if (run > target) { pick = n; break; }
                }
                if (pick < 0) {             /* rounding left the running sum at the target: last token with D2 > 0 */
                    for (int n = N - 1; n >= 0; --n)
                        if (d2[n] > 0.0) { pick = n; break; }
                }
            } else {
                pick = (int)floor(u[k] * (double)N);
            }
        }
        if (pick < 0) pick = 0;
        if (pick > N - 1) pick = N - 1;
        picked[k] = pick;
        const float *c = X + (size_t)pick * d;
#pragma omp parallel for schedule(static)
        for (int n = 0; n < N; ++n) {
            const float *x = X + (size_t)n * d;
            double a = 0.0;
            for (int j = 0; j < d; ++j) {
                double t = (double)x[j] - (double)c[j];
                a += t * t;
            }
            if (a < d2[n]) d2[n] = a;
        }
    }
    free(d2);
}

/* ------------------------------------------------------------------------
 * FP8 storage for the attention operands (the "+ FP8" rows of Table 1; the
 * paper does not say how the operands are quantised, so this is a reading):
 * OCP 8-bit floating point E4M3 -- 1 sign bit, 4 exponent bits with bias 7,
 * 3 mantissa bits, subnormals below 2^-6, no infinities, S.1111.111 is NaN,
 * largest finite value 448 -- with one scale per head and tensor,
 *     amax  = max |x| over the head's [N, d] block
 *     inv   = 448 / amax          (single precision; 1 when amax is 0)
 *     code  = E4M3(x * inv)       (single-precision product, round to
 *                                  nearest, ties to even, clamped to +-448)
 *     scale = amax / 448          (single precision; 1 when amax is 0)
 * so that x ~ decode(code) * scale.  The products are taken in single
 * precision on purpose: a rounding decision has to be taken in the same
 * precision by whoever is compared with this.
 * ------------------------------------------------------------------------ */

/* nearest E4M3 value of y (ties to even mantissa), clamped to +-448 */
double svg2o_round_e4m3(double y)
{
    if (y == 0.0 || isnan(y)) return y;
    double a = fabs(y);
    if (a >= 448.0) return copysign(448.0, y);
    double q;                               /* spacing of the representable values around a */
    if (a < ldexp(1.0, -6)) {
        q = ldexp(1.0, -9);                 /* subnormal range */
    } else {
        int e;
        (void)frexp(a, &e);                 /* a = m * 2^e, 0.5 <= m < 1: a in [2^(e-1), 2^e) */
        q = ldexp(1.0, e - 1 - 3);          /* 3 mantissa bits */
    }
    double r = nearbyint(a / q) * q;        /* default rounding mode: ties to even */
    if (r > 448.0) r = 448.0;
    return copysign(r, y);
}

/* the 8-bit code of an E4M3 value v (as returned by svg2o_round_e4m3) */
uint8_t svg2o_encode_e4m3(double v)
{
    uint8_t s = signbit(v) ? 0x80 : 0x00;
    double a = fabs(v);
    if (a == 0.0) return s;
    if (a < ldexp(1.0, -6)) return (uint8_t)(s | (uint8_t)lrint(a * 512.0));      /* exponent field 0 */
    int e;
    double m = frexp(a, &e);                /* a = (2m) * 2^(e-1), 1 <= 2m < 2 */
    int field = e - 1 + 7;
    int mant = (int)lrint((2.0 * m - 1.0) * 8.0);
    return (uint8_t)(s | (field << 3) | mant);
}

/* X [n] floats of one head and tensor -> codes [n], decoded [n] (= decode(code), unscaled), *scale */
void svg2o_quantize_e4m3(const float *X, long n, uint8_t *codes, float *decoded, float *scale)
{
    float amax = 0.0f;
    for (long i = 0; i < n; ++i) {
        float a = fabsf(X[i]);
        if (a > amax) amax = a;
    }
    volatile float inv = (amax > 0.0f) ? 448.0f / amax : 1.0f;
    volatile float sc = (amax > 0.0f) ? amax / 448.0f : 1.0f;
    for (long i = 0; i < n; ++i) {
        volatile float y = X[i] * inv;      /* single-precision product, no contraction */
        double r = svg2o_round_e4m3((double)y);
        if (codes) codes[i] = svg2o_encode_e4m3(r);
        if (decoded) decoded[i] = (float)r;
    }
    *scale = sc;
}
