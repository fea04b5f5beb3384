/*
 * CPU oracle for the VLQ-ADC build and query definitions.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against; nothing on the product path may link, load
 * or call it.  It shares no code with the HIP kernels.
 *
 * Everything is computed from the definitions, in fp64, with one loop per
 * index of the formula: squared distances are sums of squared differences,
 * candidates are scored by reconstructing the approximated point and taking
 * its distance to the query.  No lookup tables, no blocking, no fusion.
 * OpenMP only splits the outermost loop over points / queries / centroids.
 *
 * Notation follows the paper (Table 1): D dimension, k first-level centroids,
 * n graph edges per centroid, m PQ sub-spaces of 256 codewords, w1 probed
 * cells, w2 visited sub-regions, K results.
 *
 * Pins (tests/test_oracle_*.py): Eq. 7 against the direct point-to-anchor
 * distance, Eq. 8 closed forms, the term-by-term decomposition of Eq. 16-17,
 * exhaustive probing against brute force over reconstructions, lambda == 0
 * against an independent IVFADC, exactly representable data against exact
 * k-NN, brute-force enumeration of the encoder's choices on tiny inputs,
 * lambda range / anchor-error invariants, and the memory figures of Sec. 3.1.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- helpers -------------------------------------------------------- */

/* ||a - b||^2 written out (Eq. 1's summand). */
static double sqdist_ff(const float *a, const float *b, int D)
{
    double s = 0.0;
    for (int d = 0; d < D; ++d) {
        double t = (double)a[d] - (double)b[d];
        s += t * t;
    }
    return s;
}

int vlqo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void vlqo_set_num_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* lambda byte grid (Sec. 3.2, last paragraph: lambda is stored as one of 256
 * values; the paper does not give the grid, this build uses a uniform one on
 * [lo, hi] whose code z represents 0 exactly). */
static double grid_step(double lo, double hi) { return (hi - lo) / 255.0; }
static double grid_zero(double lo, double hi) { return -rint(lo / grid_step(lo, hi)); }

double vlqo_lambda_dequant(int q, double lo, double hi)
{
    return ((double)q - grid_zero(lo, hi)) * grid_step(lo, hi);
}

/* real-valued grid coordinate of lambda before rounding */
double vlqo_lambda_coord(double lambda, double lo, double hi)
{
    return lambda / grid_step(lo, hi) + grid_zero(lo, hi);
}

int vlqo_lambda_quant(double lambda, double lo, double hi)
{
    double q = rint(lambda / grid_step(lo, hi)) + grid_zero(lo, hi); /* half-even */
    if (q < 0.0) q = 0.0;
    if (q > 255.0) q = 255.0;
    return (int)q;
}

/* Eq. 8: parameter of the foot of the perpendicular from x on the line through
 * c_i (lambda = 0) and c_j (lambda = 1); a = ||x-c_i||^2, b = ||x-c_j||^2,
 * c = ||c_j-c_i||^2.  A zero-length line (duplicate centroids) has lambda 0. */
double vlqo_line_lambda(double a, double b, double c)
{
    if (c <= 0.0) return 0.0;
    return 0.5 * (a + c - b) / c;
}

/* Eq. 7: squared distance from x to the point (1-lambda) c_i + lambda c_j. */
double vlqo_line_dist2(double a, double b, double c, double lambda)
{
    return (1.0 - lambda) * a + (lambda * lambda - lambda) * c + lambda * b;
}

/* ---- n-NN graph (Sec. 3.1; Alg. 1, graph step) ---------------------- */

typedef struct { double d; int32_t j; } dj_t;

static int cmp_dj(const void *pa, const void *pb)
{
    const dj_t *a = (const dj_t *)pa, *b = (const dj_t *)pb;
    if (a->d < b->d) return -1;
    if (a->d > b->d) return 1;
    return (a->j > b->j) - (a->j < b->j);
}

/* For every centroid i listed in rows[0..nrows): S[r][0..n) = the n other
 * centroids closest to c_i, ascending by (distance, index); E[r][.] = their
 * squared distances.  rows == NULL means rows = 0..k-1 (then nrows = k). */
void vlqo_graph_rows(const float *C, int k, int D, int n,
                     const int32_t *rows, int nrows, int32_t *S, double *E)
{
#pragma omp parallel
    {
        dj_t *buf = (dj_t *)malloc((size_t)k * sizeof(dj_t));
#pragma omp for schedule(dynamic, 4)
        for (int r = 0; r < nrows; ++r) {
            int i = rows ? rows[r] : r;
            int cnt = 0;
            for (int j = 0; j < k; ++j) {
                if (j == i) continue; /* a line needs two different centroids (Sec. 2.3) */
                buf[cnt].d = sqdist_ff(C + (size_t)i * D, C + (size_t)j * D, D);
                buf[cnt].j = j;
                ++cnt;
            }
            qsort(buf, (size_t)cnt, sizeof(dj_t), cmp_dj);
            for (int e = 0; e < n; ++e) {
                S[(size_t)r * n + e] = buf[e].j;
                E[(size_t)r * n + e] = buf[e].d;
            }
        }
        free(buf);
    }
}

/* ---- encoding (Alg. 1 + Alg. 2) ------------------------------------- */

/*
 * Per point x_t:
 *   VQ   (Eq. 2)        i  = argmin_i ||x - c_i||^2                 ties -> smaller i
 *   LQ   (Alg. 1, Eq.7) j  = argmin_j d(x, l(c_i, s_ij))^2 at the   ties -> smaller j
 *                            line's own lambda (Eq. 8)
 *   lambda byte          q  = nearest grid code of lambda_ij (Eq. 13)
 *   residual (Eq. 12)   r  = x - ((1-lh) c_i + lh s_ij), lh = grid value of q
 *   PQ   (Alg. 2)       t_p = argmin_t ||r^p - P[p][t]||^2           ties -> smaller t
 *
 * S, E: full graph [k x n].  P: [m][256][D/m].
 * Optional diagnostics (may be NULL), used by the parity tests to recognise
 * near-ties: cell_d[t][2], edge_d[t][2] = best and second-best objective;
 * lam_coord[t] = unrounded grid coordinate; code_d[t][m][2].
 */
void vlqo_encode(const float *C, int k, int D, int n, const int32_t *S, const double *E,
                 const float *P, int m, double lo, double hi,
                 const float *X, int64_t N,
                 int32_t *cell, int32_t *edge, uint8_t *lamq, uint8_t *codes,
                 double *cell_d, double *edge_d, double *lam_coord, double *code_d)
{
    const int ds = D / m;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N; ++t) {
        const float *x = X + (size_t)t * D;

        /* VQ */
        int bi = -1;
        double best = INFINITY, second = INFINITY;
        for (int i = 0; i < k; ++i) {
            double d = sqdist_ff(x, C + (size_t)i * D, D);
            if (d < best) { second = best; best = d; bi = i; }
            else if (d < second) second = d;
        }
        cell[t] = bi;
        if (cell_d) { cell_d[2 * t] = best; cell_d[2 * t + 1] = second; }
        const double a = best;
        const float *ci = C + (size_t)bi * D;

        /* LQ */
        int bj = -1;
        double bestl = INFINITY, secondl = INFINITY, blam = 0.0;
        for (int j = 0; j < n; ++j) {
            const float *sj = C + (size_t)S[(size_t)bi * n + j] * D;
            double b = sqdist_ff(x, sj, D);
            double c = E[(size_t)bi * n + j];
            double lam = vlqo_line_lambda(a, b, c);
            double d2 = vlqo_line_dist2(a, b, c, lam);
            if (d2 < bestl) { secondl = bestl; bestl = d2; bj = j; blam = lam; }
            else if (d2 < secondl) secondl = d2;
        }
        edge[t] = bj;
        if (edge_d) { edge_d[2 * t] = bestl; edge_d[2 * t + 1] = secondl; }

        /* lambda byte */
        int q = vlqo_lambda_quant(blam, lo, hi);
        lamq[t] = (uint8_t)q;
        if (lam_coord) lam_coord[t] = vlqo_lambda_coord(blam, lo, hi);
        const double lh = vlqo_lambda_dequant(q, lo, hi);

        /* residual w.r.t. the anchor that the byte reproduces, then PQ */
        const float *sj = C + (size_t)S[(size_t)bi * n + bj] * D;
        for (int p = 0; p < m; ++p) {
            int bt = -1;
            double bp = INFINITY, sp = INFINITY;
            for (int c = 0; c < 256; ++c) {
                const float *w = P + ((size_t)p * 256 + c) * ds;
                double s = 0.0;
                for (int d = 0; d < ds; ++d) {
                    int g = p * ds + d;
                    double anchor = (1.0 - lh) * (double)ci[g] + lh * (double)sj[g];
                    double r = (double)x[g] - anchor;
                    double u = r - (double)w[d];
                    s += u * u;
                }
                if (s < bp) { sp = bp; bp = s; bt = c; }
                else if (s < sp) sp = s;
            }
            codes[(size_t)t * m + p] = (uint8_t)bt;
            if (code_d) {
                code_d[((size_t)t * m + p) * 2] = bp;
                code_d[((size_t)t * m + p) * 2 + 1] = sp;
            }
        }
    }
}

/* Eq. 2 alone: nearest centroid of every x_t (ties -> smaller index); cell_d
 * (optional) receives the best and second-best squared distance. */
void vlqo_vq_assign(const float *C, int k, int D, const float *X, int64_t N,
                    int32_t *cell, double *cell_d)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N; ++t) {
        int bi = -1;
        double best = INFINITY, second = INFINITY;
        for (int i = 0; i < k; ++i) {
            double d = sqdist_ff(X + (size_t)t * D, C + (size_t)i * D, D);
            if (d < best) { second = best; best = d; bi = i; }
            else if (d < second) second = d;
        }
        cell[t] = bi;
        if (cell_d) { cell_d[2 * t] = best; cell_d[2 * t + 1] = second; }
    }
}

/* Reconstruction q_1(x) + q_2(x - q_1(x)) of Eq. 14 from the stored fields. */
void vlqo_reconstruct(const float *C, int D, int n, const int32_t *S,
                      const float *P, int m, double lo, double hi,
                      const int32_t *cell, const int32_t *edge, const uint8_t *lamq,
                      const uint8_t *codes, int64_t N, double *Xhat)
{
    const int ds = D / m;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N; ++t) {
        const float *ci = C + (size_t)cell[t] * D;
        const float *sj = C + (size_t)S[(size_t)cell[t] * n + edge[t]] * D;
        double lh = vlqo_lambda_dequant(lamq[t], lo, hi);
        for (int p = 0; p < m; ++p) {
            const float *w = P + ((size_t)p * 256 + codes[(size_t)t * m + p]) * ds;
            for (int d = 0; d < ds; ++d) {
                int g = p * ds + d;
                Xhat[(size_t)t * D + g] =
                    (1.0 - lh) * (double)ci[g] + lh * (double)sj[g] + (double)w[d];
            }
        }
    }
}

/* ---- search (Alg. 3), one function per step ------------------------- */

/* Alg. 3, first loop: dist[q][i] = ||y_q - c_i||^2 for all i. */
void vlqo_coarse(const float *C, int k, int D, const float *Y, int nq, double *dist)
{
#pragma omp parallel for schedule(static)
    for (int q = 0; q < nq; ++q)
        for (int i = 0; i < k; ++i)
            dist[(size_t)q * k + i] = sqdist_ff(Y + (size_t)q * D, C + (size_t)i * D, D);
}

/* w smallest entries of each row of val[nq x len], ascending by (value, key);
 * key[q][e] is the tie-break and the reported label (NULL: the position e).
 * Rows shorter than w are padded with -1. */
void vlqo_select_smallest(const double *val, const int32_t *key, int nq, int len, int w,
                          int32_t *out)
{
#pragma omp parallel
    {
        dj_t *buf = (dj_t *)malloc((size_t)len * sizeof(dj_t));
#pragma omp for schedule(static)
        for (int q = 0; q < nq; ++q) {
            for (int e = 0; e < len; ++e) {
                buf[e].d = val[(size_t)q * len + e];
                buf[e].j = key ? key[(size_t)q * len + e] : e;
            }
            qsort(buf, (size_t)len, sizeof(dj_t), cmp_dj);
            for (int e = 0; e < w; ++e) out[(size_t)q * w + e] = e < len ? buf[e].j : -1;
        }
        free(buf);
    }
}

/* Sec. 3.3.1, second-level traversal: the query is line-quantised against every
 * edge (i, j) of every probed cell: score = Eq. 7 at the query's own lambda
 * (Eq. 8) with a = dist[q][i], b = dist[q][S_i[j]], c = E_ij.
 * Variant: the query's lambda restricted to [qlo, qhi] before Eq. 7 is evaluated
 * (the distance to that segment of the line; -inf / +inf is the literal reading,
 * the whole line).
 * score[q][e*n + j] for the e-th probed cell; label[q][e*n + j] = i*n + j. */
void vlqo_subregion_scores(const double *dist, int nq, int k, int n,
                           const int32_t *S, const double *E,
                           const int32_t *cells, int w1, double qlo, double qhi,
                           double *score, int32_t *label)
{
#pragma omp parallel for schedule(static)
    for (int q = 0; q < nq; ++q)
        for (int e = 0; e < w1; ++e) {
            int i = cells[(size_t)q * w1 + e];
            double a = dist[(size_t)q * k + i];
            for (int j = 0; j < n; ++j) {
                double b = dist[(size_t)q * k + S[(size_t)i * n + j]];
                double c = E[(size_t)i * n + j];
                double lam = vlqo_line_lambda(a, b, c);
                if (lam < qlo) lam = qlo;
                if (lam > qhi) lam = qhi;
                size_t o = ((size_t)q * w1 + e) * n + j;
                score[o] = vlqo_line_dist2(a, b, c, lam);
                label[o] = i * n + j;
            }
        }
}

typedef struct { double d; int32_t id; } cand_t;

static int cmp_cand(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->d < b->d) return -1;
    if (a->d > b->d) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

/* Alg. 3, second loop + re-ranking: for every point of every visited list,
 * rebuild the approximated point (Eq. 14) and take its squared distance to the
 * query; return the K smallest by (distance, id), padded with (+inf, -1).
 * lists[q][0..w2) are list labels i*n+j (entries < 0 are skipped).
 * Inverted lists: list_off[k*n+1], and per stored point ids / codes[m] / lamq.
 * ncand[q] (optional) = number of candidates scored. */
void vlqo_scan(const float *C, int D, int n, const int32_t *S,
               const float *P, int m, double lo, double hi,
               const int64_t *list_off, const int32_t *ids, const uint8_t *codes,
               const uint8_t *lamq,
               const float *Y, int nq, const int32_t *lists, int w2, int K,
               double *out_d, int32_t *out_id, int64_t *ncand)
{
    const int ds = D / m;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        const float *y = Y + (size_t)q * D;
        int64_t total = 0;
        for (int e = 0; e < w2; ++e) {
            int l = lists[(size_t)q * w2 + e];
            if (l >= 0) total += list_off[l + 1] - list_off[l];
        }
        cand_t *cand = (cand_t *)malloc((size_t)(total > 0 ? total : 1) * sizeof(cand_t));
        int64_t nc = 0;
        for (int e = 0; e < w2; ++e) {
            int l = lists[(size_t)q * w2 + e];
            if (l < 0) continue;
            int i = l / n, j = l % n;
            const float *ci = C + (size_t)i * D;
            const float *sj = C + (size_t)S[(size_t)i * n + j] * D;
            for (int64_t t = list_off[l]; t < list_off[l + 1]; ++t) {
                double lh = vlqo_lambda_dequant(lamq[t], lo, hi);
                double s = 0.0;
                for (int p = 0; p < m; ++p) {
                    const float *w = P + ((size_t)p * 256 + codes[(size_t)t * m + p]) * ds;
                    for (int d = 0; d < ds; ++d) {
                        int g = p * ds + d;
                        double xh = (1.0 - lh) * (double)ci[g] + lh * (double)sj[g] + (double)w[d];
                        double u = (double)y[g] - xh;
                        s += u * u;
                    }
                }
                cand[nc].d = s;
                cand[nc].id = ids[t];
                ++nc;
            }
        }
        qsort(cand, (size_t)nc, sizeof(cand_t), cmp_cand);
        for (int r = 0; r < K; ++r) {
            out_d[(size_t)q * K + r] = r < nc ? cand[r].d : INFINITY;
            out_id[(size_t)q * K + r] = r < nc ? cand[r].id : -1;
        }
        if (ncand) ncand[q] = nc;
        free(cand);
    }
}
