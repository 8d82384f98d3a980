/*
 * CPU oracle for the Frobenius-norm multiplicative-update (MU) NMF iteration.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It is never linked into, imported by or
 * called from the product path, and it shares no code, header, table or
 * helper with the HIP kernels.
 *
 * Everything is computed in IEEE double.  The data matrix A is handed over in
 * the single-precision storage the method works on (paper, section 2.3, gives
 * all matrix sizes for 4-byte elements) and every element is widened to double
 * at the point of use; the factors W and H live in double for the whole run.
 *
 * One iteration follows the order of the distributed row-partition algorithm
 * (paper, Algorithm 3, with one processing unit so that every all-reduce is
 * the identity):
 *
 *     WTA = W^T A          WTW = W^T W
 *     H   <- H * WTA / (WTW H + eps)               (H update, old H on the right)
 *     HHT = H H^T          (new H)
 *     AHT = A H^T          (new H)
 *     W   <- W * AHT / (W HHT + eps)               (W update, old W on the right)
 *
 * eps is added once, to the finished denominator (Algorithm 1 and Algorithms
 * 2/3 agree on this; the doubled eps of Algorithm 4 is taken as a slip).
 *
 * Each output element is reduced by one thread in a fixed sequential order,
 * so results do not depend on the number of OpenMP threads.
 *
 * Layout: all matrices row-major and contiguous.  A is m x n, W is m x k,
 * H is k x n.  CSR: rowptr[m+1] (int64), colidx[nnz] (int32), vals[nnz]
 * (float); columns within a row need not be sorted and repeated (i, j)
 * entries add up, i.e. the CSR arrays stand for the dense matrix they sum to.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of multiply-accumulate pairs executed since the last reset; used by
 * a test that checks the paper's FLOP model (section 3.1, list of per-line
 * counts).  Updated outside the parallel loops, from the loop bounds. */
static long long g_mac_count = 0;

void oracle_reset_mac_count(void) { g_mac_count = 0; }
long long oracle_get_mac_count(void) { return g_mac_count; }

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- the six products and two element-wise updates, one function each ---- */

/* WTW = W^T W  (k x k).  Algorithm 3, the line that forms WTW. */
void oracle_gram_w(const double *W, int64_t m, int32_t k, double *G)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int32_t a = 0; a < k; ++a)
        for (int32_t b = 0; b < k; ++b) {
            double s = 0.0;
            for (int64_t i = 0; i < m; ++i)
                s += W[i * k + a] * W[i * k + b];
            G[a * k + b] = s;
        }
    g_mac_count += (long long)m * k * k;
}

/* HHT = H H^T  (k x k).  Algorithm 3, the line that forms HHT from the new H. */
void oracle_gram_h(const double *H, int32_t k, int64_t n, double *G)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int32_t a = 0; a < k; ++a)
        for (int32_t b = 0; b < k; ++b) {
            double s = 0.0;
            for (int64_t j = 0; j < n; ++j)
                s += H[(int64_t)a * n + j] * H[(int64_t)b * n + j];
            G[a * k + b] = s;
        }
    g_mac_count += (long long)n * k * k;
}

/* WTA = W^T A  (k x n), A dense.  Algorithm 3, the line that forms WTA.
 * Threads own disjoint column ranges; every P[c][j] is summed over i = 0..m-1
 * in increasing i. */
void oracle_wta_dense(const float *A, int64_t m, int64_t n,
                      const double *W, int32_t k, double *P)
{
    const int64_t chunk = 256;
    const int64_t nchunks = (n + chunk - 1) / chunk;
#pragma omp parallel for schedule(static)
    for (int64_t ch = 0; ch < nchunks; ++ch) {
        const int64_t j0 = ch * chunk;
        const int64_t j1 = (j0 + chunk < n) ? j0 + chunk : n;
        for (int32_t c = 0; c < k; ++c)
            for (int64_t j = j0; j < j1; ++j)
                P[(int64_t)c * n + j] = 0.0;
        for (int64_t i = 0; i < m; ++i) {
            const float *Ai = A + i * n;
            for (int32_t c = 0; c < k; ++c) {
                const double w = W[i * k + c];
                double *Pc = P + (int64_t)c * n;
                for (int64_t j = j0; j < j1; ++j)
                    Pc[j] += w * (double)Ai[j];
            }
        }
    }
    g_mac_count += (long long)m * n * k;
}

/* AHT = A H^T  (m x k), A dense.  Algorithm 3, the line that forms AHT.
 * Threads own disjoint rows; every Q[i][c] is summed over j in increasing j. */
void oracle_aht_dense(const float *A, int64_t m, int64_t n,
                      const double *H, int32_t k, double *Q)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        const float *Ai = A + i * n;
        for (int32_t c = 0; c < k; ++c) {
            const double *Hc = H + (int64_t)c * n;
            double s = 0.0;
            for (int64_t j = 0; j < n; ++j)
                s += (double)Ai[j] * Hc[j];
            Q[i * k + c] = s;
        }
    }
    g_mac_count += (long long)m * n * k;
}

/* WTA from CSR.  P[c][j] = sum over stored entries (i, j, a) of W[i][c] * a.
 * Stored entries are visited in storage order (row by row), one thread, so
 * that unsorted and repeated column indices need no special handling. */
void oracle_wta_csr(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                    int64_t m, int64_t n, const double *W, int32_t k, double *P)
{
    for (int64_t t = 0; t < (int64_t)k * n; ++t)
        P[t] = 0.0;
    /* Parallel over the factor index c: thread-private rows of P. */
#pragma omp parallel for schedule(static)
    for (int32_t c = 0; c < k; ++c) {
        double *Pc = P + (int64_t)c * n;
        for (int64_t i = 0; i < m; ++i) {
            const double w = W[i * k + c];
            for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
                Pc[colidx[e]] += w * (double)vals[e];
        }
    }
    g_mac_count += (long long)rowptr[m] * k;
}

/* AHT from CSR.  Q[i][c] = sum over the stored entries of row i. */
void oracle_aht_csr(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                    int64_t m, int64_t n, const double *H, int32_t k, double *Q)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int32_t c = 0; c < k; ++c) {
            const double *Hc = H + (int64_t)c * n;
            double s = 0.0;
            for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
                s += (double)vals[e] * Hc[colidx[e]];
            Q[i * k + c] = s;
        }
    g_mac_count += (long long)rowptr[m] * k;
}

/* H <- H * WTA / (WTW H + eps).  Algorithm 3, the H-update line.  The whole
 * denominator is formed from the old H before any element is overwritten. */
void oracle_h_update(double *H, const double *P, const double *G,
                     int32_t k, int64_t n, double eps)
{
#pragma omp parallel
    {
        double *den = (double *)malloc(sizeof(double) * (size_t)k);
#pragma omp for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            for (int32_t c = 0; c < k; ++c) {
                double s = 0.0;
                for (int32_t d = 0; d < k; ++d)
                    s += G[c * k + d] * H[(int64_t)d * n + j];
                den[c] = s + eps;
            }
            for (int32_t c = 0; c < k; ++c)
                H[(int64_t)c * n + j] = H[(int64_t)c * n + j] * P[(int64_t)c * n + j] / den[c];
        }
        free(den);
    }
    g_mac_count += (long long)n * k * k;
}

/* W <- W * AHT / (W HHT + eps).  Algorithm 3, the W-update line. */
void oracle_w_update(double *W, const double *Q, const double *G,
                     int64_t m, int32_t k, double eps)
{
#pragma omp parallel
    {
        double *den = (double *)malloc(sizeof(double) * (size_t)k);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            for (int32_t c = 0; c < k; ++c) {
                double s = 0.0;
                for (int32_t d = 0; d < k; ++d)
                    s += W[i * k + d] * G[d * k + c];
                den[c] = s + eps;
            }
            for (int32_t c = 0; c < k; ++c)
                W[i * k + c] = W[i * k + c] * Q[i * k + c] / den[c];
        }
        free(den);
    }
    g_mac_count += (long long)m * k * k;
}

/* ---- whole iterations ---- */

/* which = 0: H update only; 1: W update only; 2: H then W (one iteration). */
static int mu_steps(const float *A, const int64_t *rowptr, const int32_t *colidx,
                    const float *vals, int64_t m, int64_t n, int32_t k,
                    double *W, double *H, int32_t iters, double eps, int which)
{
    double *G = (double *)malloc(sizeof(double) * (size_t)k * k);
    double *P = (which != 1) ? (double *)malloc(sizeof(double) * (size_t)k * n) : NULL;
    double *Q = (which != 0) ? (double *)malloc(sizeof(double) * (size_t)m * k) : NULL;
    if (!G || (which != 1 && !P) || (which != 0 && !Q)) {
        free(G); free(P); free(Q);
        return 1;
    }
    for (int32_t it = 0; it < iters; ++it) {
        if (which != 1) {
            oracle_gram_w(W, m, k, G);
            if (A) oracle_wta_dense(A, m, n, W, k, P);
            else   oracle_wta_csr(rowptr, colidx, vals, m, n, W, k, P);
            oracle_h_update(H, P, G, k, n, eps);
        }
        if (which != 0) {
            oracle_gram_h(H, k, n, G);
            if (A) oracle_aht_dense(A, m, n, H, k, Q);
            else   oracle_aht_csr(rowptr, colidx, vals, m, n, H, k, Q);
            oracle_w_update(W, Q, G, m, k, eps);
        }
    }
    free(G); free(P); free(Q);
    return 0;
}

int oracle_mu_dense(const float *A, int64_t m, int64_t n, int32_t k,
                    double *W, double *H, int32_t iters, double eps)
{
    return mu_steps(A, NULL, NULL, NULL, m, n, k, W, H, iters, eps, 2);
}

int oracle_mu_csr(const int64_t *rowptr, const int32_t *colidx, const float *vals,
                  int64_t m, int64_t n, int32_t k,
                  double *W, double *H, int32_t iters, double eps)
{
    return mu_steps(NULL, rowptr, colidx, vals, m, n, k, W, H, iters, eps, 2);
}

/* Half steps, exposed so that tests can look at the objective after each. */
int oracle_h_step_dense(const float *A, int64_t m, int64_t n, int32_t k,
                        double *W, double *H, double eps)
{
    return mu_steps(A, NULL, NULL, NULL, m, n, k, W, H, 1, eps, 0);
}

int oracle_w_step_dense(const float *A, int64_t m, int64_t n, int32_t k,
                        double *W, double *H, double eps)
{
    return mu_steps(A, NULL, NULL, NULL, m, n, k, W, H, 1, eps, 1);
}

/* ||A - W H||_F, the quantity the method minimises (paper, section 2.1).
 * Evaluated element by element; never forms W H as a matrix. */
double oracle_residual_dense(const float *A, int64_t m, int64_t n, int32_t k,
                             const double *W, const double *H)
{
    double *rowsum = (double *)malloc(sizeof(double) * (size_t)m);
    if (!rowsum) return -1.0;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            double x = 0.0;
            for (int32_t c = 0; c < k; ++c)
                x += W[i * k + c] * H[(int64_t)c * n + j];
            const double d = (double)A[i * n + j] - x;
            s += d * d;
        }
        rowsum[i] = s;
    }
    double total = 0.0;
    for (int64_t i = 0; i < m; ++i)
        total += rowsum[i];
    free(rowsum);
    return sqrt(total);
}
