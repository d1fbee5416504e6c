/*
 * CPU oracle for the Based sequence mixer (arXiv 2402.18668).  TEST INFRASTRUCTURE ONLY.
 *
 * Slow, plain, fp64 implementations of what the GPU hot path must compute, written
 * from the paper's equations.  Nothing here is shared with the HIP library and the
 * product path never calls into this file; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg do.
 *
 * Conventions
 *   U   independent (batch, head) units, processed one by one (OpenMP over units)
 *   N   tokens per unit, dp = d' projected feature dim, dv = value/head dim
 *   q,k [U][N][dp], v,y [U][N][dv], all double, row-major, last index fastest
 *   D = 1 + dp + dp*dp  expanded feature dim (Sec. 4 "Taylor Exponential Linear
 *       Attention": D = 1 + d' + d'^2)
 *   canonical state  S [U][D][dv],  z [U][D]   (Sec. 3.1 KV-state and K-state)
 *   feature order    row 0: constant 1; rows 1..dp: x_a; row 1+dp+a*dp+b: x_a*x_b/sqrt(2)
 *
 * Every function below is pinned by the CPU tests: closed form of Eq. 4, equality of
 * the parallel (Eq. 2) and recurrent (Eq. 3) views and of the tile split of Sec. 4,
 * a pure-Python brute force, textbook special cases, and a library softmax attention
 * for the windowed case with w >= N.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* D = 1 + d' + d'^2 (Sec. 4). */
int oracle_feature_dim(int dp) { return 1 + dp + dp * dp; }

/* Number of distinct monomials of degree <= 2 in d' variables times (dv + 1) columns:
 * the recurrent-state size formula of the appendix on state sizes,
 * (d + 1) * (1 + 3d'/2 + d'^2/2). */
long oracle_state_size_symmetric(int dp, int dv)
{
    long monomials = 1 + dp + (long)dp * (dp + 1) / 2;
    return (long)(dv + 1) * monomials;
}

/* 2nd-order Taylor feature map, Eq. 4: phi(x) = [1, x, vec(x x^T)/sqrt(2)]. */
void oracle_feature_map(const double *x, int dp, double *phi)
{
    const double r2 = sqrt(2.0);
    phi[0] = 1.0;
    for (int a = 0; a < dp; ++a) phi[1 + a] = x[a];
    for (int a = 0; a < dp; ++a)
        for (int b = 0; b < dp; ++b) phi[1 + dp + a * dp + b] = x[a] * x[b] / r2;
}

static double dot(const double *a, const double *b, int n)
{
    double s = 0.0;
    for (int i = 0; i < n; ++i) s += a[i] * b[i];
    return s;
}

/* One output row of causal Taylor linear attention in the parallel view
 * (Eq. 2 with the kernel of Eq. 4):
 *   y_i = sum_{j<=i} w_ij v_j / sum_{j<=i} w_ij,  w_ij = 1 + q_i.k_j + (q_i.k_j)^2 / 2.
 * q_i points at row i of q; k, v at row 0 of the unit. */
static void linattn_row(const double *qi, const double *k, const double *v, int i, int dp,
                        int dv, double *yi)
{
    double den = 0.0;
    for (int c = 0; c < dv; ++c) yi[c] = 0.0;
    for (int j = 0; j <= i; ++j) {
        double x = dot(qi, k + (size_t)j * dp, dp);
        double w = 1.0 + x + 0.5 * x * x;
        den += w;
        const double *vj = v + (size_t)j * dv;
        for (int c = 0; c < dv; ++c) yi[c] += w * vj[c];
    }
    for (int c = 0; c < dv; ++c) yi[c] /= den;
}

/* Parallel (quadratic) view over whole sequences, zero initial state. */
void oracle_linattn_quadratic(const double *q, const double *k, const double *v, double *y,
                              int U, int N, int dp, int dv)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (int u = 0; u < U; ++u)
        for (int i = 0; i < N; ++i) {
            const double *qu = q + (size_t)u * N * dp, *ku = k + (size_t)u * N * dp;
            const double *vu = v + (size_t)u * N * dv;
            linattn_row(qu + (size_t)i * dp, ku, vu, i, dp, dv, y + ((size_t)u * N + i) * dv);
        }
}

/* The same rows, but only at the listed token indices (for spot checks at sizes where
 * the full quadratic sweep would take too long).  y_rows is [U][nrows][dv]. */
void oracle_linattn_rows(const double *q, const double *k, const double *v,
                         const int64_t *rows, int nrows, double *y_rows, int U, int N,
                         int dp, int dv)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int u = 0; u < U; ++u)
        for (int r = 0; r < nrows; ++r) {
            int i = (int)rows[r];
            const double *qu = q + (size_t)u * N * dp, *ku = k + (size_t)u * N * dp;
            const double *vu = v + (size_t)u * N * dv;
            linattn_row(qu + (size_t)i * dp, ku, vu, i, dp, dv,
                        y_rows + ((size_t)u * nrows + r) * dv);
        }
}

/* KV-state and K-state after N tokens (Sec. 3.1): S += sum_j phi(k_j) v_j^T,
 * z += sum_j phi(k_j).  S and z are in-out (the caller zeroes them for a fresh start). */
void oracle_linattn_state(const double *k, const double *v, double *S, double *z, int U,
                          int N, int dp, int dv)
{
    const int D = oracle_feature_dim(dp);
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < U; ++u) {
        double *phi = (double *)malloc(sizeof(double) * D);
        double *Su = S + (size_t)u * D * dv, *zu = z + (size_t)u * D;
        for (int j = 0; j < N; ++j) {
            oracle_feature_map(k + ((size_t)u * N + j) * dp, dp, phi);
            const double *vj = v + ((size_t)u * N + j) * dv;
            for (int f = 0; f < D; ++f) {
                zu[f] += phi[f];
                for (int c = 0; c < dv; ++c) Su[(size_t)f * dv + c] += phi[f] * vj[c];
            }
        }
        free(phi);
    }
}

/* Recurrent view, Eq. 3, starting from (and updating in place) a given state:
 *   s_i = s_{i-1} + phi(k_i) v_i^T,  z_i = z_{i-1} + phi(k_i),
 *   y_i = phi(q_i) s_i / (phi(q_i) z_i).
 * The token updates the state before it reads it (it attends to itself). */
void oracle_linattn_recurrent(const double *q, const double *k, const double *v, double *y,
                              double *S, double *z, int U, int N, int dp, int dv)
{
    const int D = oracle_feature_dim(dp);
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < U; ++u) {
        double *pk = (double *)malloc(sizeof(double) * D);
        double *pq = (double *)malloc(sizeof(double) * D);
        double *Su = S + (size_t)u * D * dv, *zu = z + (size_t)u * D;
        for (int i = 0; i < N; ++i) {
            oracle_feature_map(k + ((size_t)u * N + i) * dp, dp, pk);
            oracle_feature_map(q + ((size_t)u * N + i) * dp, dp, pq);
            const double *vi = v + ((size_t)u * N + i) * dv;
            double *yi = y + ((size_t)u * N + i) * dv;
            double den = 0.0;
            for (int c = 0; c < dv; ++c) yi[c] = 0.0;
            for (int f = 0; f < D; ++f) {
                zu[f] += pk[f];
                den += pq[f] * zu[f];
                double *row = Su + (size_t)f * dv;
                for (int c = 0; c < dv; ++c) {
                    row[c] += pk[f] * vi[c];
                    yi[c] += pq[f] * row[c];
                }
            }
            for (int c = 0; c < dv; ++c) yi[c] /= den;
        }
        free(pk);
        free(pq);
    }
}

/* One row of causal sliding-window softmax attention (Sec. 3.2 restricting Eq. 1):
 * query i attends keys max(0, i-w+1) .. i, logits scale * q_i.k_j, max-subtracted. */
static void swa_row(const double *qi, const double *k, const double *v, int i, int dh, int w,
                    double scale, double *yi)
{
    int lo = i - w + 1;
    if (lo < 0) lo = 0;
    double m = -INFINITY;
    for (int j = lo; j <= i; ++j) {
        double s = scale * dot(qi, k + (size_t)j * dh, dh);
        if (s > m) m = s;
    }
    double den = 0.0;
    for (int c = 0; c < dh; ++c) yi[c] = 0.0;
    for (int j = lo; j <= i; ++j) {
        double p = exp(scale * dot(qi, k + (size_t)j * dh, dh) - m);
        den += p;
        const double *vj = v + (size_t)j * dh;
        for (int c = 0; c < dh; ++c) yi[c] += p * vj[c];
    }
    for (int c = 0; c < dh; ++c) yi[c] /= den;
}

void oracle_swa(const double *q, const double *k, const double *v, double *y, int U, int N,
                int dh, int w, double scale)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 64)
    for (int u = 0; u < U; ++u)
        for (int i = 0; i < N; ++i) {
            size_t base = (size_t)u * N * dh;
            swa_row(q + base + (size_t)i * dh, k + base, v + base, i, dh, w, scale,
                    y + base + (size_t)i * dh);
        }
}

void oracle_swa_rows(const double *q, const double *k, const double *v, const int64_t *rows,
                     int nrows, double *y_rows, int U, int N, int dh, int w, double scale)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (int u = 0; u < U; ++u)
        for (int r = 0; r < nrows; ++r) {
            int i = (int)rows[r];
            size_t base = (size_t)u * N * dh;
            swa_row(q + base + (size_t)i * dh, k + base, v + base, i, dh, w, scale,
                    y_rows + ((size_t)u * nrows + r) * dh);
        }
}
