/*
 * CPU oracle for the Monarch multiply  y = M x,  M = P L P^T R  (forward and backward).
 *
 * THIS IS TEST INFRASTRUCTURE, not product code.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may build, link or call it.
 * It shares no source, header, table or helper with the GPU library.
 *
 * Everything is plain double precision, one loop nest per step of the method,
 * in the order the paper states them ("Steps to multiply x by a Monarch
 * matrix", Section 3.3, steps 1-3, and Definition 3.1 for the permutation P).
 * No blocking, fusion or reordering.  OpenMP splits the batch rows only; the
 * weight-gradient sums use one private accumulator per thread, added together
 * in thread order at the end.
 *
 * Shapes (row-major, last index fastest):
 *   x  (B, k*p)      input rows, viewed (B, k, p)
 *   R  (k, q, p)     block-diagonal first factor:  R[kk][j][i] = block kk, output j, input i
 *   L  (k, s, q)     block-diagonal second factor: L[c][l][r]  = block c,  output l, input r
 *   y  (B, k*s)
 *
 * Section 3.3 step 1:  Y1[kk][j] = sum_i R[kk][j][i] * x[kk][i]
 * P^T of Def. 3.1:     U[f]      = Y1flat[pi(f)]               (the "mid" permutation)
 * Section 3.3 step 2:  W[c][l]   = sum_r L[c][l][r] * U[c*q + r]
 * Section 3.3 step 3 / outer P:  y[l*k + c] = W[c][l]
 *
 * The square case n = m^2, k = p = q = s = m reproduces the paper's formulas
 * literally: pi(c*m + r) = r*m + c, so W[j][l] = sum_k L[j][l][k] * Y1[k][j]
 * and the result is flattened as index l*m + j.
 *
 * The paper defines P only for the square case.  For k != q two readings of
 * "reshape, transpose, flatten" exist; `reading` selects one:
 *   reading 0 (A): view Y1 as a (k, q) grid, transpose it to (q, k), flatten,
 *                  cut into k chunks of length q:   pi(f) = (f mod k)*q + f div k
 *   reading 1 (B): view the flat vector as a (q, k) grid, transpose to (k, q):
 *                                                    pi(f) = (f mod q)*k + f div q
 * They are inverse permutations and agree when k == q.
 *
 * Backward is the adjoint of every step, taken in reverse order (the paper
 * relies on automatic differentiation, Section 4; the adjoints are written out
 * here):
 *   dW[c][l]   = dy[l*k + c]
 *   dL[c][l][r] += dW[c][l] * U[c*q + r]                (summed over rows)
 *   dU[c*q + r] = sum_l L[c][l][r] * dW[c][l]
 *   dY1flat[pi(f)] = dU[f]
 *   dR[kk][j][i] += dY1[kk][j] * x[kk][i]                (summed over rows)
 *   dx[kk][i]   = sum_j R[kk][j][i] * dY1[kk][j]
 */
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Mid permutation index map (Definition 3.1 for the square case; see header). */
int64_t monarch_oracle_pi(int64_t f, int k, int q, int reading)
{
    if (reading == 0)
        return (f % k) * (int64_t)q + f / k;
    return (f % q) * (int64_t)k + f / q;
}

int monarch_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One row of the forward pass.  y1, u: scratch of k*q doubles each. */
static void fwd_row(const double *x, const double *R, const double *L, double *y,
                    int k, int p, int q, int s, int reading, double *y1, double *u)
{
    /* step 1: block-diagonal R */
    for (int kk = 0; kk < k; ++kk)
        for (int j = 0; j < q; ++j) {
            double acc = 0.0;
            const double *Rrow = R + ((int64_t)kk * q + j) * p;
            for (int i = 0; i < p; ++i)
                acc += Rrow[i] * x[kk * p + i];
            y1[kk * q + j] = acc;
        }
    /* P^T */
    for (int64_t f = 0; f < (int64_t)k * q; ++f)
        u[f] = y1[monarch_oracle_pi(f, k, q, reading)];
    /* step 2: block-diagonal L, step 3: outer P folded into the store index */
    for (int c = 0; c < k; ++c)
        for (int l = 0; l < s; ++l) {
            double acc = 0.0;
            const double *Lrow = L + ((int64_t)c * s + l) * q;
            for (int r = 0; r < q; ++r)
                acc += Lrow[r] * u[c * q + r];
            y[(int64_t)l * k + c] = acc;
        }
}

/* Forward for `batch` rows.  All arrays are double, row-major.  Returns 0. */
int monarch_oracle_fwd(const double *x, const double *R, const double *L, double *y,
                       int64_t batch, int n_in, int k, int q, int s, int reading)
{
    if (k <= 0 || q <= 0 || s <= 0 || n_in <= 0 || n_in % k != 0 || batch < 0)
        return -1;
    const int p = n_in / k;
    const int64_t kq = (int64_t)k * q, n_out = (int64_t)k * s;
#pragma omp parallel
    {
        double *y1 = (double *)malloc(sizeof(double) * kq);
        double *u = (double *)malloc(sizeof(double) * kq);
#pragma omp for schedule(static)
        for (int64_t b = 0; b < batch; ++b)
            fwd_row(x + b * n_in, R, L, y + b * n_out, k, p, q, s, reading, y1, u);
        free(y1);
        free(u);
    }
    return 0;
}

/* Backward for `batch` rows: dx (batch, n_in), dR (k,q,p), dL (k,s,q); all
 * three are overwritten.  Returns 0. */
int monarch_oracle_bwd(const double *dy, const double *x, const double *R, const double *L,
                       double *dx, double *dR, double *dL,
                       int64_t batch, int n_in, int k, int q, int s, int reading)
{
    if (k <= 0 || q <= 0 || s <= 0 || n_in <= 0 || n_in % k != 0 || batch < 0)
        return -1;
    const int p = n_in / k;
    const int64_t kq = (int64_t)k * q, n_out = (int64_t)k * s;
    const int64_t nR = kq * p, nL = (int64_t)k * s * q;
    const int nthr = monarch_oracle_num_threads();
    double *dRpart = (double *)calloc((size_t)nthr * nR, sizeof(double));
    double *dLpart = (double *)calloc((size_t)nthr * nL, sizeof(double));
    if (!dRpart || !dLpart) { free(dRpart); free(dLpart); return -2; }

#pragma omp parallel num_threads(nthr)
    {
#ifdef _OPENMP
        const int t = omp_get_thread_num();
#else
        const int t = 0;
#endif
        double *dRt = dRpart + (int64_t)t * nR;
        double *dLt = dLpart + (int64_t)t * nL;
        double *y1 = (double *)malloc(sizeof(double) * kq);
        double *u = (double *)malloc(sizeof(double) * kq);
        double *du = (double *)malloc(sizeof(double) * kq);
        double *dy1 = (double *)malloc(sizeof(double) * kq);
        double *dw = (double *)malloc(sizeof(double) * n_out);
#pragma omp for schedule(static)
        for (int64_t b = 0; b < batch; ++b) {
            const double *xb = x + b * n_in;
            const double *dyb = dy + b * n_out;
            double *dxb = dx + b * n_in;
            /* recompute the forward intermediates of this row (steps 1 and P^T) */
            for (int kk = 0; kk < k; ++kk)
                for (int j = 0; j < q; ++j) {
                    double acc = 0.0;
                    const double *Rrow = R + ((int64_t)kk * q + j) * p;
                    for (int i = 0; i < p; ++i)
                        acc += Rrow[i] * xb[kk * p + i];
                    y1[kk * q + j] = acc;
                }
            for (int64_t f = 0; f < kq; ++f)
                u[f] = y1[monarch_oracle_pi(f, k, q, reading)];
            /* adjoint of step 3 (outer P) */
            for (int c = 0; c < k; ++c)
                for (int l = 0; l < s; ++l)
                    dw[c * s + l] = dyb[(int64_t)l * k + c];
            /* adjoint of step 2 */
            for (int64_t f = 0; f < kq; ++f)
                du[f] = 0.0;
            for (int c = 0; c < k; ++c)
                for (int l = 0; l < s; ++l) {
                    const double g = dw[c * s + l];
                    const double *Lrow = L + ((int64_t)c * s + l) * q;
                    double *dLrow = dLt + ((int64_t)c * s + l) * q;
                    for (int r = 0; r < q; ++r) {
                        dLrow[r] += g * u[c * q + r];
                        du[c * q + r] += Lrow[r] * g;
                    }
                }
            /* adjoint of P^T */
            for (int64_t f = 0; f < kq; ++f)
                dy1[monarch_oracle_pi(f, k, q, reading)] = du[f];
            /* adjoint of step 1 */
            for (int i = 0; i < n_in; ++i)
                dxb[i] = 0.0;
            for (int kk = 0; kk < k; ++kk)
                for (int j = 0; j < q; ++j) {
                    const double g = dy1[kk * q + j];
                    const double *Rrow = R + ((int64_t)kk * q + j) * p;
                    double *dRrow = dRt + ((int64_t)kk * q + j) * p;
                    for (int i = 0; i < p; ++i) {
                        dRrow[i] += g * xb[kk * p + i];
                        dxb[kk * p + i] += Rrow[i] * g;
                    }
                }
        }
        free(y1); free(u); free(du); free(dy1); free(dw);
    }
    for (int64_t e = 0; e < nR; ++e) {
        double acc = 0.0;
        for (int t = 0; t < nthr; ++t) acc += dRpart[(int64_t)t * nR + e];
        dR[e] = acc;
    }
    for (int64_t e = 0; e < nL; ++e) {
        double acc = 0.0;
        for (int t = 0; t < nthr; ++t) acc += dLpart[(int64_t)t * nL + e];
        dL[e] = acc;
    }
    free(dRpart);
    free(dLpart);
    return 0;
}
