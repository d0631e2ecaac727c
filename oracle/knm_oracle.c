/*
 * knm_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 CPU statement of what the preconditioned Nystrom kernel ridge
 * solver ("Falkon") of arXiv 2006.10350 computes.  It exists to check the GPU library
 * and to be timed beside it; no product code path may call it, and it shares no code,
 * header, table or constant with the HIP sources.
 *
 * Every function is the textbook definition written out: direct coordinate
 * differences for the squared distance (no norm expansion), libm exp, straight loops,
 * row-major arrays, no blocking beyond an OpenMP "parallel for" over independent
 * output rows.  Data points arrive as the fp32 values the GPU sees and are promoted
 * exactly to fp64; everything else is fp64.
 *
 * Notation follows the paper: n data points, d features, M Nystrom centres ("m" in
 * the paper), t right-hand sides, sigma the Gaussian length-scale, lambda the ridge
 * parameter.  T and A are UPPER triangular with T^T T = K_MM and
 * A^T A = T T^T / M + lambda I   (Eq. 7 and the remark K_mm = T^T T below it).
 *
 * Parity pins (tests/test_oracle_*.py): hand values, sigma->inf closed form,
 * Kronecker structure on grids, library RBF/Cholesky/solve routines, the M = n
 * closed form alpha = (K_nn + n lambda I)^-1 y, LinOp = n I when M = n, and the dense
 * solution of the Nystrom normal equations (Eq. 5).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* number of threads the parallel loops will use (reported by the CPU baseline) */
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Kernel function.  The paper works with the Gaussian kernel of a single length-scale throughout
 * (Section 2 for the estimator, Section 5 for the experiments):
 *     k(x, c) = exp(-||x - c||^2 / (2 sigma^2)).
 * Its method holds for any positive-definite kernel; beyond it this oracle has three kernels of the
 * distance r = ||x - c|| in their textbook forms, which the paper does not spell out:
 *     Laplacian     k = exp(-r / sigma)
 *     Matern 3/2    k = (1 + u) exp(-u),            u = sqrt(3) r / sigma
 *     Matern 5/2    k = (1 + u + u^2 / 3) exp(-u),  u = sqrt(5) r / sigma
 * The choice is a process-wide setting (test infrastructure: one thread of control). */
static int g_kind = 0; /* 0 Gaussian, 1 Laplacian, 2 Matern 3/2, 3 Matern 5/2 */

int orc_set_kernel(int kind)
{
    if (kind < 0 || kind > 3) return -1;
    g_kind = kind;
    return 0;
}

int orc_get_kernel(void) { return g_kind; }

static double gauss(const float *x, const float *c, int d, double sigma)
{
    double s = 0.0;
    for (int k = 0; k < d; ++k) {
        double diff = (double)x[k] - (double)c[k];
        s += diff * diff;
    }
    if (g_kind == 1) return exp(-sqrt(s) / sigma);
    if (g_kind == 2) {
        double u = sqrt(3.0) * sqrt(s) / sigma;
        return (1.0 + u) * exp(-u);
    }
    if (g_kind == 3) {
        double u = sqrt(5.0) * sqrt(s) / sigma;
        return (1.0 + u + u * u / 3.0) * exp(-u);
    }
    return exp(-s / (2.0 * sigma * sigma));
}

double orc_gauss(const float *x, const float *c, int d, double sigma)
{
    return gauss(x, c, d, sigma);
}

/* Explicit kernel matrix K[i, j] = k(x_i, c_j), n x M row-major. */
void orc_kernel_matrix(const float *X, int64_t n, int d, int64_t ldx,
                       const float *C, int64_t M, int64_t ldc, double sigma, double *K)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < M; ++j)
            K[i * M + j] = gauss(X + i * ldx, C + j * ldc, d, sigma);
}

/* W = K_nm V : W[i, :] = sum_j k(x_i, c_j) V[j, :]   (the product k(X1, X2) v of the
 * matrix-vector comparison paragraph; also the predictor of Eq. 4). V is M x t, W n x t. */
void orc_knm_v(const float *X, int64_t n, int d, int64_t ldx,
               const float *C, int64_t M, int64_t ldc, double sigma,
               const double *V, int t, double *W)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double *w = W + i * t;
        for (int c = 0; c < t; ++c) w[c] = 0.0;
        for (int64_t j = 0; j < M; ++j) {
            double k = gauss(X + i * ldx, C + j * ldc, d, sigma);
            for (int c = 0; c < t; ++c) w[c] += k * V[j * t + c];
        }
    }
}

/* U = K_nm^T W : U[j, :] = sum_i k(x_i, c_j) W[i, :].  W is n x t, U is M x t. */
void orc_knm_t_w(const float *X, int64_t n, int d, int64_t ldx,
                 const float *C, int64_t M, int64_t ldc, double sigma,
                 const double *W, int t, double *U)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < M; ++j) {
        double *u = U + j * t;
        for (int c = 0; c < t; ++c) u[c] = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double k = gauss(X + i * ldx, C + j * ldc, d, sigma);
            for (int c = 0; c < t; ++c) u[c] += k * W[i * t + c];
        }
    }
}

/* U = K_nm^T (K_nm V), Section 3.1 "Blockwise K_nm-vector product".  W (n x t) is a
 * caller-provided buffer that receives K_nm V. */
void orc_knm_prod(const float *X, int64_t n, int d, int64_t ldx,
                  const float *C, int64_t M, int64_t ldc, double sigma,
                  const double *V, int t, double *W, double *U)
{
    orc_knm_v(X, n, d, ldx, C, M, ldc, sigma, V, t, W);
    orc_knm_t_w(X, n, d, ldx, C, M, ldc, sigma, W, t, U);
}

/* Weighted product U = K_nm^T D K_nm V with D = diag(dw)  (LinOp of Alg. 2). */
void orc_knm_prod_weighted(const float *X, int64_t n, int d, int64_t ldx,
                           const float *C, int64_t M, int64_t ldc, double sigma,
                           const double *dw, const double *V, int t, double *W, double *U)
{
    orc_knm_v(X, n, d, ldx, C, M, ldc, sigma, V, t, W);
    for (int64_t i = 0; i < n; ++i)
        for (int c = 0; c < t; ++c) W[i * t + c] *= dw[i];
    orc_knm_t_w(X, n, d, ldx, C, M, ldc, sigma, W, t, U);
}

/* In-place upper Cholesky of a symmetric positive definite M x M row-major matrix:
 * on return the upper triangle holds R with R^T R = G and the strict lower triangle is
 * zero.  Returns 0, or p+1 if the p-th pivot is not positive. */
int64_t orc_chol_upper(double *G, int64_t M)
{
    for (int64_t i = 0; i < M; ++i) {
        double piv = G[i * M + i];
        if (!(piv > 0.0)) return i + 1;
        piv = sqrt(piv);
        G[i * M + i] = piv;
        for (int64_t j = i + 1; j < M; ++j) G[i * M + j] /= piv;
        /* trailing update: G[k, j] -= R[i, k] R[i, j] for i < k <= j */
#pragma omp parallel for schedule(static)
        for (int64_t k = i + 1; k < M; ++k) {
            double rik = G[i * M + k];
            for (int64_t j = k; j < M; ++j) G[k * M + j] -= rik * G[i * M + j];
        }
    }
    for (int64_t i = 1; i < M; ++i)
        for (int64_t j = 0; j < i; ++j) G[i * M + j] = 0.0;
    return 0;
}

/* Solve R Z = B (trans = 0) or R^T Z = B (trans = 1) in place; R upper M x M
 * row-major, B is M x t row-major. */
void orc_solve_upper(const double *R, int64_t M, int trans, double *B, int t)
{
    if (!trans) {
        for (int64_t i = M - 1; i >= 0; --i)
            for (int c = 0; c < t; ++c) {
                double s = B[i * t + c];
                for (int64_t j = i + 1; j < M; ++j) s -= R[i * M + j] * B[j * t + c];
                B[i * t + c] = s / R[i * M + i];
            }
    } else {
        for (int64_t i = 0; i < M; ++i)
            for (int c = 0; c < t; ++c) {
                double s = B[i * t + c];
                for (int64_t j = 0; j < i; ++j) s -= R[j * M + i] * B[j * t + c];
                B[i * t + c] = s / R[i * M + i];
            }
    }
}

/* Preconditioner of Alg. 1:  K = k(C, C) + jitter I;  T = chol(K);
 * G = T T^T / M + lambda I;  A = chol(G).  T and A are M x M row-major outputs.
 * Returns 0, or +p if the first factorisation fails at pivot p (1-based), or -p for
 * the second. */
int64_t orc_precond(const float *C, int64_t M, int d, int64_t ldc, double sigma,
                    double lambda, double jitter, double *T, double *A)
{
    orc_kernel_matrix(C, M, d, ldc, C, M, ldc, sigma, T);
    for (int64_t i = 0; i < M; ++i) T[i * M + i] += jitter;
    int64_t info = orc_chol_upper(T, M);
    if (info) return info;
    /* G[i, j] = (1/M) sum_k T[i, k] T[j, k]; T upper, so k >= max(i, j) */
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = i; j < M; ++j) {
            double s = 0.0;
            for (int64_t k = j; k < M; ++k) s += T[i * M + k] * T[j * M + k];
            s /= (double)M;
            if (i == j) s += lambda;
            A[i * M + j] = s;
            A[j * M + i] = s;
        }
    info = orc_chol_upper(A, M);
    return info ? -info : 0;
}

/* Preconditioned operator of Eq. 9:
 *   out = A^-T ( T^-T K_nm^T K_nm T^-1 A^-1 beta + lambda n A^-1 beta ).
 * beta, out: M x t.  work_w: n x t, work_m: 2 * M * t doubles. */
void orc_linop(const float *X, int64_t n, int d, int64_t ldx,
               const float *C, int64_t M, int64_t ldc, double sigma, double lambda,
               const double *T, const double *A, const double *beta, int t,
               double *work_w, double *work_m, double *out)
{
    double *v = work_m;          /* A^-1 beta */
    double *z = work_m + M * t;  /* T^-1 v    */
    memcpy(v, beta, sizeof(double) * M * t);
    orc_solve_upper(A, M, 0, v, t);
    memcpy(z, v, sizeof(double) * M * t);
    orc_solve_upper(T, M, 0, z, t);
    orc_knm_prod(X, n, d, ldx, C, M, ldc, sigma, z, t, work_w, out);
    orc_solve_upper(T, M, 1, out, t);
    for (int64_t k = 0; k < M * t; ++k) out[k] += lambda * (double)n * v[k];
    orc_solve_upper(A, M, 1, out, t);
}

/* Falkon, Alg. 1, with the centres C given by the caller:
 *   rhs = A^-T T^-T K_nm^T Y;   beta = CG(linop, rhs, iters) from beta_0 = 0
 *   (Hestenes-Stiefel, exactly `iters` steps, one step size per column);
 *   alpha = T^-1 A^-1 beta.
 * Y: n x t, alpha: M x t, resid (optional): (iters + 1) x t residual 2-norms.
 * Returns the preconditioner's status (see orc_precond). */
int64_t orc_falkon_fit(const float *X, int64_t n, int d, int64_t ldx,
                       const double *Y, int t,
                       const float *C, int64_t M, int64_t ldc,
                       double sigma, double lambda, double jitter, int iters,
                       double *alpha, double *resid)
{
    double *T = malloc(sizeof(double) * M * M);
    double *A = malloc(sizeof(double) * M * M);
    double *W = malloc(sizeof(double) * n * t);
    double *wm = malloc(sizeof(double) * 2 * M * t);
    double *beta = calloc(M * t, sizeof(double));
    double *r = malloc(sizeof(double) * M * t);
    double *p = malloc(sizeof(double) * M * t);
    double *q = malloc(sizeof(double) * M * t);
    double *rho = malloc(sizeof(double) * t);
    int64_t info = orc_precond(C, M, d, ldc, sigma, lambda, jitter, T, A);
    if (info == 0) {
        orc_knm_t_w(X, n, d, ldx, C, M, ldc, sigma, Y, t, r);
        orc_solve_upper(T, M, 1, r, t);
        orc_solve_upper(A, M, 1, r, t);
        memcpy(p, r, sizeof(double) * M * t);
        for (int c = 0; c < t; ++c) {
            double s = 0.0;
            for (int64_t k = 0; k < M; ++k) s += r[k * t + c] * r[k * t + c];
            rho[c] = s;
            if (resid) resid[c] = sqrt(s);
        }
        for (int it = 0; it < iters; ++it) {
            orc_linop(X, n, d, ldx, C, M, ldc, sigma, lambda, T, A, p, t, W, wm, q);
            for (int c = 0; c < t; ++c) {
                double pq = 0.0;
                for (int64_t k = 0; k < M; ++k) pq += p[k * t + c] * q[k * t + c];
                double a = (pq != 0.0) ? rho[c] / pq : 0.0;
                double rn = 0.0;
                for (int64_t k = 0; k < M; ++k) {
                    beta[k * t + c] += a * p[k * t + c];
                    r[k * t + c] -= a * q[k * t + c];
                    rn += r[k * t + c] * r[k * t + c];
                }
                double b = (rho[c] != 0.0) ? rn / rho[c] : 0.0;
                for (int64_t k = 0; k < M; ++k)
                    p[k * t + c] = r[k * t + c] + b * p[k * t + c];
                rho[c] = rn;
                if (resid) resid[(int64_t)(it + 1) * t + c] = sqrt(rn);
            }
        }
        memcpy(alpha, beta, sizeof(double) * M * t);
        orc_solve_upper(A, M, 0, alpha, t);
        orc_solve_upper(T, M, 0, alpha, t);
    }
    free(T); free(A); free(W); free(wm); free(beta); free(r); free(p); free(q); free(rho);
    return info;
}

/* Predictor of Eq. 4: out = k(Xtest, C) alpha. */
void orc_falkon_predict(const float *Xt, int64_t nt, int d, int64_t ldx,
                        const float *C, int64_t M, int64_t ldc, double sigma,
                        const double *alpha, int t, double *out)
{
    orc_knm_v(Xt, nt, d, ldx, C, M, ldc, sigma, alpha, t, out);
}
