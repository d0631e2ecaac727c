/*
 * knm.h -- C ABI of the MI355X (gfx950) Nystrom kernel-ridge hot path.
 *
 * Implements, on one GPU, the operations of the preconditioned Nystrom kernel ridge
 * solver ("Falkon") of arXiv 2006.10350 with the Gaussian kernel
 *     k(x, c) = exp(-||x - c||^2 / (2 sigma^2))                      (Section 2)
 * for n data points X (n x d), M Nystrom centres C (M x d) and t right-hand sides.
 *
 * Conventions for every entry point
 *  - All array arguments are DEVICE pointers owned by the caller; the library reads or
 *    writes them only during the call's enqueued work and keeps no reference afterwards.
 *    The only host pointers are the out-parameters that say so explicitly.
 *  - Matrices are row-major fp32.  X has leading dimension ldx >= d, C has ldc >= d.
 *    V, U, R, alpha are M x t with leading dimension t; W, Y, out are n x t with
 *    leading dimension t.
 *  - Work is enqueued on the context's HIP stream.  Calls return without synchronising
 *    unless a host value is needed (Cholesky status, CG scalars, timing queries).
 *  - Outputs are overwritten, never accumulated into.
 *  - The product entry points (knm_v, knm_prod, knm_prod_weighted, knm_t_y, falkon_predict) allocate
 *    only when the library-owned workspace has to grow; a repeated call with the same shapes only
 *    enqueues kernels (no memset or copy nodes, no synchronisation), so it can be captured into a
 *    HIP graph on the context's stream.  The solver entry points allocate and synchronise.
 *  - Return value: KNM_OK (0) or a negative knm_status.  No exception crosses the ABI.
 *  - Indices are 64-bit; n * d and n * M may exceed 2^32.
 *  - Results are deterministic: partial sums are merged in a fixed order (no atomics).
 */
#ifndef KNM_H
#define KNM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KNM_OK = 0,
    KNM_INVALID_ARG = -1, /* null pointer, non-positive size, sigma <= 0, lambda < 0, ld < d */
    KNM_UNSUPPORTED = -2, /* shape outside what the kernels were compiled for (see knm_max_*) */
    KNM_ALLOC = -3,       /* workspace allocation failed */
    KNM_HIP_ERROR = -4,   /* a HIP runtime call or kernel launch failed; text via knm_last_error */
    KNM_NOT_PD = -5       /* a Cholesky factorisation met a non-positive pivot */
} knm_status;

typedef struct knm_ctx knm_ctx;         /* device, stream, library-owned workspace */
typedef struct knm_precond knm_precond; /* fp64 factors T, A of the preconditioner  */

/* Create a context on HIP device `device`.  `hip_stream` is a hipStream_t passed as
 * void* (NULL = the default stream); the caller keeps ownership of the stream. */
int knm_create(knm_ctx **out, int device, void *hip_stream);
int knm_destroy(knm_ctx *ctx);
/* Static description of a status code / text of the last failing runtime call. */
const char *knm_strerror(int status);
const char *knm_last_error(const knm_ctx *ctx);
/* Largest d and t the compiled kernels accept. */
int knm_max_d(void);
int knm_max_t(void);
/* Upper bound on the device bytes of library-owned workspace that the product entry points hold
 * for this shape with the default settings (any arithmetic mode, either kernel function): W when the
 * caller passes none, the partial results of the stream chunks, and the converted operands (points, and
 * for 8 or more columns the vectors) of the split-fp16 engines.  knm_workspace_held: what the context
 * holds now. */
size_t knm_workspace_bytes(int64_t n, int64_t M, int d, int t);
size_t knm_workspace_held(const knm_ctx *ctx);

/* W[n x t] = k(X, C) V  -- the kernel-matrix-vector product k(X1, X2) v of the
 * matrix-vector comparison in the appendix on performance, and the predictor
 * f(x) = sum_j alpha_j k(x, c_j) of Eq. 4. */
int knm_v(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx,
          const float *C, int64_t M, int64_t ldc, float sigma,
          const float *V, int t, float *W);

/* U[M x t] = K_nm^T (K_nm V), the product evaluated once per conjugate-gradient
 * iteration (Section 3.1, "Blockwise K_nm-vector product"); K_nm is never formed.
 * If W_or_null is not NULL it also receives W[n x t] = K_nm V. */
int knm_prod(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx,
             const float *C, int64_t M, int64_t ldc, float sigma,
             const float *V, int t, float *W_or_null, float *U);

/* knm_prod for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments and result as knm_prod, except that
 * W (n x t) must be given.  The call allocates nothing: the chunk partials, the common shift and the
 * converted operands of the split-fp16 engines live in a static device array of
 * knm_static_scratch_bytes() bytes (64 MiB) that every GPU the library runs on holds until the process
 * ends.  Shapes whose sweeps do not fit that array (the packed operands are cut into slabs, so this is
 * mostly the partials: chunks x M x t floats) are rejected with KNM_UNSUPPORTED and the text of
 * knm_last_error says so.  All calls on one GPU share the array: calls that overlap on one GPU (other
 * streams, other contexts, other threads) race; calls on one stream are ordered.  Nothing in the
 * array needs to start at zero (every word read by a call was written by it first). */
int knm_prod_static(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx,
                    const float *C, int64_t M, int64_t ldc, float sigma,
                    const float *V, int t, float *W, float *U);
size_t knm_static_scratch_bytes(void);

/* U[M x t] = K_nm^T diag(dw) K_nm V with dw[n] >= 0: the product inside LinOp of the
 * weighted solver for generalised self-concordant losses (Alg. 2, WeightedFalkon). */
int knm_prod_weighted(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx,
                      const float *C, int64_t M, int64_t ldc, float sigma,
                      const float *dw, const float *V, int t, float *U);

/* The same product for sparse inputs (Sec. 4, "Dealing with sparse datasets"): X (n rows) and C
 * (M rows) in CSR form over d features, d < 2^31 - 1.
 *   x_indptr[n + 1], c_indptr[M + 1]: row pointers, starting at 0 and non-decreasing;
 *   x_indices, c_indices: feature of every stored entry, in [0, d) and strictly increasing
 *   within a row (canonical CSR: every feature at most once per row); x_values, c_values: fp32.
 * V (M x t), W_or_null (n x t), U (M x t) as for knm_prod.  The structure is checked on the device before it is used
 * (KNM_INVALID_ARG).  Only pairs of points that share a feature are visited: the rest of the
 * kernel matrix is a rank-one matrix and is summed in closed form.  U is accumulated with float
 * atomics, so its last bits can differ from run to run.  All pointers DEVICE; the call
 * returns after the product is complete. */
int knm_prod_csr(knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values, int64_t n,
                 const int64_t *c_indptr, const int64_t *c_indices, const float *c_values, int64_t M, int64_t d,
                 float sigma, const float *V, int t, float *W_or_null, float *U);

/* W[n x t] = k(X, C) V for CSR X and C (the predictor of Eq. 4 on sparse points); arguments as
 * for knm_prod_csr. */
int knm_v_csr(knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values, int64_t n,
              const int64_t *c_indptr, const int64_t *c_indices, const float *c_values, int64_t M, int64_t d,
              float sigma, const float *V, int t, float *W);

/* R[M x t] = K_nm^T Y, the right-hand side of the Nystrom system (Eq. 5; line
 * "R <- ..." of Alg. 1 read as k(X_m, X) y). */
int knm_t_y(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx,
            const float *C, int64_t M, int64_t ldc, float sigma,
            const float *Y, int t, float *R);

/* Preconditioner of Alg. 1 / Eq. 7, all in fp64 on the device:
 *   T = chol_upper(k(C, C) + jitter I),   A = chol_upper(T T^T / M + lambda I),
 * with T^T T = K_MM and A^T A = T T^T / M + lambda I.  The two factors share one array, as in the
 * paper's in-place preconditioner (Sec. 3.1, the paragraph and figure on its memory): T in the
 * upper triangle, the transpose of A two rows below the diagonal (so that neither diagonal is
 * lost); *out owns (M + 3) M doubles of device memory at most, plus M^2 / 8 or so for the
 * inverted diagonal blocks of the blocked solves, until precond_free.  On KNM_NOT_PD, *bad_pivot_or_null (HOST pointer)
 * receives the 1-based failing pivot, negative if it was the second factorisation. */
int precond_build(knm_ctx *ctx, const float *C, int64_t M, int d, int64_t ldc, float sigma,
                  double lambda, double jitter, knm_precond **out, int64_t *bad_pivot_or_null);
int precond_free(knm_precond *p);
/* The same preconditioner for CSR centres (M rows over d features, as for knm_prod_csr): k(C, C) is
 * formed in fp64 from the squared norms and the sparse dot products of the centres. */
int precond_build_csr(knm_ctx *ctx, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values,
                      int64_t M, int64_t d, float sigma, double lambda, double jitter, knm_precond **out,
                      int64_t *bad_pivot_or_null);
/* Copy the factors to HOST buffers of M*M doubles each (row-major, upper triangular,
 * strict lower triangle zero); either may be NULL.  For tests and inspection. */
int precond_get_factors(knm_ctx *ctx, const knm_precond *p, double *T_host, double *A_host);
/* Copy the block [row0, row0 + rows) x [col0, col0 + cols) of T (second == 0) or A (second != 0)
 * to a HOST buffer of rows*cols doubles (row-major; entries below the factor's diagonal are
 * zero).  For inspecting factors too large to copy whole. */
int precond_get_block(knm_ctx *ctx, const knm_precond *p, int second, int64_t row0, int64_t col0, int64_t rows,
                      int64_t cols, double *out_host);

/* Preconditioned operator of Eq. 9 applied to beta (M x t, fp64 DEVICE pointers):
 *   out = A^-T ( T^-T K_nm^T K_nm T^-1 A^-1 beta + lambda n A^-1 beta ). */
int falkon_linop(knm_ctx *ctx, const knm_precond *p,
                 const float *X, int64_t n, int d, int64_t ldx,
                 const float *C, int64_t M, int64_t ldc, float sigma, double lambda,
                 const double *beta, int t, double *out);

/* Symmetric rank-k update of the upper triangle of C (n x n, column-major, leading dimension
 * ldc) in fp64 on the matrix cores: the trailing-matrix step of the block Cholesky column
 * update (Sec. 4, block Cholesky paragraph, third step; appendix on out-of-core algorithms)
 * and the triangular product T diag(w) T^T of the preconditioner (Alg. 1; Alg. 2,
 * WeightedPreconditioner):
 *   C[i, j] = alpha sum_{q < k} w[q] a(i, q) a(j, q) + beta C[i, j] + shift [i == j],   i <= j < n
 *   form_nt == 0:  a(i, q) = A[q + i lda]  (A is k x n)      form_nt != 0:  a(i, q) = A[i + q lda]  (A is n x k)
 * w_or_null: k weights or NULL (all one).  triangular != 0 (form_nt only): A is upper
 * triangular (a(i, q) is taken as 0 for q < i, whatever is stored there), and the part of
 * the sum that vanishes is skipped.  The strict lower triangle of C is neither read nor written; with
 * beta == 0 C is not read.  A must not overlap the upper triangle of C.  All pointers DEVICE,
 * the call is asynchronous on the context's stream. */
int precond_rank_k_update(knm_ctx *ctx, int form_nt, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                          const double *w_or_null, int triangular, double beta, double shift, double *C, int64_t ldc);

/* General fp64 block product on the matrix cores, the building block of the first two steps of the
 * block Cholesky column update (Sec. 4, block Cholesky paragraph: factor the diagonal tile, solve
 * the block row against it) when they are carried out with products by inverted diagonal blocks:
 *   C[i, j] = alpha sum_{q < k} a(i, q) b(j, q) + beta C[i, j],   i < ni, j < nj
 *   a(i, q) = A[q + i lda] (a_nt == 0, A is k x ni) or A[i + q lda] (a_nt != 0, A is ni x k);  b(j, q) = B[q + j ldb]
 * i.e. C = alpha A^T B + beta C or C = alpha A B + beta C for column-major A, B (k x nj), C (ni x nj).
 * C must not overlap A or B; with beta == 0 C is not read.  All pointers DEVICE, asynchronous on
 * the context's stream. */
int precond_block_product(knm_ctx *ctx, int a_nt, int64_t ni, int64_t nj, int64_t k, double alpha, const double *A,
                          int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc);

/* The two triangular solves that take the preconditioned unknown to the coefficients (last
 * step of Alg. 1, alpha = T^-1 A^-1 beta) or a right-hand side into the preconditioned system
 * (its first step, A^-T T^-T r):
 *   transpose == 0:  out = T^-1 A^-1 b        transpose != 0:  out = A^-T T^-T b
 * b, out: M x t row-major fp64 DEVICE pointers, may alias; 1 <= t <= knm_max_t().  Solves on one
 * preconditioner share its staging vector: issue them from one context at a time. */
int precond_solve(knm_ctx *ctx, const knm_precond *p, int transpose, const double *b, int t, double *out);

/* The same operator with the weighted product (LinOp of Alg. 2, WeightedFalkon):
 *   out = A^-T ( T^-T K_nm^T diag(dw) K_nm T^-1 A^-1 beta + lambda n A^-1 beta ),
 * dw[n] >= 0 fp32 DEVICE pointer, NULL for the identity. */
int falkon_linop_weighted(knm_ctx *ctx, const knm_precond *p,
                          const float *X, int64_t n, int d, int64_t ldx,
                          const float *C, int64_t M, int64_t ldc, float sigma, double lambda,
                          const float *dw_or_null, const double *beta, int t, double *out);

/* Second factor of the weighted preconditioner (Alg. 2, WeightedPreconditioner), rebuilt in
 * place from the first:  A = chol_upper(T diag(dw) T^T / M + lambda I), dw[M] >= 0 fp64 DEVICE
 * pointer (NULL for the identity, which gives precond_build's A for the new lambda).  T, which
 * depends on the centres only, is kept.  On KNM_NOT_PD the factor is unusable until the next
 * successful call; *bad_pivot_or_null (HOST) receives minus the 1-based failing pivot. */
int precond_reweight(knm_ctx *ctx, knm_precond *p, double lambda, const double *dw_or_null,
                     int64_t *bad_pivot_or_null);

/* Falkon (Alg. 1) with the centres given by the caller: builds the preconditioner,
 * forms rhs = A^-T T^-T K_nm^T Y, runs exactly `iters` conjugate-gradient steps on the
 * operator of Eq. 9 from beta = 0 (one step size per column of Y), and writes
 * alpha[M x t] = T^-1 A^-1 beta (fp32).  resid_norms_or_null is a HOST buffer of
 * (iters + 1) * t doubles receiving the residual 2-norm of every column before the
 * first and after each step. */
int falkon_fit(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx,
               const float *Y, int t, const float *C, int64_t M, int64_t ldc,
               float sigma, double lambda, double jitter, int iters,
               float *alpha, double *resid_norms_or_null);

/* falkon_fit for CSR X (n rows) and CSR centres (M rows) over d features (Sec. 4, "Dealing with
 * sparse datasets"); CSR arguments as for knm_prod_csr, everything else as for falkon_fit. */
int falkon_fit_csr(knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values, int64_t n,
                   const float *Y, int t, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values,
                   int64_t M, int64_t d, float sigma, double lambda, double jitter, int iters, float *alpha,
                   double *resid_norms_or_null);

/* Approximate Newton method for the logistic loss l(z, y) = log(1 + exp(-y z)), y = +-1
 * (Appendix "Logistic Falkon Algorithm", Alg. 2).  The schedule of regularisers is not given in
 * the paper: Newton step k uses lambdas[k] and iters[k] conjugate-gradient iterations (HOST
 * arrays of n_steps entries).  Reading of Alg. 2: the objective is
 *   J(alpha) = 1/n sum_i l((K_nm alpha)_i, y_i) + lambda/2 alpha^T (K_MM + jitter I) alpha,
 * and step k, from alpha_k with g = l', D = diag l'' at K_nm alpha_k, runs CG from zero on
 *   P^T (K_nm^T D K_nm + lambda n (K_MM + jitter I)) P beta
 *        = -P^T (K_nm^T g + lambda n (K_MM + jitter I) alpha_k),      P = T^-1 A^-1,
 * with the weighted preconditioner T^T T = K_MM + jitter I, A^T A = T Dm T^T / M + lambda I,
 * Dm = diag l''((K_MM alpha_k)_j, yC_j); then alpha_{k+1} = alpha_k + P beta, from alpha_0 = 0.
 * y[n], yC[M] (labels of the rows and of the centres) and alpha[M] are fp32 DEVICE pointers;
 * loss_or_null is a HOST buffer of n_steps + 1 doubles receiving the mean loss before each
 * step and after the last. */
int logfalkon_fit(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *y,
                  const float *C, int64_t M, int64_t ldc, const float *yC, float sigma,
                  const double *lambdas, const int *iters, int n_steps, double jitter,
                  float *alpha, double *loss_or_null);

/* logfalkon_fit for CSR X (n rows) and CSR centres (M rows) over d features: the same Newton
 * iteration on the sparse sweeps (Alg. 2 with the products of Sec. 4, "Dealing with sparse
 * datasets"); CSR arguments as for knm_prod_csr, everything else as for logfalkon_fit. */
int logfalkon_fit_csr(knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values,
                      int64_t n, const float *y, const int64_t *c_indptr, const int64_t *c_indices,
                      const float *c_values, int64_t M, int64_t d, const float *yC, float sigma,
                      const double *lambdas, const int *iters, int n_steps, double jitter, float *alpha,
                      double *loss_or_null);

/* Wall-clock seconds of the phases of the most recent successful falkon_fit on this context,
 * written to the HOST array seconds[4]: [0] preconditioner, [1] right-hand side
 * (K_nm^T Y and two solves), [2] all conjugate-gradient iterations, [3] final solves. */
int knm_get_fit_timing(const knm_ctx *ctx, double *seconds);

/* out[ntest x t] = k(Xtest, C) alpha  (Eq. 4). */
int falkon_predict(knm_ctx *ctx, const float *Xtest, int64_t ntest, int d, int64_t ldx,
                   const float *C, int64_t M, int64_t ldc, float sigma,
                   const float *alpha, int t, float *out);

/* Arithmetic of the cross term <x, c> inside the kernel evaluation:
 *   KNM_CROSS_F16X3 (default) each feature, scaled by sqrt(log2 e)/sigma, is split into two
 *                   fp16 halves (22 significant bits) and the product is evaluated as
 *                   hi*hi + hi*lo + lo*hi on the f16 matrix cores with fp32 accumulation; the
 *                   norms are carried as exact fixed-point digits.  Same accuracy class as
 *                   fp32 (the dropped lo*lo term is ~2^-22 per feature; measured ~4e-7
 *                   relative L2 against the fp64 oracle).  Scaled features beyond 65000 in
 *                   magnitude and squared norms of scaled points beyond 2^22 saturate.  Uses a
 *                   library-owned workspace for the converted operands: at most 2 GiB for
 *                   d <= 44 with t = 1, at most 8 GiB otherwise.
 *   KNM_CROSS_F32   fp32 MFMA on the unsplit features: no range limits, 3 to 5 times slower
 *                   (fp32 MFMA and the exp/FMA work share the vector ALU's issue). */
typedef enum { KNM_CROSS_F32 = 0, KNM_CROSS_F16X3 = 1 } knm_cross_term;
int knm_set_cross_term(knm_ctx *ctx, int mode);
int knm_get_cross_term(const knm_ctx *ctx); /* the mode now selected, or KNM_INVALID_ARG */

/* Kernel function of the dense entry points (further kernel families on the same engines; the
 * paper's experiments use the Gaussian kernel throughout), with r = |x - c|:
 *   KNM_KERNEL_GAUSSIAN (default)  k = exp(-r^2 / (2 sigma^2))
 *   KNM_KERNEL_LAPLACIAN           k = exp(-r / sigma)
 *   KNM_KERNEL_MATERN32            k = (1 + u) exp(-u),            u = sqrt(3) r / sigma
 *   KNM_KERNEL_MATERN52            k = (1 + u + u^2 / 3) exp(-u),  u = sqrt(5) r / sigma
 * The kernels of r (all but the Gaussian) run on the K-loop engines for every shape: the matrix
 * cores accumulate -(log2(e) u)^2 from the norm expansion (u = r / sigma for the Laplacian kernel),
 * then one square root, one exp2 and the polynomial per entry.  The root magnifies the
 * cancellation error of the expansion for close pairs (every Nystrom centre coincides with a data
 * row), so pairs closer than a threshold derived from the points' norms are evaluated again from
 * fp32 differences of the two rows: the result keeps the accuracy of the Gaussian kernel.  That
 * second evaluation is rare as long as the points' distances from the mean of the centres (the
 * engines expand around it) are not many times sigma; where they are, most pairs take it and the
 * sweep slows down accordingly.  The preconditioner's k(C, C) is formed from fp64
 * differences.  The sparse (CSR) entry points support the Gaussian kernel only and return
 * KNM_UNSUPPORTED otherwise. */
typedef enum {
    KNM_KERNEL_GAUSSIAN = 0,
    KNM_KERNEL_LAPLACIAN = 1,
    KNM_KERNEL_MATERN32 = 2,
    KNM_KERNEL_MATERN52 = 3
} knm_kernel_kind;
int knm_set_kernel(knm_ctx *ctx, int kind);

/* Sparse (CSR) entry points: the features that occur in the largest share of the centres (at most
 * max_features of them, capped at 128; 0 switches this off; default 128) are taken out of the sparse
 * walk and handled by one dense product over those features, when that is estimated to be cheaper.
 * The result is the same kernel product up to rounding. */
int knm_set_sparse_head_limit(knm_ctx *ctx, int max_features);

/* Cap, in bytes, on the library-owned workspace that holds the converted operands of the
 * split-fp16 engines (0 restores the defaults: 2 GiB, or 8 GiB for the K-loop engine).  Operands
 * that do not fit are converted and swept slab by slab; results do not depend on the cap.  The
 * workspace never shrinks below what one slab needs (one stream chunk, plus the whole smaller
 * operand for the K-loop engine). */
int knm_set_pack_limit(knm_ctx *ctx, size_t bytes);

/* Range check of the split-fp16 cross term (KNM_CROSS_F16X3, the default).  Its operands hold scaled
 * features z = (x - shift) sqrt(log2 e) / sigma up to |z| = 65000 and norm terms |z|^2 / 2 below 2^21 (a
 * point about 1700 sigma from the bulk of the data); beyond that, and for features that are not finite,
 * the conversion clamps, and the kernel values of such a point are wrong wherever they are not zero
 * anyway.  Every clamped conversion of a point is counted on the device.  knm_range_exceeded waits for
 * the stream, writes the count since the last reset to the HOST pointer (several sweeps may convert
 * the same point, so only zero or non-zero is meaningful: 0 means no operand was clamped), and
 * clears it if reset != 0.  The product entry points do not synchronise and therefore cannot report
 * it themselves: check here, and repeat with knm_set_cross_term(KNM_CROSS_F32), which clamps nothing
 * and lets NaNs through (its exponent still carries about 1e-7 of the norm terms as rounding error, so
 * pairs of close points that far out are inaccurate in either mode).  falkon_fit, falkon_fit_csr and the logistic fits check after their first sweep and run the
 * whole fit with the fp32-MFMA cross term if anything was clamped. */
int knm_range_exceeded(knm_ctx *ctx, int64_t *count_host, int reset);

/* Timing aid for benchmarks: when enabled, knm_v / knm_prod / knm_t_y bracket their
 * kernels with HIP events on the context's stream.  knm_get_timing synchronises the
 * stream and writes milliseconds of the most recent call to the HOST array ms[4]:
 * [0] row sweep (W = K V), [1] column sweep (K^T W partials), [2] merge of partials,
 * [3] whole call.  Phases a call did not run are reported as 0. */
int knm_set_timing(knm_ctx *ctx, int enabled);
int knm_get_timing(knm_ctx *ctx, float *ms);

/* Measurement aid for benchmarks (not part of the method): sustained rates of the instructions the
 * tile engines are made of, measured on the context's device with register-resident loops at the
 * engines' occupancy (2 wavefronts per SIMD, all compute units), so that a roofline can be stated
 * against what the chip sustains as well as against its nominal peaks.  Writes KNM_PROBE_COUNT
 * doubles to the HOST array rates_host (count = its length); allocates two small device buffers,
 * takes about 0.5 s, and synchronises the stream. */
typedef enum {
    KNM_PROBE_MFMA_F32_TFLOPS = 0,        /* v_mfma_f32_32x32x2_f32, 4 independent chains               */
    KNM_PROBE_MFMA_F16_CONST_TFLOPS = 1,  /* v_mfma_f32_32x32x16_f16 on constant operands               */
    KNM_PROBE_MFMA_F16_RANDOM_TFLOPS = 2, /* the same on random operands (data-dependent power limit)   */
    KNM_PROBE_EXP_TOPS = 3,               /* v_exp_f32 back to back, 1e12 lane results per second       */
    KNM_PROBE_FMA_TOPS = 4,               /* v_fmac_f32, 1e12 lane results per second                   */
    /* One pair of 32 x 32 tiles of the split-fp16 register-resident engine (per wavefront 6 HU f16
     * MFMAs + 32 exp + 32 FMA in the engine's order; HU = 1, 2, 3 for d <= 12, 28, 44), random
     * operands, in nominal 2.4 GHz clocks per SIMD and tile pair: both pipes, the vector-ALU
     * instructions alone, the matrix-core instructions alone. */
    KNM_PROBE_MIX1_BOTH_CLK = 5, KNM_PROBE_MIX1_VALU_CLK = 6, KNM_PROBE_MIX1_MFMA_CLK = 7,
    KNM_PROBE_MIX2_BOTH_CLK = 8, KNM_PROBE_MIX2_VALU_CLK = 9, KNM_PROBE_MIX2_MFMA_CLK = 10,
    KNM_PROBE_MIX3_BOTH_CLK = 11, KNM_PROBE_MIX3_VALU_CLK = 12, KNM_PROBE_MIX3_MFMA_CLK = 13,
    KNM_PROBE_COUNT = 14
} knm_probe_rate;
int knm_probe_rates(knm_ctx *ctx, double *rates_host, int count);

#ifdef __cplusplus
}
#endif
#endif /* KNM_H */
