// Internal declarations shared by the HIP sources of libknm (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "knm.h"

namespace knm {

// ---- tile engine (knm_tile.hip) ---------------------------------------------------
//
// One engine serves both sweeps of K_nm^T (K_nm v) because the Gaussian kernel is
// symmetric in its two arguments:
//   out[f] = sum_s k(F_f, S_s) * vec[s]
// with "fixed" points F held in registers as the MFMA A operand and "stream" points S
// staged through LDS as the B operand.  Row sweep: F = X, S = C, vec = v.  Column
// sweep: F = C, S = X, vec = w, with the stream cut into chunks whose partial results
// are merged afterwards in a fixed order.
struct SweepArgs {
    const float *F;   // fixed points, nF x d, leading dimension ldf
    int64_t nF, ldf;
    const float *S;   // stream points, nS x d, leading dimension lds
    int64_t nS, lds;
    int d;
    // common shift of both point sets, d floats: the engines work with F - mu and S - mu (the kernels
    // depend on differences only), which keeps the norm terms of the expansion small for data that
    // is not centred; mu[d] != 0 says that the shift is not all zero
    const float *mu;
    const float *vec; // stream-side vectors: column c of stream point i is vec[i * ldv + c]
    int64_t ldv;
    int t;            // columns handled by this launch (1 for the register-resident engine)
    const float *wgt; // optional per-stream-point weight multiplied into vec (may be null)
    float *out;       // out[chunk * chunk_stride + f * ldo + c]
    // K-loop engines only: if not null the results go here instead, same indexing, in fp64 (the
    // register-resident engines ignore it and must be given `out`)
    double *out64 = nullptr;
    int64_t ldo, chunk_stride;
    int64_t chunk_len; // stream points per chunk (multiple of the stage size)
    int64_t n_chunks;
    // split-fp16 engines: incremented once per converted point whose scaled features or norm term lie
    // outside what the fp16 operands represent (|z| > 65000, |z|^2 / 2 >= 2^21, or not finite) and
    // were clamped; never null
    unsigned int *range_count;
    float sigma;      // length scale the engines work with (for the Laplacian kernel the caller's, rescaled)
    int kind;         // knm_kernel_kind (the kernels of r = |x - c|: K-loop engines only)
    // K-loop split-fp16 engine, reduction on the matrix cores: room of gemm_f16_vector_image_bytes() for the
    // vectors converted once per sweep into the layout of the LDS stage; null = every workgroup converts
    // the rows of its tiles itself
    void *vimg = nullptr;
};

// ---- kernels of r = |x - c| (Laplacian, Matern) on the K-loop engines ---------------------
//
// The engines' accumulators hold x = -s2 |f - s|^2 (s2 = log2(e) / (2 sigma^2) of the rescaled
// sigma), formed as norms minus cross term; the kernel value is 2^-sqrt(|x|).  The cancellation
// leaves an absolute error of about 1e-7 sqrt(d) N in x (N = s2 |f|^2, the norm in the same units),
// which the square root turns into error / (2 sqrt(|x|)): harmless for ordinary pairs, but 1e-4 to
// 1e-3 for coincident or nearly coincident ones, and every Nystrom centre coincides with a data
// row.  Pairs whose |x| lies below the threshold at which that error reaches about 1e-5 get their
// exponent again from fp32 differences of the two rows (exact for coincident rows, relative
// rounding error otherwise).  Such pairs are rare, so the branch is almost never taken.
__device__ __forceinline__ float near_pair_threshold(float norm_term, int d)
{
    // relative part: 1e-7 sqrt(d) N of rounding in the fp32 accumulation, at least the 2.4e-7 N that
    // the split-fp16 product leaves out; absolute part: the 2^-24 to which that engine's norm slots
    // are rounded
    const float N = fabsf(norm_term);
    return fmaxf(fmaxf(2.5e-5f * (float)d, 2.5e-4f) * N * N, 1.0e-5f);
}
__device__ __forceinline__ float exact_exponent(const float *__restrict__ f, const float *__restrict__ s, int d,
                                                float s2)
{
    float q = 0.0f;
    for (int k = 0; k < d; ++k) {
        const float diff = f[k] - s[k];
        q = fmaf(diff, diff, q);
    }
    return -s2 * q;
}
// kernel value from the exponent x = -(log2(e) u)^2 held by the accumulators
template <int KIND>
__device__ __forceinline__ float radial_from_exponent(float x)
{
    const float y = __builtin_amdgcn_sqrtf(fabsf(x)); // log2(e) u
    const float e = __builtin_amdgcn_exp2f(-y);
    if constexpr (KIND == KNM_KERNEL_LAPLACIAN) return e;
    const float u = y * 0.6931471805599453f;
    if constexpr (KIND == KNM_KERNEL_MATERN32) return fmaf(u, e, e);
    return e * fmaf(u, fmaf(u, 1.0f / 3.0f, 1.0f), 1.0f); // KNM_KERNEL_MATERN52
}

// register-resident engine (knm_tile.hip): d <= small_max_d(), one column per launch
int small_max_d();
int64_t stage_points();                 // stream points staged per LDS buffer
int64_t fixed_per_block(int d);         // fixed points one workgroup covers
hipError_t launch_sweep(const SweepArgs &a, hipStream_t stream);
// same shapes with the cross term as three f16 MFMA products (knm_tile_f16.hip): d <= f16_max_d()
int f16_max_d();
int f16_radial_max_d(); // the same for the kernels of r = |x - c|
int64_t f16_stage_points(int d, int kind); // stream points staged per LDS buffer by that engine
size_t f16_pack_bytes_per_point(int d);
// pack_buf: device workspace for the packed stream image, at least one chunk's worth
hipError_t launch_sweep_f16(const SweepArgs &a, void *pack_buf, size_t pack_bytes, hipStream_t stream);
// K-loop engine (knm_gemm.hip): any d, up to gemm_max_t() columns per launch
int gemm_max_t();
bool gemm_leading_dimension_ok(int64_t ld); // leading dimensions the fp32 K-loop engine can index
int64_t gemm_stage_points();
int64_t gemm_fixed_per_block();
hipError_t launch_sweep_gemm(const SweepArgs &a, hipStream_t stream);
// the same shapes with the cross term as three f16 MFMA products (knm_gemm_f16.hip); both
// operands are packed into the workspace, whole or slab by slab
size_t gemm_f16_pack_bytes_per_point(int d);
size_t gemm_f16_head_bytes(); // bytes of the workspace in front of the images
int gemm_f16_max_t(int kind); // columns per launch at most
int gemm_f16_group_t(int d, int t_left, int kind, bool with_vector_image); // columns the next launch should take
// bytes of the packed vector image of a launch with t columns over nS_padded stream points (0: no such image)
size_t gemm_f16_vector_image_bytes(int d, int t, int64_t nS_padded);
size_t gemm_f16_min_pack_bytes(int64_t nF, int64_t nS_padded, int64_t chunk_len, int d);
hipError_t launch_sweep_gemm_f16(const SweepArgs &a, void *pack_buf, size_t pack_bytes, hipStream_t stream);
// out[j * ldo] = sum over chunks of part[chunk * chunk_stride + j * ldp], summed in fp64 in a fixed
// order; the partials are fp32 or (part64) fp64, the result goes to `out` or, if not null, to `out64`
hipError_t launch_merge(const float *part, const double *part64, int64_t n_chunks, int64_t chunk_stride, int64_t ldp,
                        float *out, double *out64, int64_t ldo, int64_t count, hipStream_t stream);

// fp64 rank-k update of the upper triangle of C on the matrix cores (knm_dsyrk.hip):
//   C[i, j] = alpha sum_{k < K} w[k] a(i, k) a(j, k) + beta C[i, j] + shift [i == j],  i <= j < n,
// a(i, k) = A[k + i lda] (form_nt = 0) or A[i + k lda] (form_nt = 1); w may be null; with tri the
// operand is upper triangular (a(i, k) taken as 0 for k < i whatever is stored there) and the zero part
// of the contraction is skipped; with trans_c entry (i, j) goes to C[j + i ldc] (the lower triangle)
hipError_t launch_rank_k_upper(int form_nt, int64_t n, int64_t K, double alpha, const double *A, int64_t lda,
                               const double *w, int tri, double beta, double shift, double *C, int64_t ldc,
                               hipStream_t stream, int trans_c = 0);

// general fp64 product on the same kernel: C (ni x nj) = alpha sum_{k < K} a(i, k) b(j, k) + beta C with
// a(i, k) = A[k + i lda] (a_nt = 0) or A[i + k lda] (a_nt = 1) and b(j, k) = B[k + j ldb] (b_nt = 0) or
// B[j + k ldb] (b_nt = 1, only with a_nt = 1); C must not overlap A or B, except that a tile of C may be
// exactly the operand rows it reads
hipError_t launch_gemm_f64(int a_nt, int64_t ni, int64_t nj, int64_t K, double alpha, const double *A, int64_t lda,
                           const double *B, int64_t ldb, double beta, double *C, int64_t ldc, hipStream_t stream,
                           int b_nt = 0);

// Sparse inputs (knm_sparse.hip): the two sweeps of one (X, C, sigma) for CSR X and C, prepared once
// (structure check, norms, centre lists per feature, accumulators) and then applied any number
// of times; and the fp64 kernel matrix of CSR centres for the preconditioner.
struct SparseProducts {
    struct Impl;
    Impl *impl;
    SparseProducts();
    ~SparseProducts();
    SparseProducts(const SparseProducts &) = delete;
    SparseProducts &operator=(const SparseProducts &) = delete;
    int prepare(struct ::knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values, int64_t n,
                const int64_t *c_indptr, const int64_t *c_indices, const float *c_values, int64_t M, int64_t d,
                float sigma);
    int v(const float *V, int t, float *W);                       // W (n x t) = K V
    int t_w(const float *W, const float *wgt, int t, float *U);   // U (M x t) = K^T (wgt .* W)
};
int sparse_kmm(struct ::knm_ctx *ctx, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values, int64_t M,
               int64_t d, float sigma, double jitter, double *K, int64_t ldk);

} // namespace knm

struct knm_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    // workspace grown on demand and kept until knm_destroy
    float *w_buf = nullptr;
    size_t w_bytes = 0;
    float *part_buf = nullptr;
    size_t part_bytes = 0;
    float *mu_buf = nullptr;   // common shift of the two point sets of a sweep (d floats)
    size_t mu_bytes = 0;
    float *pack_buf = nullptr; // packed operand images of the split-fp16 engines
    size_t pack_bytes = 0;
    float *vimg_buf = nullptr; // packed vector image of the K-loop split-fp16 engine's matrix-core reduction
    size_t vimg_bytes = 0;
    size_t pack_limit = 0;     // cap on the image workspace chosen by the caller; 0 = engine defaults
    unsigned int *range_count = nullptr; // device word: operands the split-fp16 engines had to clamp (see SweepArgs)
    // this device's copy of the library's static scratch array (address looked up at knm_create), and
    // the state of a call that draws its workspace from it instead of allocating
    unsigned char *static_ws = nullptr;
    bool static_mode = false;
    size_t static_used = 0;
    int cross_term = KNM_CROSS_F16X3;
    int kernel_kind = KNM_KERNEL_GAUSSIAN;
    // sparse inputs: most frequent features treated densely, at most (0: none)
    int sparse_head_max = 128;
    // timing
    bool timing = false;
    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    bool ev_used[5] = {false, false, false, false, false};
    double fit_seconds[4] = {0.0, 0.0, 0.0, 0.0}; // last falkon_fit: preconditioner, rhs, iterations, tail
    std::string last_error;
    // partial sums of the solver's fp64 reductions (allocated lazily by knm_solver.hip)
    double *red_buf = nullptr;
    // second stream for the look-ahead of the blocked factorisation (created lazily by knm_solver.hip)
    hipStream_t aux_stream = nullptr;
};

namespace knm {
// Named range for profilers (rocprofv3 --marker-trace): the phases of a product or fit.  The marker
// library (librocprofiler-sdk-roctx.so, or libroctx64.so) is looked up at run time the first time a
// range opens, and only if the environment variable KNM_MARKERS is set to a non-empty value other
// than 0: libknm itself links the HIP runtime only, and a range costs nothing otherwise.
struct TraceRange {
    explicit TraceRange(const char *name);
    ~TraceRange();
    TraceRange(const TraceRange &) = delete;
    TraceRange &operator=(const TraceRange &) = delete;
    bool open;
};
int ensure(knm_ctx *ctx, float **buf, size_t *cur, size_t need);
int fail(knm_ctx *ctx, int status, const char *what, hipError_t e = hipSuccess);
// true if (d, t) runs on the K-loop engine, false for the register-resident one
bool use_gemm_engine(int d, int t, int cross_term, int kind);
// number of stream chunks for a sweep over nS stream points against nF fixed points
int64_t choose_chunks(int64_t nF, int64_t nS, int d, int t, int cross_term, int kind, int64_t *chunk_len);
int do_knm_v(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M,
             int64_t ldc, float sigma, const float *V, int t, float *W);
// U = K^T (wgt .* W) as fp32 rows (U) or, if U64 is not null, as fp64 rows (M x t, row-major) that
// never pass through fp32 after the merge of the chunk partials
int do_knm_t_w(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M,
               int64_t ldc, float sigma, const float *Wv, const float *wgt, int t, float *U, double *U64 = nullptr);
} // namespace knm
