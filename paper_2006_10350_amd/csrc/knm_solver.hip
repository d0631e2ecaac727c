// Preconditioner, preconditioned operator, conjugate gradient and predictor (Alg. 1).
//
// Everything here is fp64 and runs once per fit or is O(M^2) per iteration; the
// O(n M) work of every iteration is the fp32 kernel product of the sweep engines.
// T and A are upper triangular with T^T T = K_MM + jitter I and A^T A = T T^T / M + lambda I
// (Eq. 7 with K_mm = T^T T).  Both live in ONE column-major array of leading dimension ld = M + 2
// (M + 3 for odd M), as in the paper's in-place preconditioner (Sec. 3.1, the figure of the memory
// layout): T in the upper triangle, T(r, c) at r + c ld, and the transpose of A two rows below the
// diagonal, A(r, c) at 2 + c + r ld (a lower triangle; the two rows keep both diagonals and leave
// every column 16-byte aligned).  Code that works on either factor addresses entry (r, c), r <= c,
// of an upper factor R as base[r + c ld] ("upper storage") or base[c + r ld] ("lower storage").
// The factorisations are the block
// column update of Sec. 4 on the fp64 matrix-core products of knm_dsyrk.hip and a leaf
// kernel; the triangular solves, vector updates and reductions are kernels of this file.
#include <chrono>
#include <cmath>
#include <functional>
#include <new>
#include <type_traits>
#include <vector>

#include "knm_internal.h"

struct knm_precond {
    int device = 0;
    int64_t M = 0;
    double lambda = 0.0, jitter = 0.0;
    double *buf = nullptr; // the shared array, ld x M doubles
    int64_t ld = 0;
    double *T = nullptr;   // = buf: upper storage
    double *A = nullptr;   // = buf + 2: lower storage (what is in memory is A^T, a lower triangle)
    // inverses of the sb x sb diagonal blocks of T and A (column-major blocks, each mirrored onto
    // its lower triangle, the last one padded with the identity), used by the blocked
    // triangular solves; xw (M x kSolveCols entries) stages the solved blocks
    int sb = 0;
    double *Tdinv = nullptr;
    double *Adinv = nullptr;
    double *xw = nullptr;
    // sb x sb doubles for the solves with many right-hand sides (one block inverse with its mirror image
    // cleared); null for small M
    double *blk = nullptr;
};

namespace {

using namespace knm;

// Upper triangle (column-major with leading dimension ldk, r <= c) of K[r, c] = k(c_r, c_c) + jitter [r == c], fp64, direct
// differences: k = exp(-|c_r - c_c|^2 scale) with scale = 1 / (2 sigma^2) for the Gaussian kernel; for the
// kernels of r = |c_r - c_c|, with u = r scale: exp(-u), scale = 1 / sigma (Laplacian);
// (1 + u) exp(-u), scale = sqrt(3) / sigma; (1 + u + u^2 / 3) exp(-u), scale = sqrt(5) / sigma (Matern).  The factorisation reads nothing below the diagonal.
// One workgroup of 16 x 16 threads per 64 x 64 tile on or above the diagonal; thread (tx, ty) owns the entries
// (r0 + tx + 16 i, c0 + ty + 16 j), i, j < 4.  The rows of both sides are staged through LDS 16 features at a
// time as doubles, feature-major, so that the 16 threads of a row of the block read consecutive words; every
// squared distance is summed over the features in their order.
constexpr int kKmmTile = 64;
constexpr int kKmmChunk = 16;
__global__ __launch_bounds__(256) void kmm_kernel(const float *__restrict__ C, int64_t M, int d, int64_t ldc, int kind,
                                                  double scale, double jitter, double *__restrict__ K, int64_t ldk)
{
    if (blockIdx.x > blockIdx.y) return; // tile below the diagonal
    __shared__ double rows_r[kKmmChunk][kKmmTile];
    __shared__ double rows_c[kKmmChunk][kKmmTile];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t r0 = (int64_t)blockIdx.x * kKmmTile, c0 = (int64_t)blockIdx.y * kKmmTile;
    // staging role: row tid / 4 of the tile, features 4 (tid % 4) .. + 3 of the chunk
    const int srow = tid >> 2, sf = (tid & 3) * 4;
    const bool in_r = r0 + srow < M, in_c = c0 + srow < M;
    const float *pr = C + (in_r ? r0 + srow : 0) * ldc;
    const float *pc = C + (in_c ? c0 + srow : 0) * ldc;
    double s[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) s[i][j] = 0.0;
    for (int k0 = 0; k0 < d; k0 += kKmmChunk) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = k0 + sf + e;
            const bool kin = k < d;
            rows_r[sf + e][srow] = (in_r && kin) ? (double)pr[kin ? k : 0] : 0.0;
            rows_c[sf + e][srow] = (in_c && kin) ? (double)pc[kin ? k : 0] : 0.0;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kKmmChunk; ++k) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = rows_r[k][tx + 16 * i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = rows_c[k][ty + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const double diff = a[i] - b[j];
                    s[i][j] += diff * diff;
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t r = r0 + tx + 16 * i, c = c0 + ty + 16 * j;
            if (r > c || c >= M) continue;
            double v;
            if (kind == KNM_KERNEL_GAUSSIAN) {
                v = exp(-s[i][j] * scale);
            } else {
                const double u = sqrt(s[i][j]) * scale;
                const double poly = kind == KNM_KERNEL_MATERN32 ? 1.0 + u : kind == KNM_KERNEL_MATERN52 ? 1.0 + u + u * u / 3.0 : 1.0;
                v = poly * exp(-u);
            }
            if (r == c) v += jitter;
            K[r + c * ldk] = v;
        }
}

// first (1-based) index whose diagonal entry is not a positive finite number, else unchanged;
// catches NaN/Inf pivots, which a "pivot <= 0" test inside the factorisation lets through
__global__ void diag_check_kernel(const double *__restrict__ A, int64_t lda, int64_t M, unsigned long long *bad)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    const double v = A[i + i * lda]; // the diagonal sits at the same place in upper and lower storage
    if (!(v > 0.0) || !(v < 1.0e300)) atomicMin(bad, (unsigned long long)(i + 1));
}

// row-major (rows x t, leading dimension t) float  <->  column-major (rows x t) double
__global__ void f32_rows_to_f64_cols(const float *__restrict__ src, int64_t rows, int t, double *__restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * t) return;
    const int64_t r = i / t;
    const int c = (int)(i % t);
    dst[r + (int64_t)c * rows] = (double)src[i];
}
__global__ void f64_cols_to_f32_rows(const double *__restrict__ src, int64_t rows, int t, float *__restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * t) return;
    const int64_t r = i / t;
    const int c = (int)(i % t);
    dst[i] = (float)src[r + (int64_t)c * rows];
}
__global__ void f64_rows_to_cols(const double *__restrict__ src, int64_t rows, int t, double *__restrict__ dst, int back)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * t) return;
    const int64_t r = i / t;
    const int c = (int)(i % t);
    if (back) dst[i] = src[r + (int64_t)c * rows];
    else dst[r + (int64_t)c * rows] = src[i];
}

// dst[r * cols + c] = entry (row0 + r, col0 + c) of an upper factor stored at F (upper or lower storage,
// leading dimension ld), zero below the diagonal: a block of a factor gathered into row-major order
__global__ void gather_block_kernel(const double *__restrict__ F, int64_t ld, int lower, int64_t row0, int64_t col0,
                                    int64_t rows, int64_t cols, double *__restrict__ dst)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * cols) return;
    const int64_t r = row0 + i / cols, c = col0 + i % cols;
    dst[i] = (c >= r) ? (lower ? F[c + r * ld] : F[r + c * ld]) : 0.0;
}

// ---- blocked triangular solves -----------------------------------------------------------------
// R (upper, column-major, leading dimension M) is cut into block columns of width sb.  A solve
// walks the diagonal blocks in dependency order; each step multiplies a right-hand-side block
// by the pre-inverted diagonal block and then updates the remaining right-hand side with the
// off-diagonal panel, which is streamed once with coalesced loads.  The panels are ~all of
// the 8 M^2 / 2 bytes of the factor, so a solve is bound by HBM bandwidth; wide blocks keep the
// chain of dependent launches short (M / sb steps) and every launch large enough to fill the
// chip.
//
// Each inverted diagonal block is stored mirrored: S[i, j] = S[j, i] = inv(R_kk)[min, max].  Both
// the plain and the transposed product then read contiguous pieces of the columns of S.
inline int solve_block_width(int64_t M)
{
    int64_t b = ((M + 15) / 16 + 255) / 256 * 256;
    if (b > 2048) b = 2048;
    return (int)b;
}

// copy the upper triangle of every block onto its strict lower triangle
__global__ void mirror_upper_kernel(double *__restrict__ S, int sb)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x; // row in the lower triangle
    const int j = blockIdx.y;                            // column
    if (i >= sb || i <= j) return;
    double *blk = S + (int64_t)blockIdx.z * sb * sb;
    blk[i + (int64_t)j * sb] = blk[j + (int64_t)i * sb];
}

__device__ __forceinline__ double wave_sum(double s)
{
    s += __shfl_xor(s, 32);
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 8);
    s += __shfl_xor(s, 4);
    s += __shfl_xor(s, 2);
    s += __shfl_xor(s, 1);
    return s;
}

constexpr int kSolveCols = 8; // right-hand sides a blocked triangular solve takes through the factor together

// The three kernels of the blocked triangular solves work on TC right-hand sides at once (columns of
// a column-major M x t array, ldb apart; the staged solved blocks ldx apart), tc <= TC of them live: a
// column past tc reads the last live one and is dropped.  Every entry of the factor and of the block
// inverses is then read once per TC columns instead of once per column.

// x = inv(R_kk) b (lower = 1: x[c] = sum_{i >= c} S[i, c] b[i]) or x = inv(R_kk)^T b (lower = 0:
// x[c] = sum_{i <= c} S[i, c] b[i]) for one mirrored block S of live order nbk; one wavefront
// per entry of x, lanes along the column of S.
template <int TC>
__global__ __launch_bounds__(256) void diag_apply_kernel(const double *__restrict__ S, int sb, int nbk, int lower,
                                                        const double *__restrict__ b, int64_t ldb, int tc,
                                                        double *__restrict__ x, int64_t ldx)
{
    const int lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= nbk) return;
    const double *col = S + (int64_t)c * sb;
    const int lo = lower ? c : 0;
    const int hi = lower ? nbk : c + 1;
    const double *bq[TC];
#pragma unroll
    for (int q = 0; q < TC; ++q) bq[q] = b + (int64_t)(q < tc ? q : tc - 1) * ldb;
    double s0[TC], s1[TC];
#pragma unroll
    for (int q = 0; q < TC; ++q) s0[q] = s1[q] = 0.0;
    int i = lo + lane;
    for (; i + 64 < hi; i += 128) {
        const double a0 = col[i], a1 = col[i + 64];
#pragma unroll
        for (int q = 0; q < TC; ++q) {
            s0[q] += a0 * bq[q][i];
            s1[q] += a1 * bq[q][i + 64];
        }
    }
    if (i < hi) {
        const double a0 = col[i];
#pragma unroll
        for (int q = 0; q < TC; ++q) s0[q] += a0 * bq[q][i];
    }
#pragma unroll
    for (int q = 0; q < TC; ++q) {
        const double s = wave_sum(s0[q] + s1[q]);
        if (lane == 0 && q < tc) x[(int64_t)q * ldx + c] = s;
    }
}

constexpr int kPanelWaves = 8;  // wavefronts of a panel_update_n workgroup, sharing the columns
constexpr int kPanelRows = 64;  // rows of a panel_update_n workgroup, one per lane
constexpr int kPanelCols = 4;   // columns of one panel_update_t wavefront

// b[r] -= sum_j P[r + (k0 + j) ld] x[j] for r in [r_lo, r_hi)  (x = the solved block, nbk entries): the
// rows above the block of an upper-storage factor in its plain solve, the rows below the block of a
// lower-storage factor in its transposed solve.  Workgroups past the row range copy x into
// b[k0 : k0 + nbk].
template <int TC>
__global__ __launch_bounds__(kPanelWaves * 64) void panel_update_n_kernel(const double *__restrict__ R, int64_t M,
                                                                         int64_t k0, int nbk, int64_t r_lo,
                                                                         int64_t r_hi, const double *__restrict__ x,
                                                                         int64_t ldx, double *__restrict__ b, int64_t ldb,
                                                                         int tc)
{
    __shared__ double part[kPanelWaves][TC][kPanelRows];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t row_groups = (r_hi - r_lo + kPanelRows - 1) / kPanelRows;
    if ((int64_t)blockIdx.x >= row_groups) {
        const int64_t i = ((int64_t)blockIdx.x - row_groups) * blockDim.x + threadIdx.x;
        if (i < nbk)
            for (int q = 0; q < tc; ++q) b[(int64_t)q * ldb + k0 + i] = x[(int64_t)q * ldx + i];
        return;
    }
    const int64_t r = r_lo + (int64_t)blockIdx.x * kPanelRows + lane;
    const bool live = r < r_hi;
    const double *p = R + (live ? r : r_lo) + k0 * M;
    const double *xq[TC];
#pragma unroll
    for (int q = 0; q < TC; ++q) xq[q] = x + (int64_t)(q < tc ? q : tc - 1) * ldx;
    double s0[TC], s1[TC];
#pragma unroll
    for (int q = 0; q < TC; ++q) s0[q] = s1[q] = 0.0;
    int j = w;
    for (; j + 7 * kPanelWaves < nbk; j += 8 * kPanelWaves) {
        double a[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] = p[(int64_t)(j + u * kPanelWaves) * M];
#pragma unroll
        for (int q = 0; q < TC; ++q) {
#pragma unroll
            for (int u = 0; u < 8; u += 2) {
                s0[q] += a[u] * xq[q][j + u * kPanelWaves];
                s1[q] += a[u + 1] * xq[q][j + (u + 1) * kPanelWaves];
            }
        }
    }
    for (; j < nbk; j += kPanelWaves) {
        const double a0 = p[(int64_t)j * M];
#pragma unroll
        for (int q = 0; q < TC; ++q) s0[q] += a0 * xq[q][j];
    }
#pragma unroll
    for (int q = 0; q < TC; ++q) part[w][q][lane] = s0[q] + s1[q];
    __syncthreads();
    // wavefront q adds up right-hand side q (TC <= kPanelWaves)
    if (w < TC && w < tc && live) {
        double s = 0.0;
        for (int u = 0; u < kPanelWaves; ++u) s += part[u][w][lane];
        b[(int64_t)w * ldb + r] -= s;
    }
}

// b[j] -= sum_i P[(k0 + i) + j ld] x[i] for j in [j0, j1)  (x = the solved block, nbk entries): the
// columns right of the block of an upper-storage factor in its transposed solve, the columns left of
// the block of a lower-storage factor in its plain solve.  One wavefront per kPanelCols columns, lanes
// along the rows.  Workgroups past the column range copy x into b[k0 : k0 + nbk].
template <int TC>
__global__ __launch_bounds__(256) void panel_update_t_kernel(const double *__restrict__ R, int64_t M, int64_t k0,
                                                            int nbk, int64_t j0, int64_t j1,
                                                            const double *__restrict__ x, int64_t ldx,
                                                            double *__restrict__ b, int64_t ldb, int tc)
{
    const int lane = threadIdx.x & 63;
    const int64_t col_groups = (j1 - j0 + 4 * kPanelCols - 1) / (4 * kPanelCols);
    if ((int64_t)blockIdx.x >= col_groups) {
        const int64_t i = ((int64_t)blockIdx.x - col_groups) * blockDim.x + threadIdx.x;
        if (i < nbk)
            for (int q = 0; q < tc; ++q) b[(int64_t)q * ldb + k0 + i] = x[(int64_t)q * ldx + i];
        return;
    }
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t jb = j0 + wave * kPanelCols;
    if (jb >= j1) return;
    const double *p[kPanelCols];
    double s[kPanelCols][TC];
#pragma unroll
    for (int c = 0; c < kPanelCols; ++c) {
        const int64_t j = (jb + c < j1) ? jb + c : j1 - 1; // a clamped column is computed and dropped
        p[c] = R + k0 + j * M;
#pragma unroll
        for (int q = 0; q < TC; ++q) s[c][q] = 0.0;
    }
    const double *xq[TC];
#pragma unroll
    for (int q = 0; q < TC; ++q) xq[q] = x + (int64_t)(q < tc ? q : tc - 1) * ldx;
    int i = lane;
    for (; i + 64 < nbk; i += 128) {
        double a[kPanelCols], c2[kPanelCols];
#pragma unroll
        for (int c = 0; c < kPanelCols; ++c) {
            a[c] = p[c][i];
            c2[c] = p[c][i + 64];
        }
#pragma unroll
        for (int q = 0; q < TC; ++q) {
            const double x0 = xq[q][i], x1 = xq[q][i + 64];
#pragma unroll
            for (int c = 0; c < kPanelCols; ++c) s[c][q] += a[c] * x0 + c2[c] * x1;
        }
    }
    if (i < nbk) {
#pragma unroll
        for (int q = 0; q < TC; ++q) {
            const double x0 = xq[q][i];
#pragma unroll
            for (int c = 0; c < kPanelCols; ++c) s[c][q] += p[c][i] * x0;
        }
    }
#pragma unroll
    for (int c = 0; c < kPanelCols; ++c)
#pragma unroll
        for (int q = 0; q < TC; ++q) {
            const double tot = wave_sum(s[c][q]);
            if (lane == 0 && jb + c < j1 && q < tc) b[(int64_t)q * ldb + jb + c] -= tot;
        }
}

// ---- leaf of the blocked factorisation --------------------------------------------------------
// One workgroup factorises a diagonal block of order nb <= 128 in LDS (upper triangle packed by
// rows, right-looking, two barriers per pivot) and inverts the factor in place there.
// Everything above the leaf is products with these small inverses on the matrix cores.
// The kernel keeps to 70 KB of LDS so that it can share a CU with a workgroup of the rank-k
// kernel: during the factorisation's look-ahead it runs beside the trailing update.
constexpr int kLeaf = 128;
constexpr int kLeafThreads = 512;
constexpr int kLeafPacked = kLeaf * (kLeaf + 1) / 2;

struct LeafShared {
    double P[kLeafPacked]; // (i, j), i <= j, at i nb - i (i - 1) / 2 + (j - i)
    double rowk[kLeaf];
    double dinv[kLeaf];
    double rrow[2][kLeaf];
};

__device__ __forceinline__ int leaf_row_start(int i, int nb) { return i * nb - i * (i - 1) / 2; }

// entry (i, j), i <= j, of the block at A: A[i + j lda] (upper storage) or A[j + i lda] (lower)
__device__ __forceinline__ void leaf_load(LeafShared &sh, const double *A, int64_t lda, int nb, int lower)
{
    for (int e = threadIdx.x; e < nb * kLeaf; e += kLeafThreads) {
        // upper storage: column j of the block, row i contiguous; lower: row i, column j contiguous
        const int u = e & (kLeaf - 1), w = e >> 7;
        const int i = lower ? w : u, j = lower ? u : w;
        if (i <= j && j < nb) sh.P[leaf_row_start(i, nb) + (j - i)] = A[u + w * lda];
    }
}

// W (nb x nb, column-major, ldw; written whole, zeros below the diagonal) <- inverse of the upper
// triangular factor R packed in sh.P, whose reciprocal diagonal is in sh.dinv; sh.P is overwritten
// by the inverse.  Rows are done in lockstep, last to first:
//   W[i, c] = -(sum_{i < j <= c} R[i, j] W[j, c]) / R[i, i],
// with row i of R first copied aside (its storage then takes row i of W), so R[i, j] is a
// broadcast read and W[j, c] is contiguous across the columns c.  A column belongs to four
// adjacent lanes, which split the sum over j.  One workgroup has its CU nearly to itself, so
// the loops are unrolled by hand to keep several LDS reads in flight.
__device__ __forceinline__ void leaf_invert(LeafShared &sh, int nb, double *W, int64_t ldw)
{
    const int tid = threadIdx.x;
    const int c = tid >> 2, part = tid & 3;
    const bool live = c < nb;
    if (tid == 0) sh.P[leaf_row_start(nb - 1, nb)] = sh.dinv[nb - 1];
    for (int i = nb - 2; i >= 0; --i) {
        double *rr = sh.rrow[i & 1];
        const int ri = leaf_row_start(i, nb);
        if (tid > i && tid < nb) rr[tid] = sh.P[ri + (tid - i)];
        __syncthreads(); // row i of R is aside, row i + 1 of W is complete
        double s0 = 0.0, s1 = 0.0;
        int j = i + 1 + part;
        int pw = leaf_row_start(j, nb) + (c - j); // W[j, c]; four rows on it moves by 4 nb - 4 j - 10
        for (; j + 4 < nb; j += 8) {
            const int pw1 = pw + 4 * nb - 4 * j - 10;
            const double a0 = (live && j <= c) ? rr[j] * sh.P[pw] : 0.0;
            const double a1 = (live && j + 4 <= c) ? rr[j + 4] * sh.P[pw1] : 0.0;
            s0 += a0;
            s1 += a1;
            pw = pw1 + 4 * nb - 4 * (j + 4) - 10;
        }
        if (j < nb && live && j <= c) s0 += rr[j] * sh.P[pw];
        double s = s0 + s1;
        s += __shfl_xor(s, 1);
        s += __shfl_xor(s, 2);
        if (part == 0 && live && c > i) sh.P[ri + (c - i)] = -s * sh.dinv[i];
        if (tid == 0) sh.P[ri] = sh.dinv[i];
    }
    __syncthreads();
    for (int e = tid; e < nb * kLeaf; e += kLeafThreads) {
        const int i = e & (kLeaf - 1), j = e >> 7;
        if (i < nb) W[i + j * ldw] = (i <= j) ? sh.P[leaf_row_start(i, nb) + (j - i)] : 0.0;
    }
}

// Triangle of the nb x nb block at A (upper or lower storage, lda) <- its upper Cholesky factor R,
// R^T R = A, in the same storage; W <- R^-1 (always column-major, upper).  *bad <- min(*bad, pivot0 + k + 1) for a pivot k that is not a positive finite number
// (the factorisation then goes on with 1 in its place; the caller discards the result).
__global__ __launch_bounds__(kLeafThreads) void potrf_trtri_leaf_kernel(double *__restrict__ A, int64_t lda, int nb,
                                                                       double *__restrict__ W, int64_t ldw,
                                                                       int64_t pivot0, unsigned long long *bad,
                                                                       int lower)
{
    __shared__ LeafShared sh;
    const int tid = threadIdx.x;
    leaf_load(sh, A, lda, nb, lower);
    __syncthreads();
    const int jc = tid & (kLeaf - 1), par = tid >> 7; // trailing update: column of this thread, rows par mod 4
    for (int k = 0; k < nb; ++k) {
        const int rk = leaf_row_start(k, nb);
        const double dkk = sh.P[rk];
        const bool ok = dkk > 0.0 && dkk < 1.0e300;
        const double rinv = ok ? 1.0 / sqrt(dkk) : 1.0;
        if (tid == 0) {
            if (!ok) atomicMin(bad, (unsigned long long)(pivot0 + k + 1));
            sh.dinv[k] = rinv;
        }
        if (tid > k && tid < nb) { // row k, scaled; kept beside the packed copy for the update
            const double v = sh.P[rk + (tid - k)] * rinv;
            sh.P[rk + (tid - k)] = v;
            sh.rowk[tid] = v;
        }
        __syncthreads();
        const int j = k + 1 + jc;
        if (j < nb) {
            const double rj = sh.rowk[j];
            int i = k + 1 + par;
            int pa = leaf_row_start(i, nb) + (j - i); // (i, j); four rows on it moves by 4 nb - 4 i - 10
            for (; i + 4 <= j; i += 8) {
                const int pa1 = pa + 4 * nb - 4 * i - 10;
                const double u0 = sh.rowk[i], u1 = sh.rowk[i + 4];
                const double c0 = sh.P[pa], c1 = sh.P[pa1];
                sh.P[pa] = c0 - u0 * rj;
                sh.P[pa1] = c1 - u1 * rj;
                pa = pa1 + 4 * nb - 4 * (i + 4) - 10;
            }
            if (i <= j) sh.P[pa] -= sh.rowk[i] * rj;
        }
        __syncthreads();
    }
    // back to A, with the diagonal of R: sh.P still holds the pivots before the square root
    for (int e = tid; e < nb * kLeaf; e += kLeafThreads) {
        const int u = e & (kLeaf - 1), w = e >> 7;
        const int i = lower ? w : u, j = lower ? u : w;
        if (i <= j && j < nb) A[u + w * lda] = (i == j) ? 1.0 / sh.dinv[i] : sh.P[leaf_row_start(i, nb) + (j - i)];
    }
    __syncthreads();
    leaf_invert(sh, nb, W, ldw);
}

// W <- inverse of the upper triangular nb x nb diagonal blocks of a factor R (one workgroup per
// block): leaf g sits on the diagonal of group g / blocks_per_group, at offset (g % blocks_per_group) * 128
__global__ __launch_bounds__(kLeafThreads) void trtri_leaf_kernel(const double *__restrict__ R, int64_t ldr, int64_t M,
                                                                 int64_t step_w_block, int blocks_per_group,
                                                                 double *__restrict__ W, int64_t ldw, int lower)
{
    __shared__ LeafShared sh;
    const int64_t g = blockIdx.x;
    const int64_t r0 = g * kLeaf;
    const int nb = (int)((M - r0 < kLeaf) ? M - r0 : kLeaf);
    const double *Rb = R + r0 + r0 * ldr;
    const int64_t grp = g / blocks_per_group, off = (g % blocks_per_group) * kLeaf;
    double *Wb = W + grp * step_w_block + off + off * ldw;
    leaf_load(sh, Rb, ldr, nb, lower);
    for (int k = threadIdx.x; k < nb; k += kLeafThreads) sh.dinv[k] = 1.0 / Rb[k + k * ldr];
    __syncthreads();
    leaf_invert(sh, nb, Wb, ldw);
}

inline dim3 grid1(int64_t n, int threads = 256) { return dim3((unsigned)((n + threads - 1) / threads)); }

// ---- fp64 vector work of the CG driver -----------------------------------------------------
// Sums are taken in a fixed order (256 block partials, then one block), so a fit is
// reproducible from run to run.
constexpr int kRedBlocks = 256;

__global__ __launch_bounds__(256) void dot_partial_kernel(const double *__restrict__ x, const double *__restrict__ y,
                                                         int64_t n, double *__restrict__ part)
{
    __shared__ double sh[256];
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        s += y ? x[i] * y[i] : x[i];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = sh[0];
}

__global__ __launch_bounds__(256) void dot_finish_kernel(const double *__restrict__ part, int count, double *__restrict__ out)
{
    __shared__ double sh[256];
    sh[threadIdx.x] = ((int)threadIdx.x < count) ? part[threadIdx.x] : 0.0;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = sh[0];
}

__global__ void axpy_kernel(int64_t n, double a, const double *__restrict__ x, double *__restrict__ y)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) y[i] += a * x[i];
}

__global__ void scal_kernel(int64_t n, double b, double *__restrict__ y)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) y[i] *= b;
}

// *out_host <- sum_i x[i] y[i] (y null: sum_i x[i]); synchronises the stream
int vec_dot(knm_ctx *ctx, int64_t n, const double *x, const double *y, double *out_host)
{
    if (!ctx->red_buf) {
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&ctx->red_buf), sizeof(double) * (kRedBlocks + 1));
        if (e != hipSuccess) {
            (void)hipGetLastError();
            ctx->red_buf = nullptr;
            return fail(ctx, KNM_ALLOC, "hipMalloc(reduction buffer)", e);
        }
    }
    hipLaunchKernelGGL(dot_partial_kernel, dim3(kRedBlocks), dim3(256), 0, ctx->stream, x, y, n, ctx->red_buf);
    hipLaunchKernelGGL(dot_finish_kernel, dim3(1), dim3(256), 0, ctx->stream, ctx->red_buf, kRedBlocks,
                       ctx->red_buf + kRedBlocks);
    hipError_t e = hipMemcpyAsync(out_host, ctx->red_buf + kRedBlocks, sizeof(double), hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "vector reduction", e);
    return KNM_OK;
}

int vec_axpy(knm_ctx *ctx, int64_t n, double a, const double *x, double *y)
{
    hipLaunchKernelGGL(axpy_kernel, grid1(n), dim3(256), 0, ctx->stream, n, a, x, y);
    return hipGetLastError() == hipSuccess ? KNM_OK : fail(ctx, KNM_HIP_ERROR, "axpy launch");
}

int vec_scal(knm_ctx *ctx, int64_t n, double b, double *y)
{
    hipLaunchKernelGGL(scal_kernel, grid1(n), dim3(256), 0, ctx->stream, n, b, y);
    return hipGetLastError() == hipSuccess ? KNM_OK : fail(ctx, KNM_HIP_ERROR, "scal launch");
}


// Logistic loss l(z, y) = log(1 + exp(-y z)), y = +-1 (Appendix "Logistic Falkon Algorithm",
// Example 1a), evaluated in fp64 from fp32 predictions: first derivative g, second derivative
// dw (as float for the sweeps and/or as double for the preconditioner), loss.  Any output may
// be null.
__global__ void logistic_terms_kernel(const float *__restrict__ z, const float *__restrict__ y, int64_t n,
                                      float *__restrict__ g, float *__restrict__ dw32, double *__restrict__ dw64,
                                      double *__restrict__ loss)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const double yi = (double)y[i];
    const double m = yi * (double)z[i];
    const double s = 0.5 * (1.0 - tanh(0.5 * m)); // sigma(-m), stable for either sign
    if (g) g[i] = (float)(-yi * s);
    if (dw32) dw32[i] = (float)(s * (1.0 - s));
    if (dw64) dw64[i] = s * (1.0 - s);
    if (loss) loss[i] = (m > 0.0) ? log1p(exp(-m)) : -m + log1p(exp(m));
}

// r[j] = -(u[j] + c (zc[j] + eps a[j]))   (right-hand side of a Newton step, fp64)
__global__ void newton_rhs_kernel(const float *__restrict__ u, const float *__restrict__ zc,
                                  const double *__restrict__ a, double c, double eps, int64_t M,
                                  double *__restrict__ r)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= M) return;
    r[j] = -((double)u[j] + c * ((double)zc[j] + eps * a[j]));
}

__global__ void f64_to_f32_kernel(const double *__restrict__ a, int64_t n, float *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (float)a[i];
}

struct DevBuf {
    void *p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    int alloc(knm_ctx *ctx, size_t bytes)
    {
        hipError_t e = hipMalloc(&p, bytes ? bytes : 1);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            p = nullptr;
            return fail(ctx, KNM_ALLOC, "hipMalloc", e);
        }
        return KNM_OK;
    }
    template <class T> T *as() { return static_cast<T *>(p); }
};

// Many right-hand sides: the same blocked solve as products on the fp64 matrix cores.
constexpr int kProductSolveMinCols = 16;    // from this many right-hand sides on
constexpr int64_t kProductSolveMinM = 4096; // and this order of the factor

// out <- the upper triangle (diagonal included) of one mirrored block inverse, zeros below it
__global__ void upper_block_kernel(const double *__restrict__ S, int sb, double *__restrict__ out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int c = blockIdx.y;
    if (i < sb) out[i + (int64_t)c * sb] = (i <= c) ? S[i + (int64_t)c * sb] : 0.0;
}

// b[k0 + i + j ldb] = x[i + j ldx], i < nbk, j < tc
__global__ void block_rows_kernel(const double *__restrict__ x, int64_t ldx, int nbk, int tc, double *__restrict__ b,
                                  int64_t ldb)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int j = blockIdx.y;
    if (i < nbk && j < tc) b[i + (int64_t)j * ldb] = x[i + (int64_t)j * ldx];
}

// The blocked solve of tri_solve with both of its steps as products: per block, X = inv(R_kk) B_k or
// inv(R_kk)^T B_k (the block inverse with its mirror image cleared, so that a plain product applies the
// triangular factor), then the rows still to be solved lose the panel times X.  The factor is read once
// per group of columns (as many as the staging array holds: at least 128 from M = 4096 on), at the rate
// of the matrix cores instead of once per 8 columns.
int tri_solve_products(knm_ctx *ctx, const knm_precond *p, const double *R, const double *S, bool trans, double *B, int t)
{
    const int64_t M = p->M, ld = p->ld;
    const bool lower = (R == p->A);
    const int sb = p->sb;
    const int64_t nblk = (M + sb - 1) / sb;
    const int64_t cap = (M * kSolveCols) / sb; // columns the staging array holds at leading dimension sb
    double *X = p->xw;
    for (int c0 = 0; c0 < t;) {
        const int tc = (int)((t - c0 < cap) ? t - c0 : cap);
        double *Bc = B + (int64_t)c0 * M;
        for (int64_t step = 0; step < nblk; ++step) {
            const int64_t k = trans ? step : nblk - 1 - step; // R^T is lower: forward; R: backward
            const int64_t k0 = k * sb;
            const int nbk = (int)((M - k0 < sb) ? M - k0 : sb);
            hipLaunchKernelGGL(upper_block_kernel, dim3((unsigned)((sb + 255) / 256), (unsigned)sb), dim3(256), 0, ctx->stream,
                               S + k * sb * sb, sb, p->blk);
            // x[c] = sum_i W[c, i] b[i] (plain) or sum_i W[i, c] b[i] (transposed), W = inv(R_kk) at blk[row + col sb]
            hipError_t e = launch_gemm_f64(trans ? 0 : 1, nbk, tc, nbk, 1.0, p->blk, sb, Bc + k0, M, 0.0, X, sb, ctx->stream);
            if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "triangular solve: block product", e);
            hipLaunchKernelGGL(block_rows_kernel, dim3((unsigned)((nbk + 255) / 256), (unsigned)tc), dim3(256), 0, ctx->stream, X,
                               (int64_t)sb, nbk, tc, Bc + k0, M);
            // the rows of B still to be solved: before the block (plain) or after it (transposed)
            const int64_t lo = trans ? k0 + nbk : 0, hi = trans ? M : k0;
            if (hi > lo) {
                // panel entry (row r of the rest, column kk of the block): R[r + (k0 + kk) ld] where the panels
                // are contiguous in r, else R[(k0 + kk) + r ld]
                e = (trans == lower)
                        ? launch_gemm_f64(1, hi - lo, tc, nbk, -1.0, R + lo + k0 * ld, ld, X, sb, 1.0, Bc + lo, M, ctx->stream)
                        : launch_gemm_f64(0, hi - lo, tc, nbk, -1.0, R + k0 + lo * ld, ld, X, sb, 1.0, Bc + lo, M, ctx->stream);
                if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "triangular solve: panel product", e);
            }
        }
        c0 += tc;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "blocked triangular solve", e);
    return KNM_OK;
}

// B <- op(R)^-1 B for column-major B (M x t); S = mirrored inverses of the diagonal blocks of R
// (R = p->T, upper storage, or p->A, lower storage).  p->xw stages each solved block; solves on one
// context are stream-ordered.  Either storage streams its panels along contiguous columns of the
// array: what is a row update for one is a column update for the other.
int tri_solve(knm_ctx *ctx, const knm_precond *p, const double *R, const double *S, bool trans, double *B, int t)
{
    TraceRange range(R == p->A ? (trans ? "knm solve A^-T" : "knm solve A^-1") : (trans ? "knm solve T^-T" : "knm solve T^-1"));
    const int64_t M = p->M, ld = p->ld;
    const bool lower = (R == p->A);
    const int sb = p->sb;
    const int64_t nblk = (M + sb - 1) / sb;
    if (t >= kProductSolveMinCols && p->blk != nullptr) return tri_solve_products(ctx, p, R, S, trans, B, t);
    // right-hand sides in groups of up to kSolveCols: a group streams the factor once
    auto run = [&](auto width, int c0, int tc) {
        constexpr int TC = decltype(width)::value;
        double *b = B + (int64_t)c0 * M;
        for (int64_t step = 0; step < nblk; ++step) {
            const int64_t k = trans ? step : nblk - 1 - step; // R^T is lower: forward; R: backward
            const int64_t k0 = k * sb;
            const int nbk = (int)((M - k0 < sb) ? M - k0 : sb);
            double *x = p->xw + k0;
            hipLaunchKernelGGL(diag_apply_kernel<TC>, dim3((unsigned)((nbk + 3) / 4)), dim3(256), 0, ctx->stream,
                               S + k * sb * sb, sb, nbk, trans ? 0 : 1, b + k0, M, tc, x, M);
            // the entries of b still to be solved: before the block (plain) or after it (transposed)
            const int64_t lo = trans ? k0 + nbk : 0, hi = trans ? M : k0;
            if (trans == lower) { // panel entries R(r, k0 + j) or R(k0 + j, r) contiguous in r
                const int64_t groups = (hi - lo + kPanelRows - 1) / kPanelRows;
                const int64_t copy = (nbk + kPanelWaves * 64 - 1) / (kPanelWaves * 64);
                hipLaunchKernelGGL(panel_update_n_kernel<TC>, dim3((unsigned)(groups + copy)), dim3(kPanelWaves * 64), 0,
                                   ctx->stream, R, ld, k0, nbk, lo, hi, x, M, b, M, tc);
            } else {              // contiguous in the block's own index
                const int64_t groups = (hi - lo + 4 * kPanelCols - 1) / (4 * kPanelCols);
                const int64_t copy = (nbk + 255) / 256;
                hipLaunchKernelGGL(panel_update_t_kernel<TC>, dim3((unsigned)(groups + copy)), dim3(256), 0, ctx->stream,
                                   R, ld, k0, nbk, lo, hi, x, M, b, M, tc);
            }
        }
    };
    for (int c = 0; c < t; c += kSolveCols) {
        const int tc = (t - c < kSolveCols) ? t - c : kSolveCols;
        if (tc == 1) run(std::integral_constant<int, 1>{}, c, tc);
        else if (tc <= 4) run(std::integral_constant<int, 4>{}, c, tc);
        else run(std::integral_constant<int, kSolveCols>{}, c, tc);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "blocked triangular solve", e);
    return KNM_OK;
}

// S <- mirrored inverses of the sb x sb diagonal blocks of the upper-triangular R (p->T or p->A).  The 128 x 128
// diagonal blocks are inverted by the leaf kernel (one workgroup each); neighbouring inverses are
// then merged level by level,  inv([R11 R12; 0 R22]) = [W11, -W11 R12 W22; 0, W22],  with two
// block products per pair, until the blocks are sb wide; last the upper triangle of every
// block is copied onto its lower.  `tmp` holds (sb / 2)^2 doubles.
int invert_diag_blocks(knm_ctx *ctx, const knm_precond *p, const double *R, double *S, double *tmp)
{
    const int64_t M = p->M, ld = p->ld;
    const int lower = (R == p->A) ? 1 : 0;
    const int sb = p->sb;
    const int64_t nblk = (M + sb - 1) / sb;
    const int64_t block = (int64_t)sb * sb;
    hipError_t e = hipMemsetAsync(S, 0, sizeof(double) * nblk * block, ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemsetAsync", e);
    const int64_t leaves = (M + kLeaf - 1) / kLeaf;
    hipLaunchKernelGGL(trtri_leaf_kernel, dim3((unsigned)leaves), dim3(kLeafThreads), 0, ctx->stream, R, ld, M, block,
                       sb / kLeaf, S, (int64_t)sb, lower);
    for (int64_t h = kLeaf; h < sb; h *= 2) {
        for (int64_t k = 0; k < nblk; ++k) {
            const int64_t k0 = k * sb;
            const int64_t nbk = (M - k0 < sb) ? M - k0 : sb;
            double *Sk = S + k * block;
            for (int64_t off = 0; off + h < nbk; off += 2 * h) {
                const int64_t h2 = (nbk - off - h < h) ? nbk - off - h : h; // order of the second block of the pair
                // R12 (h x h2): entry (i, k) at R12[i + k ld] in upper storage, R12[k + i ld] in lower
                const double *R12 = lower ? R + (k0 + off + h) + (size_t)(k0 + off) * ld
                                          : R + (k0 + off) + (size_t)(k0 + off + h) * ld;
                const double *W11 = Sk + off + off * sb;
                const double *W22 = Sk + (off + h) + (off + h) * sb;
                double *W12 = Sk + off + (off + h) * sb;
                if (launch_gemm_f64(lower ? 0 : 1, h, h2, h2, 1.0, R12, ld, W22, sb, 0.0, tmp, h, ctx->stream) != hipSuccess ||
                    launch_gemm_f64(1, h, h2, h, -1.0, W11, sb, tmp, h, 0.0, W12, sb, ctx->stream) != hipSuccess)
                    return fail(ctx, KNM_HIP_ERROR, "inverse merge launch");
            }
        }
    }
    hipLaunchKernelGGL(mirror_upper_kernel, dim3((unsigned)((sb + 255) / 256), (unsigned)sb, (unsigned)nblk), dim3(256),
                       0, ctx->stream, S, sb);
    if (hipGetLastError() != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "diagonal block inversion launch");
    return KNM_OK;
}

// Workspace of one application of the operator of Eq. 9 on column-major fp64 vectors.
struct LinopWork {
    DevBuf v, z32, u32, u64;
    int alloc(knm_ctx *ctx, int64_t M, int t)
    {
        int st = v.alloc(ctx, sizeof(double) * M * t);
        if (!st) st = z32.alloc(ctx, sizeof(float) * M * t);
        if (!st) st = u32.alloc(ctx, sizeof(float) * M * t);
        if (!st) st = u64.alloc(ctx, sizeof(double) * M * t);
        return st;
    }
};

// The two sweeps of one (X, C, sigma), whatever the storage of the points: W (n x t) = K V and
// U (M x t) = K^T (wgt .* W) (wgt over the rows of X, or null)
struct KernelOps {
    int64_t n = 0, M = 0;
    std::function<int(const float *V, int t, float *W)> v;
    std::function<int(const float *W, const float *wgt, int t, float *U)> t_w;
    // the same with U as fp64 rows (M x t, row-major) that were never rounded to fp32; may be empty
    std::function<int(const float *W, const float *wgt, int t, double *U64)> t_w64;
};

// Operand conversions the split-fp16 engines have clamped so far (waits for the stream).
int read_range_count(knm_ctx *ctx, unsigned int *count)
{
    hipError_t e = hipMemcpyAsync(count, ctx->range_count, sizeof(*count), hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    return e == hipSuccess ? KNM_OK : fail(ctx, KNM_HIP_ERROR, "range counter", e);
}

// A fit runs with the context's cross-term mode unless its first sweep had to clamp operands (points
// outside the range of the split-fp16 engines): then the whole fit runs on the fp32 matrix cores,
// which have no such limits, and the context's mode comes back when the fit returns.
struct CrossTermScope {
    knm_ctx *ctx;
    int saved;
    unsigned int before = 0;
    explicit CrossTermScope(knm_ctx *c) : ctx(c), saved(c->cross_term) {}
    ~CrossTermScope() { ctx->cross_term = saved; }
    int begin() { return read_range_count(ctx, &before); }
    // after the first sweep: true if it must be repeated in the fp32 mode (now selected)
    int check(bool *repeat)
    {
        *repeat = false;
        if (ctx->cross_term != KNM_CROSS_F16X3) return KNM_OK;
        unsigned int now = 0;
        int st = read_range_count(ctx, &now);
        if (st) return st;
        if (now != before) {
            ctx->cross_term = KNM_CROSS_F32;
            *repeat = true;
        }
        return KNM_OK;
    }
};

// cols (M x t, column-major fp64) <- K^T (wgt .* W): T^-T amplifies what the solver is given by the
// conditioning of K_MM, so the result of the column sweep is taken in fp64 where the sweeps offer it
int t_w_cols(knm_ctx *ctx, const KernelOps &ops, const float *W, const float *wgt, int t, float *u32, double *u64,
             double *cols)
{
    if (ops.t_w64) {
        int st = ops.t_w64(W, wgt, t, u64);
        if (st) return st;
        hipLaunchKernelGGL(f64_rows_to_cols, grid1(ops.M * t), dim3(256), 0, ctx->stream, u64, ops.M, t, cols, 0);
    } else {
        int st = ops.t_w(W, wgt, t, u32);
        if (st) return st;
        hipLaunchKernelGGL(f32_rows_to_f64_cols, grid1(ops.M * t), dim3(256), 0, ctx->stream, u32, ops.M, t, cols);
    }
    return hipGetLastError() == hipSuccess ? KNM_OK : fail(ctx, KNM_HIP_ERROR, "column sweep result conversion");
}

KernelOps dense_ops(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *C, int64_t M, int64_t ldc,
                    float sigma)
{
    KernelOps ops;
    ops.n = n;
    ops.M = M;
    ops.v = [=](const float *V, int t, float *W) { return do_knm_v(ctx, X, n, d, ldx, C, M, ldc, sigma, V, t, W); };
    ops.t_w = [=](const float *W, const float *wgt, int t, float *U) {
        return do_knm_t_w(ctx, X, n, d, ldx, C, M, ldc, sigma, W, wgt, t, U);
    };
    ops.t_w64 = [=](const float *W, const float *wgt, int t, double *U64) {
        return do_knm_t_w(ctx, X, n, d, ldx, C, M, ldc, sigma, W, wgt, t, nullptr, U64);
    };
    return ops;
}

// out <- A^-T ( T^-T K^T D K T^-1 A^-1 beta + lambda n A^-1 beta );  beta, out column-major, may not alias;
// D = diag(wgt) over the rows of X, identity if wgt is null
int linop_cols(knm_ctx *ctx, const knm_precond *p, LinopWork &wk, const KernelOps &ops, double lambda,
               const double *beta, int t, double *out, const float *wgt = nullptr)
{
    const int64_t n = ops.n, M = ops.M;
    const size_t bytes = sizeof(double) * M * t;
    double *v = wk.v.as<double>();
    hipError_t e = hipMemcpyAsync(v, beta, bytes, hipMemcpyDeviceToDevice, ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemcpyAsync", e);
    int st = tri_solve(ctx, p, p->A, p->Adinv, false, v, t); // v = A^-1 beta
    if (st) return st;
    e = hipMemcpyAsync(out, v, bytes, hipMemcpyDeviceToDevice, ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemcpyAsync", e);
    st = tri_solve(ctx, p, p->T, p->Tdinv, false, out, t); // z = T^-1 v
    if (st) return st;
    hipLaunchKernelGGL(f64_cols_to_f32_rows, grid1(M * t), dim3(256), 0, ctx->stream, out, M, t, wk.z32.as<float>());
    // c = K_nm^T (K_nm z), the O(n M) step
    st = ensure(ctx, &ctx->w_buf, &ctx->w_bytes, sizeof(float) * (size_t)n * t);
    if (st) return st;
    st = ops.v(wk.z32.as<float>(), t, ctx->w_buf);
    if (st) return st;
    st = t_w_cols(ctx, ops, ctx->w_buf, wgt, t, wk.u32.as<float>(), wk.u64.as<double>(), out);
    if (st) return st;
    st = tri_solve(ctx, p, p->T, p->Tdinv, true, out, t); // T^-T c
    if (st) return st;
    const double ln = lambda * (double)n;
    if (vec_axpy(ctx, M * t, ln, v, out) != KNM_OK)
        return KNM_HIP_ERROR;
    return tri_solve(ctx, p, p->A, p->Adinv, true, out, t); // A^-T (...)
}

} // namespace

extern "C" {

void knm_solver_release(knm_ctx *ctx)
{
    if (ctx && ctx->red_buf) {
        (void)hipFree(ctx->red_buf);
        ctx->red_buf = nullptr;
    }
    if (ctx && ctx->aux_stream) {
        (void)hipStreamDestroy(ctx->aux_stream);
        ctx->aux_stream = nullptr;
    }
}

int precond_free(knm_precond *p)
{
    if (!p) return KNM_INVALID_ARG;
    (void)hipSetDevice(p->device);
    if (p->buf) (void)hipFree(p->buf);
    if (p->Tdinv) (void)hipFree(p->Tdinv);
    if (p->Adinv) (void)hipFree(p->Adinv);
    if (p->xw) (void)hipFree(p->xw);
    if (p->blk) (void)hipFree(p->blk);
    delete p;
    return KNM_OK;
}

// Upper Cholesky factor in place, R^T R = A (upper or lower storage, leading dimension ld): the three-step
// column update of Sec. 4 (block Cholesky paragraph) on block rows of up to 4096.
//   Steps 1 and 2 (factor the diagonal tile, solve the block row against it) are carried out
//   together, left-looking over sub-panels of 512 rows and, inside them, steps of 128 rows: a
//   row group, from its diagonal to the last column, first loses the products with the rows
//   above it (one block product, contraction over the rows already done), then the diagonal
//   block of a step is factorised and inverted by the leaf kernel, then the rest of its rows is
//   multiplied by that inverse (in place: a 128-row tile of the block product reads exactly
//   the columns it writes).
//   Step 3 (trailing update, M^3 / 3 of the flop) is one rank-k launch per block row.
// `W` is a 128 x 128 scratch block, `bad` a device word initialised by the caller to ~0;
// first_bad receives the 1-based index of the first failing pivot, or 0.
constexpr int64_t kSubPanel = 512;

// events without timing, destroyed with the set
struct EventSet {
    std::vector<hipEvent_t> ev;
    ~EventSet()
    {
        for (hipEvent_t e : ev)
            if (e) (void)hipEventDestroy(e);
    }
    bool create(int64_t count)
    {
        ev.assign((size_t)count, nullptr);
        for (auto &e : ev)
            if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return false;
        return true;
    }
    hipEvent_t operator[](int64_t i) const { return ev[(size_t)i]; }
};

// second stream of the context (default priority, no implicit ordering with the legacy default
// stream: every dependency is an event), created on first use
static int aux_stream(knm_ctx *ctx, hipStream_t *out)
{
    if (!ctx->aux_stream) {
        hipStream_t s = nullptr;
        hipError_t e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipStreamCreateWithFlags", e);
        ctx->aux_stream = s;
    }
    *out = ctx->aux_stream;
    return KNM_OK;
}

// `lower`: the factor and the matrix it replaces are in lower storage (entry (r, c), r <= c, at
// A[c + r ld]); every product below then has its two index roles exchanged, and the pieces of a
// block row that straddle the diagonal are split into a symmetric update (which writes one triangle
// only) and a rectangle, because the other triangle belongs to the other factor.
static int chol_blocked(knm_ctx *ctx, double *A, int64_t ld, int64_t M, bool lower, double *W, unsigned long long *bad,
                        int64_t *first_bad)
{
    TraceRange range(lower ? "knm Cholesky of T D T^T / M + lambda I" : "knm Cholesky of K_MM");
    int64_t b = ((M + 7) / 8 + 255) / 256 * 256;
    if (b > 4096) b = 4096;
    const int64_t nb = (M + b - 1) / b;
    const unsigned long long none = ~0ull;
    hipError_t e = hipMemcpyAsync(bad, &none, sizeof(none), hipMemcpyHostToDevice, ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemcpyAsync", e);
    hipStream_t aux = nullptr;
    int st = aux_stream(ctx, &aux);
    if (st) return st;
    EventSet ev_rows, ev_rest;
    if (!ev_rows.create(nb) || !ev_rest.create(nb)) return fail(ctx, KNM_HIP_ERROR, "hipEventCreate");
    std::vector<char> have_rest(nb, 0);
    // entry (r, c) of the matrix, r <= c
    auto at = [&](int64_t r, int64_t c) { return lower ? A + c + (size_t)r * ld : A + r + (size_t)c * ld; };
    // rows [row, row + nr) of the columns from `col` on lose the products with rows [top, top + K)
    // of the same columns: R(row + i, col + j) -= sum_k R(top + k, row + i) R(top + k, col + j).
    // Here col == row: the nr x nr block on the diagonal and the rectangle to its right.
    auto update_rows = [&](int64_t top, int64_t K, int64_t row, int64_t nr) -> bool {
        const int64_t ncols = M - row;
        if (!lower) // upper storage: one product; what it writes below the diagonal block's diagonal is unused space
            return launch_gemm_f64(0, nr, ncols, K, -1.0, at(top, row), ld, at(top, row), ld, 1.0, at(row, row), ld,
                                   ctx->stream) == hipSuccess;
        const double *P = at(top, row); // element (top + k, row + x) at P[x + k ld]
        if (launch_rank_k_upper(1, nr, K, -1.0, P, ld, nullptr, 0, 1.0, 0.0, at(row, row), ld, ctx->stream, 1) != hipSuccess)
            return false;
        return ncols == nr || launch_gemm_f64(1, ncols - nr, nr, K, -1.0, P + nr, ld, P, ld, 1.0, at(row, row + nr), ld,
                                              ctx->stream, 1) == hipSuccess;
    };
    for (int64_t k = 0; k < nb; ++k) {
        const int64_t r0 = k * b;
        const int64_t w = (M - r0 < b) ? M - r0 : b;
        for (int64_t S0 = 0; S0 < w; S0 += kSubPanel) {
            // the sub-panel's rows lose the products with the block row's rows above them at once
            // (four tile rows per launch); inside it the 128-row steps only reach back to its top
            const int64_t sw = (w - S0 < kSubPanel) ? w - S0 : kSubPanel;
            const int64_t prow = r0 + S0;
            if (S0 > 0 && !update_rows(r0, S0, prow, sw)) return fail(ctx, KNM_HIP_ERROR, "block row update launch");
            for (int64_t s0 = 0; s0 < sw; s0 += kLeaf) {
                const int64_t row = prow + s0;
                const int nbk = (int)((sw - s0 < kLeaf) ? sw - s0 : kLeaf);
                const int64_t ncols = M - row;
                if (s0 > 0 && !update_rows(prow, s0, row, nbk)) return fail(ctx, KNM_HIP_ERROR, "block row update launch");
                hipLaunchKernelGGL(potrf_trtri_leaf_kernel, dim3(1), dim3(kLeafThreads), 0, ctx->stream, at(row, row), ld, nbk,
                                   W, (int64_t)kLeaf, row, bad, lower ? 1 : 0);
                if (ncols > nbk) {
                    // the rest of the rows times the inverse: R(row + i, c) <- sum_k W(k, i) R(row + k, c)
                    double *right = at(row, row + nbk);
                    const hipError_t le =
                        lower ? launch_gemm_f64(1, ncols - nbk, nbk, nbk, 1.0, right, ld, W, kLeaf, 0.0, right, ld, ctx->stream)
                              : launch_gemm_f64(0, nbk, ncols - nbk, nbk, 1.0, W, kLeaf, right, ld, 0.0, right, ld, ctx->stream);
                    if (le != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "block row solve launch");
                }
            }
        }
        const int64_t rest = M - r0 - w;
        if (rest == 0) break;
        // Step 3 with one block row of look-ahead.  The part of the trailing matrix that the next
        // block row needs (its own rows) is updated on the main stream, which then goes on to
        // steps 1 and 2 of that block row; the remainder (most of the flop) runs on the second
        // stream meanwhile and fills the chip, which those short dependent launches cannot.
        const int64_t w2 = (rest < b) ? rest : b;
        const int64_t c0 = r0 + w;                 // first trailing row and column
        const double *Akr = at(r0, c0);            // block row to the right of the diagonal block
        const double *Akr2 = at(r0, c0 + w2);
        const int form = lower ? 1 : 0, tc = lower ? 1 : 0;
        if (hipEventRecord(ev_rows[k], ctx->stream) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipEventRecord");
        if (k > 0 && have_rest[k - 1] && hipStreamWaitEvent(ctx->stream, ev_rest[k - 1], 0) != hipSuccess)
            return fail(ctx, KNM_HIP_ERROR, "hipStreamWaitEvent");
        if (launch_rank_k_upper(form, w2, w, -1.0, Akr, ld, nullptr, 0, 1.0, 0.0, at(c0, c0), ld, ctx->stream, tc) != hipSuccess)
            return fail(ctx, KNM_HIP_ERROR, "trailing update launch");
        if (rest > w2) {
            // R(c0 + i, c0 + w2 + j) -= sum_k R(r0 + k, c0 + i) R(r0 + k, c0 + w2 + j)
            const hipError_t le =
                lower ? launch_gemm_f64(1, rest - w2, w2, w, -1.0, Akr2, ld, Akr, ld, 1.0, at(c0, c0 + w2), ld, ctx->stream, 1)
                      : launch_gemm_f64(0, w2, rest - w2, w, -1.0, Akr, ld, Akr2, ld, 1.0, at(c0, c0 + w2), ld, ctx->stream);
            if (le != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "trailing update launch");
            if (hipStreamWaitEvent(aux, ev_rows[k], 0) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipStreamWaitEvent");
            if (launch_rank_k_upper(form, rest - w2, w, -1.0, Akr2, ld, nullptr, 0, 1.0, 0.0, at(c0 + w2, c0 + w2), ld, aux,
                                    tc) != hipSuccess)
                return fail(ctx, KNM_HIP_ERROR, "trailing update launch");
            if (hipEventRecord(ev_rest[k], aux) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipEventRecord");
            have_rest[k] = 1;
        }
    }
    // the second stream's last update (its stream order makes it the last of all) before anything else
    for (int64_t k = nb - 1; k >= 0; --k)
        if (have_rest[k]) {
            if (hipStreamWaitEvent(ctx->stream, ev_rest[k], 0) != hipSuccess)
                return fail(ctx, KNM_HIP_ERROR, "hipStreamWaitEvent");
            break;
        }
    unsigned long long got = none;
    e = hipMemcpyAsync(&got, bad, sizeof(got), hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "factorisation", e);
    *first_bad = (got == none) ? 0 : (int64_t)got;
    return KNM_OK;
}

// A <- upper Cholesky factor of T D T^T / M + lambda I, D = diag(dw) (identity if dw is null), and
// the inverses of its diagonal blocks.  T is upper triangular, so entry (i, j) of the product
// only sums over k >= max(i, j): M^3 / 3 flop instead of the M^3 of a dense rank-M update,
// in one launch of the rank-k kernel, which skips the vanishing part tile by tile.  The product is
// written mirrored, into the lower storage of A beside T, and factorised there in place.
static int build_second_factor(knm_ctx *ctx, knm_precond *p, double lambda, const double *dw,
                               int64_t *bad_pivot)
{
    const int64_t M = p->M;
    *bad_pivot = 0;
    DevBuf leaf, badbuf;
    int st = leaf.alloc(ctx, sizeof(double) * kLeaf * kLeaf);
    if (!st) st = badbuf.alloc(ctx, sizeof(unsigned long long));
    if (st) return st;
    {
        TraceRange range("knm triangular product T D T^T");
        if (launch_rank_k_upper(1, M, M, 1.0 / (double)M, p->T, p->ld, dw, 1, 0.0, lambda, p->A, p->ld, ctx->stream, 1) !=
            hipSuccess)
            return fail(ctx, KNM_HIP_ERROR, "triangular product launch");
    }
    int64_t pivot = 0;
    st = chol_blocked(ctx, p->A, p->ld, M, true, leaf.as<double>(), badbuf.as<unsigned long long>(), &pivot);
    if (st) return st;
    if (pivot == 0) {
        const unsigned long long none = ~0ull;
        unsigned long long got = none;
        hipError_t err = hipMemcpyAsync(badbuf.p, &none, sizeof(none), hipMemcpyHostToDevice, ctx->stream);
        if (err == hipSuccess) {
            hipLaunchKernelGGL(diag_check_kernel, grid1(M), dim3(256), 0, ctx->stream, p->A, p->ld, M,
                               badbuf.as<unsigned long long>());
            err = hipMemcpyAsync(&got, badbuf.p, sizeof(got), hipMemcpyDeviceToHost, ctx->stream);
        }
        if (err == hipSuccess) err = hipStreamSynchronize(ctx->stream);
        if (err != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "diagonal check", err);
        pivot = (got == none) ? 0 : (int64_t)got;
    }
    if (pivot != 0) {
        *bad_pivot = pivot;
        return fail(ctx, KNM_NOT_PD, "T D T^T / M + lambda I is not positive definite");
    }
    DevBuf merge;
    st = merge.alloc(ctx, sizeof(double) * (size_t)(p->sb / 2) * (size_t)(p->sb / 2));
    if (!st) st = invert_diag_blocks(ctx, p, p->A, p->Adinv, merge.as<double>());
    if (st) return st;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "second factor"); // scratch is freed on return
    if (hipGetLastError() != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "preconditioner kernel launch");
    p->lambda = lambda;
    return KNM_OK;
}

// fill_kmm(K, ldk) writes the upper triangle of K_MM + jitter I (column-major, leading dimension ldk)
static int precond_build_from(knm_ctx *ctx, int64_t M, const std::function<int(double *, int64_t)> &fill_kmm, double lambda,
                              double jitter, bool second_factor, knm_precond **out, int64_t *bad_pivot_or_null)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!out) return fail(ctx, KNM_INVALID_ARG, "null output");
    *out = nullptr;
    if (bad_pivot_or_null) *bad_pivot_or_null = 0;
    if (M <= 0 || !(lambda >= 0.0) || !(jitter >= 0.0)) return fail(ctx, KNM_INVALID_ARG, "bad preconditioner argument");
    if (M > 2000000000LL / 1) return fail(ctx, KNM_UNSUPPORTED, "M too large");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    int st = KNM_OK;

    knm_precond *p = new (std::nothrow) knm_precond();
    if (!p) return fail(ctx, KNM_ALLOC, "host allocation");
    p->device = ctx->device;
    p->M = M;
    p->lambda = lambda;
    p->jitter = jitter;
    p->ld = M + 2 + (M & 1); // even: every column of either factor starts 16-byte aligned
    const size_t bytes = sizeof(double) * (size_t)p->ld * (size_t)M;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&p->buf), bytes);
    p->T = p->buf;
    p->A = p->buf ? p->buf + 2 : nullptr;
    p->sb = solve_block_width(M);
    const int64_t nblk = (M + p->sb - 1) / p->sb;
    const size_t dbytes = sizeof(double) * (size_t)nblk * p->sb * p->sb;
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&p->Tdinv), dbytes);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&p->Adinv), dbytes);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&p->xw), sizeof(double) * (size_t)M * kSolveCols);
    if (e == hipSuccess && M >= kProductSolveMinM)
        e = hipMalloc(reinterpret_cast<void **>(&p->blk), sizeof(double) * (size_t)p->sb * p->sb);
    DevBuf leaf;
    if (e != hipSuccess || leaf.alloc(ctx, sizeof(double) * kLeaf * kLeaf)) {
        (void)hipGetLastError();
        precond_free(p);
        return fail(ctx, KNM_ALLOC, "hipMalloc(preconditioner)", e);
    }
    auto bail = [&](int status, const char *what) {
        precond_free(p);
        return fail(ctx, status, what);
    };

    st = fill_kmm(p->T, p->ld);
    if (st) {
        precond_free(p);
        return st;
    }

    DevBuf badbuf;
    if (badbuf.alloc(ctx, sizeof(unsigned long long))) return bail(KNM_ALLOC, "hipMalloc");
    // returns the failing pivot (1-based) of the factor in `F`, or 0
    auto bad_diagonal = [&](const double *F, int64_t *pivot) -> hipError_t {
        const unsigned long long none = ~0ull;
        unsigned long long got = none;
        hipError_t err = hipMemcpyAsync(badbuf.p, &none, sizeof(none), hipMemcpyHostToDevice, ctx->stream);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(diag_check_kernel, grid1(M), dim3(256), 0, ctx->stream, F, p->ld, M,
                           badbuf.as<unsigned long long>());
        err = hipMemcpyAsync(&got, badbuf.p, sizeof(got), hipMemcpyDeviceToHost, ctx->stream);
        if (err == hipSuccess) err = hipStreamSynchronize(ctx->stream);
        *pivot = (got == none) ? 0 : (int64_t)got;
        return err;
    };

    int64_t host_info = 0;
    {
        int st2 = chol_blocked(ctx, p->T, p->ld, M, false, leaf.as<double>(), badbuf.as<unsigned long long>(), &host_info);
        if (st2) {
            precond_free(p);
            return st2;
        }
    }
    int64_t pivot = host_info;
    if (pivot == 0 && bad_diagonal(p->T, &pivot) != hipSuccess) return bail(KNM_HIP_ERROR, "diagonal check");
    if (pivot != 0) {
        if (bad_pivot_or_null) *bad_pivot_or_null = pivot;
        return bail(KNM_NOT_PD, "K_MM + jitter I is not positive definite");
    }
    if (hipGetLastError() != hipSuccess) return bail(KNM_HIP_ERROR, "preconditioner kernel launch");
    DevBuf merge;
    st = merge.alloc(ctx, sizeof(double) * (size_t)(p->sb / 2) * (size_t)(p->sb / 2));
    if (!st) st = invert_diag_blocks(ctx, p, p->T, p->Tdinv, merge.as<double>());
    if (!st && hipStreamSynchronize(ctx->stream) != hipSuccess) st = fail(ctx, KNM_HIP_ERROR, "first factor");
    if (st) {
        precond_free(p);
        return st;
    }
    if (second_factor) {
        int64_t bad = 0;
        st = build_second_factor(ctx, p, lambda, nullptr, &bad);
        if (st) {
            if (bad_pivot_or_null) *bad_pivot_or_null = -bad;
            precond_free(p);
            return st;
        }
    }
    *out = p;
    return KNM_OK;
}

static int precond_build_impl(knm_ctx *ctx, const float *C, int64_t M, int d, int64_t ldc, float sigma, double lambda,
                              double jitter, bool second_factor, knm_precond **out, int64_t *bad_pivot_or_null)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!C || M <= 0 || d <= 0 || ldc < d || !(sigma > 0.0f))
        return fail(ctx, KNM_INVALID_ARG, "bad preconditioner argument");
    auto fill = [=](double *K, int64_t ldk) {
        const dim3 tb(256);
        const dim3 tg((unsigned)((M + kKmmTile - 1) / kKmmTile), (unsigned)((M + kKmmTile - 1) / kKmmTile));
        const int kind = ctx->kernel_kind;
        const double scale = kind == KNM_KERNEL_GAUSSIAN   ? 1.0 / (2.0 * (double)sigma * (double)sigma)
                             : kind == KNM_KERNEL_MATERN32 ? sqrt(3.0) / (double)sigma
                             : kind == KNM_KERNEL_MATERN52 ? sqrt(5.0) / (double)sigma
                                                           : 1.0 / (double)sigma;
        hipLaunchKernelGGL(kmm_kernel, tg, tb, 0, ctx->stream, C, M, d, ldc, kind, scale, jitter, K, ldk);
        return hipGetLastError() == hipSuccess ? KNM_OK : fail(ctx, KNM_HIP_ERROR, "kmm_kernel launch");
    };
    return precond_build_from(ctx, M, fill, lambda, jitter, second_factor, out, bad_pivot_or_null);
}

int precond_build(knm_ctx *ctx, const float *C, int64_t M, int d, int64_t ldc, float sigma, double lambda,
                  double jitter, knm_precond **out, int64_t *bad_pivot_or_null)
{
    return precond_build_impl(ctx, C, M, d, ldc, sigma, lambda, jitter, true, out, bad_pivot_or_null);
}

int precond_build_csr(knm_ctx *ctx, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values, int64_t M,
                      int64_t d, float sigma, double lambda, double jitter, knm_precond **out,
                      int64_t *bad_pivot_or_null)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!c_indptr || M <= 0 || d <= 0 || d >= 0x7fffffffLL || !(sigma > 0.0f))
        return fail(ctx, KNM_INVALID_ARG, "bad preconditioner argument");
    auto fill = [=](double *K, int64_t ldk) {
        return sparse_kmm(ctx, c_indptr, c_indices, c_values, M, d, sigma, jitter, K, ldk);
    };
    return precond_build_from(ctx, M, fill, lambda, jitter, true, out, bad_pivot_or_null);
}

int precond_get_factors(knm_ctx *ctx, const knm_precond *p, double *T_host, double *A_host)
{
    if (!ctx || !p) return KNM_INVALID_ARG;
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    const int64_t M = p->M;
    std::vector<double> tmp((size_t)M * M);
    const double *src[2] = {p->T, p->A};
    double *dst[2] = {T_host, A_host};
    for (int k = 0; k < 2; ++k) {
        if (!dst[k]) continue;
        hipError_t e = hipStreamSynchronize(ctx->stream);
        if (e == hipSuccess)
            e = hipMemcpy2D(tmp.data(), sizeof(double) * M, src[k], sizeof(double) * p->ld, sizeof(double) * M, (size_t)M,
                            hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemcpy(factor)", e);
        // T: upper storage, entry (i, j) at i + j M of the copy; A: lower storage, at j + i M
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < M; ++j) dst[k][i * M + j] = (j >= i) ? (k == 0 ? tmp[i + j * M] : tmp[j + i * M]) : 0.0;
    }
    return KNM_OK;
}

int precond_get_block(knm_ctx *ctx, const knm_precond *p, int second, int64_t row0, int64_t col0, int64_t rows,
                      int64_t cols, double *out_host)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!p || !out_host || row0 < 0 || col0 < 0 || rows <= 0 || cols <= 0 || row0 + rows > p->M || col0 + cols > p->M)
        return fail(ctx, KNM_INVALID_ARG, "bad factor block");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    // gathered on the device (a row of an upper-storage factor is strided in memory), then one copy
    DevBuf tmp;
    int st = tmp.alloc(ctx, sizeof(double) * (size_t)rows * (size_t)cols);
    if (st) return st;
    hipLaunchKernelGGL(gather_block_kernel, grid1(rows * cols), dim3(256), 0, ctx->stream, second ? p->A : p->T, p->ld,
                       second ? 1 : 0, row0, col0, rows, cols, tmp.as<double>());
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess) e = hipMemcpy(out_host, tmp.p, sizeof(double) * (size_t)rows * (size_t)cols, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "factor block copy", e);
    return KNM_OK;
}

int falkon_linop_weighted(knm_ctx *ctx, const knm_precond *p, const float *X, int64_t n, int d, int64_t ldx,
                          const float *C, int64_t M, int64_t ldc, float sigma, double lambda, const float *dw_or_null,
                          const double *beta, int t, double *out)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!p || !X || !C || !beta || !out || n <= 0 || M <= 0 || d <= 0 || t <= 0 || ldx < d || ldc < d ||
        !(sigma > 0.0f) || p->M != M)
        return fail(ctx, KNM_INVALID_ARG, "bad linop argument");
    if (d > knm_max_d() || t > knm_max_t()) return fail(ctx, KNM_UNSUPPORTED, "d or t above compiled maximum");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    int st = KNM_OK;
    LinopWork wk;
    DevBuf bc, oc;
    st = wk.alloc(ctx, M, t);
    if (!st) st = bc.alloc(ctx, sizeof(double) * M * t);
    if (!st) st = oc.alloc(ctx, sizeof(double) * M * t);
    if (st) return st;
    hipLaunchKernelGGL(f64_rows_to_cols, grid1(M * t), dim3(256), 0, ctx->stream, beta, M, t, bc.as<double>(), 0);
    st = linop_cols(ctx, p, wk, dense_ops(ctx, X, n, d, ldx, C, M, ldc, sigma), lambda, bc.as<double>(), t, oc.as<double>(),
                    dw_or_null);
    if (st) return st;
    hipLaunchKernelGGL(f64_rows_to_cols, grid1(M * t), dim3(256), 0, ctx->stream, oc.as<double>(), M, t, out, 1);
    hipError_t e = hipStreamSynchronize(ctx->stream); // temporaries are freed on return
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "falkon_linop", e);
    return KNM_OK;
}

int falkon_linop(knm_ctx *ctx, const knm_precond *p, const float *X, int64_t n, int d, int64_t ldx, const float *C,
                 int64_t M, int64_t ldc, float sigma, double lambda, const double *beta, int t, double *out)
{
    return falkon_linop_weighted(ctx, p, X, n, d, ldx, C, M, ldc, sigma, lambda, nullptr, beta, t, out);
}

int precond_rank_k_update(knm_ctx *ctx, int form_nt, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                          const double *w_or_null, int triangular, double beta, double shift, double *C, int64_t ldc)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (n < 0 || k < 0 || !C || ldc < (n > 1 ? n : 1) || (n > 0 && k > 0 && !A))
        return fail(ctx, KNM_INVALID_ARG, "bad rank-k update argument");
    if (n > 0 && k > 0 && lda < (form_nt ? n : k)) return fail(ctx, KNM_INVALID_ARG, "leading dimension too small");
    if (triangular && !form_nt) return fail(ctx, KNM_INVALID_ARG, "triangular operand needs the row-contiguous form");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    hipError_t e = launch_rank_k_upper(form_nt, n, k, alpha, A, lda, w_or_null, triangular, beta, shift, C, ldc,
                                       ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "rank-k update launch", e);
    return KNM_OK;
}

int precond_block_product(knm_ctx *ctx, int a_nt, int64_t ni, int64_t nj, int64_t k, double alpha, const double *A,
                          int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (ni < 0 || nj < 0 || k < 0 || !C || ldc < (ni > 1 ? ni : 1) || (ni > 0 && nj > 0 && k > 0 && (!A || !B)))
        return fail(ctx, KNM_INVALID_ARG, "bad block product argument");
    if (ni > 0 && nj > 0 && k > 0 && (lda < (a_nt ? ni : k) || ldb < k))
        return fail(ctx, KNM_INVALID_ARG, "leading dimension too small");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    hipError_t e = launch_gemm_f64(a_nt, ni, nj, k, alpha, A, lda, B, ldb, beta, C, ldc, ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "block product launch", e);
    return KNM_OK;
}

int precond_solve(knm_ctx *ctx, const knm_precond *p, int transpose, const double *b, int t, double *out)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!p || !b || !out || t <= 0 || t > knm_max_t()) return fail(ctx, KNM_INVALID_ARG, "bad solve argument");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    const int64_t M = p->M;
    DevBuf bc;
    int st = bc.alloc(ctx, sizeof(double) * M * t);
    if (st) return st;
    double *v = bc.as<double>();
    hipLaunchKernelGGL(f64_rows_to_cols, grid1(M * t), dim3(256), 0, ctx->stream, b, M, t, v, 0);
    if (transpose) {
        st = tri_solve(ctx, p, p->T, p->Tdinv, true, v, t);
        if (!st) st = tri_solve(ctx, p, p->A, p->Adinv, true, v, t);
    } else {
        st = tri_solve(ctx, p, p->A, p->Adinv, false, v, t);
        if (!st) st = tri_solve(ctx, p, p->T, p->Tdinv, false, v, t);
    }
    if (st) return st;
    hipLaunchKernelGGL(f64_rows_to_cols, grid1(M * t), dim3(256), 0, ctx->stream, v, M, t, out, 1);
    hipError_t e = hipStreamSynchronize(ctx->stream); // the temporary is freed on return
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "precond_solve", e);
    return KNM_OK;
}

int precond_reweight(knm_ctx *ctx, knm_precond *p, double lambda, const double *dw_or_null, int64_t *bad_pivot_or_null)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (bad_pivot_or_null) *bad_pivot_or_null = 0;
    if (!p || !(lambda >= 0.0)) return fail(ctx, KNM_INVALID_ARG, "bad preconditioner argument");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    int st = KNM_OK;
    int64_t bad = 0;
    st = build_second_factor(ctx, p, lambda, dw_or_null, &bad);
    if (bad_pivot_or_null) *bad_pivot_or_null = -bad;
    return st;
}

// Alg. 1 from the right-hand side on, with the preconditioner built: exactly `iters` steps of
// preconditioned CG on the operator of Eq. 9, then alpha = T^-1 A^-1 beta.  Takes ownership of p.
static int fit_core(knm_ctx *ctx, const KernelOps &ops, knm_precond *p, const float *Y, int t, double lambda, int iters,
                    float *alpha, double *resid_norms_or_null, std::chrono::steady_clock::time_point t_start)
{
    using clk = std::chrono::steady_clock;
    auto secs = [](clk::time_point a, clk::time_point b) { return std::chrono::duration<double>(b - a).count(); };
    const clk::time_point t_precond = clk::now();
    struct Guard {
        knm_precond *p;
        ~Guard() { precond_free(p); }
    } guard{p};
    const int64_t M = ops.M;
    int st = KNM_OK;

    const int64_t len = M * t;
    LinopWork wk;
    DevBuf beta, r, pv, q, r32;
    st = wk.alloc(ctx, M, t);
    if (!st) st = beta.alloc(ctx, sizeof(double) * len);
    if (!st) st = r.alloc(ctx, sizeof(double) * len);
    if (!st) st = pv.alloc(ctx, sizeof(double) * len);
    if (!st) st = q.alloc(ctx, sizeof(double) * len);
    if (!st) st = r32.alloc(ctx, sizeof(float) * len);
    if (st) return st;
    double *db = beta.as<double>(), *dr = r.as<double>(), *dp = pv.as<double>(), *dq = q.as<double>();

    // rhs = A^-T T^-T K_nm^T Y
    CrossTermScope cross(ctx);
    st = cross.begin();
    if (st) return st;
    st = t_w_cols(ctx, ops, Y, nullptr, t, r32.as<float>(), wk.u64.as<double>(), dr);
    if (st) return st;
    bool repeat = false;
    st = cross.check(&repeat);
    if (!st && repeat) st = t_w_cols(ctx, ops, Y, nullptr, t, r32.as<float>(), wk.u64.as<double>(), dr);
    if (st) return st;
    st = tri_solve(ctx, p, p->T, p->Tdinv, true, dr, t);
    if (!st) st = tri_solve(ctx, p, p->A, p->Adinv, true, dr, t);
    if (st) return st;
    hipError_t e = hipMemsetAsync(db, 0, sizeof(double) * len, ctx->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(dp, dr, sizeof(double) * len, hipMemcpyDeviceToDevice, ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "CG initialisation", e);

    auto vec_ok = [&](int status) { return status == KNM_OK; };
    std::vector<double> rho(t), pq(t);
    for (int c = 0; c < t; ++c) {
        if (!vec_ok(vec_dot(ctx, M, dr + c * M, dr + c * M, &rho[c])))
            return fail(ctx, KNM_HIP_ERROR, "vector reduction");
        if (resid_norms_or_null) resid_norms_or_null[c] = std::sqrt(rho[c]);
    }
    const clk::time_point t_rhs = clk::now(); // the host-pointer dot products above synchronise
    for (int it = 0; it < iters; ++it) {
        TraceRange range("knm CG iteration");
        st = linop_cols(ctx, p, wk, ops, lambda, dp, t, dq);
        if (st) return st;
        for (int c = 0; c < t; ++c) {
            double *pc = dp + c * M, *qc = dq + c * M, *rc = dr + c * M, *bc = db + c * M;
            if (!vec_ok(vec_dot(ctx, M, pc, qc, &pq[c]))) return fail(ctx, KNM_HIP_ERROR, "vector reduction");
            const double a = (pq[c] != 0.0) ? rho[c] / pq[c] : 0.0;
            const double ma = -a;
            double rn = 0.0;
            if (!vec_ok(vec_axpy(ctx, M, a, pc, bc)) ||
                !vec_ok(vec_axpy(ctx, M, ma, qc, rc)) ||
                !vec_ok(vec_dot(ctx, M, rc, rc, &rn)))
                return fail(ctx, KNM_HIP_ERROR, "CG vector update");
            const double b = (rho[c] != 0.0) ? rn / rho[c] : 0.0;
            const double one = 1.0;
            if (!vec_ok(vec_scal(ctx, M, b, pc)) ||
                !vec_ok(vec_axpy(ctx, M, one, rc, pc)))
                return fail(ctx, KNM_HIP_ERROR, "CG vector update");
            rho[c] = rn;
            if (resid_norms_or_null) resid_norms_or_null[(int64_t)(it + 1) * t + c] = std::sqrt(rn);
        }
    }
    // alpha = T^-1 A^-1 beta
    st = tri_solve(ctx, p, p->A, p->Adinv, false, db, t);
    if (!st) st = tri_solve(ctx, p, p->T, p->Tdinv, false, db, t);
    if (st) return st;
    hipLaunchKernelGGL(f64_cols_to_f32_rows, grid1(len), dim3(256), 0, ctx->stream, db, M, t, alpha);
    const clk::time_point t_iters = clk::now(); // each iteration ends with synchronising dot products
    e = hipStreamSynchronize(ctx->stream); // temporaries are freed on return
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "falkon_fit", e);
    ctx->fit_seconds[0] = secs(t_start, t_precond);
    ctx->fit_seconds[1] = secs(t_precond, t_rhs);
    ctx->fit_seconds[2] = secs(t_rhs, t_iters);
    ctx->fit_seconds[3] = secs(t_iters, clk::now());
    return KNM_OK;
}

int falkon_fit(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *Y, int t, const float *C,
               int64_t M, int64_t ldc, float sigma, double lambda, double jitter, int iters, float *alpha,
               double *resid_norms_or_null)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!X || !Y || !C || !alpha || n <= 0 || M <= 0 || d <= 0 || t <= 0 || iters <= 0 || ldx < d || ldc < d ||
        !(sigma > 0.0f) || !(lambda >= 0.0) || !(jitter >= 0.0))
        return fail(ctx, KNM_INVALID_ARG, "bad fit argument");
    if (d > knm_max_d() || t > knm_max_t()) return fail(ctx, KNM_UNSUPPORTED, "d or t above compiled maximum");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    const std::chrono::steady_clock::time_point t_start = std::chrono::steady_clock::now();
    knm_precond *p = nullptr;
    int st = precond_build(ctx, C, M, d, ldc, sigma, lambda, jitter, &p, nullptr); // synchronises
    if (st) return st;
    return fit_core(ctx, dense_ops(ctx, X, n, d, ldx, C, M, ldc, sigma), p, Y, t, lambda, iters, alpha,
                    resid_norms_or_null, t_start);
}

int falkon_fit_csr(knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values, int64_t n,
                   const float *Y, int t, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values,
                   int64_t M, int64_t d, float sigma, double lambda, double jitter, int iters, float *alpha,
                   double *resid_norms_or_null)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!x_indptr || !c_indptr || !Y || !alpha || n <= 0 || M <= 0 || d <= 0 || t <= 0 || iters <= 0 ||
        !(sigma > 0.0f) || !(lambda >= 0.0) || !(jitter >= 0.0))
        return fail(ctx, KNM_INVALID_ARG, "bad fit argument");
    if (d >= 0x7fffffffLL || M >= 0x7fffffffLL || t > knm_max_t())
        return fail(ctx, KNM_UNSUPPORTED, "d, M or t above the supported maximum");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    const std::chrono::steady_clock::time_point t_start = std::chrono::steady_clock::now();
    SparseProducts sp; // outlives the fit: the sweeps use its workspace
    int st = sp.prepare(ctx, x_indptr, x_indices, x_values, n, c_indptr, c_indices, c_values, M, d, sigma);
    if (st) return st;
    knm_precond *p = nullptr;
    st = precond_build_csr(ctx, c_indptr, c_indices, c_values, M, d, sigma, lambda, jitter, &p, nullptr);
    if (st) return st;
    KernelOps ops;
    ops.n = n;
    ops.M = M;
    ops.v = [&sp](const float *V, int tt, float *W) { return sp.v(V, tt, W); };
    ops.t_w = [&sp](const float *W, const float *wgt, int tt, float *U) { return sp.t_w(W, wgt, tt, U); };
    return fit_core(ctx, ops, p, Y, t, lambda, iters, alpha, resid_norms_or_null, t_start);
}

int knm_v_csr(knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values, int64_t n,
              const int64_t *c_indptr, const int64_t *c_indices, const float *c_values, int64_t M, int64_t d,
              float sigma, const float *V, int t, float *W)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!x_indptr || !c_indptr || !V || !W || n <= 0 || M <= 0 || d <= 0 || t <= 0 || !(sigma > 0.0f))
        return fail(ctx, KNM_INVALID_ARG, "bad shape or pointer");
    if (d >= 0x7fffffffLL || M >= 0x7fffffffLL || t > knm_max_t())
        return fail(ctx, KNM_UNSUPPORTED, "d, M or t above the supported maximum");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    SparseProducts sp;
    int st = sp.prepare(ctx, x_indptr, x_indices, x_values, n, c_indptr, c_indices, c_values, M, d, sigma);
    if (!st) st = sp.v(V, t, W);
    if (st) return st;
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "knm_v_csr", e);
    return KNM_OK;
}

int knm_get_fit_timing(const knm_ctx *ctx, double *seconds)
{
    if (!ctx || !seconds) return KNM_INVALID_ARG;
    for (int i = 0; i < 4; ++i) seconds[i] = ctx->fit_seconds[i];
    return KNM_OK;
}

int falkon_predict(knm_ctx *ctx, const float *Xtest, int64_t ntest, int d, int64_t ldx, const float *C, int64_t M,
                   int64_t ldc, float sigma, const float *alpha, int t, float *out)
{
    return knm_v(ctx, Xtest, ntest, d, ldx, C, M, ldc, sigma, alpha, t, out);
}

// Newton iteration of the logistic fit (Alg. 2) on whatever storage the points have: `ops` are the
// two sweeps of k(X, C), `centres_v` gives k(C, C) a (M floats); p holds T (its second factor is
// rebuilt at every step) and is freed on return.
static int logfalkon_core(knm_ctx *ctx, const KernelOps &ops, const std::function<int(const float *, float *)> &centres_v,
                          knm_precond *p, const float *y, const float *yC, const double *lambdas, const int *iters,
                          int n_steps, double jitter, float *alpha, double *loss_or_null)
{
    const int64_t n = ops.n, M = ops.M;
    int st = KNM_OK;
    struct Guard {
        knm_precond *p;
        ~Guard() { precond_free(p); }
    } guard{p};

    LinopWork wk;
    DevBuf a64, a32, z, zc, g, dw, dm, lossv, u32, beta, r, pv, q;
    st = wk.alloc(ctx, M, 1);
    if (!st) st = a64.alloc(ctx, sizeof(double) * M);
    if (!st) st = a32.alloc(ctx, sizeof(float) * M);
    if (!st) st = z.alloc(ctx, sizeof(float) * n);
    if (!st) st = zc.alloc(ctx, sizeof(float) * M);
    if (!st) st = g.alloc(ctx, sizeof(float) * n);
    if (!st) st = dw.alloc(ctx, sizeof(float) * n);
    if (!st) st = dm.alloc(ctx, sizeof(double) * M);
    if (!st && loss_or_null) st = lossv.alloc(ctx, sizeof(double) * n);
    if (!st) st = u32.alloc(ctx, sizeof(float) * M);
    if (!st) st = beta.alloc(ctx, sizeof(double) * M);
    if (!st) st = r.alloc(ctx, sizeof(double) * M);
    if (!st) st = pv.alloc(ctx, sizeof(double) * M);
    if (!st) st = q.alloc(ctx, sizeof(double) * M);
    if (st) return st;
    double *da = a64.as<double>(), *db = beta.as<double>(), *dr = r.as<double>(), *dp = pv.as<double>(),
           *dq = q.as<double>();
    hipError_t e = hipMemsetAsync(da, 0, sizeof(double) * M, ctx->stream);
    if (e == hipSuccess) e = hipMemsetAsync(a32.p, 0, sizeof(float) * M, ctx->stream);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemsetAsync", e);
    auto vec_ok = [&](int status) { return status == KNM_OK; };
    // predictions at the rows and at the centres for the current alpha, and the loss terms
    auto evaluate = [&](bool derivatives, double *mean_loss) -> int {
        int s2 = ops.v(a32.as<float>(), 1, z.as<float>());
        if (s2) return s2;
        hipLaunchKernelGGL(logistic_terms_kernel, grid1(n), dim3(256), 0, ctx->stream, z.as<float>(), y, n,
                           derivatives ? g.as<float>() : nullptr, derivatives ? dw.as<float>() : nullptr,
                           (double *)nullptr, mean_loss ? lossv.as<double>() : nullptr);
        if (mean_loss) {
            // sum in pieces that fit the 32-bit BLAS interface
            double total = 0.0;
            for (int64_t o = 0; o < n; o += (1 << 30)) {
                const int64_t len = (n - o < (1 << 30)) ? n - o : (1 << 30);
                double part = 0.0;
                if (!vec_ok(vec_dot(ctx, len, lossv.as<double>() + o, nullptr, &part)))
                    return fail(ctx, KNM_HIP_ERROR, "loss reduction");
                total += part;
            }
            *mean_loss = total / (double)n;
        }
        return KNM_OK;
    };

    CrossTermScope cross(ctx);
    st = cross.begin();
    if (st) return st;
    for (int k = 0; k < n_steps; ++k) {
        const double mu = lambdas[k];
        st = evaluate(true, loss_or_null ? loss_or_null + k : nullptr);
        if (st) return st;
        if (k == 0) {
            bool repeat = false;
            st = cross.check(&repeat);
            if (!st && repeat) st = evaluate(true, loss_or_null ? loss_or_null : nullptr);
            if (st) return st;
        }
        // weights at the centres -> second factor of the preconditioner for this step
        st = centres_v(a32.as<float>(), zc.as<float>());
        if (st) return st;
        hipLaunchKernelGGL(logistic_terms_kernel, grid1(M), dim3(256), 0, ctx->stream, zc.as<float>(), yC, M,
                           (float *)nullptr, (float *)nullptr, dm.as<double>(), (double *)nullptr);
        int64_t bad = 0;
        st = build_second_factor(ctx, p, mu, dm.as<double>(), &bad);
        if (st) return st;
        // right-hand side  -P^T (K^T g + mu n (K_MM + eps I) alpha)
        st = ops.t_w(g.as<float>(), nullptr, 1, u32.as<float>());
        if (st) return st;
        hipLaunchKernelGGL(newton_rhs_kernel, grid1(M), dim3(256), 0, ctx->stream, u32.as<float>(), zc.as<float>(), da,
                           mu * (double)n, jitter, M, dr);
        st = tri_solve(ctx, p, p->T, p->Tdinv, true, dr, 1);
        if (!st) st = tri_solve(ctx, p, p->A, p->Adinv, true, dr, 1);
        if (st) return st;
        e = hipMemsetAsync(db, 0, sizeof(double) * M, ctx->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(dp, dr, sizeof(double) * M, hipMemcpyDeviceToDevice, ctx->stream);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "CG initialisation", e);
        double rho = 0.0;
        if (!vec_ok(vec_dot(ctx, M, dr, dr, &rho))) return fail(ctx, KNM_HIP_ERROR, "vector reduction");
        for (int it = 0; it < iters[k]; ++it) {
            st = linop_cols(ctx, p, wk, ops, mu, dp, 1, dq, dw.as<float>());
            if (st) return st;
            double pq = 0.0, rn = 0.0;
            if (!vec_ok(vec_dot(ctx, M, dp, dq, &pq))) return fail(ctx, KNM_HIP_ERROR, "vector reduction");
            const double a = (pq != 0.0) ? rho / pq : 0.0, ma = -a, one = 1.0;
            if (!vec_ok(vec_axpy(ctx, M, a, dp, db)) ||
                !vec_ok(vec_axpy(ctx, M, ma, dq, dr)) ||
                !vec_ok(vec_dot(ctx, M, dr, dr, &rn)))
                return fail(ctx, KNM_HIP_ERROR, "CG vector update");
            const double b = (rho != 0.0) ? rn / rho : 0.0;
            if (!vec_ok(vec_scal(ctx, M, b, dp)) ||
                !vec_ok(vec_axpy(ctx, M, one, dr, dp)))
                return fail(ctx, KNM_HIP_ERROR, "CG vector update");
            rho = rn;
        }
        // alpha += T^-1 A^-1 beta
        st = tri_solve(ctx, p, p->A, p->Adinv, false, db, 1);
        if (!st) st = tri_solve(ctx, p, p->T, p->Tdinv, false, db, 1);
        if (st) return st;
        const double one = 1.0;
        if (!vec_ok(vec_axpy(ctx, M, one, db, da))) return fail(ctx, KNM_HIP_ERROR, "vector update");
        hipLaunchKernelGGL(f64_to_f32_kernel, grid1(M), dim3(256), 0, ctx->stream, da, M, a32.as<float>());
    }
    if (loss_or_null) {
        st = evaluate(false, loss_or_null + n_steps);
        if (st) return st;
    }
    e = hipMemcpyAsync(alpha, a32.p, sizeof(float) * M, hipMemcpyDeviceToDevice, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream); // temporaries are freed on return
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "logfalkon_fit", e);
    return KNM_OK;
}


int logfalkon_fit(knm_ctx *ctx, const float *X, int64_t n, int d, int64_t ldx, const float *y, const float *C, int64_t M,
                  int64_t ldc, const float *yC, float sigma, const double *lambdas, const int *iters, int n_steps,
                  double jitter, float *alpha, double *loss_or_null)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!X || !y || !C || !yC || !alpha || !lambdas || !iters || n <= 0 || M <= 0 || d <= 0 || n_steps <= 0 ||
        ldx < d || ldc < d || !(sigma > 0.0f) || !(jitter >= 0.0))
        return fail(ctx, KNM_INVALID_ARG, "bad fit argument");
    for (int k = 0; k < n_steps; ++k)
        if (!(lambdas[k] >= 0.0) || iters[k] <= 0) return fail(ctx, KNM_INVALID_ARG, "bad Newton schedule");
    if (d > knm_max_d()) return fail(ctx, KNM_UNSUPPORTED, "d above compiled maximum");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    int st = KNM_OK;
    // T depends on the centres only: built once; A is rebuilt per Newton step
    knm_precond *p = nullptr;
    st = precond_build_impl(ctx, C, M, d, ldc, sigma, lambdas[0], jitter, false, &p, nullptr);
    if (st) return st;
    const KernelOps ops = dense_ops(ctx, X, n, d, ldx, C, M, ldc, sigma);
    auto centres_v = [=](const float *a, float *zc) { return do_knm_v(ctx, C, M, d, ldc, C, M, ldc, sigma, a, 1, zc); };
    return logfalkon_core(ctx, ops, centres_v, p, y, yC, lambdas, iters, n_steps, jitter, alpha, loss_or_null);
}

int logfalkon_fit_csr(knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values, int64_t n,
                      const float *y, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values, int64_t M,
                      int64_t d, const float *yC, float sigma, const double *lambdas, const int *iters, int n_steps,
                      double jitter, float *alpha, double *loss_or_null)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!x_indptr || !c_indptr || !y || !yC || !alpha || !lambdas || !iters || n <= 0 || M <= 0 || d <= 0 ||
        n_steps <= 0 || !(sigma > 0.0f) || !(jitter >= 0.0))
        return fail(ctx, KNM_INVALID_ARG, "bad fit argument");
    for (int k = 0; k < n_steps; ++k)
        if (!(lambdas[k] >= 0.0) || iters[k] <= 0) return fail(ctx, KNM_INVALID_ARG, "bad Newton schedule");
    if (d >= 0x7fffffffLL || M >= 0x7fffffffLL) return fail(ctx, KNM_UNSUPPORTED, "d or M above the supported maximum");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    // the sweeps of k(X, C) and of k(C, C); both outlive the fit, which uses their workspaces
    SparseProducts sp, spc;
    int st = sp.prepare(ctx, x_indptr, x_indices, x_values, n, c_indptr, c_indices, c_values, M, d, sigma);
    if (!st) st = spc.prepare(ctx, c_indptr, c_indices, c_values, M, c_indptr, c_indices, c_values, M, d, sigma);
    if (st) return st;
    knm_precond *p = nullptr;
    auto fill = [=](double *K, int64_t ldk) {
        return sparse_kmm(ctx, c_indptr, c_indices, c_values, M, d, sigma, jitter, K, ldk);
    };
    st = precond_build_from(ctx, M, fill, lambdas[0], jitter, false, &p, nullptr);
    if (st) return st;
    KernelOps ops;
    ops.n = n;
    ops.M = M;
    ops.v = [&sp](const float *V, int tt, float *W) { return sp.v(V, tt, W); };
    ops.t_w = [&sp](const float *W, const float *wgt, int tt, float *U) { return sp.t_w(W, wgt, tt, U); };
    auto centres_v = [&spc](const float *a, float *zc) { return spc.v(a, 1, zc); };
    return logfalkon_core(ctx, ops, centres_v, p, y, yC, lambdas, iters, n_steps, jitter, alpha, loss_or_null);
}

} // extern "C"
