// Kernel product for sparse inputs (Sec. 4, "Dealing with sparse datasets"): X and C in CSR
// form with a feature dimension far beyond what a dense row can hold.
//
// The kernel matrix of sparse points is still dense, but most of it is a rank-one matrix:
// with a_i = exp(-|x_i|^2 / 2 sigma^2), b_j = exp(-|c_j|^2 / 2 sigma^2) and g_ij = x_i . c_j,
//   K_ij = a_i b_j exp(g_ij / sigma^2),
// and g_ij = 0 unless the two points share a feature.  So
//   (K v)_i   = a_i sum_j b_j v_j  +  sum_{j : g_ij != 0} (K_ij - a_i b_j) v_j
//   (K^T w)_j = b_j sum_i a_i w_i  +  sum_{i : g_ij != 0} (K_ij - a_i b_j) w_i,
// exactly (up to rounding order), and only the pairs that share a feature are ever visited:
// no dense n x M sweep, no dense tile of the cross term.  The paper forms the dense kernel
// blocks from a sparse matrix product; this is the same result with the all-ones part of
// exp(g / sigma^2) summed in closed form.
//
// One wavefront owns a row of X at a time and a private dense accumulator over the M centres
// (in HBM / L2): it walks the row's features, and for each feature the list of centres that
// have it (C transposed to CSC once per call), adding x_if c_jf into the accumulator; a second
// walk takes every touched entry out again (atomic exchange with zero, so a centre reached
// through several features is consumed once), turns it into K_ij - a_i b_j and adds it to the
// row's sum (row sweep) or scatters it into a fp64 image of U (column sweep, fp64 atomics: the
// summation order varies from run to run, which the rounding to fp32 at the end mostly hides).  Long centre lists are walked by the whole
// wavefront, short ones by the lane that owns the feature.  The additions are the hardware's
// fp32 atomic add (the accumulators and U live in ordinary device memory).
//
// What a row has to walk is prepared once per (X, C): a work list with the start and length of
// the centre list of every entry whose feature occurs in a centre at all.  A row with few pair
// updates accumulates in a small table in LDS instead of the accumulator in device memory.  The few features that
// occur in a large share of the centres are not walked: their pairs are covered by one dense
// product over those features (see "head features" below), which takes the place of the
// rank-one term.
#include <algorithm>
#include <cstring>
#include <vector>

#include "knm_internal.h"

namespace knm {
namespace {

constexpr int kSpThreads = 256;
constexpr int kSpWaves = kSpThreads / 64;
constexpr int kLongList = 32;     // centre lists at least this long are walked by the whole wavefront
constexpr int kScanChunk = 4096;  // elements per workgroup of the prefix sum
constexpr int64_t kFillGroup = 128; // rows of C per launch of the CSC fill
constexpr int kHashBits = 9;        // slots (2^9) of a wavefront's accumulator table in LDS
constexpr int kHashSlots = 1 << kHashBits;
constexpr int kHashMaxPairs = 320; // a row with at most this many pair updates uses the table (load <= 5/8)
constexpr int kMaxHead = 128;       // features treated densely, at most (one dense row of X^H and C^H each)

// flag |= 1 if the CSR structure is not usable: indptr not starting at 0, decreasing, running
// past nnz, or the column indices of a row not strictly increasing inside [0, d)
__global__ void csr_check_kernel(const int64_t *__restrict__ indptr, const int64_t *__restrict__ indices, int64_t rows,
                                 int64_t nnz, int64_t d, int *flag)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    const int64_t p0 = indptr[r], p1 = indptr[r + 1];
    bool bad = (r == 0 && p0 != 0) || p0 < 0 || p1 < p0 || p1 > nnz;
    if (!bad) {
        int64_t prev = -1;
        for (int64_t p = p0; p < p1; ++p) {
            const int64_t c = indices[p];
            if (c <= prev || c >= d) bad = true; // strictly increasing: every feature at most once in a row
            prev = c;
        }
    }
    if (bad) atomicOr(flag, 1);
}

__global__ void row_norms_kernel(const int64_t *__restrict__ indptr, const float *__restrict__ values, int64_t rows,
                                 float *__restrict__ norms)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    double s = 0.0;
    for (int64_t p = indptr[r]; p < indptr[r + 1]; ++p) s += (double)values[p] * (double)values[p];
    norms[r] = (float)s;
}

__global__ void col_count_kernel(const int64_t *__restrict__ indices, int64_t nnz, int *__restrict__ count)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < nnz) atomicAdd(&count[indices[p]], 1);
}

// exclusive prefix sum of `in` (len entries) in three passes; out may alias in
__global__ __launch_bounds__(256) void scan_local_kernel(const int *__restrict__ in, int64_t len, int *__restrict__ out,
                                                        int *__restrict__ sums)
{
    __shared__ int sh[256];
    constexpr int kPer = kScanChunk / 256;
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kPer;
    int v[kPer];
    int tot = 0;
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        v[e] = (base + e < len) ? in[base + e] : 0;
        tot += v[e];
    }
    sh[threadIdx.x] = tot;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const int add = ((int)threadIdx.x >= off) ? sh[threadIdx.x - off] : 0;
        __syncthreads();
        sh[threadIdx.x] += add;
        __syncthreads();
    }
    int run = sh[threadIdx.x] - tot; // exclusive prefix of this thread inside the workgroup
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        if (base + e < len) out[base + e] = run;
        run += v[e];
    }
    if (threadIdx.x == 255) sums[blockIdx.x] = sh[255];
}

__global__ __launch_bounds__(256) void scan_sums_kernel(int *__restrict__ sums, int64_t count)
{
    __shared__ int sh[256];
    const int64_t per = (count + 255) / 256;
    const int64_t b0 = (int64_t)threadIdx.x * per;
    int tot = 0;
    for (int64_t i = b0; i < b0 + per && i < count; ++i) tot += sums[i];
    sh[threadIdx.x] = tot;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const int add = ((int)threadIdx.x >= off) ? sh[threadIdx.x - off] : 0;
        __syncthreads();
        sh[threadIdx.x] += add;
        __syncthreads();
    }
    int run = sh[threadIdx.x] - tot;
    for (int64_t i = b0; i < b0 + per && i < count; ++i) {
        const int v = sums[i];
        sums[i] = run;
        run += v;
    }
}

__global__ void scan_add_kernel(int *__restrict__ out, int64_t len, const int *__restrict__ sums)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < len) out[i] += sums[i / kScanChunk];
}

// scatter the entries of rows [row0, row1) of C (CSR) into its CSC image; cursor starts as a copy
// of col_ptr.  Launched for one group of rows after the other, so that a feature's centre list
// comes out ordered by group: neighbouring list entries then update neighbouring accumulator
// entries (the same cache lines) when the whole wavefront walks a long list.
__global__ void csc_fill_kernel(const int64_t *__restrict__ indptr, const int64_t *__restrict__ indices,
                                const float *__restrict__ values, int64_t row0, int64_t row1, int64_t p0, int64_t p1,
                                int *__restrict__ cursor, int *__restrict__ csc_row, float *__restrict__ csc_val)
{
    const int64_t p = p0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; // one stored entry of the group
    if (p >= p1) return;
    int64_t lo = row0, hi = row1; // its row: the last r in [row0, row1) with indptr[r] <= p
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (indptr[mid] <= p) lo = mid;
        else hi = mid;
    }
    const int pos = atomicAdd(&cursor[indices[p]], 1);
    csc_row[pos] = (int)lo;
    csc_val[pos] = values[p];
}

// e[r] = exp(-norm[r] / 2 sigma^2)
__global__ void norm_factor_kernel(const float *__restrict__ norms, int64_t rows, float inv2s2, float *__restrict__ e)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < rows) e[r] = expf(-norms[r] * inv2s2);
}

// partial sums of e[r] * vec[r * ldv] in fp64, fixed order: one partial per workgroup
__global__ __launch_bounds__(256) void weighted_sum_kernel(const float *__restrict__ e, const float *__restrict__ vec,
                                                          int64_t ldv, int64_t rows, double *__restrict__ part)
{
    __shared__ double sh[256];
    double s = 0.0;
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < rows; r += (int64_t)gridDim.x * 256)
        s += (double)e[r] * (double)vec[r * ldv];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = sh[0];
}

// Column sweep: the all-pairs part of U in fp64, base[j] = e[j] * s (rank-one form, x null) or
// e[j] * x[j] (dense head product).  The sparse walk scatters its terms into a separate fp64
// buffer and the two are added at the end: float atomics onto the all-pairs part, which is
// orders of magnitude larger than a single term, would lose the terms' low bits at every add.
__global__ void column_base_kernel(const float *__restrict__ e, const float *__restrict__ x, double s, int64_t rows,
                                   double *__restrict__ base)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < rows) base[r] = (double)e[r] * (x ? (double)x[r] : s);
}

// out[j * ldo] = base[j] + scattered[j]
__global__ void column_finish_kernel(const double *__restrict__ base, const double *__restrict__ scattered, int64_t rows,
                                     float *__restrict__ out, int64_t ldo)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < rows) out[r * ldo] = (float)(base[r] + scattered[r]);
}

// Orders a wavefront's accesses to its private accumulator: everything it has issued (atomics
// without a return value included) has been performed at the L2, where all accesses to the
// accumulator take place, before anything that follows.  A workgroup-scope fence is that wait and
// nothing else; a device-scope one would also write back and invalidate the XCD's whole L2 at every
// row, which evicts the accumulator lines the next pass is about to hit.
__device__ __forceinline__ void accumulator_fence() { __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup"); }

// ---- head features ---------------------------------------------------------------------
//
// A feature that occurs in a large share of the centres (and hence of the rows) makes nearly every
// pair of points share a feature: its centre list is long and is walked for every row that has
// the feature, and a handful of such features carry most of the pair updates.  They are taken out
// of the sparse walk and treated densely instead.  With H the set of head features, x^H / c^H the
// dense head parts of the points and g = g^H + g^T split accordingly,
//   K_ij = KH_ij + KH_ij (exp(g^T_ij / sigma^2) - 1),    KH_ij = a_i b_j exp(g^H_ij / sigma^2),
// the first term over all pairs and the second only over pairs that share a tail feature.  KH is
// the Gaussian kernel of the head parts times the factors a^T_i = exp(-|x^T_i|^2 / 2 sigma^2) and
// b^T_j of the tail parts' norms, so its sweep is one dense product with d = |H| on the dense
// engines; the second term is the sparse walk over the tail features, whose pairs read g^H from
// the dense head rows of the few head features their row has.

// features whose centre list has at least min_len entries: (feature, list start, length)
__global__ void head_candidates_kernel(const int *__restrict__ col_ptr, int64_t d, int min_len, int cap,
                                       int *__restrict__ count, int *__restrict__ cand)
{
    const int64_t f = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= d) return;
    const int q0 = col_ptr[f], len = col_ptr[f + 1] - q0;
    if (len < min_len) return;
    const int at = atomicAdd(count, 1);
    if (at < cap) {
        cand[3 * at] = (int)f;
        cand[3 * at + 1] = q0;
        cand[3 * at + 2] = len;
    }
}

struct HeadLists {
    int q0[kMaxHead], len[kMaxHead];
};

// CH[j, h] = c_j's value of head feature h (CH zeroed before); blockIdx.y = h
__global__ void head_centres_kernel(HeadLists hl, int Hn, const int *__restrict__ csc_row,
                                    const float *__restrict__ csc_val, float *__restrict__ CH)
{
    const int h = blockIdx.y;
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < hl.len[h]) CH[(int64_t)csc_row[hl.q0[h] + k] * Hn + h] = csc_val[hl.q0[h] + k];
}

// e[r] = exp(-(norm[r] - |row r of PH|^2) / 2 sigma^2): the factor of the tail part's norm; *worst =
// bits of the largest |row of PH|^2 / 2 sigma^2 (non-negative floats order like their bit patterns)
__global__ void tail_factor_kernel(const float *__restrict__ norms, const float *__restrict__ PH, int Hn, int64_t rows,
                                   float inv2s2, float *__restrict__ e, unsigned *__restrict__ worst)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    float hn = 0.0f;
    for (int h = 0; h < Hn; ++h) hn = fmaf(PH[r * Hn + h], PH[r * Hn + h], hn);
    e[r] = expf(-fmaxf(norms[r] - hn, 0.0f) * inv2s2);
    atomicMax(worst, __float_as_uint(hn * inv2s2));
}

// out[r * ldo] = e[r] * x[r * ldx]
__global__ void scale_kernel(const float *__restrict__ e, const float *__restrict__ x, int64_t ldx, int64_t rows,
                             float *__restrict__ out, int64_t ldo)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < rows) out[r * ldo] = e[r] * x[r * ldx];
}

// Work list of X (see SparseArgs): one wavefront per row looks every entry's feature up in the
// centre lists once, so that the sweeps stream (start, length, value) instead of reading the
// d + 1 list pointers at random for every entry, pass and sweep; entries whose feature occurs in no
// centre drop out.  Entries of head features (head_feat: Hn ids, ascending) go to the back of
// the row's range as (head index, value) and into the dense row XH[row, :] (zeroed before).
__global__ __launch_bounds__(kSpThreads) void build_work_kernel(const int64_t *__restrict__ x_indptr,
                                                               const int64_t *__restrict__ x_indices,
                                                               const float *__restrict__ x_values, int64_t n,
                                                               const int *__restrict__ col_ptr,
                                                               const int *__restrict__ head_feat, int Hn, int head_min_len,
                                                               int *__restrict__ work_count, int *__restrict__ work_pairs,
                                                               int *__restrict__ head_count,
                                                               int *__restrict__ work_q0, int *__restrict__ work_len,
                                                               float *__restrict__ work_val, float *__restrict__ XH)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * kSpWaves + (threadIdx.x >> 6);
    const int64_t waves = (int64_t)gridDim.x * kSpWaves;
    for (int64_t row = wave; row < n; row += waves) {
        const int64_t p0 = x_indptr[row], p1 = x_indptr[row + 1];
        int64_t kept = 0, heads = 0, pairs = 0;
        for (int64_t p = p0; p < p1; p += 64) {
            int q0 = 0, len = 0, h = -1;
            float xv = 0.0f;
            if (p + lane < p1) {
                const int64_t col = x_indices[p + lane];
                xv = x_values[p + lane];
                q0 = col_ptr[col];
                len = col_ptr[col + 1] - q0;
                if (Hn > 0 && len >= head_min_len) { // binary search among the head features
                    int lo = 0, hi = Hn - 1;
                    while (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if ((int64_t)head_feat[mid] < col) lo = mid + 1;
                        else hi = mid;
                    }
                    if ((int64_t)head_feat[lo] == col) h = lo;
                }
            }
            const unsigned long long below = (1ull << lane) - 1ull;
            const unsigned long long keep = __ballot(len > 0 && h < 0);
            const unsigned long long head = __ballot(h >= 0);
            if (len > 0 && h < 0) {
                const int64_t at = p0 + kept + __popcll(keep & below);
                work_q0[at] = q0;
                work_len[at] = len;
                work_val[at] = xv;
            }
            if (h >= 0) {
                const int64_t at = p1 - 1 - heads - __popcll(head & below);
                work_q0[at] = h;
                work_val[at] = xv;
                XH[row * Hn + h] = xv;
            }
            kept += __popcll(keep);
            heads += __popcll(head);
            pairs += (len > 0 && h < 0) ? len : 0;
        }
        for (int w = 32; w > 0; w >>= 1) pairs += __shfl_xor(pairs, w);
        if (lane == 0) {
            work_count[row] = (int)kept;
            work_pairs[row] = (int)(pairs < 0x7fffffffLL ? pairs : 0x7fffffffLL);
            head_count[row] = (int)heads;
        }
    }
}

struct SparseArgs {
    const int64_t *x_indptr;
    // work list of X: per row the entries whose feature occurs in some centre, packed to the front
    // of the row's own range [x_indptr[r], x_indptr[r] + work_count[r]): start and length of the
    // feature's centre list and the entry's value
    const int *work_count, *work_q0, *work_len;
    const float *work_val;
    const int *work_pairs; // per row: sum of the list lengths of its work list (saturating)
    // head features (Hn = 0: none): per row the last head_count[r] slots of its range hold (head
    // index, value); CH is the dense M x Hn image of the centres' head parts; tail_factor the
    // factor a^T of the rows (row sweep); dense the head-kernel product of the row sweep
    int Hn;
    const int *head_count;
    const float *CH, *tail_factor, *dense;
    int64_t n, M;
    const int *csc_row;
    const float *csc_val;
    const float *xn, *cn; // squared norms
    const float *xa;      // a_i
    const float *vec;     // row sweep: v over the centres; column sweep: w over the rows
    int64_t ldv;
    float *out;           // row sweep: W over the rows
    double *scattered;    // column sweep: the walk's terms of U over the centres (zero before)
    int64_t ldo;
    float *acc;           // one dense accumulator of M floats per wavefront of the grid, all zero
    float inv2s2, inv_s2;
    double s_rank_one;    // row sweep: sum_j b_j v_j
};

// K_ij - KH_ij from the tail part gt and the head part gh of the dot product and the squared norms
// (no head features: gh = 0 and KH_ij = a_i b_j).  With e0 = -log KH_ij >= 0 and a = gt / sigma^2 the
// excess is exp(a - e0) - exp(-e0), where a - e0 = log K_ij <= 0: neither term can overflow.  For
// small a the difference is taken as exp(-e0) expm1(a), which keeps its leading digits.
__device__ __forceinline__ float pair_excess(float gt, float gh, float xn, float cn, float inv2s2, float inv_s2)
{
    const float e0 = (xn + cn) * inv2s2 - gh * inv_s2;
    const float a = gt * inv_s2;
    if (a < 1.0f) return expf(-e0) * expm1f(a);
    return expf(a - e0) - expf(-e0);
}

// Adds v to the entry of key j of a wavefront's table (open addressing, linear probing; the
// table never holds more than kHashMaxPairs keys, so a free slot is always found)
__device__ __forceinline__ void table_add(int *keys, float *vals, int j, float v)
{
    unsigned slot = ((unsigned)j * 2654435761u) >> (32 - kHashBits);
    for (;;) {
        const int prev = atomicCAS(&keys[slot], -1, j);
        if (prev == -1 || prev == j) {
            unsafeAtomicAdd(&vals[slot], v);
            return;
        }
        slot = (slot + 1) & (kHashSlots - 1);
    }
}

template <int COLUMN_SWEEP>
__global__ __launch_bounds__(kSpThreads) void sparse_sweep_kernel(SparseArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * kSpWaves + (threadIdx.x >> 6);
    const int64_t waves = (int64_t)gridDim.x * kSpWaves;
    float *acc = a.acc + wave * a.M;
    // the head features of the row in hand, for every lane of the wavefront to read
    __shared__ int head_idx_all[kSpWaves][kMaxHead];
    __shared__ float head_val_all[kSpWaves][kMaxHead];
    int *const head_idx = head_idx_all[threadIdx.x >> 6];
    float *const head_val = head_val_all[threadIdx.x >> 6];
    // Rows with few pair updates accumulate in a table in LDS instead of the dense accumulator in
    // device memory: (centre, sum) pairs, all slots empty (key -1, sum 0) between rows.
    __shared__ int keys_all[kSpWaves][kHashSlots];
    __shared__ float vals_all[kSpWaves][kHashSlots];
    int *const keys = keys_all[threadIdx.x >> 6];
    float *const vals = vals_all[threadIdx.x >> 6];
    for (int k = lane; k < kHashSlots; k += 64) {
        keys[k] = -1;
        vals[k] = 0.0f;
    }
    accumulator_fence();
    for (int64_t row = wave; row < a.n; row += waves) {
        const int64_t p0 = a.x_indptr[row], p1 = p0 + a.work_count[row];
        const float xn = a.xn[row];
        const float wrow = COLUMN_SWEEP ? a.vec[row * a.ldv] : 0.0f;
        const bool in_lds = a.work_pairs[row] <= kHashMaxPairs; // same for the whole wavefront
        float sum = 0.0f;
        int hc = 0;
        if (a.Hn > 0) {
            hc = a.head_count[row];
            const int64_t back = a.x_indptr[row + 1] - hc;
            for (int k = lane; k < hc; k += 64) { // hc <= Hn <= kMaxHead, which may exceed the 64 lanes
                head_idx[k] = a.work_q0[back + k];
                head_val[k] = a.work_val[back + k];
            }
            accumulator_fence(); // the wavefront's own LDS writes, before any lane reads them
        }
        // g^H_ij of the row in hand against centre j
        auto head_dot = [&](int j) -> float {
            float gh = 0.0f;
            for (int k = 0; k < hc; ++k) gh = fmaf(head_val[k], a.CH[(int64_t)j * a.Hn + head_idx[k]], gh);
            return gh;
        };
        // one term x_if c_jf of g^T_ij
        auto add = [&](int j, float v) {
            if (in_lds) table_add(keys, vals, j, v);
            else unsafeAtomicAdd(&acc[j], v);
        };
        // the finished g^T_ij of a pair that shares a tail feature
        auto consume = [&](int j, float g) {
            if (g == 0.0f) return; // nothing beyond KH_ij (or, in device memory, taken out before)
            const float ex = pair_excess(g, head_dot(j), xn, a.cn[j], a.inv2s2, a.inv_s2);
            if (COLUMN_SWEEP) unsafeAtomicAdd(&a.scattered[j], (double)ex * (double)wrow);
            else sum += ex * a.vec[j * a.ldv];
        };
        // pass 0 adds x_if c_jf into the accumulator; pass 1 takes every touched entry out again:
        // in device memory by walking the lists a second time (atomic exchange with zero, so a
        // centre reached through several features is consumed once), in LDS by a sweep over the table
        for (int pass = 0; pass < (in_lds ? 1 : 2); ++pass) {
            for (int64_t p = p0; p < p1; p += 64) {
                const bool mine = p + lane < p1;
                int q0 = 0, q1 = 0;
                float xv = 0.0f;
                if (mine) {
                    q0 = a.work_q0[p + lane];
                    q1 = q0 + a.work_len[p + lane];
                    xv = a.work_val[p + lane];
                }
                const int len = q1 - q0;
                unsigned long long longs = __ballot(len >= kLongList);
                while (longs) {
                    const int src = __ffsll((long long)longs) - 1;
                    longs &= longs - 1;
                    const int b0 = __shfl(q0, src), b1 = __shfl(q1, src);
                    const float bx = __shfl(xv, src);
                    for (int q = b0 + lane; q < b1; q += 64) {
                        const int j = a.csc_row[q];
                        if (pass == 0) add(j, bx * a.csc_val[q]);
                        else consume(j, atomicExch(&acc[j], 0.0f));
                    }
                }
                if (len < kLongList)
                    for (int q = q0; q < q1; ++q) {
                        const int j = a.csc_row[q];
                        if (pass == 0) add(j, xv * a.csc_val[q]);
                        else consume(j, atomicExch(&acc[j], 0.0f));
                    }
            }
            accumulator_fence(); // every lane's updates are done before the next pass or row
        }
        if (in_lds) {
            for (int k = lane; k < kHashSlots; k += 64) {
                const int j = keys[k];
                if (j >= 0) {
                    const float g = vals[k];
                    keys[k] = -1;
                    vals[k] = 0.0f;
                    consume(j, g);
                }
            }
            accumulator_fence();
        }
        if (!COLUMN_SWEEP) {
            sum += __shfl_xor(sum, 32);
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 8);
            sum += __shfl_xor(sum, 4);
            sum += __shfl_xor(sum, 2);
            sum += __shfl_xor(sum, 1);
            if (lane == 0) {
                const float all_pairs = a.Hn > 0 ? a.tail_factor[row] * a.dense[row] : (float)((double)a.xa[row] * a.s_rank_one);
                a.out[row * a.ldo] = all_pairs + sum;
            }
        }
    }
}

inline dim3 grid_for(int64_t n, int threads = 256) { return dim3((unsigned)((n + threads - 1) / threads)); }

// fp64 entries of the centres' kernel matrix, for the preconditioner: row i of the upper triangle
// (column-major K, leading dimension ldk) = exp(-(|c_i|^2 + |c_j|^2 - 2 g_ij) / 2 sigma^2) + jitter [i == j],
// j >= i, with g_ij accumulated in a private fp64 accumulator exactly as in the sweeps (every
// entry of the accumulator is read and cleared when the row is written out).
__global__ __launch_bounds__(kSpThreads) void sparse_kmm_kernel(const int64_t *__restrict__ c_indptr,
                                                               const int64_t *__restrict__ c_indices,
                                                               const float *__restrict__ c_values, int64_t M,
                                                               const int *__restrict__ col_ptr,
                                                               const int *__restrict__ csc_row,
                                                               const float *__restrict__ csc_val,
                                                               const double *__restrict__ cn, double inv2s2,
                                                               double jitter, double *__restrict__ acc_all,
                                                               double *__restrict__ K, int64_t ldk)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * kSpWaves + (threadIdx.x >> 6);
    const int64_t waves = (int64_t)gridDim.x * kSpWaves;
    double *acc = acc_all + wave * M;
    for (int64_t row = wave; row < M; row += waves) {
        const int64_t p0 = c_indptr[row], p1 = c_indptr[row + 1];
        for (int64_t p = p0; p < p1; p += 64) {
            const bool mine = p + lane < p1;
            int q0 = 0, q1 = 0;
            double xv = 0.0;
            if (mine) {
                const int64_t col = c_indices[p + lane];
                xv = (double)c_values[p + lane];
                q0 = col_ptr[col];
                q1 = col_ptr[col + 1];
            }
            const int len = q1 - q0;
            unsigned long long longs = __ballot(len >= kLongList);
            while (longs) {
                const int src = __ffsll((long long)longs) - 1;
                longs &= longs - 1;
                const int b0 = __shfl(q0, src), b1 = __shfl(q1, src);
                const double bx = __shfl(xv, src);
                for (int q = b0 + lane; q < b1; q += 64) unsafeAtomicAdd(&acc[csc_row[q]], bx * (double)csc_val[q]);
            }
            if (len < kLongList)
                for (int q = q0; q < q1; ++q) unsafeAtomicAdd(&acc[csc_row[q]], xv * (double)csc_val[q]);
        }
        accumulator_fence();
        const double ci = cn[row];
        for (int64_t j = lane; j < M; j += 64) {
            // written by atomics (at the L2): read and cleared there too, past the first-level cache
            const double g = __hip_atomic_load(&acc[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (g != 0.0) __hip_atomic_store(&acc[j], 0.0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (j >= row) K[row + j * ldk] = exp(-(ci + cn[j] - 2.0 * g) * inv2s2) + (j == row ? jitter : 0.0);
        }
        accumulator_fence();
    }
}

__global__ void row_norms_f64_kernel(const int64_t *__restrict__ indptr, const float *__restrict__ values, int64_t rows,
                                     double *__restrict__ norms)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    double s = 0.0;
    for (int64_t p = indptr[r]; p < indptr[r + 1]; ++p) s += (double)values[p] * (double)values[p];
    norms[r] = s;
}

// out[r] = w[r] * x[r * ldx]
__global__ void weigh_kernel(const float *__restrict__ x, int64_t ldx, const float *__restrict__ w, int64_t rows,
                             float *__restrict__ out)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < rows) out[r] = w[r] * x[r * ldx];
}

struct DevMem {
    void *p = nullptr;
    ~DevMem() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 1); }
    template <class T> T *as() { return static_cast<T *>(p); }
};

// structure check of one CSR matrix before anything indexes with the caller's numbers; *nnz_out
// receives indptr[rows]
int check_csr(knm_ctx *ctx, const int64_t *indptr, const int64_t *indices, int64_t rows, int64_t d, int64_t *nnz_out)
{
    hipStream_t st = ctx->stream;
    int64_t nnz = 0;
    hipError_t e = hipMemcpyAsync(&nnz, indptr + rows, sizeof(int64_t), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "reading the CSR size", e);
    if (nnz < 0 || nnz >= 0x7fffffffLL * 64) return fail(ctx, KNM_INVALID_ARG, "bad CSR size");
    DevMem flag;
    if (flag.alloc(sizeof(int)) != hipSuccess) return fail(ctx, KNM_ALLOC, "hipMalloc");
    int bad = 0;
    e = hipMemsetAsync(flag.p, 0, sizeof(int), st);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemsetAsync", e);
    hipLaunchKernelGGL(csr_check_kernel, grid_for(rows), dim3(256), 0, st, indptr, indices, rows, nnz, d, flag.as<int>());
    e = hipMemcpyAsync(&bad, flag.p, sizeof(int), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "CSR check", e);
    if (bad)
        return fail(ctx, KNM_INVALID_ARG,
                    "CSR structure: row pointers not monotone from 0, or feature ids of a row not strictly increasing in [0, d)");
    *nnz_out = nnz;
    return KNM_OK;
}

// CSC image of the centres: col_ptr (d + 1), csc_row / csc_val (nnz_c)
struct CentreLists {
    DevMem col_ptr, csc_row, csc_val;
    int build(knm_ctx *ctx, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values, int64_t M,
              int64_t d, int64_t nnz_c)
    {
        hipStream_t st = ctx->stream;
        if (nnz_c >= 0x7fffffffLL) return fail(ctx, KNM_UNSUPPORTED, "more than 2^31 - 2 stored entries in C");
        DevMem cursor, sums;
        const int64_t scan_blocks = (d + 1 + kScanChunk - 1) / kScanChunk;
        if (col_ptr.alloc(sizeof(int) * (d + 1)) != hipSuccess || cursor.alloc(sizeof(int) * (d + 1)) != hipSuccess ||
            sums.alloc(sizeof(int) * scan_blocks) != hipSuccess || csc_row.alloc(sizeof(int) * nnz_c) != hipSuccess ||
            csc_val.alloc(sizeof(float) * nnz_c) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, KNM_ALLOC, "hipMalloc(centre lists)");
        }
        hipError_t e = hipMemsetAsync(col_ptr.p, 0, sizeof(int) * (d + 1), st);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemsetAsync", e);
        if (nnz_c > 0)
            hipLaunchKernelGGL(col_count_kernel, grid_for(nnz_c), dim3(256), 0, st, c_indices, nnz_c, col_ptr.as<int>());
        hipLaunchKernelGGL(scan_local_kernel, dim3((unsigned)scan_blocks), dim3(256), 0, st, col_ptr.as<int>(), d + 1,
                           col_ptr.as<int>(), sums.as<int>());
        hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(256), 0, st, sums.as<int>(), scan_blocks);
        hipLaunchKernelGGL(scan_add_kernel, grid_for(d + 1), dim3(256), 0, st, col_ptr.as<int>(), d + 1, sums.as<int>());
        e = hipMemcpyAsync(cursor.p, col_ptr.p, sizeof(int) * (d + 1), hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemcpyAsync", e);
        std::vector<int64_t> c_ptr_host((size_t)M + 1);
        e = hipMemcpyAsync(c_ptr_host.data(), c_indptr, sizeof(int64_t) * (M + 1), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "reading the row pointers of C", e);
        for (int64_t r0 = 0; r0 < M; r0 += kFillGroup) {
            const int64_t r1 = (r0 + kFillGroup < M) ? r0 + kFillGroup : M;
            const int64_t q0 = c_ptr_host[(size_t)r0], q1 = c_ptr_host[(size_t)r1]; // checked: monotone, within nnz
            if (q1 > q0)
                hipLaunchKernelGGL(csc_fill_kernel, grid_for(q1 - q0), dim3(256), 0, st, c_indptr, c_indices, c_values, r0,
                                   r1, q0, q1, cursor.as<int>(), csc_row.as<int>(), csc_val.as<float>());
        }
        e = hipStreamSynchronize(st); // cursor and sums are freed on return
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "centre lists", e);
        return KNM_OK;
    }
};

} // namespace

// Everything the two sweeps of one (X, C, sigma) need, prepared once: validated structure, norms,
// centre lists, accumulators.
struct SparseProducts::Impl {
    knm_ctx *ctx = nullptr;
    const int64_t *x_indptr = nullptr, *x_indices = nullptr;
    const float *x_values = nullptr;
    int64_t n = 0, M = 0;
    float inv2s2 = 0.0f, inv_s2 = 0.0f;
    int64_t wgs = 0;
    CentreLists lists;
    DevMem xn, cn, xa, cb, acc, part, tmp, work_count, work_pairs, work_q0, work_len, work_val;
    // head features: dense head parts XH (n x Hn), CH (M x Hn), factors of the tail norms, per-row
    // head counts, and the vectors of the dense product (tmp_m over the centres, dense_n / tmp_n over
    // the rows)
    int Hn = 0;
    float sigma = 0.0f;
    DevMem head_feat, head_count, XH, CH, xat, cbt, tmp_m, dense_n, dense_m, tmp_n;
    DevMem col_base, col_scattered; // column sweep: all-pairs part and scattered terms, fp64 over the centres

    int rank_one_sum(const float *ev, const float *vec, int64_t ldv, int64_t rows, double *out)
    {
        double host[256];
        hipStream_t st = ctx->stream;
        hipLaunchKernelGGL(weighted_sum_kernel, dim3(256), dim3(256), 0, st, ev, vec, ldv, rows, part.as<double>());
        hipError_t err = hipMemcpyAsync(host, part.p, sizeof(double) * 256, hipMemcpyDeviceToHost, st);
        if (err == hipSuccess) err = hipStreamSynchronize(st);
        if (err != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "rank-one sum", err);
        double s = 0.0;
        for (int i = 0; i < 256; ++i) s += host[i];
        *out = s;
        return KNM_OK;
    }
    // Chooses the head features from the centre lists and builds CH.  A feature qualifies with a
    // list of at least max(16, M / 160) centres; the kMaxHead longest are taken if, on the estimate
    // that a feature is as frequent in the rows as in the centres, they would cost more pair updates
    // (n / M sum_h len_h^2) than the dense product costs entries (n M / 128 at the measured rates).
    int choose_head(int64_t d, int64_t nnz_c, int max_head, int *min_len_out)
    {
        hipStream_t st = ctx->stream;
        Hn = 0;
        const int min_len = (int)(M / 160 > 16 ? M / 160 : 16);
        *min_len_out = min_len;
        if (max_head <= 0 || nnz_c < min_len) return KNM_OK;
        if (max_head > kMaxHead) max_head = kMaxHead;
        const int cap = (int)(nnz_c / min_len) + 1; // no more features than this can have such lists
        DevMem count, cand;
        if (count.alloc(sizeof(int)) != hipSuccess || cand.alloc(sizeof(int) * 3 * (size_t)cap) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, KNM_ALLOC, "hipMalloc(head candidates)");
        }
        hipError_t e = hipMemsetAsync(count.p, 0, sizeof(int), st);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemsetAsync", e);
        hipLaunchKernelGGL(head_candidates_kernel, grid_for(d), dim3(256), 0, st, lists.col_ptr.as<int>(), d, min_len, cap,
                           count.as<int>(), cand.as<int>());
        int found = 0;
        e = hipMemcpyAsync(&found, count.p, sizeof(int), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "head candidates", e);
        if (found <= 0) return KNM_OK;
        if (found > cap) found = cap;
        std::vector<int> host(3 * (size_t)found);
        e = hipMemcpy(host.data(), cand.p, sizeof(int) * host.size(), hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "head candidates", e);
        struct Cand { int feat, q0, len; };
        std::vector<Cand> cs((size_t)found);
        for (int i = 0; i < found; ++i) cs[i] = {host[3 * i], host[3 * i + 1], host[3 * i + 2]};
        // longest first; equal lengths by feature id, so the choice does not depend on the order
        // in which the candidates were found
        std::sort(cs.begin(), cs.end(), [](const Cand &x, const Cand &y) { return x.len != y.len ? x.len > y.len : x.feat < y.feat; });
        if ((int)cs.size() > max_head) cs.resize((size_t)max_head);
        double sq = 0.0;
        for (const Cand &c : cs) sq += (double)c.len * (double)c.len;
        if (sq * 128.0 < (double)M * (double)M) return KNM_OK;
        std::sort(cs.begin(), cs.end(), [](const Cand &x, const Cand &y) { return x.feat < y.feat; });
        Hn = (int)cs.size();
        HeadLists hl;
        int feats[kMaxHead], longest = 0;
        for (int h = 0; h < kMaxHead; ++h) {
            hl.q0[h] = h < Hn ? cs[h].q0 : 0;
            hl.len[h] = h < Hn ? cs[h].len : 0;
            feats[h] = h < Hn ? cs[h].feat : 0;
            if (hl.len[h] > longest) longest = hl.len[h];
        }
        if (head_feat.alloc(sizeof(int) * kMaxHead) != hipSuccess || CH.alloc(sizeof(float) * (size_t)M * Hn) != hipSuccess ||
            XH.alloc(sizeof(float) * (size_t)n * Hn) != hipSuccess || xat.alloc(sizeof(float) * n) != hipSuccess ||
            cbt.alloc(sizeof(float) * M) != hipSuccess || tmp_m.alloc(sizeof(float) * M) != hipSuccess ||
            dense_m.alloc(sizeof(float) * M) != hipSuccess || dense_n.alloc(sizeof(float) * n) != hipSuccess ||
            tmp_n.alloc(sizeof(float) * n) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, KNM_ALLOC, "hipMalloc(head features)");
        }
        e = hipMemcpy(head_feat.p, feats, sizeof(int) * kMaxHead, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemsetAsync(CH.p, 0, sizeof(float) * (size_t)M * Hn, st);
        if (e == hipSuccess) e = hipMemsetAsync(XH.p, 0, sizeof(float) * (size_t)n * Hn, st);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "head features", e);
        hipLaunchKernelGGL(head_centres_kernel, dim3((unsigned)((longest + 255) / 256), (unsigned)Hn), dim3(256), 0, st, hl, Hn,
                           lists.csc_row.as<int>(), lists.csc_val.as<float>(), CH.as<float>());
        return hipGetLastError() == hipSuccess ? KNM_OK : fail(ctx, KNM_HIP_ERROR, "head_centres_kernel launch");
    }
    SparseArgs args()
    {
        SparseArgs a;
        a.x_indptr = x_indptr;
        a.work_count = work_count.as<int>();
        a.work_q0 = work_q0.as<int>();
        a.work_len = work_len.as<int>();
        a.work_val = work_val.as<float>();
        a.work_pairs = work_pairs.as<int>();
        a.scattered = nullptr;
        a.Hn = Hn;
        a.head_count = head_count.as<int>();
        a.CH = CH.as<float>();
        a.tail_factor = xat.as<float>();
        a.dense = dense_n.as<float>();
        a.n = n;
        a.M = M;
        a.csc_row = lists.csc_row.as<int>();
        a.csc_val = lists.csc_val.as<float>();
        a.xn = xn.as<float>();
        a.cn = cn.as<float>();
        a.xa = xa.as<float>();
        a.acc = acc.as<float>();
        a.inv2s2 = inv2s2;
        a.inv_s2 = inv_s2;
        return a;
    }
};

SparseProducts::SparseProducts() : impl(new Impl()) {}
SparseProducts::~SparseProducts()
{
    if (impl && impl->ctx) (void)hipStreamSynchronize(impl->ctx->stream); // kernels may still use the workspace
    delete impl;
}

int SparseProducts::prepare(knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values,
                            int64_t n, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values,
                            int64_t M, int64_t d, float sigma)
{
    // the closed form of the rank-one part belongs to the Gaussian kernel
    if (ctx->kernel_kind != KNM_KERNEL_GAUSSIAN)
        return fail(ctx, KNM_UNSUPPORTED, "sparse inputs: Gaussian kernel only");
    Impl &s = *impl;
    s.ctx = ctx;
    s.x_indptr = x_indptr;
    s.x_indices = x_indices;
    s.x_values = x_values;
    s.n = n;
    s.M = M;
    s.inv2s2 = 1.0f / (2.0f * sigma * sigma);
    s.inv_s2 = 1.0f / (sigma * sigma);
    hipStream_t st = ctx->stream;
    int64_t nnz_x = 0, nnz_c = 0;
    int stat = check_csr(ctx, x_indptr, x_indices, n, d, &nnz_x);
    if (!stat) stat = check_csr(ctx, c_indptr, c_indices, M, d, &nnz_c);
    if (stat) return stat;
    // grid: enough wavefronts to fill the chip, each with a private accumulator over the centres
    s.wgs = (n + kSpWaves - 1) / kSpWaves;
    if (s.wgs > 2048) s.wgs = 2048; // 8 workgroups per CU: the sweep is bound by memory latency
    const int64_t waves = s.wgs * kSpWaves;
    if (s.xn.alloc(sizeof(float) * n) != hipSuccess || s.cn.alloc(sizeof(float) * M) != hipSuccess ||
        s.xa.alloc(sizeof(float) * n) != hipSuccess || s.cb.alloc(sizeof(float) * M) != hipSuccess ||
        s.acc.alloc(sizeof(float) * waves * M) != hipSuccess || s.part.alloc(sizeof(double) * 256) != hipSuccess ||
        s.tmp.alloc(sizeof(float) * n) != hipSuccess || s.col_base.alloc(sizeof(double) * M) != hipSuccess ||
        s.col_scattered.alloc(sizeof(double) * M) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, KNM_ALLOC, "hipMalloc(sparse workspace)");
    }
    hipLaunchKernelGGL(row_norms_kernel, grid_for(n), dim3(256), 0, st, x_indptr, x_values, n, s.xn.as<float>());
    hipLaunchKernelGGL(row_norms_kernel, grid_for(M), dim3(256), 0, st, c_indptr, c_values, M, s.cn.as<float>());
    hipLaunchKernelGGL(norm_factor_kernel, grid_for(n), dim3(256), 0, st, s.xn.as<float>(), n, s.inv2s2, s.xa.as<float>());
    hipLaunchKernelGGL(norm_factor_kernel, grid_for(M), dim3(256), 0, st, s.cn.as<float>(), M, s.inv2s2, s.cb.as<float>());
    stat = s.lists.build(ctx, c_indptr, c_indices, c_values, M, d, nnz_c);
    if (stat) return stat;
    s.sigma = sigma;
    int head_min_len = 0;
    stat = s.choose_head(d, nnz_c, ctx->sparse_head_max, &head_min_len);
    if (stat) return stat;
    const size_t work = (size_t)(nnz_x > 0 ? nnz_x : 1);
    if (s.work_count.alloc(sizeof(int) * n) != hipSuccess || s.head_count.alloc(sizeof(int) * n) != hipSuccess ||
        s.work_pairs.alloc(sizeof(int) * n) != hipSuccess ||
        s.work_q0.alloc(sizeof(int) * work) != hipSuccess || s.work_len.alloc(sizeof(int) * work) != hipSuccess ||
        s.work_val.alloc(sizeof(float) * work) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, KNM_ALLOC, "hipMalloc(sparse work list)");
    }
    auto build_work = [&]() {
        hipLaunchKernelGGL(build_work_kernel, dim3((unsigned)s.wgs), dim3(kSpThreads), 0, st, x_indptr, x_indices, x_values, n,
                           s.lists.col_ptr.as<int>(), s.head_feat.as<int>(), s.Hn, head_min_len, s.work_count.as<int>(),
                           s.work_pairs.as<int>(), s.head_count.as<int>(), s.work_q0.as<int>(), s.work_len.as<int>(),
                           s.work_val.as<float>(), s.XH.as<float>());
        return hipGetLastError() == hipSuccess ? KNM_OK : fail(ctx, KNM_HIP_ERROR, "work list launch");
    };
    stat = build_work();
    if (stat) return stat;
    if (s.Hn > 0) {
        // The dense product forms its exponent from the norm expansion, whose rounding error grows
        // with the head parts' norm terms |x^H|^2 / 2 sigma^2 (about 1e-7 of them): beyond 50 the
        // head features go back into the sparse walk, which has no such cancellation.
        unsigned worst_bits = 0;
        hipError_t e = hipMemsetAsync(s.part.p, 0, sizeof(unsigned), st);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemsetAsync", e);
        hipLaunchKernelGGL(tail_factor_kernel, grid_for(n), dim3(256), 0, st, s.xn.as<float>(), s.XH.as<float>(), s.Hn, n,
                           s.inv2s2, s.xat.as<float>(), s.part.as<unsigned>());
        hipLaunchKernelGGL(tail_factor_kernel, grid_for(M), dim3(256), 0, st, s.cn.as<float>(), s.CH.as<float>(), s.Hn, M,
                           s.inv2s2, s.cbt.as<float>(), s.part.as<unsigned>());
        e = hipMemcpyAsync(&worst_bits, s.part.p, sizeof(unsigned), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "head norm terms", e);
        float worst = 0.0f;
        memcpy(&worst, &worst_bits, sizeof(float));
        if (!(worst <= 50.0f)) {
            s.Hn = 0;
            stat = build_work();
            if (stat) return stat;
        }
    }
    hipError_t e = hipMemsetAsync(s.acc.p, 0, sizeof(float) * waves * M, st);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemsetAsync", e);
    return KNM_OK;
}

// W (n x t, row-major) = K V
int SparseProducts::v(const float *V, int t, float *W)
{
    Impl &s = *impl;
    for (int c = 0; c < t; ++c) {
        double sum = 0.0;
        if (s.Hn > 0) {
            // all pairs: a^T_i sum_j k(x^H_i, c^H_j) b^T_j v_j on the dense engine
            hipLaunchKernelGGL(scale_kernel, grid_for(s.M), dim3(256), 0, s.ctx->stream, s.cbt.as<float>(), V + c, (int64_t)t,
                               s.M, s.tmp_m.as<float>(), (int64_t)1);
            int stat = do_knm_v(s.ctx, s.XH.as<float>(), s.n, s.Hn, s.Hn, s.CH.as<float>(), s.M, s.Hn, s.sigma,
                                s.tmp_m.as<float>(), 1, s.dense_n.as<float>());
            if (stat) return stat;
        } else {
            int stat = s.rank_one_sum(s.cb.as<float>(), V + c, t, s.M, &sum);
            if (stat) return stat;
        }
        SparseArgs a = s.args();
        a.vec = V + c;
        a.ldv = t;
        a.out = W + c;
        a.ldo = t;
        a.s_rank_one = sum;
        hipLaunchKernelGGL(sparse_sweep_kernel<0>, dim3((unsigned)s.wgs), dim3(kSpThreads), 0, s.ctx->stream, a);
    }
    return hipGetLastError() == hipSuccess ? KNM_OK : fail(s.ctx, KNM_HIP_ERROR, "sparse row sweep launch");
}

// U (M x t, row-major) = K^T (wgt .* W), wgt over the rows of X or null
int SparseProducts::t_w(const float *W, const float *wgt, int t, float *U)
{
    Impl &s = *impl;
    hipStream_t st = s.ctx->stream;
    for (int c = 0; c < t; ++c) {
        const float *w = W + c;
        int64_t ldw = t;
        if (wgt) {
            hipLaunchKernelGGL(weigh_kernel, grid_for(s.n), dim3(256), 0, st, W + c, (int64_t)t, wgt, s.n, s.tmp.as<float>());
            w = s.tmp.as<float>();
            ldw = 1;
        }
        if (s.Hn > 0) {
            // all pairs: b^T_j sum_i k(x^H_i, c^H_j) a^T_i w_i on the dense engine
            hipLaunchKernelGGL(scale_kernel, grid_for(s.n), dim3(256), 0, st, s.xat.as<float>(), w, ldw, s.n,
                               s.tmp_n.as<float>(), (int64_t)1);
            int stat = do_knm_t_w(s.ctx, s.XH.as<float>(), s.n, s.Hn, s.Hn, s.CH.as<float>(), s.M, s.Hn, s.sigma,
                                  s.tmp_n.as<float>(), nullptr, 1, s.dense_m.as<float>());
            if (stat) return stat;
            hipLaunchKernelGGL(column_base_kernel, grid_for(s.M), dim3(256), 0, st, s.cbt.as<float>(), s.dense_m.as<float>(), 0.0,
                               s.M, s.col_base.as<double>());
        } else {
            double sum = 0.0;
            int stat = s.rank_one_sum(s.xa.as<float>(), w, ldw, s.n, &sum);
            if (stat) return stat;
            hipLaunchKernelGGL(column_base_kernel, grid_for(s.M), dim3(256), 0, st, s.cb.as<float>(), (const float *)nullptr, sum,
                               s.M, s.col_base.as<double>());
        }
        hipError_t e = hipMemsetAsync(s.col_scattered.p, 0, sizeof(double) * s.M, st);
        if (e != hipSuccess) return fail(s.ctx, KNM_HIP_ERROR, "hipMemsetAsync", e);
        SparseArgs a = s.args();
        a.vec = w;
        a.ldv = ldw;
        a.out = nullptr;
        a.ldo = 0;
        a.scattered = s.col_scattered.as<double>();
        a.s_rank_one = 0.0;
        hipLaunchKernelGGL(sparse_sweep_kernel<1>, dim3((unsigned)s.wgs), dim3(kSpThreads), 0, st, a);
        hipLaunchKernelGGL(column_finish_kernel, grid_for(s.M), dim3(256), 0, st, s.col_base.as<double>(),
                           s.col_scattered.as<double>(), s.M, U + c, (int64_t)t);
    }
    return hipGetLastError() == hipSuccess ? KNM_OK : fail(s.ctx, KNM_HIP_ERROR, "sparse column sweep launch");
}

// Upper triangle of K (M x M, column-major with leading dimension ldk, fp64) = k(C, C) + jitter I for CSR centres
int sparse_kmm(knm_ctx *ctx, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values, int64_t M,
               int64_t d, float sigma, double jitter, double *K, int64_t ldk)
{
    if (ctx->kernel_kind != KNM_KERNEL_GAUSSIAN)
        return fail(ctx, KNM_UNSUPPORTED, "sparse inputs: Gaussian kernel only");
    hipStream_t st = ctx->stream;
    int64_t nnz_c = 0;
    int stat = check_csr(ctx, c_indptr, c_indices, M, d, &nnz_c);
    if (stat) return stat;
    CentreLists lists;
    stat = lists.build(ctx, c_indptr, c_indices, c_values, M, d, nnz_c);
    if (stat) return stat;
    int64_t wgs = (M + kSpWaves - 1) / kSpWaves;
    if (wgs > 1024) wgs = 1024;
    const int64_t waves = wgs * kSpWaves;
    DevMem cn, acc;
    if (cn.alloc(sizeof(double) * M) != hipSuccess || acc.alloc(sizeof(double) * waves * M) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, KNM_ALLOC, "hipMalloc(sparse K_MM workspace)");
    }
    hipLaunchKernelGGL(row_norms_f64_kernel, grid_for(M), dim3(256), 0, st, c_indptr, c_values, M, cn.as<double>());
    hipError_t e = hipMemsetAsync(acc.p, 0, sizeof(double) * waves * M, st);
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipMemsetAsync", e);
    hipLaunchKernelGGL(sparse_kmm_kernel, dim3((unsigned)wgs), dim3(kSpThreads), 0, st, c_indptr, c_indices, c_values, M,
                       lists.col_ptr.as<int>(), lists.csc_row.as<int>(), lists.csc_val.as<float>(), cn.as<double>(),
                       1.0 / (2.0 * (double)sigma * (double)sigma), jitter, acc.as<double>(), K, ldk);
    e = hipStreamSynchronize(st); // the workspace is freed on return
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "sparse K_MM", e);
    return KNM_OK;
}

} // namespace knm

extern "C" int knm_prod_csr(knm_ctx *ctx, const int64_t *x_indptr, const int64_t *x_indices, const float *x_values,
                            int64_t n, const int64_t *c_indptr, const int64_t *c_indices, const float *c_values,
                            int64_t M, int64_t d, float sigma, const float *V, int t, float *W_or_null, float *U)
{
    using namespace knm;
    if (!ctx) return KNM_INVALID_ARG;
    if (!x_indptr || !c_indptr || !V || !U || n <= 0 || M <= 0 || d <= 0 || t <= 0 || !(sigma > 0.0f))
        return fail(ctx, KNM_INVALID_ARG, "bad shape or pointer");
    if (d >= 0x7fffffffLL || M >= 0x7fffffffLL) return fail(ctx, KNM_UNSUPPORTED, "d or M beyond 2^31 - 2");
    if (t > knm_max_t()) return fail(ctx, KNM_UNSUPPORTED, "t above compiled maximum");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    SparseProducts ops;
    int st = ops.prepare(ctx, x_indptr, x_indices, x_values, n, c_indptr, c_indices, c_values, M, d, sigma);
    if (st) return st;
    float *W = W_or_null;
    if (!W) {
        st = ensure(ctx, &ctx->w_buf, &ctx->w_bytes, sizeof(float) * (size_t)n * t);
        if (st) return st;
        W = ctx->w_buf;
    }
    st = ops.v(V, t, W);
    if (!st) st = ops.t_w(W, nullptr, t, U);
    if (st) return st;
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "sparse product", e);
    return KNM_OK;
}
