// fp64 symmetric rank-k updates on the matrix cores: the bulk of the preconditioner's flop.
//
// Both factorisations of the preconditioner (Alg. 1, the two Cholesky lines) spend M^3 / 3 flop
// each in the third step of the block Cholesky column update (Sec. 4, block Cholesky
// paragraph; appendix on the out-of-core algorithms): the trailing matrix loses the product
// of the just-solved block row with itself.  The triangular product between them (the same
// algorithm's T T^T line, with the diagonal weights of Alg. 2's WeightedPreconditioner) is the
// same contraction over a triangular operand.  One kernel serves both:
//
//   C[i, j] = alpha * sum_{k in [k0(j), K)} w[k] * a(i, k) * a(j, k) + beta * C[i, j] + shift * [i == j],   i <= j < n
//
//   form TN:  a(i, k) = A[k + i * lda]   (block row of the factor: contraction index contiguous)
//   form NT:  a(i, k) = A[i + k * lda]   (columns of the triangular factor: row index contiguous)
//
// The result goes to the upper triangle of C, or (trans_c) mirrored to C[j + i * ldc], i <= j: the lower
// triangle of the same array.  The two factors of the preconditioner share one array that way (the
// first in the upper triangle, the transpose of the second two rows below it), and a triangular operand
// is masked below its diagonal while it is staged, because what lies there belongs to the other factor.
//
// and, with the triangle test and the patch enumeration switched off, the general product
//   C[i, j] = alpha * sum_k a(i, k) * b(j, k) + beta * C[i, j]   over a rectangular C with its own
// column operand b (always TN), which carries the first two steps of the column update (products
// with the rows above and with inverted diagonal blocks) and the merging of block inverses.
//
// A workgroup of 4 wavefronts owns a 128 x 128 tile of C, each wavefront a 64 x 64 piece as
// 4 x 4 accumulators of v_mfma_f64_16x16x4_f64.  Operand tiles (16 deep) are staged through
// LDS, double buffered, with the global loads issued a stage and a half ahead.  Two
// workgroups share a CU (72 KB of LDS and 4 x ~225 registers each), so that one runs while the
// other sits at its per-stage barrier: 256 x 128 tiles with one 8-wavefront workgroup per CU
// were 4 % slower.
//
// On this chip the fp64 matrix instruction and the vector ALU do not overlap: every VALU
// cycle of either wavefront of a SIMD is taken from the matrix pipe (8 dependent fp64 adds per
// 16 products cost 7 % in a micro-benchmark).  The loop is therefore written to issue next
// to no VALU work: operands are fetched with buffer loads whose range check replaces the
// bounds tests (rows past the matrix read zeros or neighbouring rows, and only ever reach
// entries of C that are not stored), per-thread offsets are computed once, the per-stage
// advance is scalar arithmetic on the buffer descriptor, and every LDS address is a fixed
// per-thread base plus an immediate.
//
// Workgroups are numbered so that the 64 that run together on an XCD (and share its L2) cover
// a 1024 x 1024 patch of C and re-use each other's operand rows.
#include "knm_internal.h"

namespace knm {
namespace {

typedef double d4 __attribute__((ext_vector_type(4)));
typedef double d2 __attribute__((ext_vector_type(2)));

#ifndef KNM_RANKK_TI
#define KNM_RANKK_TI 128
#endif
constexpr int kTI = KNM_RANKK_TI; // tile rows of C
constexpr int kTJ = 128;      // tile columns of C
constexpr int kTK = 16;       // contraction depth of a stage
constexpr int kWavesI = kTI / 64, kWavesJ = kTJ / 64; // wavefront grid of a workgroup
constexpr int kThreads = 64 * kWavesI * kWavesJ;
// LDS image of an operand tile: element (k, i) at k * stride + i, for the k-contiguous form at
// k * stride + (i ^ k).  The strides are 16 mod 32 doubles, so the four 16-lane groups of an
// operand read (four consecutive k) fall on alternating halves of the banks; the XOR spreads
// the 16 k of one column, which the k-contiguous form writes at once, over 16 bank pairs.
constexpr int kSA = kTI + 16;
constexpr int kSB = kTJ + 16;
constexpr int kStageDoubles = kTK * (kSA + kSB);
constexpr int kPatchI = 1024 / kTI, kPatchJ = 1024 / kTJ; // tiles of a patch: 1024 x 1024 entries of C
constexpr int kPatchWgs = kPatchI * kPatchJ;
constexpr int kXcds = 8;

struct RankKArgs {
    const double *A; // operand of the rows of C
    int64_t lda;
    int64_t extent;  // elements from A to one past the last one of the operand
    const double *B; // operand of the columns of C (= A for the symmetric update)
    int64_t ldb;
    int64_t extent_b;
    const double *w; // weights along the contraction, or null
    double *C;
    int64_t ldc;
    int64_t n, nj, K; // C is n x nj (nj = n for the symmetric update)
    double alpha, beta, shift;
    int tri;           // operand is upper triangular (what is stored below its diagonal is ignored): tile column j0 starts at k = j0
    int trans_c;       // store entry (i, j) at C[j + i * ldc]
    int patch_i;       // general product: tiles of a patch along i (kPatchWgs / patch_i along j)
    int64_t n_patch_i; // general product: patches along i
    int64_t n_patches; // patches in all (symmetric update: the upper-triangular ones)
};

// Stage loader of one operand: a (kTK x R) tile, kPer elements per thread in kPer / VEC loads of
// VEC consecutive doubles, held in registers between the buffer loads and the LDS stores.
// VEC = 2 needs every load 16-byte aligned (even leading dimension, 16-byte aligned operand).
//   TN (FORM 0): thread -> k = VEC (tid % (16 / VEC)) .. + VEC (contiguous in memory), rows tid / (16 / VEC) + kPass r
//   NT (FORM 1): thread -> rows VEC (tid % (R / VEC)) .. + VEC (contiguous in memory), k = tid / (R / VEC) + kStepK r
template <int FORM, int R, int VEC> struct Fetch {
    static constexpr int kPer = kTK * R / kThreads;
    static constexpr int kLoads = kPer / VEC;
    static constexpr int kPass = kThreads / (kTK / VEC);  // TN: row advance per load
    static constexpr int kStepK = kThreads / (R / VEC);   // NT: k advance per load
    double v[kPer];        // element e of load r at v[r * VEC + e]
    unsigned voff[kLoads]; // byte offsets of this thread's loads from the stage base
    const double *base;    // uniform: first element of the current stage of this tile
    int64_t left;          // uniform: elements from base to the end of the operand
    int64_t stage;         // uniform: elements per stage advance
    int row, k;            // tile-relative row and k of element 0

    __device__ __forceinline__ int row_of(int r, int e) const { return FORM == 0 ? row + kPass * r : row + e; }
    __device__ __forceinline__ int k_of(int r, int e) const { return FORM == 0 ? k + e : k + kStepK * r; }

    __device__ __forceinline__ void init(const double *P, int64_t ld, int64_t extent, int64_t row0, int64_t kbeg)
    {
        const int tid = threadIdx.x;
        int64_t first;
        if (FORM == 0) {
            k = VEC * (tid % (kTK / VEC));
            row = tid / (kTK / VEC);
            first = kbeg + row0 * ld;
            stage = kTK;
        } else {
            row = VEC * (tid % (R / VEC));
            k = tid / (R / VEC);
            first = row0 + kbeg * ld;
            stage = kTK * ld;
        }
#pragma unroll
        for (int r = 0; r < kLoads; ++r)
            voff[r] = (unsigned)((FORM == 0 ? (int64_t)k_of(r, 0) + (int64_t)row_of(r, 0) * ld
                                            : (int64_t)row_of(r, 0) + (int64_t)k_of(r, 0) * ld) * 8);
        base = P + first;
        left = extent - first;
    }
    // issue the loads of the next stage; reads past the operand's last element return zero
    __device__ __forceinline__ void load()
    {
        // left > 0 for every stage that is loaded; the descriptor's range is 32 bits
        const unsigned records = ((uint64_t)left >> 29) != 0 ? 0xffffffffu : (unsigned)left * 8u;
        const __amdgpu_buffer_rsrc_t rs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<double *>(base), 0, (int)records, 0x00020000);
#pragma unroll
        for (int r = 0; r < kLoads; ++r) {
            if (VEC == 1) {
                v[r] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(rs, (int)voff[r], 0, 0));
            } else {
                const d2 x = __builtin_bit_cast(d2, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff[r], 0, 0));
                v[2 * r] = x[0];
                v[2 * r + 1] = x[1];
            }
        }
        base += stage;
        left -= stage;
    }
    // the k-contiguous form can run past K inside the operand: zero k >= k_left (last stage only)
    __device__ __forceinline__ void mask_tail(int k_left)
    {
        if (FORM == 0) {
#pragma unroll
            for (int r = 0; r < kLoads; ++r)
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    if (k_of(r, e) >= k_left) v[r * VEC + e] = 0.0;
        }
    }
    // upper-triangular operand: zero the elements below the diagonal, row > k + delta in tile-relative
    // terms (delta = global k of the stage's first element minus global row of the tile's first row)
    __device__ __forceinline__ void mask_lower(int delta)
    {
#pragma unroll
        for (int r = 0; r < kLoads; ++r)
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                if (row_of(r, e) > k_of(r, e) + delta) v[r * VEC + e] = 0.0;
    }
    // weights of the stage's k, fetched together with the operand (buffer loads: zero past K)
    static constexpr int kW = FORM == 0 ? VEC : kLoads;
    double wv[kW];
    __device__ __forceinline__ void load_weights(const double *w_stage, int64_t w_left)
    {
        const unsigned records = ((uint64_t)w_left >> 29) != 0 ? 0xffffffffu : (unsigned)w_left * 8u;
        const __amdgpu_buffer_rsrc_t rs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<double *>(w_stage), 0, (int)records, 0x00020000);
#pragma unroll
        for (int q = 0; q < kW; ++q) {
            const int kk = FORM == 0 ? k + q : k + kStepK * q;
            wv[q] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(rs, kk * 8, 0, 0));
        }
    }
    __device__ __forceinline__ void scale()
    {
#pragma unroll
        for (int r = 0; r < kLoads; ++r)
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[r * VEC + e] *= wv[FORM == 0 ? e : r];
    }
    __device__ __forceinline__ void store(double *lds, int stride) const
    {
#pragma unroll
        for (int r = 0; r < kLoads; ++r) {
            if (FORM == 1 && VEC == 2) {
                *reinterpret_cast<d2 *>(lds + k_of(r, 0) * stride + row_of(r, 0)) = d2{v[2 * r], v[2 * r + 1]};
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int i = row_of(r, e), kk = k_of(r, e);
                    lds[kk * stride + (FORM == 0 ? (i ^ kk) : i)] = v[r * VEC + e];
                }
            }
        }
    }
};

// FA, FB: forms of the row and column operands; SYM: symmetric update (B = A, upper triangle of C
// only, triangular patch enumeration); otherwise the general product C = alpha a b^T + beta C
template <int FA, int FB, bool WEIGHTED, int VEC, bool SYM>
__global__ __launch_bounds__(kThreads) void rank_k_upper_kernel(RankKArgs a)
{
    __shared__ double lds[2 * kStageDoubles];
    // workgroup -> patch -> tile: consecutive workgroup ids go to consecutive XCDs, so the
    // workgroups of one patch are those with equal id % 8 and equal (id / 8) / kPatchWgs
    const int64_t g = blockIdx.x;
    const int64_t slot = g / kXcds;
    const int64_t q = (slot / kPatchWgs) * kXcds + g % kXcds;
    if (q >= a.n_patches) return;
    const int wq = (int)(slot % kPatchWgs);
    int64_t i0, j0;
    if (SYM) {
        // q = pj (pj + 1) / 2 + pi, pi <= pj
        int64_t pj = (int64_t)((sqrt(8.0 * (double)q + 1.0) - 1.0) * 0.5);
        while (pj * (pj + 1) / 2 > q) --pj;
        while ((pj + 1) * (pj + 2) / 2 <= q) ++pj;
        const int64_t pi = q - pj * (pj + 1) / 2;
        i0 = (pi * kPatchI + wq % kPatchI) * kTI;
        j0 = (pj * kPatchJ + wq / kPatchI) * kTJ;
        if (i0 >= a.n || j0 >= a.n || i0 > j0 + (kTJ - 1)) return; // outside C or strictly below its diagonal
    } else {
        const int64_t pi = q % a.n_patch_i, pj = q / a.n_patch_i;
        const int patch_j = kPatchWgs / a.patch_i;
        i0 = (pi * a.patch_i + wq % a.patch_i) * kTI;
        j0 = (pj * patch_j + wq / a.patch_i) * kTJ;
        if (i0 >= a.n || j0 >= a.nj) return;
    }

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wi = (wave % kWavesI) * 64, wj = (wave / kWavesI) * 64;
    const int64_t kbeg = (SYM && a.tri) ? j0 : 0; // a multiple of kTK
    const int64_t span = (a.K - kbeg + kTK - 1) / kTK;
    const int stages = span > 0x7fffffff ? 0x7fffffff : (int)span; // launch_rank_k_upper bounds K

    d4 acc[4][4];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int nn = 0; nn < 4; ++nn) acc[m][nn] = d4{0.0, 0.0, 0.0, 0.0};

    if (stages > 0) {
        Fetch<FA, kTI, VEC> fa;
        Fetch<FB, kTJ, VEC> fb;
        fa.init(a.A, a.lda, a.extent, i0, kbeg);
        fb.init(a.B, a.ldb, a.extent_b, j0, kbeg);
        // operand registers of k-step ks of the stage in `buf`: lane l takes k = 4 ks + l / 16
        const int qk = lane >> 4, l15 = lane & 15;
        auto read_ops = [&](const double *buf, int ks, double (&av)[4], double (&bv)[4]) {
            const int krow = ks * 4 + qk;
            const double *pa = buf + krow * kSA + wi + (FA == 0 ? (l15 ^ krow) : l15);
            const double *pb = buf + kTK * kSA + krow * kSB + wj + (FB == 0 ? (l15 ^ krow) : l15);
#pragma unroll
            for (int m = 0; m < 4; ++m) av[m] = pa[m * 16];
#pragma unroll
            for (int nn = 0; nn < 4; ++nn) bv[nn] = pb[nn * 16];
        };
        auto products = [&](const double (&av)[4], const double (&bv)[4]) {
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int nn = 0; nn < 4; ++nn)
                    acc[m][nn] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[m], bv[nn], acc[m][nn], 0, 0, 0);
        };
        // registers -> LDS for stage s (whose loads were issued earlier)
        const int k_total = (int)(a.K - kbeg);
        auto commit = [&](int s, double *buf) {
            const int k_left = k_total - s * kTK;
            if (k_left < kTK) {
                fa.mask_tail(k_left);
                fb.mask_tail(k_left);
            }
            if (SYM && a.tri) {
                // stages that still overlap the diagonal band of a tile's rows (the first few of a tile)
                const int64_t kk0 = kbeg + (int64_t)s * kTK;
                if (kk0 < i0 + kTI) fa.mask_lower((int)(kk0 - i0));
                if (kk0 < j0 + kTJ) fb.mask_lower((int)(kk0 - j0));
            }
            if (WEIGHTED) fb.scale();
            fa.store(buf, kSA);
            fb.store(buf + kTK * kSA, kSB);
        };

        const double *w_stage = WEIGHTED ? a.w + kbeg : nullptr;
        int64_t w_left = a.K - kbeg;
        auto fetch = [&]() {
            fa.load();
            fb.load();
            if (WEIGHTED) {
                fb.load_weights(w_stage, w_left);
                w_stage += kTK;
                w_left -= kTK;
            }
        };
        double a0[4], b0[4], a1[4], b1[4];
        fetch();
        commit(0, lds);
        if (stages > 1) fetch();
        __syncthreads();
        read_ops(lds, 0, a0, b0);
        // Per stage: the operands of a k-step are read while the products of the one before
        // run; the next stage's tile goes to the other LDS buffer in mid-stage (its loads were
        // issued a stage earlier) and the loads of the stage after that follow; the one
        // barrier sits before the last k-step, after which the first operands of the next
        // stage are read under the last products.  Two stages per trip keep the buffer
        // offsets compile-time constants.
        // The products have no side effects the compiler must order against LDS traffic or
        // barriers, and left alone it sinks them below the barrier, which then waits for the
        // LDS stores with nothing to run; the scheduling fences keep each group where it is.
        auto stage_body = [&](int s, const double *cur, double *nxt) {
            read_ops(cur, 1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            products(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            read_ops(cur, 2, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            products(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            if (s + 1 < stages) {
                commit(s + 1, nxt);
                if (s + 2 < stages) fetch();
            }
            read_ops(cur, 3, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            products(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            if (s + 1 < stages) read_ops(nxt, 0, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            products(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        };
        for (int s = 0; s < stages; s += 2) {
            stage_body(s, lds, lds + kStageDoubles);
            if (s + 1 < stages) stage_body(s + 1, lds + kStageDoubles, lds);
        }
    }

    // accumulator entry r of lane l is C[4 r + l / 16][l % 16] of its 16 x 16 block
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int nn = 0; nn < 4; ++nn) {
            const int64_t j = j0 + wj + nn * 16 + (lane & 15);
            const int64_t ib = i0 + wi + m * 16 + (lane >> 4);
            if (j >= a.nj) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t i = ib + 4 * r;
                if ((SYM && i > j) || i >= a.n) continue;
                double *dst = a.trans_c ? a.C + j + i * a.ldc : a.C + i + j * a.ldc;
                double v = a.alpha * acc[m][nn][r];
                if (a.beta != 0.0) v += a.beta * *dst;
                if (SYM && i == j) v += a.shift;
                *dst = v;
            }
        }
}

} // namespace

hipError_t launch_rank_k_upper(int form_nt, int64_t n, int64_t K, double alpha, const double *A, int64_t lda,
                               const double *w, int tri, double beta, double shift, double *C, int64_t ldc,
                               hipStream_t stream, int trans_c)
{
    if (n <= 0) return hipSuccess;
    RankKArgs a;
    a.A = a.B = A;
    a.lda = a.ldb = lda;
    a.w = w;
    a.C = C;
    a.ldc = ldc;
    a.n = a.nj = n;
    a.K = K;
    a.alpha = alpha;
    a.beta = beta;
    a.shift = shift;
    a.tri = tri;
    a.trans_c = trans_c;
    a.extent = a.extent_b = K <= 0 ? 0 : (form_nt ? (K - 1) * lda + n : (n - 1) * lda + K);
    const int64_t patch = (int64_t)kPatchI * kTI; // = kPatchJ * kTJ
    const int64_t n_patch = (n + patch - 1) / patch;
    a.patch_i = kPatchI;
    a.n_patch_i = n_patch;
    a.n_patches = n_patch * (n_patch + 1) / 2;
    const int64_t groups = (a.n_patches + kXcds - 1) / kXcds;
    const int64_t wgs = groups * kXcds * kPatchWgs;
    if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    // a thread's byte offsets inside a stage must fit the 32-bit buffer offset
    const int64_t span = form_nt ? (int64_t)kTK * lda + kTI : (int64_t)kTI * lda + kTK;
    if (span * 8 >= 0xffffffffLL || K >= (int64_t)0x7fffffff * kTK) return hipErrorInvalidValue;
    const dim3 grid((unsigned)wgs), block(kThreads);
    // 16-byte loads when every one of them is aligned: tile origins are multiples of 128
    const bool vec2 = lda % 2 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0;
    const int which = (form_nt ? 4 : 0) + (w ? 2 : 0) + (vec2 ? 1 : 0);
    switch (which) {
    case 0: hipLaunchKernelGGL((rank_k_upper_kernel<0, 0, false, 1, true>), grid, block, 0, stream, a); break;
    case 1: hipLaunchKernelGGL((rank_k_upper_kernel<0, 0, false, 2, true>), grid, block, 0, stream, a); break;
    case 2: hipLaunchKernelGGL((rank_k_upper_kernel<0, 0, true, 1, true>), grid, block, 0, stream, a); break;
    case 3: hipLaunchKernelGGL((rank_k_upper_kernel<0, 0, true, 2, true>), grid, block, 0, stream, a); break;
    case 4: hipLaunchKernelGGL((rank_k_upper_kernel<1, 1, false, 1, true>), grid, block, 0, stream, a); break;
    case 5: hipLaunchKernelGGL((rank_k_upper_kernel<1, 1, false, 2, true>), grid, block, 0, stream, a); break;
    case 6: hipLaunchKernelGGL((rank_k_upper_kernel<1, 1, true, 1, true>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((rank_k_upper_kernel<1, 1, true, 2, true>), grid, block, 0, stream, a); break;
    }
    return hipGetLastError();
}

hipError_t launch_gemm_f64(int a_nt, int64_t ni, int64_t nj, int64_t K, double alpha, const double *A, int64_t lda,
                           const double *B, int64_t ldb, double beta, double *C, int64_t ldc, hipStream_t stream, int b_nt)
{
    if (b_nt && !a_nt) return hipErrorInvalidValue; // not instantiated
    if (ni <= 0 || nj <= 0) return hipSuccess;
    RankKArgs a;
    a.A = A;
    a.lda = lda;
    a.B = B;
    a.ldb = ldb;
    a.w = nullptr;
    a.C = C;
    a.ldc = ldc;
    a.n = ni;
    a.nj = nj;
    a.K = K;
    a.alpha = alpha;
    a.beta = beta;
    a.shift = 0.0;
    a.tri = 0;
    a.trans_c = 0;
    a.extent = K <= 0 ? 0 : (a_nt ? (K - 1) * lda + ni : (ni - 1) * lda + K);
    a.extent_b = K <= 0 ? 0 : (b_nt ? (K - 1) * ldb + nj : (nj - 1) * ldb + K);
    // patches of 64 tiles, as square as the shape of C allows
    const int64_t tiles_i = (ni + kTI - 1) / kTI;
    int patch_i = 1;
    while (patch_i < 8 && patch_i < tiles_i) patch_i *= 2;
    const int patch_j = kPatchWgs / patch_i;
    a.patch_i = patch_i;
    a.n_patch_i = (tiles_i + patch_i - 1) / patch_i;
    const int64_t tiles_j = (nj + kTJ - 1) / kTJ;
    a.n_patches = a.n_patch_i * ((tiles_j + patch_j - 1) / patch_j);
    const int64_t groups = (a.n_patches + kXcds - 1) / kXcds;
    const int64_t wgs = groups * kXcds * kPatchWgs;
    if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    const int64_t span_a = a_nt ? (int64_t)kTK * lda + kTI : (int64_t)kTI * lda + kTK;
    const int64_t span_b = b_nt ? (int64_t)kTK * ldb + kTJ : (int64_t)kTJ * ldb + kTK;
    if (span_a * 8 >= 0xffffffffLL || span_b * 8 >= 0xffffffffLL || K >= (int64_t)0x7fffffff * kTK)
        return hipErrorInvalidValue;
    const dim3 grid((unsigned)wgs), block(kThreads);
    const bool vec2 = lda % 2 == 0 && ldb % 2 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0 &&
                      reinterpret_cast<uintptr_t>(B) % 16 == 0;
    if (b_nt && vec2)
        hipLaunchKernelGGL((rank_k_upper_kernel<1, 1, false, 2, false>), grid, block, 0, stream, a);
    else if (b_nt)
        hipLaunchKernelGGL((rank_k_upper_kernel<1, 1, false, 1, false>), grid, block, 0, stream, a);
    else if (a_nt && vec2)
        hipLaunchKernelGGL((rank_k_upper_kernel<1, 0, false, 2, false>), grid, block, 0, stream, a);
    else if (a_nt)
        hipLaunchKernelGGL((rank_k_upper_kernel<1, 0, false, 1, false>), grid, block, 0, stream, a);
    else if (vec2)
        hipLaunchKernelGGL((rank_k_upper_kernel<0, 0, false, 2, false>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((rank_k_upper_kernel<0, 0, false, 1, false>), grid, block, 0, stream, a);
    return hipGetLastError();
}

} // namespace knm
