// Gaussian-kernel tile engine with the cross term on the f16 matrix cores:
//     out[f] = sum_s k(F_f, S_s) vec[s]          (d <= 44, one column per launch)
//
// Same computation as knm_tile.hip (Section 3.1, "Blockwise K_nm-vector product"; Gaussian
// kernel of Section 2), different arithmetic for the contraction over d.  Measured on
// gfx950, fp32 MFMA shares the vector ALU's issue with the exp/FMA work that finishes
// every kernel entry, so the fp32 engine is bound by MFMA time PLUS VALU time.  The f16
// MFMA (v_mfma_f32_32x32x16_f16, 16x the rate, products exact, fp32 accumulation, fp16
// subnormal inputs honoured -- all checked on the device) runs beside the VALU instead.
// To keep fp32-level accuracy every scaled feature z = x sqrt(log2(e)) / sigma is split
// into two halves, z = zh + zl (22 significant bits), and the cross term is evaluated as
//     <f, x>  ~=  fh.xh + fh.xl + fl.xh                        (drops fl.xl ~ 2^-22)
// i.e. three "planes" of the same MFMA shape.  With this scaling the base-2 exponent is
//     log2 k(f, x) = <zf, zx> - |zf|^2 / 2 - |zx|^2 / 2 .
// The two norm terms ride in four spare K-slots per side as 4-digit fixed-point numbers,
//     n = q1 2^10 + q2 2^-1 + q3 2^-12 + q4 2^-23,   q_i integers <= 2048 (exact in fp16),
// multiplied by the constants 2^10, 2^-1, 2^-12, 2^-23 on the other operand, so the MFMA
// accumulator again holds the exponent itself (resolution 2^-24, range 2^21; the last constant
// is an fp16 subnormal, which the MFMA honours).
// Inputs outside that range (|z| > 65000, norm term |z|^2 / 2 >= 2^21) saturate.
//
// Layout.  A K=16 MFMA takes 8 halves ("unit") from each half-wave.  Unit u holds
// features 8u .. 8u+7; the last four slots of the last unit are the special slots.
// Plane 1 = (fh | -q^f) x (xh | consts), plane 2 = (fh | consts) x (xl | -q^x),
// plane 3 = (fl | 0) x (xh | consts); the stream side keeps two register sets (xh, xl), the
// fixed side three (fh, a variant of fh's last MFMA operand with the constants, fl).
//
// Packing.  Converting a stream point (scale, split, norm digits) costs ~10 VALU
// instructions per feature, and every workgroup of a sweep would repeat it for the same
// points.  A small pre-pass (`pack_stream_kernel`) therefore converts the stream points
// once into a packed image in device memory, laid out exactly as the LDS stage (per
// 32-point tile: [plane xh/xl][MFMA][lane] units of 8 halves); the sweep's staging is then
// a straight 16-byte copy, done by loads that write LDS directly (no staging registers, no
// LDS write instructions), one stage ahead.  The image is built slab by slab (bounded
// workspace) and the sweep is launched once per slab.
//
// Schedule.  Accumulators are double-buffered across stream tiles: while the matrix
// cores run the 3 NU MFMAs of tile k (two fixed blocks), the VALU finishes tile k-1
// (exp, FMA), spread behind the MFMAs.  The hot instructions are volatile inline
// assembly so this order survives the compiler; no MFMA result is read until a whole
// tile after it was issued, and no exp result by the instruction right after it.

#include <type_traits>

#include "knm_internal.h"
#include "knm_operands.h"

namespace knm {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
// stream points per LDS stage: 256 (eight tiles between barriers) while two workgroups' double buffers
// still fit a CU's LDS, 128 for the six-unit layout
constexpr int stage_of(int nu, int /*kind*/) { return nu <= 4 ? 256 : 128; }
// ---- one MFMA followed by G (exp, FMA) pairs of the previous tile -------------------------
#define KNM_MFMA_FIRST "v_mfma_f32_32x32x16_f16 %[acc], %[a], %[b], 0\n\t"
#define KNM_MFMA_NEXT "v_mfma_f32_32x32x16_f16 %[acc], %[a], %[b], %[acc]\n\t"
#define KNM_EXP(i) "v_exp_f32_e64 %[p" #i "], %[x" #i "] clamp\n\t"
#define KNM_FMA(i) "v_fmac_f32_e32 %[s" #i "], %[p" #i "], %[vl]\n\t"
#define KNM_P(i) [p##i] "=&v"(p##i)
#define KNM_S(i) [s##i] "+v"(s[R0 + i])
#define KNM_X(i) [x##i] "v"(pa[R0 + i])

template <bool FIRST, int G, int R0>
__device__ __forceinline__ void mfma_step(f32x16 &acc, const f16x8 &a, const f16x8 &b, const f32x16 &pa, float vl,
                                          float (&s)[16])
{
    float p0, p1, p2, p3, p4, p5;
    (void)p0; (void)p1; (void)p2; (void)p3; (void)p4; (void)p5;
    if constexpr (FIRST) {
        static_assert(G == 1 || G == 2 || G == 3 || G == 5, "first step of a chain");
        if constexpr (G == 1)
            asm volatile(KNM_MFMA_FIRST KNM_EXP(0) "s_nop 0\n\t" KNM_FMA(0)
                         : [acc] "=&v"(acc), KNM_P(0), KNM_S(0)
                         : [a] "v"(a), [b] "v"(b), KNM_X(0), [vl] "v"(vl));
        else if constexpr (G == 2)
            asm volatile(KNM_MFMA_FIRST KNM_EXP(0) KNM_EXP(1) KNM_FMA(0) KNM_FMA(1)
                         : [acc] "=&v"(acc), KNM_P(0), KNM_P(1), KNM_S(0), KNM_S(1)
                         : [a] "v"(a), [b] "v"(b), KNM_X(0), KNM_X(1), [vl] "v"(vl));
        else if constexpr (G == 3)
            asm volatile(KNM_MFMA_FIRST KNM_EXP(0) KNM_EXP(1) KNM_EXP(2) KNM_FMA(0) KNM_FMA(1) KNM_FMA(2)
                         : [acc] "=&v"(acc), KNM_P(0), KNM_P(1), KNM_P(2), KNM_S(0), KNM_S(1), KNM_S(2)
                         : [a] "v"(a), [b] "v"(b), KNM_X(0), KNM_X(1), KNM_X(2), [vl] "v"(vl));
        else
            asm volatile(KNM_MFMA_FIRST KNM_EXP(0) KNM_EXP(1) KNM_EXP(2) KNM_EXP(3) KNM_EXP(4) KNM_FMA(0) KNM_FMA(1)
                             KNM_FMA(2) KNM_FMA(3) KNM_FMA(4)
                         : [acc] "=&v"(acc), KNM_P(0), KNM_P(1), KNM_P(2), KNM_P(3), KNM_P(4), KNM_S(0), KNM_S(1),
                           KNM_S(2), KNM_S(3), KNM_S(4)
                         : [a] "v"(a), [b] "v"(b), KNM_X(0), KNM_X(1), KNM_X(2), KNM_X(3), KNM_X(4), [vl] "v"(vl));
    } else {
        static_assert(G >= 1 && G <= 6 && G != 4, "group size");
        if constexpr (G == 1)
            asm volatile(KNM_MFMA_NEXT KNM_EXP(0) "s_nop 0\n\t" KNM_FMA(0)
                         : [acc] "+v"(acc), KNM_P(0), KNM_S(0)
                         : [a] "v"(a), [b] "v"(b), KNM_X(0), [vl] "v"(vl));
        else if constexpr (G == 2)
            asm volatile(KNM_MFMA_NEXT KNM_EXP(0) KNM_EXP(1) KNM_FMA(0) KNM_FMA(1)
                         : [acc] "+v"(acc), KNM_P(0), KNM_P(1), KNM_S(0), KNM_S(1)
                         : [a] "v"(a), [b] "v"(b), KNM_X(0), KNM_X(1), [vl] "v"(vl));
        else if constexpr (G == 3)
            asm volatile(KNM_MFMA_NEXT KNM_EXP(0) KNM_EXP(1) KNM_EXP(2) KNM_FMA(0) KNM_FMA(1) KNM_FMA(2)
                         : [acc] "+v"(acc), KNM_P(0), KNM_P(1), KNM_P(2), KNM_S(0), KNM_S(1), KNM_S(2)
                         : [a] "v"(a), [b] "v"(b), KNM_X(0), KNM_X(1), KNM_X(2), [vl] "v"(vl));
        else if constexpr (G == 5)
            asm volatile(KNM_MFMA_NEXT KNM_EXP(0) KNM_EXP(1) KNM_EXP(2) KNM_EXP(3) KNM_EXP(4) KNM_FMA(0) KNM_FMA(1)
                             KNM_FMA(2) KNM_FMA(3) KNM_FMA(4)
                         : [acc] "+v"(acc), KNM_P(0), KNM_P(1), KNM_P(2), KNM_P(3), KNM_P(4), KNM_S(0), KNM_S(1),
                           KNM_S(2), KNM_S(3), KNM_S(4)
                         : [a] "v"(a), [b] "v"(b), KNM_X(0), KNM_X(1), KNM_X(2), KNM_X(3), KNM_X(4), [vl] "v"(vl));
        else
            asm volatile(KNM_MFMA_NEXT KNM_EXP(0) KNM_EXP(1) KNM_EXP(2) KNM_EXP(3) KNM_EXP(4) KNM_EXP(5) KNM_FMA(0)
                             KNM_FMA(1) KNM_FMA(2) KNM_FMA(3) KNM_FMA(4) KNM_FMA(5)
                         : [acc] "+v"(acc), KNM_P(0), KNM_P(1), KNM_P(2), KNM_P(3), KNM_P(4), KNM_P(5), KNM_S(0),
                           KNM_S(1), KNM_S(2), KNM_S(3), KNM_S(4), KNM_S(5)
                         : [a] "v"(a), [b] "v"(b), KNM_X(0), KNM_X(1), KNM_X(2), KNM_X(3), KNM_X(4), KNM_X(5),
                           [vl] "v"(vl));
    }
}

// ---- kernels of r = |f - x| (Laplacian, Matern): one MFMA followed by the finish of G entries ----
// The accumulator holds x = -(log2(e) u)^2; the kernel value is 2^-sqrt(|x|) (times a polynomial in u
// for the Matern kernels).  Entries whose |x| lies below the lane's threshold `thr` (pairs so close
// that the cancellation error of the norm expansion would show after the square root) get the
// value 0 here and are noted in `near` (a wave mask); the caller evaluates them again from
// differences.  Every instruction is its own volatile statement, in program order; a transcendental
// result is never read by the instruction right after it.
struct RadialConsts {
    float big;   // replaces the exponent of a near pair: 2^-sqrt(big) = 0
    float ln2;   // u = y ln 2 for y = log2(e) u
    float third; // Matern 5/2
};

template <int KIND, int G, int R0>
__device__ __forceinline__ void radial_group(const f32x16 &pa, float thr, float vl, const RadialConsts &rc, float (&s)[16],
                                             uint64_t &near)
{
    float p[G], q[G];
#pragma unroll
    for (int i = 0; i < G; ++i)
        asm volatile("v_cmp_lt_f32_e64 vcc, |%2|, %3\n\t"
                     "s_or_b64 %1, %1, vcc\n\t"
                     "v_cndmask_b32_e32 %0, %2, %4, vcc"
                     : "=&v"(p[i]), "+s"(near)
                     : "v"(pa[R0 + i]), "v"(thr), "v"(rc.big)
                     : "vcc");
#pragma unroll
    for (int i = 0; i < G; ++i) asm volatile("v_sqrt_f32_e64 %0, |%1|" : "=v"(q[i]) : "v"(p[i]));
    if constexpr (G == 1) asm volatile("s_nop 0");
#pragma unroll
    for (int i = 0; i < G; ++i) asm volatile("v_exp_f32_e64 %0, -%1" : "=v"(p[i]) : "v"(q[i]));
    if constexpr (KIND == KNM_KERNEL_LAPLACIAN) {
        if constexpr (G == 1) asm volatile("s_nop 0");
    } else {
#pragma unroll
        for (int i = 0; i < G; ++i) asm volatile("v_mul_f32_e32 %0, %1, %0" : "+v"(q[i]) : "v"(rc.ln2)); // u
        if constexpr (KIND == KNM_KERNEL_MATERN32) {
#pragma unroll
            for (int i = 0; i < G; ++i) asm volatile("v_fmac_f32_e32 %0, %1, %0" : "+v"(p[i]) : "v"(q[i])); // e + u e
        } else {
            float w[G];
#pragma unroll
            for (int i = 0; i < G; ++i) asm volatile("v_fma_f32 %0, %1, %2, 1.0" : "=v"(w[i]) : "v"(q[i]), "v"(rc.third));
#pragma unroll
            for (int i = 0; i < G; ++i) asm volatile("v_fma_f32 %0, %1, %0, 1.0" : "+v"(w[i]) : "v"(q[i])); // 1 + u + u^2 / 3
#pragma unroll
            for (int i = 0; i < G; ++i) asm volatile("v_mul_f32_e32 %0, %0, %1" : "+v"(p[i]) : "v"(w[i]));
        }
    }
#pragma unroll
    for (int i = 0; i < G; ++i) asm volatile("v_fmac_f32_e32 %0, %1, %2" : "+v"(s[R0 + i]) : "v"(p[i]), "v"(vl));
}

template <bool FIRST>
__device__ __forceinline__ void mfma_only(f32x16 &acc, const f16x8 &a, const f16x8 &b)
{
    if constexpr (FIRST) asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

// The 3 HU MFMAs of one fixed block on one stream tile, with the finish of the 16 entries of the
// same block's accumulator of the previous tile (`pa`, weight `vl_prev`; for the kernels of r also
// that tile's threshold `thr_prev`) spread behind them.
template <int HU, int KIND, int I = 0>
__device__ __forceinline__ void block_tile(f32x16 &acc, const f16x8 (&fh)[HU], const f16x8 &fhv,
                                           const f16x8 (&fl)[HU], const f16x8 (&bh)[HU], const f16x8 (&bl)[HU],
                                           const f32x16 &pa, float vl_prev, float thr_prev, const RadialConsts &rc,
                                           float (&s)[16], uint64_t &near)
{
    constexpr int NM = 3 * HU;
    if constexpr (I < NM) {
        constexpr int R0 = (16 * I) / NM;
        constexpr int G = (16 * (I + 1)) / NM - R0;
        constexpr int plane = I / HU, m = I % HU;
        const f16x8 &a = plane == 0 ? fh[m] : (plane == 1 ? (m == HU - 1 ? fhv : fh[m]) : fl[m]);
        const f16x8 &b = plane == 1 ? bl[m] : bh[m];
        if constexpr (KIND == KNM_KERNEL_GAUSSIAN) {
            mfma_step<I == 0, G, R0>(acc, a, b, pa, vl_prev, s);
        } else {
            mfma_only<I == 0>(acc, a, b);
            radial_group<KIND, G, R0>(pa, thr_prev, vl_prev, rc, s, near);
        }
        block_tile<HU, KIND, I + 1>(acc, fh, fhv, fl, bh, bl, pa, vl_prev, thr_prev, rc, s, near);
    }
}

// Packed image of stream points [row0, row0 + rows) (rows beyond nS are zero points):
// tile g of the slab occupies 2 * HU * 64 units at packed + g * 2 * HU * 64.
template <int NU, int VW>
__global__ __launch_bounds__(kThreads) void pack_stream_kernel(const float *__restrict__ S, int64_t nS, int64_t lds,
                                                               const float *__restrict__ mu, int d, float sigma,
                                                               int64_t row0, int64_t rows, f16x8 *__restrict__ packed,
                                                               unsigned int *__restrict__ range_count)
{
    constexpr int HU = NU / 2;
    constexpr int FPT = 8 * HU;
    const int tid = threadIdx.x;
    const int part = tid & 1;
    const int64_t rel = (int64_t)blockIdx.x * (kThreads / 2) + (tid >> 1); // point within the slab
    if (rel >= rows) return;
    const int64_t idx = row0 + rel;
    const bool valid = idx < nS;
    const float gamma = sqrtf(kLog2e) / sigma;
    float xs[FPT];
    load_features<FPT, VW>(S + (valid ? idx : 0) * lds, mu, true, part * FPT, d, valid, xs);
    float nrm = 0.0f;
    bool clamped = false;
#pragma unroll
    for (int k = 0; k < FPT; ++k) {
        xs[k] *= gamma;
        nrm = fmaf(xs[k], xs[k], nrm);
        clamped |= out_of_half_range(xs[k]);
    }
    nrm += __shfl_xor(nrm, 1);
    clamped |= !(0.5f * nrm <= kNormMax);
    clamped |= (__shfl_xor((int)clamped, 1) != 0); // the two threads of a point
    if (clamped && valid && part == 0) atomicAdd(range_count, 1u); // rare: one count per point
    _Float16 q[4];
    norm_digits(0.5f * nrm, q);
    f16x8 *tile = packed + (rel >> 5) * (2 * HU * 64);
    const int prow = (int)(rel & 31);
#pragma unroll
    for (int j = 0; j < HU; ++j) {
        const int u = part * HU + j; // unit of the point
        f16x8 hi, lo;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            f16x2 ph, pl;
            split_pair(xs[8 * j + e], xs[8 * j + e + 1], ph, pl);
            hi[e] = (_Float16)ph[0]; hi[e + 1] = (_Float16)ph[1];
            lo[e] = (_Float16)pl[0]; lo[e + 1] = (_Float16)pl[1];
        }
        if (j == HU - 1 && part == 1) { // last unit: constants beside xh, norm digits beside xl
            hi[4] = (_Float16)kC1; hi[5] = (_Float16)kC2; hi[6] = (_Float16)kC3; hi[7] = (_Float16)kC4;
            lo[4] = q[0]; lo[5] = q[1]; lo[6] = q[2]; lo[7] = q[3];
        }
        tile[(0 * HU + (u >> 1)) * 64 + (u & 1) * 32 + prow] = hi;
        tile[(1 * HU + (u >> 1)) * 64 + (u & 1) * 32 + prow] = lo;
    }
}

// `packed` is the image of the stream chunks [chunk0, chunk0 + n_chunks) built by pack_stream_kernel.
// Workgroup -> (fixed block, chunk of the slab).  Workgroups are dealt round-robin to the 8 XCDs (each with
// its own L2) in launch order; the first 8 floor(n_chunks / 8) chunks are numbered so that all fixed blocks
// of a chunk run on one XCD, one chunk after the other, and the chunk's image is fetched into one L2 instead
// of eight; the remaining chunks are spread over all XCDs, so that every XCD gets the same work.
template <int NU, int KIND>
__global__ __launch_bounds__(kThreads, 2) void gauss_sweep_f16_kernel(SweepArgs a, const f16x8 *__restrict__ packed,
                                                                      int64_t chunk0, int n_fblocks, int n_chunks)
{
    int64_t fblock, chunk_local;
    const int grouped = n_chunks & ~7; // chunks that are dealt to one XCD each
    if ((int64_t)blockIdx.x < (int64_t)grouped * n_fblocks) {
        const int64_t slot = (int64_t)blockIdx.x >> 3;
        chunk_local = (slot / n_fblocks) * 8 + (blockIdx.x & 7);
        fblock = slot % n_fblocks;
    } else {
        const int64_t rest = (int64_t)blockIdx.x - (int64_t)grouped * n_fblocks;
        fblock = rest % n_fblocks;
        chunk_local = grouped + rest / n_fblocks;
    }

    constexpr bool kRadial = KIND != KNM_KERNEL_GAUSSIAN;
    constexpr int HU = NU / 2;                      // MFMAs per plane
    constexpr int kStage = stage_of(NU, KIND);
    constexpr int kTilesPerStage = kStage / 32;
    constexpr int UPS = kTilesPerStage * 2 * HU * 64; // 16-byte units per stage
    constexpr int UPT = UPS / kThreads;             // units copied per thread and stage
    static_assert(NU % 2 == 0 && NU >= 2, "an MFMA takes two units");

    __shared__ f16x8 img[2][kTilesPerStage][2][HU][64]; // [buffer][tile][plane xh/xl][mfma][lane]
    __shared__ float vv[2][kStage];
    __shared__ float tt[kRadial ? 2 : 1][kRadial ? kStage : 1]; // per stream point: threshold of a near pair

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row = lane & 31;
    const int h = lane >> 5;
    const float gamma = sqrtf(kLog2e) / a.sigma;
    const int d = a.d;

    // ---- fixed operand: 2 blocks of 32 points per wavefront, in registers -----------------
    const int64_t fixed0 = (fblock * kWaves + wave) * 64;
    f16x8 fh[2][HU], fl[2][HU], fhv[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int64_t idx = fixed0 + rb * 32 + row;
        const bool valid = idx < a.nF;
        const float *p = a.F + (valid ? idx : 0) * a.ldf;
        float nrm = 0.0f;
        bool clamped = false;
#pragma unroll
        for (int m = 0; m < HU; ++m) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = 8 * (2 * m + h) + e;
                const float z = (valid && k < d) ? gamma * (p[k] - a.mu[k < d ? k : 0]) : 0.0f;
                nrm = fmaf(z, z, nrm);
                clamped |= out_of_half_range(z);
                _Float16 zh, zl;
                split_half(z, zh, zl);
                fh[rb][m][e] = zh;
                fl[rb][m][e] = zl;
            }
        }
        nrm += __shfl_xor(nrm, 32);
        clamped |= !(0.5f * nrm <= kNormMax);
        clamped |= (__shfl_xor((int)clamped, 32) != 0); // the two lanes of a point
        // one count per point and sweep: the workgroups of the first chunk report (every chunk's
        // workgroups convert the same fixed points)
        if (clamped && valid && h == 0 && chunk_local == 0 && chunk0 == 0) atomicAdd(a.range_count, 1u);
        _Float16 q[4];
        norm_digits(valid ? 0.5f * nrm : 0.0f, q);
        fhv[rb] = fh[rb][HU - 1];
        if (h == 1) { // the special slots live in the last unit, which half-wave 1 supplies
            fh[rb][HU - 1][4] = q[0]; fh[rb][HU - 1][5] = q[1]; fh[rb][HU - 1][6] = q[2]; fh[rb][HU - 1][7] = q[3];
            fhv[rb][4] = (_Float16)kC1; fhv[rb][5] = (_Float16)kC2; fhv[rb][6] = (_Float16)kC3; fhv[rb][7] = (_Float16)kC4;
        }
    }

    float sum[2][16];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[rb][r] = 0.0f;

    // ---- stream staging: a straight copy of the packed image, 16 bytes per thread and unit --------
    const int64_t chunk = chunk0 + chunk_local;
    const int64_t chunk_begin = chunk * a.chunk_len;
    int64_t chunk_end = chunk_begin + a.chunk_len;
    if (chunk_end > a.nS) chunk_end = a.nS;
    const int n_stages = (int)((chunk_end - chunk_begin + kStage - 1) / kStage);
    const f16x8 *src = packed + (chunk_local * a.chunk_len / kStage) * UPS + tid;

    // The image goes from memory into LDS by loads that write LDS directly (a wavefront's 64 units land in
    // the 1 KB at the address in M0), started one stage ahead; vmcnt counts them, and since the compiler
    // does not look inside inline assembly the wait for them is written out where a stage begins.
    const unsigned lds_wave = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) f16x8 *)&img[0][0][0][0][0] + (unsigned)wave * 1024u);
    const unsigned src_off = (unsigned)tid * 16u;
    auto issue = [&](int stage, int buf) {
        const f16x8 *const b = uniform_pointer(src - tid + (int64_t)stage * UPS);
        const unsigned l = __builtin_amdgcn_readfirstlane(lds_wave + (unsigned)buf * (unsigned)(UPS * 16));
        unsigned m0_saved;
        static_assert(UPT == 4 || UPT == 6 || UPT == 8, "one block of inline assembly per count");
        // (one wait state between a scalar write of M0 and the load that reads it)
#define KNM_DMA_FIRST "s_mov_b32 %[keep], m0\n\ts_mov_b32 m0, %[l]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[o], %[b0]\n\t"
#define KNM_DMA_NEXT(k) "s_add_u32 m0, m0, 0x1000\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[o], %[b" #k "]\n\t"
#define KNM_DMA_LAST "s_mov_b32 m0, %[keep]"
        if constexpr (UPT == 4)
            asm volatile(KNM_DMA_FIRST KNM_DMA_NEXT(1) KNM_DMA_NEXT(2) KNM_DMA_NEXT(3) KNM_DMA_LAST
                         : [keep] "=&s"(m0_saved)
                         : [l] "s"(l), [o] "v"(src_off), [b0] "s"(b), [b1] "s"(b + kThreads), [b2] "s"(b + 2 * kThreads),
                           [b3] "s"(b + 3 * kThreads)
                         : "memory", "scc");
        else if constexpr (UPT == 6)
            asm volatile(KNM_DMA_FIRST KNM_DMA_NEXT(1) KNM_DMA_NEXT(2) KNM_DMA_NEXT(3) KNM_DMA_NEXT(4) KNM_DMA_NEXT(5) KNM_DMA_LAST
                         : [keep] "=&s"(m0_saved)
                         : [l] "s"(l), [o] "v"(src_off), [b0] "s"(b), [b1] "s"(b + kThreads), [b2] "s"(b + 2 * kThreads),
                           [b3] "s"(b + 3 * kThreads), [b4] "s"(b + 4 * kThreads), [b5] "s"(b + 5 * kThreads)
                         : "memory", "scc");
        else
            asm volatile(KNM_DMA_FIRST KNM_DMA_NEXT(1) KNM_DMA_NEXT(2) KNM_DMA_NEXT(3) KNM_DMA_NEXT(4) KNM_DMA_NEXT(5)
                             KNM_DMA_NEXT(6) KNM_DMA_NEXT(7) KNM_DMA_LAST
                         : [keep] "=&s"(m0_saved)
                         : [l] "s"(l), [o] "v"(src_off), [b0] "s"(b), [b1] "s"(b + kThreads), [b2] "s"(b + 2 * kThreads),
                           [b3] "s"(b + 3 * kThreads), [b4] "s"(b + 4 * kThreads), [b5] "s"(b + 5 * kThreads),
                           [b6] "s"(b + 6 * kThreads), [b7] "s"(b + 7 * kThreads)
                         : "memory", "scc");
#undef KNM_DMA_FIRST
#undef KNM_DMA_NEXT
#undef KNM_DMA_LAST
    };
    float vs = 0.0f;
    typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
    f16x4 digits = {(_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f};
    auto fetch = [&](int stage) {
        const int sp = tid & (kStage - 1); // stream point of the stage this thread brings the vector entry of
        const int64_t idx = chunk_begin + (int64_t)stage * kStage + sp;
        const bool valid = idx < chunk_end;
        const int64_t vi = valid ? idx : 0;
        const float vraw = a.vec[vi * a.ldv];
        const float wraw = (a.wgt != nullptr) ? a.wgt[vi] : 1.0f;
        vs = valid ? vraw * wraw : 0.0f;
        if constexpr (kRadial) {
            // the point's norm term, as the four digits the packing kernel left in the last unit of
            // the lo plane (half-wave 1, slots 4..7): unit (tile, plane 1, MFMA HU - 1, lane 32 + row)
            const f16x8 *unit = src - tid + (int64_t)stage * UPS + ((sp >> 5) * 2 * HU + HU + (HU - 1)) * 64 + 32 + (sp & 31);
            digits = reinterpret_cast<const f16x4 *>(unit)[1];
        }
    };
    auto commit = [&](int buf) {
        if (tid < kStage) vv[buf][tid] = vs;
        if constexpr (kRadial) {
            // the digits hold -n; a near pair has nearly equal norms, so the stream point's own
            // norm stands for both
            const float nrm = -(kC1 * (float)digits[0] + kC2 * (float)digits[1] + kC3 * (float)digits[2] + kC4 * (float)digits[3]);
            if (tid < kStage) tt[buf][tid] = near_pair_threshold(nrm, d);
        }
    };

    // accumulators of the tile in flight (cur) and of the tile being finished (prev)
    f32x16 accA[2], accB[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) { accA[rb][r] = 0.0f; accB[rb][r] = 0.0f; }
    float vl_prev = 0.0f; // zero weight: the first "previous tile" contributes nothing
    // kernels of r: threshold and stream point of the tile being finished (no entry of the first
    // "previous tile" lies below a zero threshold), the wave's mask of near pairs seen, constants
    float thr_prev = 0.0f;
    int64_t j_prev = 0;
    uint64_t near = 0;
    RadialConsts rc;
    rc.big = 1.0e30f;
    rc.ln2 = 0.6931471805599453f;
    rc.third = 1.0f / 3.0f;
    const float s2 = kLog2e / (2.0f * a.sigma * a.sigma); // exponent per squared distance, for the second evaluation
    // Second evaluation of the near pairs of one finished tile (rare: behind a wave-uniform branch):
    // their exponents again from fp32 differences of the two rows, exact for coincident rows.
    auto refine = [&](const f32x16 (&acc)[2], float thr_t, float vl_t, int64_t j) {
        const bool in = j < chunk_end; // a padding point has a zero vector entry
        const float *srow = a.S + (in ? j : 0) * a.lds;
        uint32_t m = 0; // bit 16 rb + r: entry r of block rb is a near pair of this lane
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (fabsf(acc[rb][r]) < thr_t) m |= 1u << (16 * rb + r);
        if (!in) m = 0;
        while (__builtin_amdgcn_ballot_w64(m != 0) != 0) {
            int b = -1;
            float term = 0.0f;
            if (m != 0) {
                b = __builtin_ctz(m);
                m &= m - 1;
                const int64_t fi = fixed0 + (b >> 4) * 32 + 8 * ((b & 15) >> 2) + 4 * h + (b & 3);
                if (fi < a.nF) term = radial_from_exponent<KIND>(exact_exponent(a.F + fi * a.ldf, srow, d, s2)) * vl_t;
            }
#pragma unroll
            for (int k = 0; k < 32; ++k) sum[k >> 4][k & 15] += (b == k) ? term : 0.0f;
        }
    };

    if (n_stages > 0) {
        issue(0, 0);
        fetch(0);
    }
    for (int st = 0; st < n_stages; ++st) {
        const int buf = st & 1;
        commit(buf);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this thread's share of the stage has landed
        __syncthreads();                                 // everyone's has, and the other buffer is free
        if (st + 1 < n_stages) {
            issue(st + 1, buf ^ 1);
            fetch(st + 1);
        }

        f16x8 bh[2][HU], bl[2][HU];
        float vl[2], th[2] = {0.0f, 0.0f};
        auto read_tile = [&](int tile, int slot) {
#pragma unroll
            for (int m = 0; m < HU; ++m) {
                bh[slot][m] = img[buf][tile][0][m][lane];
                bl[slot][m] = img[buf][tile][1][m][lane];
            }
            vl[slot] = vv[buf][tile * 32 + row];
            if constexpr (kRadial) th[slot] = tt[buf][tile * 32 + row];
        };
        read_tile(0, 0);
#pragma unroll
        for (int tile = 0; tile < kTilesPerStage; ++tile) {
            const int cur = tile & 1;
            if (tile + 1 < kTilesPerStage) read_tile(tile + 1, cur ^ 1);
            if (cur == 0) {
                block_tile<HU, KIND>(accA[0], fh[0], fhv[0], fl[0], bh[cur], bl[cur], accB[0], vl_prev, thr_prev, rc, sum[0], near);
                block_tile<HU, KIND>(accA[1], fh[1], fhv[1], fl[1], bh[cur], bl[cur], accB[1], vl_prev, thr_prev, rc, sum[1], near);
            } else {
                block_tile<HU, KIND>(accB[0], fh[0], fhv[0], fl[0], bh[cur], bl[cur], accA[0], vl_prev, thr_prev, rc, sum[0], near);
                block_tile<HU, KIND>(accB[1], fh[1], fhv[1], fl[1], bh[cur], bl[cur], accA[1], vl_prev, thr_prev, rc, sum[1], near);
            }
            if constexpr (kRadial) {
                if (near != 0) { // the finished tile (the set this tile's MFMAs do not write) had near pairs
                    if (cur == 0) refine(accB, thr_prev, vl_prev, j_prev);
                    else refine(accA, thr_prev, vl_prev, j_prev);
                    near = 0;
                }
                thr_prev = th[cur];
                j_prev = chunk_begin + (int64_t)st * kStage + tile * 32 + row;
            }
            vl_prev = vl[cur];
        }
    }
    // the last tile's accumulators (tiles per stage is even, so they are in set B); the wait states
    // an MFMA result needs before ordinary code may read it are explicit, because the compiler
    // does not know that the inline assembly above contains MFMAs
    static_assert(kTilesPerStage % 2 == 0, "accumulator sets alternate per tile");
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3" : "+v"(accB[0]), "+v"(accB[1]));
    bool any_near = false;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p;
            if constexpr (kRadial) {
                const bool nr = fabsf(accB[rb][r]) < thr_prev;
                any_near |= nr;
                p = nr ? 0.0f : radial_from_exponent<KIND>(accB[rb][r]);
            } else {
                p = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(accB[rb][r]), 0.0f, 1.0f);
            }
            sum[rb][r] = fmaf(p, vl_prev, sum[rb][r]);
        }
    if constexpr (kRadial) {
        if (__builtin_amdgcn_ballot_w64(any_near) != 0) refine(accB, thr_prev, vl_prev, j_prev);
    }

    // ---- reduce over the 32 stream lanes of each half-wave and store ----------------------
    float *out = a.out + chunk * a.chunk_stride;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float v = sum[rb][r];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 8);
            v += __shfl_xor(v, 4);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 1);
            const int64_t idx = fixed0 + rb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
            if (row == 0 && idx < a.nF) out[idx * a.ldo] = v;
        }
}

template <int NU, int KIND>
hipError_t launch_nu(const SweepArgs &a, void *pack_buf, size_t pack_bytes, hipStream_t stream)
{
    constexpr int HU = NU / 2;
    constexpr size_t bytes_per_point = 2 * HU * 2 * 16; // two planes, HU MFMAs, two half-waves, 16 B units / 32 rows * 32
    const int64_t per_block = (int64_t)kWaves * 64;
    const int64_t blocks = (a.nF + per_block - 1) / per_block;
    // slab = whole chunks whose packed image fits the workspace
    int64_t slab_chunks = (int64_t)(pack_bytes / bytes_per_point) / a.chunk_len;
    if (slab_chunks < 1) return hipErrorInvalidValue;
    const bool a16 = (a.d % 4 == 0) && (a.lds % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.S) & 15) == 0);
    const bool a8 = (a.d % 2 == 0) && (a.lds % 2 == 0) && ((reinterpret_cast<uintptr_t>(a.S) & 7) == 0);
    f16x8 *packed = static_cast<f16x8 *>(pack_buf);
    for (int64_t c0 = 0; c0 < a.n_chunks; c0 += slab_chunks) {
        const int64_t nc = (a.n_chunks - c0 < slab_chunks) ? a.n_chunks - c0 : slab_chunks;
        const int64_t row0 = c0 * a.chunk_len, rows = nc * a.chunk_len;
        const dim3 pgrid((unsigned)((rows + kThreads / 2 - 1) / (kThreads / 2)));
        if (a16)
            hipLaunchKernelGGL((pack_stream_kernel<NU, 4>), pgrid, dim3(kThreads), 0, stream, a.S, a.nS, a.lds, a.mu, a.d,
                               a.sigma, row0, rows, packed, a.range_count);
        else if (a8)
            hipLaunchKernelGGL((pack_stream_kernel<NU, 2>), pgrid, dim3(kThreads), 0, stream, a.S, a.nS, a.lds, a.mu, a.d,
                               a.sigma, row0, rows, packed, a.range_count);
        else
            hipLaunchKernelGGL((pack_stream_kernel<NU, 1>), pgrid, dim3(kThreads), 0, stream, a.S, a.nS, a.lds, a.mu, a.d,
                               a.sigma, row0, rows, packed, a.range_count);
        const int64_t wgs = blocks * nc;
        if (wgs > 0x7fffffff) return hipErrorInvalidValue;
        hipLaunchKernelGGL((gauss_sweep_f16_kernel<NU, KIND>), dim3((unsigned)wgs), dim3(kThreads), 0, stream, a, packed, c0,
                           (int)blocks, (int)nc);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

} // namespace

int f16_max_d() { return 44; } // 6 units of 8 features; larger images exceed 64 KB of static LDS
int64_t f16_stage_points(int d, int kind) { return stage_of(d <= 12 ? 2 : (d <= 28 ? 4 : 6), kind); }
int f16_radial_max_d() { return 28; } // the kernels of r need more registers per entry: 4 units

// bytes of packed image per stream point for this d
size_t f16_pack_bytes_per_point(int d) { return d <= 12 ? 64 : (d <= 28 ? 128 : 192); }

hipError_t launch_sweep_f16(const SweepArgs &a, void *pack_buf, size_t pack_bytes, hipStream_t stream)
{
    if (a.nF <= 0 || a.nS <= 0 || a.n_chunks <= 0 || a.t != 1 || a.d > f16_max_d()) return hipErrorInvalidValue;
    if (a.kind != KNM_KERNEL_GAUSSIAN && a.d > f16_radial_max_d()) return hipErrorInvalidValue;
    if (a.chunk_len % f16_stage_points(a.d, a.kind) != 0 || a.n_chunks * a.chunk_len < a.nS) return hipErrorInvalidValue;
    if (a.n_chunks > 65535) return hipErrorInvalidValue;
    if (a.kind < KNM_KERNEL_GAUSSIAN || a.kind > KNM_KERNEL_MATERN52) return hipErrorInvalidValue;
    // units of 8 features; the last unit keeps 4 slots for the norm digits
    auto launch = [&](auto kind) {
        constexpr int K = decltype(kind)::value;
        if (a.d <= 12) return launch_nu<2, K>(a, pack_buf, pack_bytes, stream);
        if (a.d <= 28) return launch_nu<4, K>(a, pack_buf, pack_bytes, stream);
        return launch_nu<6, K>(a, pack_buf, pack_bytes, stream);
    };
    switch (a.kind) {
    case KNM_KERNEL_LAPLACIAN: return launch(std::integral_constant<int, KNM_KERNEL_LAPLACIAN>{});
    case KNM_KERNEL_MATERN32: return launch(std::integral_constant<int, KNM_KERNEL_MATERN32>{});
    case KNM_KERNEL_MATERN52: return launch(std::integral_constant<int, KNM_KERNEL_MATERN52>{});
    default: return launch(std::integral_constant<int, KNM_KERNEL_GAUSSIAN>{});
    }
}

} // namespace knm
