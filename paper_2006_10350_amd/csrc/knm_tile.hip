// Gaussian-kernel tile engine for gfx950 (CDNA4): out[f] = sum_s k(F_f, S_s) vec[s].
//
// Computes the blockwise, never-materialised kernel-matrix-vector products of
// Section 3.1 ("Blockwise K_nm-vector product"): the cross term of the squared distance
// is a dense contraction over the d features and runs on fp32 MFMA
// (v_mfma_f32_32x32x2_f32); the norms, the exponential and the reduction against the
// vector are fused behind it in registers, so no kernel block ever reaches memory.
//
// Formulation.  With s2 = log2(e) / (2 sigma^2),
//     log2 k(f, x) = 2 s2 <f, x> - s2 |f|^2 - s2 |x|^2 .
// Both operands are extended by one contraction step ("augmented step") carrying
//     fixed side : [ -s2 |f|^2 , 1 ]        stream side : [ 1 , -s2 |x|^2 ]
// and the fixed side's features are pre-multiplied by 2 s2, so the MFMA accumulator
// holds the base-2 exponent directly; one v_exp_f32 (clamped to [0, 1]) and one FMA
// against the stream-side vector finish an entry.
//
// Work decomposition.  A workgroup is 4 wavefronts.  Each wavefront keeps R blocks of
// 32 fixed points in registers as MFMA A operands for its whole life.  Stream points
// are staged cooperatively through LDS, 128 at a time (double buffered, one barrier
// per stage), already laid out as MFMA B operands, and every wavefront runs all its
// fixed blocks against each 32-point stream tile.  Per lane, the 16 accumulator
// registers of a 32x32 tile belong to 16 different fixed points and one stream point,
// so the running sums are per-lane and the only cross-lane reduction happens once,
// at the end of the chunk.
//
// Slot mapping.  A K-step s of the MFMA takes one value from each half-wave h:
// slot (s, h) holds "virtual feature" k = 4 (s / 2) + 2 h + (s % 2).  Virtual features
// 0..d-1 are the real ones, the rest are zero except the augmented step s = KS - 1.
// This makes a lane's slots pairs of adjacent features, which keeps the global loads
// and LDS accesses 8 or 16 bytes wide.

#include "knm_internal.h"
#include "knm_operands.h"

namespace knm {
namespace {


constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kStage = 128; // stream points per LDS stage (2 threads per point)
constexpr int kTilesPerStage = kStage / 32;

template <int KS>
struct Geo {
    static constexpr int KS2 = (KS + 1) / 2;      // slot pairs per half-wave
    static constexpr int G = (KS2 + 1) / 2;       // 16-byte units per lane per tile
    static constexpr int VPT = 4 * G;             // virtual features per staging thread
    static constexpr int SA = KS - 1;             // augmented step
    static constexpr int K0 = 4 * (SA / 2) + (SA % 2); // virtual feature of slot (SA, 0)
    static constexpr int K1 = K0 + 2;                  // virtual feature of slot (SA, 1)
    static constexpr int TILE_FLOATS = G * 64 * 4;
};

__host__ __device__ constexpr int ks_for_d(int d)
{
    // smallest KS whose augmented slots lie beyond the real features
    int ks = 2;
    while (4 * ((ks - 1) / 2) + ((ks - 1) % 2) < d) ++ks;
    return ks;
}

// The hot instructions are issued through volatile inline assembly: the compiler keeps
// volatile statements in program order, which is what the schedule below relies on.
//
// Measured on gfx950: fp32 MFMA and VALU instructions of one SIMD do not overlap in time,
// so the best order for a stream tile is simply one in which nothing waits:
//     chain(block 0), chain(block 1), finish(block 0), finish(block 1).
// An MFMA result may be read by the VALU only after the MFMA has retired (16 passes); the
// compiler cannot see into the assembly, so the order itself guarantees it: block 0's
// accumulator is read a whole 15-MFMA chain after its last MFMA, block 1's after the 32
// VALU instructions that finish block 0.  Each exp is separated from the FMA consuming it
// by three instructions (a transcendental result needs one idle issue slot).
// acc = sum_{s < KS} a[s] (x) b[s] as one dependent chain of 32x32x2 fp32 MFMAs, emitted in
// assembly blocks of up to four instructions (operand-count limit of an asm statement).
// `guard` is the accumulator of another block whose MFMA chain may still be in flight: naming it as
// an operand of every statement keeps the compiler from placing a copy or spill of it (a read the
// hardware does not interlock) between these statements.
template <int KS, int S0>
__device__ __forceinline__ void mfma_chain_from(f32x16 &acc, const float *a, const float *b, f32x16 &guard)
{
    constexpr int n = KS - S0 >= 4 ? 4 : KS - S0;
    if constexpr (n == 4)
        asm volatile("v_mfma_f32_32x32x2_f32 %[c], %[a0], %[b0], %[c]\n\t"
                     "v_mfma_f32_32x32x2_f32 %[c], %[a1], %[b1], %[c]\n\t"
                     "v_mfma_f32_32x32x2_f32 %[c], %[a2], %[b2], %[c]\n\t"
                     "v_mfma_f32_32x32x2_f32 %[c], %[a3], %[b3], %[c]"
                     : [c] "+v"(acc), "+v"(guard)
                     : [a0] "v"(a[S0]), [b0] "v"(b[S0]), [a1] "v"(a[S0 + 1]), [b1] "v"(b[S0 + 1]), [a2] "v"(a[S0 + 2]),
                       [b2] "v"(b[S0 + 2]), [a3] "v"(a[S0 + 3]), [b3] "v"(b[S0 + 3]));
    else if constexpr (n == 3)
        asm volatile("v_mfma_f32_32x32x2_f32 %[c], %[a0], %[b0], %[c]\n\t"
                     "v_mfma_f32_32x32x2_f32 %[c], %[a1], %[b1], %[c]\n\t"
                     "v_mfma_f32_32x32x2_f32 %[c], %[a2], %[b2], %[c]"
                     : [c] "+v"(acc), "+v"(guard)
                     : [a0] "v"(a[S0]), [b0] "v"(b[S0]), [a1] "v"(a[S0 + 1]), [b1] "v"(b[S0 + 1]), [a2] "v"(a[S0 + 2]),
                       [b2] "v"(b[S0 + 2]));
    else if constexpr (n == 2)
        asm volatile("v_mfma_f32_32x32x2_f32 %[c], %[a0], %[b0], %[c]\n\t"
                     "v_mfma_f32_32x32x2_f32 %[c], %[a1], %[b1], %[c]"
                     : [c] "+v"(acc), "+v"(guard)
                     : [a0] "v"(a[S0]), [b0] "v"(b[S0]), [a1] "v"(a[S0 + 1]), [b1] "v"(b[S0 + 1]));
    else if constexpr (n == 1)
        asm volatile("v_mfma_f32_32x32x2_f32 %[c], %[a0], %[b0], %[c]" : [c] "+v"(acc), "+v"(guard) : [a0] "v"(a[S0]), [b0] "v"(b[S0]));
    if constexpr (S0 + n < KS) mfma_chain_from<KS, S0 + n>(acc, a, b, guard);
}
template <int KS>
__device__ __forceinline__ void mfma_chain(f32x16 &acc, const float *a, const float *b, f32x16 &guard)
{
    // first instruction takes the literal 0 as its C operand
    asm volatile("v_mfma_f32_32x32x2_f32 %0, %2, %3, 0" : "=&v"(acc), "+v"(guard) : "v"(a[0]), "v"(b[0]));
    if constexpr (KS > 1) mfma_chain_from<KS, 1>(acc, a, b, guard);
}
// s_i += min(max(2^x_i, 0), 1) * vl for four entries; the clamp keeps kernel values in [0, 1]
// (`guard`: see mfma_chain_from)
__device__ __forceinline__ void exp_fma4(float x0, float x1, float x2, float x3, float vl, float &s0, float &s1,
                                         float &s2, float &s3, f32x16 &guard)
{
    float p0, p1, p2, p3;
    asm volatile("v_exp_f32_e64 %[p0], %[x0] clamp\n\t"
                 "v_exp_f32_e64 %[p1], %[x1] clamp\n\t"
                 "v_exp_f32_e64 %[p2], %[x2] clamp\n\t"
                 "v_exp_f32_e64 %[p3], %[x3] clamp\n\t"
                 "v_fmac_f32_e32 %[s0], %[p0], %[vl]\n\t"
                 "v_fmac_f32_e32 %[s1], %[p1], %[vl]\n\t"
                 "v_fmac_f32_e32 %[s2], %[p2], %[vl]\n\t"
                 "v_fmac_f32_e32 %[s3], %[p3], %[vl]"
                 : [p0] "=&v"(p0), [p1] "=&v"(p1), [p2] "=&v"(p2), [p3] "=&v"(p3), [s0] "+v"(s0), [s1] "+v"(s1),
                   [s2] "+v"(s2), [s3] "+v"(s3), "+v"(guard)
                 : [x0] "v"(x0), [x1] "v"(x1), [x2] "v"(x2), [x3] "v"(x3), [vl] "v"(vl));
}

template <int KS, int R, int VW>
__global__ __launch_bounds__(kThreads, (KS <= 15 ? 3 : 1)) void gauss_sweep_kernel(SweepArgs a)
{
    using geo = Geo<KS>;
    constexpr int G = geo::G;
    constexpr int VPT = geo::VPT;

    __shared__ __attribute__((aligned(16))) float img[2][kTilesPerStage * geo::TILE_FLOATS];
    __shared__ float vv[2][kStage];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row = lane & 31;
    const int h = lane >> 5;
    const float s2 = kLog2e / (2.0f * a.sigma * a.sigma);
    const int d = a.d;
    const bool shifted = a.mu[d] != 0.0f; // same for every thread of the grid

    // ---- fixed operand: R blocks of 32 points per wavefront, in registers -------------
    const int64_t fixed0 = ((int64_t)blockIdx.x * kWaves + wave) * (32 * R);
    float af[R][KS];
#pragma unroll
    for (int rb = 0; rb < R; ++rb) {
        const int64_t idx = fixed0 + rb * 32 + row;
        const bool valid = idx < a.nF;
        const float *p = a.F + (valid ? idx : 0) * a.ldf;
        float nrm = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int k = 4 * (s / 2) + 2 * h + (s % 2);
            float v = (valid && k < d) ? p[k] - a.mu[k < d ? k : 0] : 0.0f;
            nrm = fmaf(v, v, nrm);
            af[rb][s] = 2.0f * s2 * v;
        }
        nrm += __shfl_xor(nrm, 32);
        af[rb][geo::SA] = valid ? (h == 0 ? -s2 * nrm : 1.0f) : 0.0f;
    }

    float sum[R][16];
#pragma unroll
    for (int rb = 0; rb < R; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[rb][r] = 0.0f;

    // ---- stream staging: thread (p, part) owns half of one point per stage --------------
    const int sp = tid >> 1;   // point within the stage
    const int part = tid & 1;  // which half of the virtual features
    const int64_t chunk_begin = (int64_t)blockIdx.y * a.chunk_len;
    int64_t chunk_end = chunk_begin + a.chunk_len;
    if (chunk_end > a.nS) chunk_end = a.nS;
    const int n_stages = (int)((chunk_end - chunk_begin + kStage - 1) / kStage);

    float xs[VPT];
    float vs = 0.0f;
    auto fetch = [&](int stage) {
        const int64_t idx = chunk_begin + (int64_t)stage * kStage + sp;
        const bool valid = idx < chunk_end;
        const float *p = a.S + (valid ? idx : 0) * a.lds;
        load_features<VPT, VW>(p, a.mu, shifted, part * VPT, d, valid, xs);
        const int64_t vi = valid ? idx : 0;
        const float vraw = a.vec[vi * a.ldv];
        const float wraw = (a.wgt != nullptr) ? a.wgt[vi] : 1.0f;
        vs = valid ? vraw * wraw : 0.0f;
    };
    auto commit = [&](int buf) {
        float nrm = 0.0f;
#pragma unroll
        for (int k = 0; k < VPT; ++k) nrm = fmaf(xs[k], xs[k], nrm);
        nrm += __shfl_xor(nrm, 1);
        if (geo::K0 / VPT == 0) { if (part == 0) xs[geo::K0 % VPT] = 1.0f; }
        else                    { if (part == 1) xs[geo::K0 % VPT] = 1.0f; }
        if (geo::K1 / VPT == 0) { if (part == 0) xs[geo::K1 % VPT] = -s2 * nrm; }
        else                    { if (part == 1) xs[geo::K1 % VPT] = -s2 * nrm; }
        const int tile = sp >> 5;
        const int prow = sp & 31;
        float *base = &img[buf][tile * geo::TILE_FLOATS];
#pragma unroll
        for (int q = 0; q < 2 * G; ++q) {
            const int hh = q & 1;                 // pair index part*2G + q; 2G is even
            const int j = part * G + (q >> 1);
            const int g = j >> 1;
            const int e0 = (j & 1) * 2;
            f32x2 v;
            v[0] = xs[2 * q];
            v[1] = xs[2 * q + 1];
            *reinterpret_cast<f32x2 *>(base + ((g * 64 + hh * 32 + prow) * 4 + e0)) = v;
        }
        if (part == 0) vv[buf][sp] = vs;
    };

    if (n_stages > 0) fetch(0);
    for (int st = 0; st < n_stages; ++st) {
        const int buf = st & 1;
        commit(buf);
        __syncthreads();
        if (st + 1 < n_stages) fetch(st + 1);

        // B operands are read one tile ahead so the LDS latency hides under the MFMA chains
        float b[2][4 * G];
        float vl[2];
        auto read_tile = [&](int tile, int slot) {
            const float *tb = &img[buf][tile * geo::TILE_FLOATS];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                f32x4 u = *reinterpret_cast<const f32x4 *>(tb + (g * 64 + lane) * 4);
                b[slot][4 * g] = u[0]; b[slot][4 * g + 1] = u[1]; b[slot][4 * g + 2] = u[2]; b[slot][4 * g + 3] = u[3];
            }
            vl[slot] = vv[buf][tile * 32 + row];
        };
        read_tile(0, 0);
#pragma unroll
        for (int tile = 0; tile < kTilesPerStage; ++tile) {
            const int cur = tile & 1;
            if (tile + 1 < kTilesPerStage) read_tile(tile + 1, cur ^ 1);
            // chain(0), chain(1), finish(0), finish(1): every statement that runs while the other
            // block's chain may be in flight names that block's accumulator as its guard
            static_assert(R == 2, "the order of chains and finishes below is written for two blocks");
            f32x16 acc[R];
            mfma_chain<KS>(acc[0], af[0], b[cur], acc[1]); // acc[1]: not yet written, a harmless guard
            mfma_chain<KS>(acc[1], af[1], b[cur], acc[0]);
#pragma unroll
            for (int rb = 0; rb < R; ++rb)
#pragma unroll
                for (int r = 0; r < 16; r += 4)
                    exp_fma4(acc[rb][r], acc[rb][r + 1], acc[rb][r + 2], acc[rb][r + 3], vl[cur], sum[rb][r],
                             sum[rb][r + 1], sum[rb][r + 2], sum[rb][r + 3], acc[rb ^ 1]);
        }
    }
    // ---- reduce over the 32 stream lanes of each half-wave and store ----------------------
    float *out = a.out + (int64_t)blockIdx.y * a.chunk_stride;
#pragma unroll
    for (int rb = 0; rb < R; ++rb)
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

template <typename TI, typename TO>
__global__ void merge_kernel(const TI *__restrict__ part, int64_t n_chunks, int64_t chunk_stride, int64_t ldp,
                             TO *__restrict__ out, int64_t ldo, int64_t count)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= count) return;
    double s = 0.0;
    for (int64_t c = 0; c < n_chunks; ++c) s += (double)part[c * chunk_stride + j * ldp];
    out[j * ldo] = (TO)s;
}

constexpr int kR = 2;

template <int KS>
hipError_t launch_ks(const SweepArgs &a, hipStream_t stream)
{
    const int64_t per_block = (int64_t)kWaves * 32 * kR;
    const int64_t blocks = (a.nF + per_block - 1) / per_block;
    dim3 grid((unsigned)blocks, (unsigned)a.n_chunks);
    const bool a16 = (a.d % 4 == 0) && (a.lds % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.S) & 15) == 0);
    const bool a8 = (a.d % 2 == 0) && (a.lds % 2 == 0) && ((reinterpret_cast<uintptr_t>(a.S) & 7) == 0);
    if (a16)
        hipLaunchKernelGGL((gauss_sweep_kernel<KS, kR, 4>), grid, dim3(kThreads), 0, stream, a);
    else if (a8)
        hipLaunchKernelGGL((gauss_sweep_kernel<KS, kR, 2>), grid, dim3(kThreads), 0, stream, a);
    else
        hipLaunchKernelGGL((gauss_sweep_kernel<KS, kR, 1>), grid, dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

} // namespace

int small_max_d() { return 64; }
int64_t stage_points() { return kStage; }
int64_t fixed_per_block(int) { return (int64_t)kWaves * 32 * kR; }

hipError_t launch_sweep(const SweepArgs &a, hipStream_t stream)
{
    if (a.nF <= 0 || a.nS <= 0 || a.n_chunks <= 0 || a.t != 1 || a.d > small_max_d()) return hipErrorInvalidValue;
    if (a.chunk_len % kStage != 0 || a.n_chunks * a.chunk_len < a.nS) return hipErrorInvalidValue;
    if (a.n_chunks > 65535) return hipErrorInvalidValue;
    const int ks = ks_for_d(a.d);
    // compiled step counts; a larger KS than needed only adds zero-padded steps
    if (ks <= 3) return launch_ks<3>(a, stream);
    if (ks <= 5) return launch_ks<5>(a, stream);
    if (ks <= 7) return launch_ks<7>(a, stream);
    if (ks <= 9) return launch_ks<9>(a, stream);
    if (ks <= 11) return launch_ks<11>(a, stream);
    if (ks <= 15) return launch_ks<15>(a, stream);
    if (ks <= 19) return launch_ks<19>(a, stream);
    if (ks <= 25) return launch_ks<25>(a, stream);
    if (ks <= 33) return launch_ks<33>(a, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_merge(const float *part, const double *part64, int64_t n_chunks, int64_t chunk_stride, int64_t ldp,
                        float *out, double *out64, int64_t ldo, int64_t count, hipStream_t stream)
{
    if ((part == nullptr) == (part64 == nullptr) || (out == nullptr) == (out64 == nullptr)) return hipErrorInvalidValue;
    const dim3 threads(256), blocks((unsigned)((count + 255) / 256));
    if (part64 != nullptr && out64 != nullptr)
        hipLaunchKernelGGL((merge_kernel<double, double>), blocks, threads, 0, stream, part64, n_chunks, chunk_stride, ldp, out64, ldo, count);
    else if (part64 != nullptr)
        hipLaunchKernelGGL((merge_kernel<double, float>), blocks, threads, 0, stream, part64, n_chunks, chunk_stride, ldp, out, ldo, count);
    else if (out64 != nullptr)
        hipLaunchKernelGGL((merge_kernel<float, double>), blocks, threads, 0, stream, part, n_chunks, chunk_stride, ldp, out64, ldo, count);
    else
        hipLaunchKernelGGL((merge_kernel<float, float>), blocks, threads, 0, stream, part, n_chunks, chunk_stride, ldp, out, ldo, count);
    return hipGetLastError();
}

} // namespace knm
