// Gaussian-kernel tile engine, K-loop variant: out[f, c] = sum_s k(F_f, S_s) vec[s, c]
// for any number of features d and up to 16 right-hand sides per launch.
//
// Used where the register-resident engine of knm_tile.hip does not apply: d too large
// to keep a block of points in registers (the image-like workload, d = 784), or several
// output columns sharing every kernel evaluation (multi-class targets).  Same
// formulation (Section 3.1, "Blockwise K_nm-vector product"; Gaussian kernel of
// Section 2): the cross term runs on fp32 MFMA with the contraction over d split into
// chunks of 16 features staged through LDS for BOTH operands, one augmented K-step adds
// the two norms, and exp plus the reduction against the vectors are fused behind it.
//
// Tile shape.  Workgroup = 4 wavefronts = 256 fixed points x 128 stream points per tile;
// each wavefront owns 64 fixed points (2 blocks of 32) x all 128 stream points (4 blocks)
// = 8 accumulators of 32x32.  Arithmetic intensity against L2 is
// 256*128 / (2*(256+128)) = 43 flop/B.
//
// Orientation.  The stream block is the MFMA A operand and the fixed block the B operand,
// so a lane's accumulator registers run over 16 stream points of ONE fixed point.  The
// reduction over stream points is then in-lane: t running sums per fixed block and lane,
// with the vector rows read from LDS as broadcasts.  The two half-waves hold different
// stream rows of the same fixed point and are added once, when the workgroup finishes.

#include <type_traits>

#include "knm_internal.h"
#include "knm_operands.h"

namespace knm {
namespace {


constexpr int kThreads = 256;
constexpr int kFixed = 256;            // fixed points per workgroup
constexpr int kStream = 128;           // stream points per tile
constexpr int kPts = kFixed + kStream; // points staged per K-chunk
constexpr int kBlocks = kPts / 32;     // 32-point blocks in LDS: 8 fixed then 4 stream
constexpr int kChunk = 16;             // features per K-chunk = 8 K-steps
constexpr int kLoads = kPts * (kChunk / 4) / kThreads; // float4 loads per thread and chunk (6)
constexpr int kBlockFloats = 2 * 64 * 4; // one block, one chunk: 2 units x 64 lanes x 4 K-steps

static_assert(kLoads * kThreads == kPts * (kChunk / 4), "staging must divide evenly");

// The eight 32x32 accumulators of a wavefront are pinned to the accumulation registers
// (AGPRs) through the asm constraint, which leaves the architectural VGPRs to staging,
// operands and running sums: 128 + <= 128 registers = two wavefronts per SIMD.
__device__ __forceinline__ void mfma_zero(f32x16 &acc, float a, float b)
{
    asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, 0" : "=&a"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_acc(f32x16 &acc, float a, float b)
{
    asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// exp2 of an accumulator element with the clamp modifier (Gaussian kernel value in [0, 1]).  Volatile
// and reading the accumulation register itself: the compiler does not look inside inline assembly,
// so it must neither move this read up towards the MFMA that produces the element nor be
// relied on for the wait state a transcendental result needs before its first use.
__device__ __forceinline__ float exp2_clamped(const float &x)
{
    float p;
    asm volatile("v_accvgpr_read_b32 %0, %1\n\tv_exp_f32_e64 %0, %0 clamp\n\ts_nop 0" : "=v"(p) : "a"(x));
    return p;
}
// the accumulator element itself, for code the compiler schedules (same ordering argument)
__device__ __forceinline__ float acc_read(const float &x)
{
    float p;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(p) : "a"(x));
    return p;
}

// TP: number of vector columns, padded to a multiple of 4.  VW: 4 if rows can be read
// with aligned 16-byte loads, else 1.
template <int TP, int VW, int KIND>
__global__ __launch_bounds__(kThreads, 2) void gauss_gemm_kernel(SweepArgs a)
{
    __shared__ __attribute__((aligned(16))) float img[2][kBlocks * kBlockFloats]; // 2 x 24 KB
    __shared__ float aug[kBlocks * 64];                                            // last K-step
    __shared__ __attribute__((aligned(16))) float vimg[kStream * TP];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int h = lane >> 5;
    const int t = a.t;
    const int d = a.d;
    const float s2 = kLog2e / (2.0f * a.sigma * a.sigma);
    const int n_kc = (d + kChunk - 1) / kChunk;
    const bool shifted = a.mu[d] != 0.0f; // same for every thread of the grid

    const int64_t fixed0 = (int64_t)blockIdx.x * kFixed;
    const int64_t chunk_begin = (int64_t)blockIdx.y * a.chunk_len;
    int64_t chunk_end = chunk_begin + a.chunk_len;
    if (chunk_end > a.nS) chunk_end = a.nS;
    const int n_tiles = (int)((chunk_end - chunk_begin + kStream - 1) / kStream);

    // staging role of this thread for load i: point (0..383) and feature quad (0..3)
    // id = tid + 256 i  ->  point = id / 4 = tid / 4 + 64 i,  quad = tid % 4
    const int sq = tid & 3;
    const int sp0 = tid >> 2;

    // Two levels of summation: the terms of one tile (64 per lane and fixed point) in fp32 from zero,
    // the tile sums into fp64 running sums, so that the rounding of a long sum of same-sign terms
    // does not grow with the chunk (with 16 columns the registers hold only the fp32 sums, which
    // then run through the chunk).
    constexpr bool kWide = TP <= 12;
    float sum[2][TP];
    double wide[2][kWide ? TP : 1];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int c = 0; c < TP; ++c) {
            sum[fb][c] = 0.0f;
            if constexpr (kWide) wide[fb][c] = 0.0;
        }

    for (int tile = 0; tile < n_tiles; ++tile) {
        const int64_t stream0 = chunk_begin + (int64_t)tile * kStream;

        // staged points of this thread (4 fixed, 2 stream): uniform base pointer of the
        // block plus a 32-bit element offset of the (clamped) row
        const float *const fbase = a.F + fixed0 * a.ldf;
        const float *const sbase = a.S + stream0 * a.lds;
        const int f_rows = (int)((a.nF - fixed0 < kFixed) ? a.nF - fixed0 : kFixed);
        const int s_rows = (int)((chunk_end - stream0 < kStream) ? chunk_end - stream0 : kStream);
        int roff[kLoads];
        bool valid[kLoads];
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            const int p = sp0 + 64 * i;
            if (i < kFixed / 64) {
                valid[i] = p < f_rows;
                roff[i] = (valid[i] ? p : 0) * (int)a.ldf;
            } else {
                valid[i] = (p - kFixed) < s_rows;
                roff[i] = (valid[i] ? p - kFixed : 0) * (int)a.lds;
            }
        }
        auto rowp = [&](int i) { return (i < kFixed / 64 ? fbase : sbase) + roff[i]; };

        f32x16 acc[2][4];
        float nrm[kLoads];
#pragma unroll
        for (int i = 0; i < kLoads; ++i) nrm[i] = 0.0f;

        f32x4 pre[kLoads];
        auto fetch = [&](int kc) {
            const int f0 = kc * kChunk + sq * 4;
            // the common shift of this thread's four features (the same for all its points)
            f32x4 m4 = {0.0f, 0.0f, 0.0f, 0.0f};
            if (shifted) {
#pragma unroll
                for (int e = 0; e < 4; ++e) m4[e] = a.mu[f0 + e < d ? f0 + e : 0];
            }
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
                if constexpr (VW == 4) {
                    const bool in = valid[i] && (f0 < d); // d % 4 == 0 in this mode
                    const f32x4 v = *reinterpret_cast<const f32x4 *>(rowp(i) + (in ? f0 : 0));
                    pre[i][0] = in ? v[0] - m4[0] : 0.0f; pre[i][1] = in ? v[1] - m4[1] : 0.0f;
                    pre[i][2] = in ? v[2] - m4[2] : 0.0f; pre[i][3] = in ? v[3] - m4[3] : 0.0f;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool in = valid[i] && (f0 + e < d);
                        const float v = rowp(i)[in ? f0 + e : 0];
                        pre[i][e] = in ? v - m4[e] : 0.0f;
                    }
                }
            }
        };
        // K-step s of a chunk takes feature 4 (s / 2) + 2 h + (s % 2) from half-wave h, so the
        // quad of features `sq` lands in unit sq / 2, entries 2 (sq % 2) + {0, 1}, for h = 0, 1.
        auto commit = [&](int buf) {
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
                const int p = sp0 + 64 * i;
                const float scale = (i < kFixed / 64) ? 2.0f * s2 : 1.0f;
                nrm[i] = fmaf(pre[i][0], pre[i][0], nrm[i]);
                nrm[i] = fmaf(pre[i][1], pre[i][1], nrm[i]);
                nrm[i] = fmaf(pre[i][2], pre[i][2], nrm[i]);
                nrm[i] = fmaf(pre[i][3], pre[i][3], nrm[i]);
                float *base = &img[buf][(p >> 5) * kBlockFloats + (sq >> 1) * 256 + (sq & 1) * 2];
                f32x2 lo, hi;
                lo[0] = scale * pre[i][0]; lo[1] = scale * pre[i][1];
                hi[0] = scale * pre[i][2]; hi[1] = scale * pre[i][3];
                *reinterpret_cast<f32x2 *>(base + (p & 31) * 4) = lo;        // half-wave 0
                *reinterpret_cast<f32x2 *>(base + (32 + (p & 31)) * 4) = hi; // half-wave 1
            }
        };

        fetch(0);
        for (int kc = 0; kc < n_kc; ++kc) {
            const int buf = kc & 1;
            commit(buf);
            __syncthreads();
            if (kc + 1 < n_kc) fetch(kc + 1);
            const float *ib = img[buf];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                f32x4 av[4], bv[2];
#pragma unroll
                for (int sb = 0; sb < 4; ++sb)
                    av[sb] = *reinterpret_cast<const f32x4 *>(ib + (kFixed / 32 + sb) * kBlockFloats + g * 256 + lane * 4);
#pragma unroll
                for (int fb = 0; fb < 2; ++fb)
                    bv[fb] = *reinterpret_cast<const f32x4 *>(ib + (wave * 2 + fb) * kBlockFloats + g * 256 + lane * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                        for (int sb = 0; sb < 4; ++sb) {
                            if (kc == 0 && g == 0 && e == 0) mfma_zero(acc[fb][sb], av[sb][e], bv[fb][e]);
                            else mfma_acc(acc[fb][sb], av[sb][e], bv[fb][e]);
                        }
            }
        }

        // augmented K-step: stream side [1, -s2 |x|^2], fixed side [-s2 |f|^2, 1]; plus the vectors
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            float v = nrm[i];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            if (sq == 0) {
                const int p = sp0 + 64 * i;
                const bool fixed = i < kFixed / 64;
                float *ab = &aug[(p >> 5) * 64 + (p & 31)];
                ab[0] = fixed ? -s2 * v : 1.0f;
                ab[32] = fixed ? 1.0f : -s2 * v;
            }
        }
        for (int k = tid; k < kStream * TP; k += kThreads) {
            const int j = k / TP, c = k % TP;
            const int64_t idx = stream0 + j;
            const bool in = idx < chunk_end && c < t;
            const int64_t vi = in ? idx : 0;
            float v = a.vec[vi * a.ldv + (in ? c : 0)];
            if (a.wgt != nullptr) v *= a.wgt[vi];
            vimg[k] = in ? v : 0.0f;
        }
        __syncthreads();
        {
            float av[4], bv[2];
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) av[sb] = aug[(kFixed / 32 + sb) * 64 + lane];
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) bv[fb] = aug[(wave * 2 + fb) * 64 + lane];
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                for (int sb = 0; sb < 4; ++sb)
                    mfma_acc(acc[fb][sb], av[sb], bv[fb]);
        }

        // finish: register r of a lane is stream row 8 (r / 4) + 4 h + r % 4 of its block
        mfma_results_ready();
        // Laplacian: per fixed point of this lane, the row and the |exponent| below which a pair is
        // taken again from differences (never for a padding row).  The unrolled pass leaves such
        // pairs out (kernel value 0) and only notes that there are some; the rare second pass
        // finds them again and adds their terms.
        const float *frow[2] = {nullptr, nullptr};
        float near[2] = {0.0f, 0.0f};
        bool any_near = false;
        if constexpr (KIND != KNM_KERNEL_GAUSSIAN) {
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) {
                const int64_t idx = fixed0 + (wave * 2 + fb) * 32 + (lane & 31);
                const bool in = idx < a.nF;
                frow[fb] = a.F + (in ? idx : 0) * a.ldf;
                near[fb] = in ? near_pair_threshold(aug[(wave * 2 + fb) * 64 + (lane & 31)], d) : -INFINITY;
            }
        }
        auto kernel_value = [&](int fb, int sb, int r) -> float {
            if constexpr (KIND != KNM_KERNEL_GAUSSIAN) {
                const float x = acc_read(acc[fb][sb][r]);
                const bool nr = x > -near[fb];
                any_near |= nr;
                return nr ? 0.0f : radial_from_exponent<KIND>(x);
            } else {
                // exponent <= 0 up to rounding; the clamp modifier keeps the kernel value in [0, 1]
                return exp2_clamped(acc[fb][sb][r]);
            }
        };
#pragma unroll
        for (int sb = 0; sb < 4; ++sb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = sb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                float vr[TP];
#pragma unroll
                for (int c4 = 0; c4 < TP; c4 += 4) {
                    const f32x4 u = *reinterpret_cast<const f32x4 *>(&vimg[j * TP + c4]);
                    vr[c4] = u[0]; vr[c4 + 1] = u[1]; vr[c4 + 2] = u[2]; vr[c4 + 3] = u[3];
                }
#pragma unroll
                for (int fb = 0; fb < 2; ++fb) {
                    const float p = kernel_value(fb, sb, r);
#pragma unroll
                    for (int c = 0; c < TP; ++c) sum[fb][c] = fmaf(p, vr[c], sum[fb][c]);
                }
            }
        if constexpr (KIND != KNM_KERNEL_GAUSSIAN) {
            if (__builtin_amdgcn_ballot_w64(any_near) != 0) {
#pragma unroll
                for (int fb = 0; fb < 2; ++fb) {
                    // bit 16 (sb % 2) + r of word sb / 2: register r of stream block sb is a near pair
                    uint32_t m[2] = {0u, 0u};
#pragma unroll
                    for (int sb = 0; sb < 4; ++sb)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (acc_read(acc[fb][sb][r]) > -near[fb]) m[sb >> 1] |= 1u << ((sb & 1) * 16 + r);
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        uint32_t mm = m[half];
                        while (mm != 0u) {
                            const int b = __builtin_ctz(mm);
                            mm &= mm - 1u;
                            const int sb = half * 2 + (b >> 4), r = b & 15;
                            const int jl = sb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                            const int64_t j = stream0 + jl;
                            if (j < chunk_end) { // a padding row has zero vectors
                                const float p = radial_from_exponent<KIND>(exact_exponent(frow[fb], a.S + j * a.lds, d, s2));
#pragma unroll
                                for (int c = 0; c < TP; ++c) sum[fb][c] = fmaf(p, vimg[jl * TP + c], sum[fb][c]);
                            }
                        }
                    }
                }
            }
        }
        if constexpr (kWide) {
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                for (int c = 0; c < TP; ++c) {
                    wide[fb][c] += (double)sum[fb][c];
                    sum[fb][c] = 0.0f;
                }
        }
        __syncthreads(); // aug / vimg / img are rewritten by the next tile
    }

    // the two half-waves hold different stream rows of the same fixed point
    // partials in fp64 if asked for (a uniform choice: one base address, two element sizes)
    const bool wide_out = a.out64 != nullptr;
    char *const obase = wide_out ? reinterpret_cast<char *>(a.out64 + (int64_t)blockIdx.y * a.chunk_stride)
                                 : reinterpret_cast<char *>(a.out + (int64_t)blockIdx.y * a.chunk_stride);
#pragma unroll
    for (int fb = 0; fb < 2; ++fb) {
        const int64_t idx = fixed0 + (wave * 2 + fb) * 32 + (lane & 31);
#pragma unroll
        for (int c = 0; c < TP; ++c) {
            double v;
            if constexpr (kWide) v = wide[fb][c];
            else v = (double)sum[fb][c];
            v += __shfl_xor(v, 32);
            if (h == 0 && idx < a.nF && c < t) {
                const int64_t at = idx * a.ldo + c;
                if (wide_out) *reinterpret_cast<double *>(obase + at * 8) = v;
                else *reinterpret_cast<float *>(obase + at * 4) = (float)v;
            }
        }
    }
}

template <int TP>
hipError_t launch_tp(const SweepArgs &a, hipStream_t stream)
{
    const int64_t blocks = (a.nF + kFixed - 1) / kFixed;
    dim3 grid((unsigned)blocks, (unsigned)a.n_chunks);
    const bool a16 = (a.d % 4 == 0) && (a.lds % 4 == 0) && (a.ldf % 4 == 0) &&
                     ((reinterpret_cast<uintptr_t>(a.S) & 15) == 0) && ((reinterpret_cast<uintptr_t>(a.F) & 15) == 0);
    auto launch = [&](auto kind) {
        constexpr int K = decltype(kind)::value;
        if (a16) hipLaunchKernelGGL((gauss_gemm_kernel<TP, 4, K>), grid, dim3(kThreads), 0, stream, a);
        else hipLaunchKernelGGL((gauss_gemm_kernel<TP, 1, K>), grid, dim3(kThreads), 0, stream, a);
    };
    switch (a.kind) {
    case KNM_KERNEL_LAPLACIAN: launch(std::integral_constant<int, KNM_KERNEL_LAPLACIAN>{}); break;
    case KNM_KERNEL_MATERN32: launch(std::integral_constant<int, KNM_KERNEL_MATERN32>{}); break;
    case KNM_KERNEL_MATERN52: launch(std::integral_constant<int, KNM_KERNEL_MATERN52>{}); break;
    default: launch(std::integral_constant<int, KNM_KERNEL_GAUSSIAN>{}); break;
    }
    return hipGetLastError();
}

} // namespace

int gemm_max_t() { return 16; }
// the stagers form row offsets within a block of 256 fixed + 128 stream points in 32 bits
bool gemm_leading_dimension_ok(int64_t ld) { return ld <= (int64_t)0x7fffffff / 384; }
int64_t gemm_stage_points() { return kStream; }
int64_t gemm_fixed_per_block() { return kFixed; }

hipError_t launch_sweep_gemm(const SweepArgs &a, hipStream_t stream)
{
    if (a.nF <= 0 || a.nS <= 0 || a.n_chunks <= 0 || a.t <= 0 || a.t > gemm_max_t()) return hipErrorInvalidValue;
    if (a.kind < KNM_KERNEL_GAUSSIAN || a.kind > KNM_KERNEL_MATERN52) return hipErrorInvalidValue;
    if (a.chunk_len % kStream != 0 || a.n_chunks * a.chunk_len < a.nS) return hipErrorInvalidValue;
    if (a.n_chunks > 65535) return hipErrorInvalidValue;
    if (!gemm_leading_dimension_ok(a.ldf) || !gemm_leading_dimension_ok(a.lds)) return hipErrorInvalidValue;
    if (a.t <= 4) return launch_tp<4>(a, stream);
    if (a.t <= 8) return launch_tp<8>(a, stream);
    if (a.t <= 12) return launch_tp<12>(a, stream);
    return launch_tp<16>(a, stream);
}

} // namespace knm
