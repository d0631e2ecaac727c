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

namespace knm {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kStage = 128; // stream points per LDS stage (2 threads per point)
constexpr int kTilesPerStage = kStage / 32;
constexpr float kLog2e = 1.4426950408889634f;

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

// Loads virtual features [base, base + N) of one point into registers (zero beyond d).
template <int N, int VW>
__device__ __forceinline__ void load_features(const float *__restrict__ row, int base, int d, bool valid,
                                              float (&x)[N])
{
#pragma unroll
    for (int k = 0; k < N; ++k) x[k] = 0.0f;
    if (!valid) return;
    if constexpr (VW == 4) {
#pragma unroll
        for (int k = 0; k < N; k += 4) {
            if (base + k < d) { // d % 4 == 0 in this mode
                f32x4 v = *reinterpret_cast<const f32x4 *>(row + base + k);
                x[k] = v[0]; x[k + 1] = v[1]; x[k + 2] = v[2]; x[k + 3] = v[3];
            }
        }
    } else if constexpr (VW == 2) {
#pragma unroll
        for (int k = 0; k < N; k += 2) {
            if (base + k < d) { // d % 2 == 0 in this mode
                f32x2 v = *reinterpret_cast<const f32x2 *>(row + base + k);
                x[k] = v[0]; x[k + 1] = v[1];
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < N; ++k)
            if (base + k < d) x[k] = row[base + k];
    }
}

template <int KS, int R, int VW>
__global__ __launch_bounds__(kThreads) void gauss_sweep_kernel(SweepArgs a)
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
            float v = (valid && k < d) ? p[k] : 0.0f;
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
        load_features<VPT, VW>(p, part * VPT, d, valid, xs);
        if (part == 0) {
            vs = valid ? a.vec[idx * a.ldv] : 0.0f;
            if (a.wgt != nullptr && valid) vs *= a.wgt[idx];
        }
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

#pragma unroll
        for (int tile = 0; tile < kTilesPerStage; ++tile) {
            const float *tb = &img[buf][tile * geo::TILE_FLOATS];
            float b[4 * G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                f32x4 u = *reinterpret_cast<const f32x4 *>(tb + (g * 64 + lane) * 4);
                b[4 * g] = u[0]; b[4 * g + 1] = u[1]; b[4 * g + 2] = u[2]; b[4 * g + 3] = u[3];
            }
            const float vl = vv[buf][tile * 32 + row];
            f32x16 acc[R];
#pragma unroll
            for (int rb = 0; rb < R; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rb][r] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int rb = 0; rb < R; ++rb)
                    acc[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[rb][s], b[s], acc[rb], 0, 0, 0);
#pragma unroll
            for (int rb = 0; rb < R; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    // exponent <= 0 up to rounding; med3 keeps the kernel value in [0, 1]
                    float p = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(acc[rb][r]), 0.0f, 1.0f);
                    sum[rb][r] = fmaf(p, vl, sum[rb][r]);
                }
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

__global__ void merge_kernel(const float *__restrict__ part, int64_t n_chunks, int64_t chunk_stride, int64_t ldp,
                             float *__restrict__ out, int64_t ldo, int64_t count)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= count) return;
    double s = 0.0;
    for (int64_t c = 0; c < n_chunks; ++c) s += (double)part[c * chunk_stride + j * ldp];
    out[j * ldo] = (float)s;
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

int max_d() { return 64; }
int64_t stage_points() { return kStage; }
int64_t fixed_per_block(int) { return (int64_t)kWaves * 32 * kR; }

hipError_t launch_sweep(const SweepArgs &a, hipStream_t stream)
{
    if (a.nF <= 0 || a.nS <= 0 || a.n_chunks <= 0) return hipErrorInvalidValue;
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

hipError_t launch_merge(const float *part, int64_t n_chunks, int64_t chunk_stride, int64_t ldp, float *out,
                        int64_t ldo, int64_t count, hipStream_t stream)
{
    const int threads = 256;
    const int64_t blocks = (count + threads - 1) / threads;
    hipLaunchKernelGGL(merge_kernel, dim3((unsigned)blocks), dim3(threads), 0, stream, part, n_chunks,
                       chunk_stride, ldp, out, ldo, count);
    return hipGetLastError();
}

} // namespace knm
