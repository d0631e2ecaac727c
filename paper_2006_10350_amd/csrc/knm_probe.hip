// Sustained instruction rates of the device the library runs on, measured with register-resident
// loops: the matrix-core and vector-ALU instructions the tile engines are made of, alone and in
// the engines' own mix.  A measurement aid for the benchmark (it states the rooflines against what
// the chip sustains as well as against the nominal peaks); not part of the method.
#include <type_traits>
#include <vector>

#include "knm_internal.h"

namespace knm {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int kBlocks = 256 * 2; // two workgroups per compute unit = 2 wavefronts per SIMD, as the engines run

// 4 independent chains of v_mfma_f32_32x32x2_f32; 8 x 4 instructions per trip
__global__ __launch_bounds__(kThreads, 2) void probe_mfma_f32_kernel(float *out, int iters, float a0, float b0)
{
    f32x16 acc[4];
    for (int c = 0; c < 4; ++c)
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.0f;
    const float a = a0 + 1.0e-3f * threadIdx.x, b = b0;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.0f;
    for (int c = 0; c < 4; ++c)
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    out[blockIdx.x * kThreads + threadIdx.x] = s;
}

// 4 independent chains of v_mfma_f32_32x32x16_f16 on operands read from `in` (their bit patterns
// decide how much power the matrix cores draw); 6 x 4 instructions per trip
__global__ __launch_bounds__(kThreads, 2) void probe_mfma_f16_kernel(const f16x8 *in, float *out, int iters)
{
    f16x8 a[6], b[6];
    for (int i = 0; i < 6; ++i) {
        a[i] = in[(threadIdx.x * 16 + i) % 4096];
        b[i] = in[(threadIdx.x * 16 + i + 8) % 4096];
    }
    f32x16 acc[4];
    for (int c = 0; c < 4; ++c)
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.0f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int m = 0; m < 6; ++m)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[m], b[(m + c) % 6], acc[c], 0, 0, 0);
    }
    float s = 0.0f;
    for (int c = 0; c < 4; ++c)
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    out[blockIdx.x * kThreads + threadIdx.x] = s;
}

// 8 independent v_exp_f32 (WHAT = 0) or v_fmac_f32 (WHAT = 1) per trip and lane
template <int WHAT>
__global__ __launch_bounds__(kThreads, 2) void probe_valu_kernel(float *out, int iters, float x0)
{
    float x[8], p[8];
    for (int k = 0; k < 8; ++k) {
        x[k] = x0 - 1.0e-3f * (threadIdx.x + k);
        p[k] = 0.0f;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if constexpr (WHAT == 0) asm volatile("v_exp_f32_e64 %0, %1 clamp" : "=v"(p[k]) : "v"(x[k]));
            else asm volatile("v_fmac_f32_e32 %0, %1, %1" : "+v"(p[k]) : "v"(x[k]));
        }
    }
    float s = 0.0f;
    for (int k = 0; k < 8; ++k) s += p[k];
    out[blockIdx.x * kThreads + threadIdx.x] = s;
}

// The instruction mix of the split-fp16 register-resident engine on one pair of 32 x 32 tiles (one
// wavefront, two blocks of fixed points against one stream tile): per block 3 HU
// v_mfma_f32_32x32x16_f16 in one chain (HU = 1, 2, 3 for d <= 12, 28, 44) and 16 (v_exp_f32,
// v_fmac_f32) pairs spread behind them in groups, on registers that no MFMA writes.
// MODE 0: both, 1: vector ALU only, 2: matrix cores only.
template <int MODE, int HU>
__global__ __launch_bounds__(kThreads, 2) void probe_mix_kernel(const f16x8 *in, float *out, int iters)
{
    constexpr int NM = 3 * HU;
    f16x8 a[6], b[6];
    for (int i = 0; i < 6; ++i) {
        a[i] = in[(threadIdx.x * 16 + i) % 4096];
        b[i] = in[(threadIdx.x * 16 + i + 8) % 4096];
    }
    float x[6], p[6], s[6];
    for (int g = 0; g < 6; ++g) {
        x[g] = -0.5f * (g + 1) - threadIdx.x * 1e-3f;
        p[g] = 0.0f;
        s[g] = 0.0f;
    }
    const float w = 0.5f;
    f32x16 c[2];
    for (int r = 0; r < 16; ++r) {
        c[0][r] = 0.0f;
        c[1][r] = 0.0f;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                const int g_count = (16 * (i + 1)) / NM - (16 * i) / NM; // as the engine spreads them
                if constexpr (MODE != 1)
                    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(c[blk]) : "v"(a[i % 6]), "v"(b[(i + blk) % 6]));
                if constexpr (MODE != 2) {
#pragma unroll
                    for (int g = 0; g < g_count; ++g) asm volatile("v_exp_f32_e64 %0, %1 clamp" : "=v"(p[g]) : "v"(x[g]));
                    if (g_count == 1) asm volatile("s_nop 0"); // a transcendental result is not read by the next instruction
#pragma unroll
                    for (int g = 0; g < g_count; ++g) asm volatile("v_fmac_f32_e32 %0, %1, %2" : "+v"(s[g]) : "v"(p[g]), "v"(w));
                }
            }
        }
    }
    // the accumulators are read by ordinary code: give the last MFMA its wait states first
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3" : "+v"(c[0]), "+v"(c[1]));
    float t = 0.0f;
    for (int g = 0; g < 6; ++g) t += s[g];
    for (int r = 0; r < 16; ++r) t += c[0][r] + c[1][r];
    out[blockIdx.x * kThreads + threadIdx.x] = t;
}

struct Timer {
    hipStream_t stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok = true;
    explicit Timer(hipStream_t s) : stream(s)
    {
        ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
    }
    ~Timer()
    {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
    // milliseconds of the second of two identical launches (the first warms the clocks up)
    template <class F>
    double run(F launch)
    {
        launch();
        if (hipEventRecord(e0, stream) != hipSuccess) ok = false;
        launch();
        if (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) ok = false;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) ok = false;
        if (hipGetLastError() != hipSuccess) ok = false;
        return (double)ms;
    }
};

} // namespace
} // namespace knm

using namespace knm;

extern "C" int knm_probe_rates(knm_ctx *ctx, double *rates_host, int count)
{
    if (!ctx) return KNM_INVALID_ARG;
    if (!rates_host || count < KNM_PROBE_COUNT) return fail(ctx, KNM_INVALID_ARG, "probe output too short");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, KNM_HIP_ERROR, "hipSetDevice");
    float *out = nullptr;
    f16x8 *in = nullptr;
    if (hipMalloc(&out, sizeof(float) * kBlocks * kThreads) != hipSuccess || hipMalloc(&in, 4096 * sizeof(f16x8)) != hipSuccess) {
        (void)hipGetLastError();
        if (out) (void)hipFree(out);
        return fail(ctx, KNM_ALLOC, "hipMalloc(probe buffers)");
    }
    auto fill = [&](bool random) {
        std::vector<_Float16> h(4096 * 8);
        uint32_t state = 12345u;
        for (auto &v : h) {
            state = state * 1664525u + 1013904223u;
            v = (_Float16)(random ? ((float)(state >> 8) * (1.0f / 8388608.0f) - 1.0f) * 0.01f : 0.001f);
        }
        return hipMemcpy(in, h.data(), h.size() * sizeof(_Float16), hipMemcpyHostToDevice) == hipSuccess;
    };
    Timer tm(ctx->stream);
    bool ok = tm.ok;
    const double waves = (double)kBlocks * (kThreads / 64);
    {
        const int iters = 4000;
        const double ms = tm.run([&] { hipLaunchKernelGGL(probe_mfma_f32_kernel, dim3(kBlocks), dim3(kThreads), 0, ctx->stream, out, iters, 1.0f, 2.0f); });
        rates_host[KNM_PROBE_MFMA_F32_TFLOPS] = waves * iters * 32.0 * (32.0 * 32.0 * 2.0 * 2.0) / (ms * 1e-3) / 1e12;
    }
    for (int random = 0; random < 2; ++random) {
        ok = ok && fill(random != 0);
        const int iters = 20000;
        const double ms = tm.run([&] { hipLaunchKernelGGL(probe_mfma_f16_kernel, dim3(kBlocks), dim3(kThreads), 0, ctx->stream, in, out, iters); });
        rates_host[random ? KNM_PROBE_MFMA_F16_RANDOM_TFLOPS : KNM_PROBE_MFMA_F16_CONST_TFLOPS] =
            waves * iters * 24.0 * (32.0 * 32.0 * 16.0 * 2.0) / (ms * 1e-3) / 1e12;
    }
    {
        const int iters = 40000;
        const double lanes = (double)kBlocks * kThreads * iters * 8.0;
        const double ms_exp = tm.run([&] { hipLaunchKernelGGL(probe_valu_kernel<0>, dim3(kBlocks), dim3(kThreads), 0, ctx->stream, out, iters, -0.5f); });
        const double ms_fma = tm.run([&] { hipLaunchKernelGGL(probe_valu_kernel<1>, dim3(kBlocks), dim3(kThreads), 0, ctx->stream, out, iters, 0.5f); });
        rates_host[KNM_PROBE_EXP_TOPS] = lanes / (ms_exp * 1e-3) / 1e12;
        rates_host[KNM_PROBE_FMA_TOPS] = lanes / (ms_fma * 1e-3) / 1e12;
    }
    {
        // the engine's mix on random operands (the fill above): nominal 2.4 GHz clocks a SIMD needs per
        // tile pair (each SIMD runs two wavefronts, so a wavefront's trip takes twice this)
        const int iters = 20000;
        const double per = 2.4e9 * 1e-3 / iters / 2.0;
        auto mix = [&](auto hu, int base) {
            constexpr int HU = decltype(hu)::value;
            rates_host[base + 0] = per * tm.run([&] { hipLaunchKernelGGL((probe_mix_kernel<0, HU>), dim3(kBlocks), dim3(kThreads), 0, ctx->stream, in, out, iters); });
            rates_host[base + 1] = per * tm.run([&] { hipLaunchKernelGGL((probe_mix_kernel<1, HU>), dim3(kBlocks), dim3(kThreads), 0, ctx->stream, in, out, iters); });
            rates_host[base + 2] = per * tm.run([&] { hipLaunchKernelGGL((probe_mix_kernel<2, HU>), dim3(kBlocks), dim3(kThreads), 0, ctx->stream, in, out, iters); });
        };
        mix(std::integral_constant<int, 1>{}, KNM_PROBE_MIX1_BOTH_CLK);
        mix(std::integral_constant<int, 2>{}, KNM_PROBE_MIX2_BOTH_CLK);
        mix(std::integral_constant<int, 3>{}, KNM_PROBE_MIX3_BOTH_CLK);
    }
    ok = ok && tm.ok && hipStreamSynchronize(ctx->stream) == hipSuccess;
    (void)hipFree(out);
    (void)hipFree(in);
    return ok ? KNM_OK : fail(ctx, KNM_HIP_ERROR, "instruction-rate probe");
}
