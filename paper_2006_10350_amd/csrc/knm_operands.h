// Device helpers shared by the tile engines: operand conversion for the split-fp16 cross term
// (scaling, hi/lo split, fixed-point norm digits), branch-free row loads, and the wait states an
// MFMA issued from inline assembly needs before ordinary code reads its result.
#pragma once

#include <hip/hip_runtime.h>

namespace knm {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __fp16 f16x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
// weights of the four fixed-point digits of a norm term: 2^10, 2^-1, 2^-12, 2^-23
constexpr float kC1 = 1024.0f, kC2 = 0.5f, kC3 = 0.000244140625f, kC4 = 1.1920928955078125e-07f;
constexpr float kHalfMax = 65000.0f;   // scaled features are clamped to +-this before the split
constexpr float kNormMax = 2097151.0f; // norm terms are clamped to this (four digits of 11 bits)

// hi = nearest half of z (clamped to the finite range first), lo = nearest half of the exact
// remainder z - hi; hi + lo carries 22-23 significant bits of z
__device__ __forceinline__ void split_half(float z, _Float16 &hi, _Float16 &lo)
{
    z = fminf(fmaxf(z, -kHalfMax), kHalfMax);
    hi = (_Float16)z;
    lo = (_Float16)(z - (float)hi);
}
// two features at once
__device__ __forceinline__ void split_pair(float z0, float z1, f16x2 &hi, f16x2 &lo)
{
    f32x2 z;
    z[0] = fminf(fmaxf(z0, -kHalfMax), kHalfMax);
    z[1] = fminf(fmaxf(z1, -kHalfMax), kHalfMax);
    hi = __builtin_convertvector(z, f16x2);
    f32x2 rem;
    rem[0] = z[0] - (float)hi[0];
    rem[1] = z[1] - (float)hi[1];
    lo = __builtin_convertvector(rem, f16x2);
}
// true if the conversion of z clamps it (also for a NaN)
__device__ __forceinline__ bool out_of_half_range(float z) { return !(fabsf(z) <= kHalfMax); }

// -n as four fixed-point digits, n = q1 2^10 + q2 2^-1 + q3 2^-12 + q4 2^-23 with integer
// q_i <= 2048 (exact in fp16); n >= 0, clamped to kNormMax
__device__ __forceinline__ void norm_digits(float n, _Float16 (&q)[4])
{
    n = fminf(n, kNormMax);
    const float q1 = floorf(n * (1.0f / 1024.0f));
    float r = fmaf(-q1, 1024.0f, n);
    const float q2 = floorf(r * 2.0f);
    r = fmaf(-q2, 0.5f, r);
    const float q3 = floorf(r * 4096.0f);
    r = fmaf(-q3, kC3, r);
    const float q4 = rintf(r * 8388608.0f);
    q[0] = (_Float16)(-q1); q[1] = (_Float16)(-q2); q[2] = (_Float16)(-q3); q[3] = (_Float16)(-q4);
}

// Branch-free row loads: virtual features [base, base + N) of `row` minus the common shift `mu`
// (skipped if !shifted), zero beyond d or for an invalid row.  Out-of-range features read element 0
// of the row and are zeroed by a select, so all loads issue back to back; `row` must point at a
// readable row.  VW = 4, 2: 16- and 8-byte loads (d, the leading dimension and the base address
// must be multiples of VW elements); VW = 1: scalar loads.
template <int N, int VW>
__device__ __forceinline__ void load_features(const float *__restrict__ row, const float *__restrict__ mu, bool shifted,
                                              int base, int d, bool valid, float (&x)[N])
{
    if constexpr (VW == 4) {
#pragma unroll
        for (int k = 0; k < N; k += 4) {
            const bool in = valid && (base + k < d);
            const f32x4 v = *reinterpret_cast<const f32x4 *>(row + (in ? base + k : 0));
            f32x4 m = {0.0f, 0.0f, 0.0f, 0.0f};
            if (shifted) m = *reinterpret_cast<const f32x4 *>(mu + (in ? base + k : 0));
            x[k] = in ? v[0] - m[0] : 0.0f; x[k + 1] = in ? v[1] - m[1] : 0.0f;
            x[k + 2] = in ? v[2] - m[2] : 0.0f; x[k + 3] = in ? v[3] - m[3] : 0.0f;
        }
    } else if constexpr (VW == 2) {
#pragma unroll
        for (int k = 0; k < N; k += 2) {
            const bool in = valid && (base + k < d);
            const f32x2 v = *reinterpret_cast<const f32x2 *>(row + (in ? base + k : 0));
            f32x2 m = {0.0f, 0.0f};
            if (shifted) m = *reinterpret_cast<const f32x2 *>(mu + (in ? base + k : 0));
            x[k] = in ? v[0] - m[0] : 0.0f; x[k + 1] = in ? v[1] - m[1] : 0.0f;
        }
    } else {
#pragma unroll
        for (int k = 0; k < N; ++k) {
            const bool in = valid && (base + k < d);
            const float v = row[in ? base + k : 0];
            x[k] = in ? v - (shifted ? mu[in ? base + k : 0] : 0.0f) : 0.0f;
        }
    }
}

// Wait states between the last 32 x 32 MFMA written in inline assembly and the first read of its
// result by other instructions (the compiler cannot insert them for instructions it does not see).
__device__ __forceinline__ void mfma_results_ready()
{
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3" ::: "memory");
}

// A pointer that is the same in every lane, as a value the compiler keeps in scalar registers (an "s"
// operand of inline assembly does not by itself move a value there).
template <typename T>
__device__ __forceinline__ const T *uniform_pointer(const T *p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const T *>(((uint64_t)hi << 32) | lo);
}

} // namespace knm
