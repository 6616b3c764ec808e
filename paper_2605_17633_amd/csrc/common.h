// Internal helpers shared by the HIP sources of libssam (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ssam.h"

typedef __bf16 bf16;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define SSAM_WAVE 64

// Workgroup barrier that orders LDS traffic only: unlike __syncthreads() it does not drain the
// global-memory counter, so prefetches of later K slabs stay in flight across it.
#define LDS_BARRIER()                                                         \
    do {                                                                      \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");       \
        __builtin_amdgcn_s_barrier();                                         \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");       \
    } while (0)

#define SSAM_CHECK_LAUNCH()                                   \
    do {                                                      \
        if (hipGetLastError() != hipSuccess) return SSAM_EHIP; \
    } while (0)

static inline bool ssam_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static inline int ssam_div_up(long a, long b) { return (int)((a + b - 1) / b); }

// Number of dense prefix tiles of the A-shape mask (Alg. 1): floor(r*T), with a
// 1e-6 guard against r*T falling just below an integer, clamped to [0, T].
static inline int ssam_prefix_tiles(int T, double r)
{
    long n = (long)__builtin_floor(r * (double)T + 1e-6);
    if (n < 0) n = 0;
    if (n > T) n = T;
    return (int)n;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

// 8 bf16 packed in a uint4 -> 8 floats
__device__ __forceinline__ void unpack_bf16x8(const uint4 &v, float *f)
{
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

// two floats -> two bf16 (round to nearest even) packed low|high
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v = { (__bf16)lo, (__bf16)hi };
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ uint4 pack_bf16x8(const float *f)
{
    return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]),
                      pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// erf GELU, 0.5 t (1 + erf(t / sqrt 2)).  erf by the rational approximation 7.1.26 of Abramowitz & Stegun,
// erf(x) = 1 - (a1 u + ... + a5 u^5) exp(-x^2), u = 1 / (1 + p x) for x >= 0, odd in x; absolute error below
// 1.5e-7, far under the bf16 rounding of the stored activation.  One reciprocal and one exp2 per element.
__device__ __forceinline__ float gelu_erf(float t)
{
    const float x = fabsf(t) * 0.70710678118654752440f;
    const float u = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float poly = fmaf(1.061405429f, u, -1.453152027f);
    poly = fmaf(poly, u, 1.421413741f);
    poly = fmaf(poly, u, -0.284496736f);
    poly = fmaf(poly, u, 0.254829592f);
    poly *= u;
    const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * x * x);
    const float erf_abs = fmaf(-poly, e, 1.0f);                 // erf(|t| / sqrt 2)
    const float erf_signed = copysignf(erf_abs, t);
    return 0.5f * t * (1.0f + erf_signed);
}
