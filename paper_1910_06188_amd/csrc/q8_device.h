// Device-side helpers shared by the q8 HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace q8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// The rounding bracket of Eq. 1 on a binary32 value: nearest integer, ties away
// from zero.  p - trunc(p) is exact, so the comparison with 0.5 is exact too
// (adding 0.5 before truncating is not: it rounds 0.49999997 up to 1).
__device__ __forceinline__ float round_half_away(float p)
{
    float t = __builtin_truncf(p);
    float d = p - t;
    float one = __builtin_copysignf(1.0f, p);
    return (__builtin_fabsf(d) >= 0.5f) ? t + one : t;
}

// Eq. 1 with M = 127: one separately rounded multiply, round, clamp, convert.
__device__ __forceinline__ int quantize_code(float x, float scale)
{
    float p = __fmul_rn(x, scale);
    float r = round_half_away(p);
    r = __builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

// Eq. 3 with M = 127; an all-zero tensor takes S = 1 so that every code is 0.
__device__ __forceinline__ float scale_from_amax(float amax)
{
    return (amax == 0.0f) ? 1.0f : __fdiv_rn(127.0f, amax);
}

// Int32 bias of Section 3: round(b * (S_x * S_W)), clamped to +-(2^31 - 1)
// (Eq. 2 with b = 32).  Floats at or beyond 2^31 saturate before the conversion.
__device__ __forceinline__ int quantize_bias(float b, float sx, float sw)
{
    float sb = __fmul_rn(sx, sw);
    float r = round_half_away(__fmul_rn(b, sb));
    if (r >= 2147483648.0f) return 2147483647;
    if (r <= -2147483648.0f) return -2147483647;
    return (int)r;
}

// Reciprocal of S_x * S_W, formed in binary64 and rounded once, so that
// float(acc) * r stays within ~1.5 ulp of acc / (S_x * S_W).
__device__ __forceinline__ float dequant_factor(float sx, float sw)
{
    return (float)(1.0 / ((double)sx * (double)sw));
}

// GELU(v) = v * Phi(v), Phi the standard normal CDF (exact-erf GELU, kept in fp32:
// Section 3).  Written through erfc so that the negative tail does not cancel: with
// g = 0.5 |v| erfc(|v|/sqrt 2) >= 0,
//   v <  0 : GELU = -g          v >= 0 : GELU = v - g          i.e. GELU = max(v, 0) - g.
// erfc(z) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-z^2), t = 1/(1 + p z), is the
// classical 5-term rational fit (Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7, about one
// fp32 ulp of 1.0).  The factors 0.5, 1/sqrt 2 and log2 e are folded into the constants:
// 13 VALU operations and two transcendentals per element.  In the fused GEMM epilogue this
// arithmetic, not the store, is what the GELU variants wait for.
__device__ __forceinline__ float gelu_erf(float v)
{
    const float a = __builtin_fabsf(v);
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f * 0.70710678118654752440f, a, 1.0f));
    const float e = __builtin_amdgcn_exp2f((v * v) * (-0.5f * 1.44269504088896340736f));
    float p = __builtin_fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
    p = __builtin_fmaf(p, t, 0.5f * 1.421413741f);
    p = __builtin_fmaf(p, t, 0.5f * -0.284496736f);
    p = __builtin_fmaf(p, t, 0.5f * 0.254829592f);
    const float g = a * ((p * t) * e);
    return __builtin_fmaxf(v, 0.0f) - g;
}

__device__ __forceinline__ unsigned wave_max_u32(unsigned v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        unsigned o = (unsigned)__shfl_xor((int)v, off, 64);
        v = v > o ? v : o;
    }
    return v;
}

}  // namespace q8
