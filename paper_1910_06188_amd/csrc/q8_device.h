// Device-side helpers shared by the q8 HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace q8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// The rounding bracket of Eq. 1 on a binary32 value: nearest integer, ties away from zero.
// Adding 0.5 before truncating is wrong (it rounds 0.49999997 up to 1); adding the float just
// below 0.5, 0.5 - 2^-25, is right for every binary32 p: below a tie the sum stays below the
// next integer, at a tie it lands half-way between two floats whose even neighbour is that
// integer, and from 2^23 on p is an integer that the addend cannot move.  (Checked
// exhaustively against the trunc / compare-the-fraction definition on all 1.27e9 floats of
// [0, 2^24]; the form is odd in p.)
__device__ __forceinline__ float round_half_away(float p)
{
    return __builtin_truncf(__fadd_rn(p, __builtin_copysignf(0.49999997f, p)));
}

// Eq. 1 with M = 127: one separately rounded multiply, round, clamp, convert.  The
// float-to-int conversion truncates, which the rounding needs anyway; clamping the sum to
// +-127 first gives the same code (truncation is monotone and 127 is an integer) and keeps
// the conversion in range for any finite input.
__device__ __forceinline__ int quantize_code(float x, float scale)
{
    const float p = __fmul_rn(x, scale);
    const float r = __fadd_rn(p, __builtin_copysignf(0.49999997f, p));
    return (int)__builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
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
// Section 3).  Written through the upper tail Q(a) = 1 - Phi(a) = 0.5 erfc(a / sqrt 2) so that
// the negative side does not cancel:
//     GELU(v) = max(v, 0) - |v| Q(|v|).
// log2 Q is smooth on [0, 6] (from -1 down to -29.9) and is fitted there by a degree-6
// polynomial p.  An error dp of the exponent moves the GELU by a Q(a) ln2 dp, so the fit
// minimises the largest a Q(a) |p - log2 Q| instead of the largest |p - log2 Q| (gelu_fit.py
// beside the package regenerates the constants): GELU error <= 9e-8 absolute on the negative
// side and one rounding of the result on the positive side, a twentieth of the tolerance the
// tests allow; beyond 6 the term is below 6e-9 and |v| is clamped.  Nine VALU operations and
// one transcendental per element.
__device__ __forceinline__ float gelu_erf(float v)
{
    const float a = __builtin_fminf(__builtin_fabsf(v), 6.0f);
    float p = __builtin_fmaf(3.309277963e-05f, a, -7.692193612e-04f);
    p = __builtin_fmaf(p, a, 8.080715314e-03f);
    p = __builtin_fmaf(p, a, -5.341210216e-02f);
    p = __builtin_fmaf(p, a, -4.587709606e-01f);
    p = __builtin_fmaf(p, a, -1.151201725e+00f);
    p = __builtin_fmaf(p, a, -9.999930859e-01f);
    return __builtin_fmaf(-a, __builtin_amdgcn_exp2f(p), __builtin_fmaxf(v, 0.0f));  // one rounding, one operation less
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
