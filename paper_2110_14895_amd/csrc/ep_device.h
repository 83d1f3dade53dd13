// Small device helpers shared by the bf16 kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float ep_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 ep_bf16x2 __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16 (lo in bits 0..15), round to nearest even: one v_cvt_pk_bf16_f32
__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    const ep_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, ep_bf16x2));
}

// GELU with the exact (erf) definition, gelu(u) = u/2 * (1 + erf(u / sqrt 2)), evaluated as
//   max(u, 0) - a * Q(a),   a = min(|u|, 6),   Q(a) = erfc(a / sqrt 2) / 2 = 2^P(a),
// where P is a degree-6 polynomial fit of log2 Q on [0, 6] (log2 Q is smooth and nearly
// quadratic, so a short polynomial under one exp2 replaces the reciprocal, the exponential and
// the five-term rational of the textbook erfc formulas).  The absolute error of a * Q(a) in fp32
// arithmetic is below 1.2e-7 over the whole line (a * Q(a) < 6e-9 beyond the clamp), far below
// bf16 resolution.  11 instruction slots.
#define EP_GELU_LOG2Q_COEFFS                                                                           \
    {-0.999993085861206f, -1.1512017250061035f, -0.4587709605693817f, -0.05341213569045067f,        \
     0.008080736733973026f, -0.0007692259387113154f, 3.309352905489504e-05f}
__device__ inline float gelu_erf(float u)
{
    constexpr float c[7] = EP_GELU_LOG2Q_COEFFS;
    const float a = fminf(fabsf(u), 6.0f);
    float p = fmaf(c[6], a, c[5]);
    p = fmaf(p, a, c[4]);
    p = fmaf(p, a, c[3]);
    p = fmaf(p, a, c[2]);
    p = fmaf(p, a, c[1]);
    p = fmaf(p, a, c[0]);
    return fmaf(-__builtin_amdgcn_exp2f(p), a, fmaxf(u, 0.0f));
}
