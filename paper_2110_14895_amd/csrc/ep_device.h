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
// where P is a degree-4 polynomial fit of log2 Q on [0, 6] (log2 Q is smooth and nearly
// quadratic, so a short polynomial under one exp2 replaces the reciprocal, the exponential and
// the five-term rational of the textbook erfc formulas).  The result goes to bf16 (steps of
// 3.9e-3 relative), and the degree is matched to that: the absolute error of a * Q(a) in fp32
// arithmetic is below 6.5e-6 over the whole line and the relative error of gelu(u) below 3.5e-4
// for u > 0 (a * Q(a) < 6e-9 beyond the clamp).  9 instruction slots; every slot counts, the
// first MLP layer's epilogue is bound by the vector ALU (degree 6, 1.5e-7 absolute, cost 5 us
// more per launch at 16448 x 5120).
#define EP_GELU_LOG2Q_COEFFS                                                                           \
    {-1.0004799365997314f, -1.1473703384399414f, -0.46801844239234924f, -0.04407674819231033f,       \
     0.0038656943943351507f}
__device__ inline float gelu_erf(float u)
{
    constexpr float c[5] = EP_GELU_LOG2Q_COEFFS;
    // the NaN-propagating minimum (one v_minimum3_f32, the cost of v_min_f32): a NaN pre-activation
    // makes a, P(a) and the result NaN instead of vanishing in fminf / fmaxf
    const float a = __builtin_elementwise_minimum(fabsf(u), 6.0f);
    float p = fmaf(c[4], a, c[3]);
    p = fmaf(p, a, c[2]);
    p = fmaf(p, a, c[1]);
    p = fmaf(p, a, c[0]);
    return fmaf(-__builtin_amdgcn_exp2f(p), a, fmaxf(u, 0.0f));
}
