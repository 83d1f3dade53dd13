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
//   max(u, 0) - |u| * E(|u| / sqrt 2) / 2,   E(x) = 1 - erf(x) = t * P(t) * exp(-x^2),
//   t = 1 / (1 + p x)
// with the five-term polynomial of Abramowitz & Stegun 7.1.26 (|error of erf| < 1.5e-7, so the
// absolute error of gelu stays below 1e-7 * |u|, far below bf16 resolution).  The halving is
// folded into the coefficients and the 1 / sqrt 2 into p and into the exponent.
__device__ inline float gelu_erf(float u)
{
    const float au = fabsf(u);
    const float t = __builtin_amdgcn_rcpf(fmaf(au, 0.3275911f * 0.70710678118654752440f, 1.0f));
    const float ex = __builtin_amdgcn_exp2f(u * u * (-0.5f * 1.4426950408889634f));
    float q = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
    q = fmaf(q, t, 0.5f * 1.421413741f);
    q = fmaf(q, t, 0.5f * -0.284496736f);
    q = fmaf(q, t, 0.5f * 0.254829592f);
    const float h = q * t * ex;                      // E / 2
    return fmaf(-h, au, fmaxf(u, 0.0f));
}
