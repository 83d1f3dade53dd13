// HBM-bound row kernels of the bf16 path: LayerNorm over the fp32 residual
// stream producing the bf16 GEMM operand (paper section 2.1: the two layer
// normalisations of a layer), and dtype conversion at the stage boundary.
//
// LayerNorm: one wavefront per row, the whole row held in registers (float4
// loads, D <= 64*4*MAXV), mean then centred variance (two passes over
// registers, one pass over memory), fp32 statistics, round-to-nearest-even
// narrowing.  Algorithmic traffic per row: 4*D bytes read, 2*D written.
#include "ep_kernels.h"
#include "ep_device.h"

namespace {

constexpr int WAVE = 64;

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}

// What a dense layer whose K was cut into ranges left to do: ((part[0] + ... + part[splits-1]) + bias) + resid,
// the ranges in index order (the same association as the epilogue of the uncut layer: sum, bias, residual).
// The number of ranges is a template argument (2, 4 or 8) so that all loads of a lane are in flight together:
// these kernels run on a few hundred rows, where latency is all there is.
template <int S>
__device__ inline float4 ranges_bias_resid(const float4 *part, size_t range_stride4, float4 bias, float4 resid)
{
    float4 p[S];
#pragma unroll
    for (int r = 0; r < S; ++r) p[r] = part[(size_t)r * range_stride4];
    float4 a = p[0];
#pragma unroll
    for (int r = 1; r < S; ++r) { a.x += p[r].x; a.y += p[r].y; a.z += p[r].z; a.w += p[r].w; }
    a.x += bias.x; a.y += bias.y; a.z += bias.z; a.w += bias.w;
    return make_float4(a.x + resid.x, a.y + resid.y, a.z + resid.z, a.w + resid.w);
}

// NV = number of float4 per lane (D = 256 * NV exactly, or ragged when GUARD).  SUM > 0: x is first brought up to
// date in place from the SUM K ranges of the dense layer before it (part [SUM, rows, D], bias), then normalised.
template <int NV, bool GUARD, int SUM>
__global__ __launch_bounds__(256) void ln_bf16_kernel(float *__restrict__ x, const float *__restrict__ part,
                                                      const float *__restrict__ bias,
                                                      const float *__restrict__ g,
                                                      const float *__restrict__ b, float eps,
                                                      uint16_t *__restrict__ y, int64_t rows, int D)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x / WAVE) + (threadIdx.x / WAVE);
    if (row >= rows) return;
    float4 *xr = reinterpret_cast<float4 *>(x + row * D);
    const int nvec = D >> 2;
    float4 v[NV];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + i * WAVE;
        if (!GUARD || c < nvec) {
            v[i] = xr[c];
            if (SUM > 0) {
                v[i] = ranges_bias_resid<SUM ? SUM : 1>(reinterpret_cast<const float4 *>(part + row * D) + c,
                                                       (size_t)rows * D / 4, reinterpret_cast<const float4 *>(bias)[c], v[i]);
                xr[c] = v[i];
            }
            s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
        } else {
            v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    const float mean = wave_sum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + i * WAVE;
        if (!GUARD || c < nvec) {
            v[i].x -= mean; v[i].y -= mean; v[i].z -= mean; v[i].w -= mean;
            q += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
        }
    }
    const float inv = 1.0f / sqrtf(wave_sum(q) / (float)D + eps);
    const float4 *g4 = reinterpret_cast<const float4 *>(g);
    const float4 *b4 = reinterpret_cast<const float4 *>(b);
    uint2 *yr = reinterpret_cast<uint2 *>(y + row * D);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + i * WAVE;
        if (!GUARD || c < nvec) {
            const float4 gg = g4[c], bb = b4[c];
            uint2 o;
            o.x = pack_bf16x2(v[i].x * inv * gg.x + bb.x, v[i].y * inv * gg.y + bb.y);
            o.y = pack_bf16x2(v[i].z * inv * gg.z + bb.z, v[i].w * inv * gg.w + bb.w);
            yr[c] = o;
        }
    }
}

template <int S>
__global__ __launch_bounds__(256) void residual_sum_kernel(const float *resid, const float *__restrict__ part,
                                                           const float *__restrict__ bias, float *out,
                                                           int64_t n4, int d4)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    reinterpret_cast<float4 *>(out)[i] =
        ranges_bias_resid<S>(reinterpret_cast<const float4 *>(part) + i, (size_t)n4,
                             reinterpret_cast<const float4 *>(bias)[i % d4], reinterpret_cast<const float4 *>(resid)[i]);
}

__global__ __launch_bounds__(256) void bf16_to_f32_kernel(const uint16_t *__restrict__ in,
                                                          float *__restrict__ out, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    const uint2 p = reinterpret_cast<const uint2 *>(in)[i];
    float4 o;
    o.x = __uint_as_float(p.x << 16);
    o.y = __uint_as_float(p.x & 0xFFFF0000u);
    o.z = __uint_as_float(p.y << 16);
    o.w = __uint_as_float(p.y & 0xFFFF0000u);
    reinterpret_cast<float4 *>(out)[i] = o;
}

__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float *__restrict__ in,
                                                          uint16_t *__restrict__ out, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    const float4 v = reinterpret_cast<const float4 *>(in)[i];
    uint2 o;
    o.x = pack_bf16x2(v.x, v.y);
    o.y = pack_bf16x2(v.z, v.w);
    reinterpret_cast<uint2 *>(out)[i] = o;
}

// part == nullptr: plain LayerNorm of x (which is then only read)
template <int NV>
hipError_t launch_ln(float *x, const float *part, int splits, const float *bias, const float *g, const float *b,
                     float eps, uint16_t *y, int64_t rows, int D, hipStream_t s)
{
    const unsigned grid = (unsigned)((rows + 3) / 4);
    const bool ragged = D != NV * 256;
#define EP_LN_LAUNCH(GUARD, SUM) \
    hipLaunchKernelGGL((ln_bf16_kernel<NV, GUARD, SUM>), dim3(grid), dim3(256), 0, s, x, part, bias, g, b, eps, y, rows, D)
#define EP_LN_LAUNCH_SUM(SUM) do { if (ragged) EP_LN_LAUNCH(true, SUM); else EP_LN_LAUNCH(false, SUM); } while (0)
    switch (part ? splits : 0) {
    case 0: EP_LN_LAUNCH_SUM(0); break;
    case 2: EP_LN_LAUNCH_SUM(2); break;
    case 4: EP_LN_LAUNCH_SUM(4); break;
    case 8: EP_LN_LAUNCH_SUM(8); break;
    default: return hipErrorInvalidValue;
    }
#undef EP_LN_LAUNCH_SUM
#undef EP_LN_LAUNCH
    return hipGetLastError();
}

hipError_t layernorm_any(float *x, const float *part, int splits, const float *bias, const float *g, const float *b,
                         float eps, uint16_t *y, int64_t rows, int D, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    if (D % 4 != 0 || D <= 0 || D > 8 * 256) return hipErrorInvalidValue;
    const int nv = (D + 255) / 256;
    switch (nv) {
    case 1: return launch_ln<1>(x, part, splits, bias, g, b, eps, y, rows, D, s);
    case 2: return launch_ln<2>(x, part, splits, bias, g, b, eps, y, rows, D, s);
    case 3: return launch_ln<3>(x, part, splits, bias, g, b, eps, y, rows, D, s);
    case 4: return launch_ln<4>(x, part, splits, bias, g, b, eps, y, rows, D, s);
    case 5: return launch_ln<5>(x, part, splits, bias, g, b, eps, y, rows, D, s);
    case 6: return launch_ln<6>(x, part, splits, bias, g, b, eps, y, rows, D, s);
    case 7: return launch_ln<7>(x, part, splits, bias, g, b, eps, y, rows, D, s);
    default: return launch_ln<8>(x, part, splits, bias, g, b, eps, y, rows, D, s);
    }
}

}  // namespace

hipError_t ep_bf16_layernorm(const float *x, const float *g, const float *b, float eps,
                             uint16_t *y, int64_t rows, int D, hipStream_t s)
{
    // without ranges to add the kernel only reads x
    return layernorm_any(const_cast<float *>(x), nullptr, 0, nullptr, g, b, eps, y, rows, D, s);
}

hipError_t ep_bf16_layernorm_sum(float *x, const float *part, int splits, const float *bias, const float *g,
                                 const float *b, float eps, uint16_t *y, int64_t rows, int D, hipStream_t s)
{
    if (!part || !bias || (splits != 2 && splits != 4 && splits != 8)) return hipErrorInvalidValue;
    return layernorm_any(x, part, splits, bias, g, b, eps, y, rows, D, s);
}

hipError_t ep_f32_residual_sum(const float *resid, const float *part, int splits, const float *bias, float *out,
                               int64_t rows, int D, hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    if (!part || !bias || D <= 0 || D % 4 != 0) return hipErrorInvalidValue;
    const int64_t n4 = rows * D / 4;
    const dim3 grid((unsigned)((n4 + 255) / 256));
    switch (splits) {
    case 2: hipLaunchKernelGGL(residual_sum_kernel<2>, grid, dim3(256), 0, s, resid, part, bias, out, n4, D / 4); break;
    case 4: hipLaunchKernelGGL(residual_sum_kernel<4>, grid, dim3(256), 0, s, resid, part, bias, out, n4, D / 4); break;
    case 8: hipLaunchKernelGGL(residual_sum_kernel<8>, grid, dim3(256), 0, s, resid, part, bias, out, n4, D / 4); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t ep_bf16_to_f32(const uint16_t *in, float *out, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    if (n % 4) return hipErrorInvalidValue;
    const int64_t n4 = n / 4;
    hipLaunchKernelGGL(bf16_to_f32_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, in, out, n4);
    return hipGetLastError();
}

hipError_t ep_f32_to_bf16(const float *in, uint16_t *out, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    if (n % 4) return hipErrorInvalidValue;
    const int64_t n4 = n / 4;
    hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, in, out, n4);
    return hipGetLastError();
}
