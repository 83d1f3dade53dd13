// bf16 MFMA GEMM for a short stack of rows (the remainder of M after the last
// full 256-row tile of a dense layer, paper section 2.1):
//
//   C[M, N] = A[M, K] . W[N, K]^T + bias[N]   (+ erf GELU | + fp32 residual),  M small
//
// Such a problem has too few output tiles to fill the chip and a long K, so it
// is latency-bound.  Each workgroup owns a 64 x 32 output tile (narrow, so that
// many compute units pull the weights in parallel) and splits K eight ways over
// its 8 waves; a wave streams its K range straight from global memory into MFMA
// fragments (no LDS staging: every byte is used once), ten 16-wide slices
// (30 loads) in flight at a time, and accumulates a private 64 x 32 partial.  The eight partials are summed through LDS in a fixed order
// (wave 0 .. 7, so the result does not depend on timing), then bias / GELU /
// residual are applied and 4 consecutive columns per thread are stored.
//
// Requirements: K % 128 == 0, N % 8 == 0.  Rows past M and columns past N are
// read as zeros (per-lane buffer offsets past the end) and never stored.
#include "ep_kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int TM = 64, TN = 32, NW = 8, U = 10;
constexpr size_t SMEM = (size_t)NW * TM * TN * sizeof(float);

__device__ inline float gelu_fast(float u)
{
    // erf by Abramowitz & Stegun 7.1.26, absolute error < 1.5e-7
    const float x = fabsf(u) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    const float e = p * t * __builtin_amdgcn_exp2f(-x * x * 1.4426950408889634f);
    return 0.5f * u * (1.0f + copysignf(1.0f - e, u));
}

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    const __bf16 a = (__bf16)lo, b = (__bf16)hi;
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

template <int EPI>
__global__ __launch_bounds__(NW * 64) void gemm_bf16_skinny_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, const float *__restrict__ bias,
    const float *resid, void *Cout, int M, int N, int K)
{
#if defined(__HIP_DEVICE_COMPILE__)
    extern __shared__ float part_raw[];              // [NW][TM][TN] fp32 = 64 KB
    float (*part)[TM][TN] = reinterpret_cast<float (*)[TM][TN]>(part_raw);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, g = lane >> 5;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;

    const __amdgpu_buffer_rsrc_t a_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(A), 0, (int)((size_t)M * K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(W), 0, (int)((size_t)N * K * 2), 0x00020000);
    constexpr int OOB = 0x7FFFFFF0;
    const int kw = K / NW;                           // this wave's K range: [wave*kw, (wave+1)*kw)
    const int nsl = kw / 16;
    // fragment f (0,1): rows f*32 + l31 of the tile, 8 elements at k + g*8
    int a_off[2], w_off;
#pragma unroll
    for (int f = 0; f < 2; ++f) {
        const int am = m0 + f * 32 + l31;
        a_off[f] = am < M ? (am * K + wave * kw + g * 8) * 2 : OOB;
    }
    w_off = n0 + l31 < N ? ((n0 + l31) * K + wave * kw + g * 8) * 2 : OOB;

    f32x16 acc[2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mi][i] = 0.f;

    for (int s0 = 0; s0 < nsl; s0 += U) {
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 fa[U][2], fw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool live = s0 + u < nsl;          // wave-uniform
            const int ko = (s0 + u) * 32;            // bytes
            fw[u] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(w_rs, live ? w_off + ko : OOB, 0, 0));
#pragma unroll
            for (int f = 0; f < 2; ++f)
                fa[u][f] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(a_rs, live ? a_off[f] + ko : OOB, 0, 0));
        }
        __builtin_amdgcn_sched_barrier(0);           // all loads of the batch are issued before the first MFMA
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
                acc[mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[u], fa[u][mi], acc[mi], 0, 0, 0);
    }

    // acc[mi][i] <-> column 8*(i/4) + 4*g + (i%4), row mi*32 + l31
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<float4 *>(&part[wave][mi * 32 + l31][q * 8 + g * 4]) =
                make_float4(acc[mi][q * 4 + 0], acc[mi][q * 4 + 1], acc[mi][q * 4 + 2], acc[mi][q * 4 + 3]);
    __syncthreads();

    // thread t: row t/8, columns (t%8)*4 .. +3
    const int r = tid >> 3, c = (tid & 7) * 4;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const float4 p0 = *reinterpret_cast<const float4 *>(&part[w][r][c]);
        v[0] += p0.x; v[1] += p0.y; v[2] += p0.z; v[3] += p0.w;
    }
    const int m = m0 + r, n = n0 + c;
    if (m >= M || n >= N) return;
    const float4 b0 = *reinterpret_cast<const float4 *>(bias + n);
    v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w;
    const size_t off = (size_t)m * N + n;
    if (EPI == EPI_BIAS_RESID) {
        const float4 x0 = *reinterpret_cast<const float4 *>(resid + off);
        float *C = reinterpret_cast<float *>(Cout);
        *reinterpret_cast<float4 *>(C + off) = make_float4(v[0] + x0.x, v[1] + x0.y, v[2] + x0.z, v[3] + x0.w);
    } else {
        if (EPI == EPI_BIAS_GELU) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = gelu_fast(v[j]);
        }
        uint2 o;
        o.x = pack_bf16x2(v[0], v[1]); o.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(Cout) + off) = o;
    }
#endif
}

template <int EPI>
hipError_t launch_skinny(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid, void *C,
                         int M, int N, int K, hipStream_t s)
{
    auto kern = gemm_bf16_skinny_kernel<EPI>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 grid((N + TN - 1) / TN, (M + TM - 1) / TM);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), SMEM, s, A, W, bias, resid, C, M, N, K);
    return hipGetLastError();
}

}  // namespace

bool ep_bf16_gemm_skinny_supported(int64_t M, int N, int K)
{
    return M > 0 && M <= 4096 && N > 0 && N % 8 == 0 && K >= 128 && K % 128 == 0 &&
           M * (int64_t)K * 2 < 0x7FFFFFF0ll && (int64_t)N * K * 2 < 0x7FFFFFF0ll;
}

hipError_t ep_bf16_gemm_skinny(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                               void *C, int64_t M, int N, int K, int epi, hipStream_t s)
{
    if (!ep_bf16_gemm_skinny_supported(M, N, K)) return hipErrorInvalidValue;
    if (epi == EPI_BIAS_RESID && !resid) return hipErrorInvalidValue;
    switch (epi) {
    case EPI_BIAS: return launch_skinny<EPI_BIAS>(A, W, bias, resid, C, (int)M, N, K, s);
    case EPI_BIAS_GELU: return launch_skinny<EPI_BIAS_GELU>(A, W, bias, resid, C, (int)M, N, K, s);
    case EPI_BIAS_RESID: return launch_skinny<EPI_BIAS_RESID>(A, W, bias, resid, C, (int)M, N, K, s);
    }
    return hipErrorInvalidValue;
}
