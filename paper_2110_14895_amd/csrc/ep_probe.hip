// Measurement hook: what the matrix cores of this device sustain on a loop of
// nothing but matrix instructions (no loads, no LDS, no stores until the end),
// as the yardstick next to the published peak for the dense layers of a stage
// (paper section 5.1 attributes a layer's time to them).  The rate depends on
// the operand data (the chip lowers its clock under the switching activity of
// random operands) and on the instruction form, so both are arguments.
//
// One workgroup of 8 waves per compute unit (two waves per SIMD, like the
// dense-layer kernels); every wave multiplies 4 x 4 fragment pairs round and
// round into 16 (form 0) or 4 (form 1) accumulators taken in rotation, so consecutive
// matrix instructions are independent and see different operand data.  Each
// workgroup reads the shader clock counter and the constant 100 MHz counter
// before and after its loop: their ratio is the clock the loop ran at.
#include <hip/hip_runtime.h>

#include "edgepipe.h"
#include "ep_error.h"
#include "ep_kernels.h"
#include "ep_launch.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int WAVES = 8;
constexpr int NFRAG = 4;                      // fragments per operand side
constexpr double REALTIME_HZ = 100e6;         // s_memrealtime counts at 100 MHz

// operand words: a hash of the word index, shaped into bf16 values with magnitude in [0.5, 2)
// and random sign and mantissa (random == 0: every value is 1.0)
__global__ void probe_fill_kernel(uint32_t *ops, int n_words, int random)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_words) return;
    uint32_t h = (uint32_t)i * 0x9E3779B9u + 0x7F4A7C15u;
    h ^= h >> 16; h *= 0x85EBCA6Bu; h ^= h >> 13; h *= 0xC2B2AE35u; h ^= h >> 16;
    auto bf = [](uint32_t r) -> uint32_t {      // 16 random bits -> sign, exponent 126 or 127, 7 mantissa bits
        return (r & 0x8000u) | ((126u + ((r >> 7) & 1u)) << 7) | (r & 0x7Fu);
    };
    ops[i] = random ? (bf(h & 0xFFFFu) | (bf(h >> 16) << 16)) : 0x3F803F80u;
}

template <int FORM>
__global__ __launch_bounds__(WAVES * 64, 1) void mfma_peak_kernel(const uint4 *__restrict__ ops, float *sink,
                                                                  unsigned long long *clk, int iters)
{
    const int lane = threadIdx.x & 63;
    bf16x8 a[NFRAG], b[NFRAG];
#pragma unroll
    for (int i = 0; i < NFRAG; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, ops[i * 64 + lane]);
        b[i] = __builtin_bit_cast(bf16x8, ops[(NFRAG + i) * 64 + lane]);
    }
    float total = 0.f;
    const unsigned long long c0 = clock64(), r0 = wall_clock64();
    if (FORM == 0) {
        f32x4 acc[NFRAG][NFRAG] = {};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < NFRAG; ++i)
#pragma unroll
                for (int j = 0; j < NFRAG; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < NFRAG; ++i)
#pragma unroll
            for (int j = 0; j < NFRAG; ++j) total += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    } else {
        f32x16 acc[2][2] = {};
        for (int it = 0; it < iters; ++it) {
            // the same 16 operand pairs per iteration, four per accumulator, the accumulators in rotation
#pragma unroll
            for (int i = 0; i < NFRAG; ++i)
#pragma unroll
                for (int j = 0; j < NFRAG; ++j)
                    acc[j >> 1][j & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[j >> 1][j & 1], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int k = 0; k < 16; ++k) total += acc[i][j][k];
    }
    const unsigned long long c1 = clock64(), r1 = wall_clock64();
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = total;
    if (threadIdx.x == 0) {
        clk[blockIdx.x * 2 + 0] = c1 - c0;
        clk[blockIdx.x * 2 + 1] = r1 - r0;
    }
}

}  // namespace

extern "C" ep_status ep_mfma_peak(int32_t form, int32_t random_operands, int32_t iters, void *stream,
                                  double *tflops, double *shader_mhz)
{
    if (!tflops) return ep_fail(EP_ERR_INVALID_ARG, "ep_mfma_peak: null output");
    if ((form != 0 && form != 1) || iters < 1 || iters > (1 << 24))
        return ep_fail(EP_ERR_INVALID_ARG, "ep_mfma_peak: form must be 0 or 1 and 1 <= iters <= 2^24");
    hipStream_t s = (hipStream_t)stream;
    int cus = 0;
    hipError_t e = ep_device_cu_count(&cus);
    if (e != hipSuccess) return ep_fail(EP_ERR_HIP, "device query failed: %s", hipGetErrorString(e));

    const int n_words = 2 * NFRAG * 64 * 4;                       // uint32 words of operand data
    const size_t ops_bytes = (size_t)n_words * 4, sink_bytes = (size_t)cus * WAVES * 64 * 4,
                 clk_bytes = (size_t)cus * 2 * 8;
    char *buf = nullptr;
    e = hipMalloc((void **)&buf, ops_bytes + sink_bytes + clk_bytes);
    if (e != hipSuccess) return ep_fail(EP_ERR_OOM, "ep_mfma_peak: hipMalloc failed: %s", hipGetErrorString(e));
    uint32_t *ops = (uint32_t *)buf;
    float *sink = (float *)(buf + ops_bytes);
    unsigned long long *clk = (unsigned long long *)(buf + ops_bytes + sink_bytes);
    hipEvent_t t0 = nullptr, t1 = nullptr;
    ep_status rc = EP_OK;
    auto fail = [&](const char *what, hipError_t err) { rc = ep_fail(EP_ERR_HIP, "%s failed: %s", what, hipGetErrorString(err)); };
    do {
        if ((e = hipEventCreate(&t0)) != hipSuccess) { fail("hipEventCreate", e); break; }
        if ((e = hipEventCreate(&t1)) != hipSuccess) { fail("hipEventCreate", e); break; }
        hipLaunchKernelGGL(probe_fill_kernel, dim3((n_words + 255) / 256), dim3(256), 0, s, ops, n_words, random_operands);
        auto launch = [&](int n) {
            if (form == 0)
                hipLaunchKernelGGL(mfma_peak_kernel<0>, dim3(cus), dim3(WAVES * 64), 0, s, (const uint4 *)ops, sink, clk, n);
            else
                hipLaunchKernelGGL(mfma_peak_kernel<1>, dim3(cus), dim3(WAVES * 64), 0, s, (const uint4 *)ops, sink, clk, n);
        };
        launch(iters < 64 ? iters : 64);                           // warm-up: code and clocks
        if ((e = hipEventRecord(t0, s)) != hipSuccess) { fail("hipEventRecord", e); break; }
        launch(iters);
        if ((e = hipGetLastError()) != hipSuccess) { fail("probe launch", e); break; }
        if ((e = hipEventRecord(t1, s)) != hipSuccess) { fail("hipEventRecord", e); break; }
        if ((e = hipEventSynchronize(t1)) != hipSuccess) { fail("hipEventSynchronize", e); break; }
        float ms = 0.f;
        if ((e = hipEventElapsedTime(&ms, t0, t1)) != hipSuccess) { fail("hipEventElapsedTime", e); break; }
        const double flop_per_mfma = form == 0 ? 2.0 * 16 * 16 * 32 : 2.0 * 32 * 32 * 16;
        const double flops = (double)cus * WAVES * (double)iters * NFRAG * NFRAG * flop_per_mfma;
        *tflops = flops / ((double)ms * 1e-3) / 1e12;
        if (shader_mhz) {
            unsigned long long h[2 * 1024];
            const int n = cus < 1024 ? cus : 1024;
            if ((e = hipMemcpy(h, clk, (size_t)n * 16, hipMemcpyDeviceToHost)) != hipSuccess) { fail("hipMemcpy", e); break; }
            double sum = 0.0;
            int cnt = 0;
            for (int i = 0; i < n; ++i)
                if (h[2 * i + 1] > 0) { sum += (double)h[2 * i] / (double)h[2 * i + 1] * REALTIME_HZ; ++cnt; }
            *shader_mhz = cnt ? sum / cnt / 1e6 : 0.0;
        }
    } while (0);
    if (t0) (void)hipEventDestroy(t0);
    if (t1) (void)hipEventDestroy(t1);
    (void)hipFree(buf);
    return rc;
}

extern "C" ep_status ep_gemm_clock_sample(double *shader_mhz, double *seconds)
{
    if (!shader_mhz || !seconds) return ep_fail(EP_ERR_INVALID_ARG, "ep_gemm_clock_sample: null output");
    const hipError_t e = ep_bf16_gemm_persistent_clock(shader_mhz, seconds);
    if (e == hipErrorNotReady)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_gemm_clock_sample: no large dense-layer launch has finished on this device");
    if (e != hipSuccess) return ep_fail(EP_ERR_HIP, "reading the clock sample failed: %s", hipGetErrorString(e));
    return EP_OK;
}
