// bf16 MFMA GEMM for a short stack of rows (a dense layer on few rows, paper
// section 2.1: the classifier on the class tokens of a batch; the same tile
// routine serves the row remainder inside the persistent kernel):
//
//   C[M, N] = A[M, K] . W[N, K]^T + bias[N]   (+ erf GELU | + fp32 residual | fp32 store),  M small
//
// Such a problem has few output tiles and a long K, so it is bound by latency
// and by how many compute units pull the weights at once.  The work is cut
// three ways: 64 x 32 output tiles (narrow, many of them), for long K (>= 2560)
// K split over up to 8 workgroups per tile (so that there are about two
// workgroups per compute unit), and inside a workgroup the 16-wide K slices
// dealt round-robin to its 8 waves.  A wave streams its slices straight from global memory into MFMA
// fragments (no LDS staging: every byte is used once), up to ten slices
// (30 loads) in flight, and accumulates a private 64 x 32 partial.  The eight
// partials of a workgroup are summed through LDS in a fixed order (wave 0 .. 7).
// Without a K split the workgroup then applies bias / GELU / residual and
// stores; with one it writes its partial tile to a workspace and a second small
// kernel sums the splits, again in a fixed order, and applies the epilogue.
// The result does not depend on timing in either case.
//
// Requirements: K % 16 == 0, N % 8 == 0, M <= 4096.  Rows past M and columns
// past N are read as zeros (per-lane buffer offsets past the end) and never
// stored.
#include "ep_kernels.h"
#include "ep_device.h"
#include "ep_gemm_bf16_skinny_tile.h"

namespace {

using ep_skinny::TM;
using ep_skinny::TN;
using ep_skinny::NW;
using ep_skinny::SMEM;
using ep_skinny::store_epilogue;
constexpr int MAX_SPLIT = 8;

// grid: x = column tiles, y = row tiles, z = K splits of kw elements each.  part == nullptr: no split.
template <int EPI>
__global__ __launch_bounds__(NW * 64) void gemm_bf16_skinny_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, const float *__restrict__ bias,
    const float *resid, void *Cout, float *__restrict__ part, int M, int N, int K, int kw)
{
    extern __shared__ float part_raw[];              // [NW][TM][TN] fp32 = 64 KB
    ep_skinny::tile<EPI>(A, W, bias, resid, Cout, part ? part + (size_t)blockIdx.z * M * N : nullptr, M, N, K,
                         blockIdx.y * TM, blockIdx.x * TN, blockIdx.z * kw, kw, part_raw);
}

// sums the K splits (in order) and applies the epilogue; one thread per 4 columns
template <int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_skinny_reduce_kernel(const float *__restrict__ part, int splits,
                                                                      const float *__restrict__ bias,
                                                                      const float *resid, void *Cout, int M, int N)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int n4 = N / 4;
    if (i >= (int64_t)M * n4) return;
    const int m = (int)(i / n4), n = (int)(i % n4) * 4;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    for (int z = 0; z < splits; ++z) {
        const float4 p = *reinterpret_cast<const float4 *>(part + ((size_t)z * M + m) * N + n);
        v[0] += p.x; v[1] += p.y; v[2] += p.z; v[3] += p.w;
    }
    store_epilogue<EPI>(v, bias, resid, Cout, m, n, N);
}

int pick_splits(int M, int N, int K, size_t ws_floats)
{
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
            n_cu = 256;
    }
    const int tiles = ((N + TN - 1) / TN) * ((M + TM - 1) / TM);
    int splits = 1;
    // a second launch costs about as much as 20 slices per wave take: split long K only
    if (K < 2560) return 1;
    // double while that keeps every split a whole number of slices, at least one slice per wave,
    // inside the workspace, and the grid at or below about two workgroups per compute unit
    while (splits * 2 <= MAX_SPLIT && K % (splits * 2 * 16) == 0 && K / (splits * 2) >= NW * 16 &&
           (size_t)(splits * 2) * M * N <= ws_floats && tiles * splits * 2 <= 2 * n_cu + n_cu / 4)
        splits *= 2;
    return splits;
}

template <int EPI>
hipError_t launch_skinny(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid, void *C,
                         int M, int N, int K, float *ws, size_t ws_floats, hipStream_t s)
{
    auto kern = gemm_bf16_skinny_kernel<EPI>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int splits = ws ? pick_splits(M, N, K, ws_floats) : 1;
    const dim3 grid((N + TN - 1) / TN, (M + TM - 1) / TM, splits);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), SMEM, s, A, W, bias, resid, C, splits > 1 ? ws : nullptr, M, N, K,
                       K / splits);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || splits == 1) return e;
    const int64_t threads = (int64_t)M * (N / 4);
    hipLaunchKernelGGL(gemm_bf16_skinny_reduce_kernel<EPI>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                       ws, splits, bias, resid, C, M, N);
    return hipGetLastError();
}

}  // namespace

bool ep_bf16_gemm_skinny_supported(int64_t M, int N, int K)
{
    return M > 0 && M <= 4096 && N > 0 && N % 8 == 0 && K >= 16 && K % 16 == 0 &&
           M * (int64_t)K * 2 < 0x7FFFFFF0ll && (int64_t)N * K * 2 < 0x7FFFFFF0ll;
}

size_t ep_bf16_gemm_skinny_workspace_floats(int64_t M, int N) { return (size_t)MAX_SPLIT * (size_t)M * (size_t)N; }

hipError_t ep_bf16_gemm_skinny(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                               void *C, int64_t M, int N, int K, int epi, float *ws, size_t ws_floats,
                               hipStream_t s)
{
    if (!ep_bf16_gemm_skinny_supported(M, N, K)) return hipErrorInvalidValue;
    if (epi == EPI_BIAS_RESID && !resid) return hipErrorInvalidValue;
    switch (epi) {
    case EPI_BIAS: return launch_skinny<EPI_BIAS>(A, W, bias, resid, C, (int)M, N, K, ws, ws_floats, s);
    case EPI_BIAS_GELU: return launch_skinny<EPI_BIAS_GELU>(A, W, bias, resid, C, (int)M, N, K, ws, ws_floats, s);
    case EPI_BIAS_RESID: return launch_skinny<EPI_BIAS_RESID>(A, W, bias, resid, C, (int)M, N, K, ws, ws_floats, s);
    case EPI_BIAS_F32: return launch_skinny<EPI_BIAS_F32>(A, W, bias, resid, C, (int)M, N, K, ws, ws_floats, s);
    }
    return hipErrorInvalidValue;
}
