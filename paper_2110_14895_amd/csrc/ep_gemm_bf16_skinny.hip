// bf16 MFMA GEMM for a short stack of rows (a dense layer on few rows, paper
// section 2.1: the classifier on the class tokens of a batch; the same tile
// routine serves the row remainder inside the persistent kernel):
//
//   C[M, N] = A[M, K] . W[N, K]^T + bias[N]   (+ erf GELU | + fp32 residual | fp32 store),  M small
//
// Such a problem has few output tiles and a long K, so it is bound by latency
// and by how many compute units pull the weights at once.  The work is cut into
// narrow 64 x 32 output tiles (many of them), and inside a workgroup the 16-wide
// K slices are dealt round-robin to its 8 waves.  A wave streams its slices
// straight from global memory into MFMA fragments (no LDS staging: every byte is
// used once), up to ten slices (30 loads) in flight, and accumulates a private
// 64 x 32 partial.  The eight partials of a workgroup are summed through LDS in a
// fixed order (wave 0 .. 7), then bias / GELU / residual are applied and the tile
// is stored.  The result does not depend on timing.
//
// Requirements: K % 16 == 0, N % 8 == 0, M <= 4096.  Rows past M and columns
// past N are read as zeros (per-lane buffer offsets past the end) and never
// stored.
#include "ep_kernels.h"
#include "ep_device.h"
#include "ep_launch.h"
#include "ep_gemm_bf16_skinny_tile.h"

namespace {

using ep_skinny::TM;
using ep_skinny::TN;
using ep_skinny::NW;
using ep_skinny::SMEM;

// grid: x = column tiles, y = row tiles
template <int EPI>
__global__ __launch_bounds__(NW * 64) void gemm_bf16_skinny_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, const float *__restrict__ bias,
    const float *resid, void *Cout, int M, int N, int K)
{
    extern __shared__ float part_raw[];              // [NW][TM][TN] fp32 = 64 KB
    ep_skinny::tile<EPI>(A, W, bias, resid, Cout, M, N, K, blockIdx.y * TM, blockIdx.x * TN, part_raw);
}

template <int EPI>
hipError_t launch_skinny(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid, void *C,
                         int M, int N, int K, hipStream_t s)
{
    auto kern = gemm_bf16_skinny_kernel<EPI>;
    static EpSmemLimit smem_limit;
    const hipError_t e = smem_limit.ensure(reinterpret_cast<const void *>(kern), (int)SMEM);
    if (e != hipSuccess) return e;
    const dim3 grid((N + TN - 1) / TN, (M + TM - 1) / TM);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), SMEM, s, A, W, bias, resid, C, M, N, K);
    return hipGetLastError();
}

}  // namespace

bool ep_bf16_gemm_skinny_supported(int64_t M, int N, int K)
{
    return M > 0 && M <= 4096 && N > 0 && N % 8 == 0 && K >= 16 && K % 16 == 0 &&
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
    case EPI_BIAS_F32: return launch_skinny<EPI_BIAS_F32>(A, W, bias, resid, C, (int)M, N, K, s);
    }
    return hipErrorInvalidValue;
}
