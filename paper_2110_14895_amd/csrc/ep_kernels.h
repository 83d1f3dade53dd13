// Launchers of the stage's HIP kernels (gfx950).  Every launcher enqueues on the
// given stream, allocates nothing and returns the launch status.  Shapes are
// validated by the caller (ep_stage.hip); the launchers re-check the
// divisibility assumptions their kernels make and refuse otherwise.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// GEMM epilogues: C = A . W^T + bias, then ...
enum EpEpilogue {
    EPI_BIAS = 0,       // store (bf16 on the bf16 path, fp32 on the fp32 path)
    EPI_BIAS_GELU = 1,  // exact erf GELU, store
    EPI_BIAS_RESID = 2, // add the fp32 residual, store fp32 (out may alias resid)
    EPI_BIAS_F32 = 3,   // store fp32 (short-M bf16 kernel only: the classifier's logits)
    EPI_PARTIAL = 4     // no bias: the bare fp32 sum over one range of K (ep_bf16_gemm_partial only)
};

// ---- fp32 path -------------------------------------------------------------
hipError_t ep_f32_layernorm(const float *x, const float *g, const float *b, float eps, float *y,
                            int64_t rows, int D, hipStream_t s);
hipError_t ep_f32_gemm(const float *A, const float *W, const float *bias, const float *resid,
                       float *C, int64_t M, int N, int K, int epi, hipStream_t s);
hipError_t ep_f32_attention(const float *qkv, float *o, int B, int T, int D, int H, hipStream_t s);

// ---- bf16 path -------------------------------------------------------------
// x fp32 [rows, D] -> y bf16, fp32 statistics
hipError_t ep_bf16_layernorm(const float *x, const float *g, const float *b, float eps,
                             uint16_t *y, int64_t rows, int D, hipStream_t s);
// The same after a dense layer whose K was cut into ranges (ep_bf16_gemm_partial): first
// x[r, :] = ((part[0] + part[1] + ... + part[splits-1]) + bias) + x[r, :] in place, in that order, then as above.
// part is [splits, rows, D] fp32; splits 2, 4 or 8.
hipError_t ep_bf16_layernorm_sum(float *x, const float *part, int splits, const float *bias, const float *g,
                                 const float *b, float eps, uint16_t *y, int64_t rows, int D, hipStream_t s);
// Only the sum: out = ((part[0] + ... + part[splits-1]) + bias) + resid, n = rows * D elements, D % 4 == 0
// (out may alias resid).
hipError_t ep_f32_residual_sum(const float *resid, const float *part, int splits, const float *bias, float *out,
                               int64_t rows, int D, hipStream_t s);
hipError_t ep_bf16_to_f32(const uint16_t *in, float *out, int64_t n, hipStream_t s);
hipError_t ep_f32_to_bf16(const float *in, uint16_t *out, int64_t n, hipStream_t s);
// A bf16 [M, K], W bf16 [N, K]; out bf16 (EPI_BIAS, EPI_BIAS_GELU) or fp32 (EPI_BIAS_RESID).
// after_main: if non-null, recorded on s right after the launch (it covers the rows
// ep_bf16_gemm_main_rows reports: all of them).
hipError_t ep_bf16_gemm(const uint16_t *A, const uint16_t *W, const float *bias,
                        const float *resid, void *C, int64_t M, int N, int K, int epi,
                        hipEvent_t after_main, hipStream_t s);
int64_t ep_bf16_gemm_main_rows(int64_t M, int N, int K);
// qkv bf16 [B*T, 3D] -> o bf16 [B*T, D]; d_head 64 or 80, T <= 4096 (K and V stream through LDS in chunks)
hipError_t ep_bf16_attention(const uint16_t *qkv, uint16_t *o, int B, int T, int D, int H,
                             hipStream_t s);
bool ep_bf16_attention_supported(int T, int d_head);

// deterministic fill used by the profiler (values in [-1, 1])
hipError_t ep_fill_pattern(float *x, int64_t n, hipStream_t s);

// one tile per workgroup (64 x 64, 64 x 128 or 128 x 128 by the size of the problem): what is too small for the
// persistent kernel
hipError_t ep_bf16_gemm_small(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                              void *C, int64_t M, int N, int K, int epi, hipStream_t s);

// the same kernel with K cut into `splits` ranges: part[r] = A[:, range r] . W[:, range r]^T, fp32 [splits, M, N];
// K % (64 * splits) == 0
hipError_t ep_bf16_gemm_partial(const uint16_t *A, const uint16_t *W, float *part, int64_t M, int N, int K,
                                int splits, hipStream_t s);
// how many ranges the dispatcher wants for a dense layer with fp32 output (1: ep_bf16_gemm as it is)
int ep_bf16_gemm_splits(int64_t M, int N, int K);

// persistent kernel for large problems (ep_gemm_bf16_persist.hip): 256 x BN tiles, BN = tile_bn
// (256 or 320; 0 = pick the one with fewer weighted rounds).  The tile walk covers rows
// [0, m_rows); with fuse_tail the same launch also computes rows [m_rows, M) as 64 x 32 tiles.
bool ep_bf16_gemm_persistent_supported(int64_t M, int N, int K);
// rounds of tiles over the compute units times the tile width (lower is better); writes the
// tile width it would pick
int64_t ep_bf16_gemm_persistent_cost(int64_t rows, int N, int *tile_bn);
// resident workgroups of a launch on the current device: one per compute unit (256 if the device cannot be asked)
int ep_bf16_gemm_persistent_workgroups();
hipError_t ep_bf16_gemm_persistent(const uint16_t *A, const uint16_t *W, const float *bias,
                                   const float *resid, void *C, int64_t M, int64_t m_rows, int N,
                                   int K, int epi, int tile_bn, bool fuse_tail, hipStream_t s);

// Shader clock (MHz) and duration of workgroup 0 of the most recent persistent launch that has finished on the
// current device (hipErrorNotReady if none has); copies four counters from the device, so it synchronises.
hipError_t ep_bf16_gemm_persistent_clock(double *shader_mhz, double *seconds);

// short-M kernel (ep_gemm_bf16_skinny.hip): 64 x 32 tiles, K dealt to the 8 waves of a workgroup
bool ep_bf16_gemm_skinny_supported(int64_t M, int N, int K);
hipError_t ep_bf16_gemm_skinny(const uint16_t *A, const uint16_t *W, const float *bias,
                               const float *resid, void *C, int64_t M, int N, int K, int epi,
                               hipStream_t s);
