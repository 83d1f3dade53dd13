// One 64 x 32 output tile of the short-M bf16 GEMM as a device function, shared by the short-M
// kernel and by the tail phase of the persistent kernel (paper section 2.1: a dense layer of a
// stage on the rows of a micro-batch):
//
//   C[m0 .. m0+63, n0 .. n0+31] = A[m0 .. m0+63, :] . W[n0 .. n0+31, :]^T  (+ bias, epilogue)
//
// The 16-wide K slices are dealt round-robin to the 8 waves of the workgroup; a wave
// streams its slices straight from global memory into MFMA fragments (no LDS staging: every byte is
// used once), up to ten slices (30 loads) in flight, and accumulates a private 64 x 32 partial.  The
// eight partials are summed through LDS in a fixed order (wave 0 .. 7), so the result does not depend
// on timing.  Rows past M and columns past N are read as zeros (per-lane buffer offsets past the end)
// and never stored.
#pragma once
#include "ep_kernels.h"
#include "ep_device.h"

namespace ep_skinny {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int TM = 64, TN = 32, NW = 8, U = 10;
constexpr size_t SMEM = (size_t)NW * TM * TN * sizeof(float);      // 64 KB of LDS per workgroup

template <int EPI>
__device__ inline void store_epilogue(float v[4], const float *bias, const float *resid, void *Cout, int m, int n,
                                      int N)
{
    const float4 b0 = *reinterpret_cast<const float4 *>(bias + n);
    v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w;
    const size_t off = (size_t)m * N + n;
    if (EPI == EPI_BIAS_RESID) {
        const float4 x0 = *reinterpret_cast<const float4 *>(resid + off);
        float *C = reinterpret_cast<float *>(Cout);
        *reinterpret_cast<float4 *>(C + off) = make_float4(v[0] + x0.x, v[1] + x0.y, v[2] + x0.z, v[3] + x0.w);
    } else if (EPI == EPI_BIAS_F32) {
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(Cout) + off) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        if (EPI == EPI_BIAS_GELU) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = gelu_erf(v[j]);
        }
        uint2 o;
        o.x = pack_bf16x2(v[0], v[1]); o.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(Cout) + off) = o;
    }
}

// All 512 threads of the workgroup call this together.  TMU = 64 or 32: rows of the tile (two or one
// 32x32x16 MFMA blocks).  lds: SMEM bytes, free on entry; the caller synchronises before it reuses them.
template <int EPI, int TMU = TM>
__device__ inline void tile(const uint16_t *__restrict__ A, const uint16_t *__restrict__ W,
                            const float *__restrict__ bias, const float *resid, void *Cout, int M, int N, int K,
                            int m0, int n0, float *lds)
{
#if defined(__HIP_DEVICE_COMPILE__)
    static_assert(TMU == 64 || TMU == 32, "tile rows");
    constexpr int MI = TMU / 32;
    float (*wsum)[TMU][TN] = reinterpret_cast<float (*)[TMU][TN]>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, g = lane >> 5;

    const __amdgpu_buffer_rsrc_t a_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(A), 0, (int)((size_t)M * K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(W), 0, (int)((size_t)N * K * 2), 0x00020000);
    constexpr int OOB = 0x7FFFFFF0;
    const int nsl = K / 16;                          // slices of this tile; wave w takes w, w+8, ...
    const int my_nsl = (nsl - wave + NW - 1) / NW;
    // fragment f: rows f*32 + l31 of the tile, 8 elements at k + g*8
    int a_off[MI], w_off;
#pragma unroll
    for (int f = 0; f < MI; ++f) {
        const int am = m0 + f * 32 + l31;
        a_off[f] = am < M ? (am * K + wave * 16 + g * 8) * 2 : OOB;
    }
    w_off = n0 + l31 < N ? ((n0 + l31) * K + wave * 16 + g * 8) * 2 : OOB;

    f32x16 acc[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mi][i] = 0.f;

    for (int s0 = 0; s0 < my_nsl; s0 += U) {
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 fa[U][MI], fw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool live = s0 + u < my_nsl;       // wave-uniform
            const int ko = (s0 + u) * NW * 32;       // bytes: my slices are NW * 16 elements apart
            fw[u] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(w_rs, live ? w_off + ko : OOB, 0, 0));
#pragma unroll
            for (int f = 0; f < MI; ++f)
                fa[u][f] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(a_rs, live ? a_off[f] + ko : OOB, 0, 0));
        }
        __builtin_amdgcn_sched_barrier(0);           // all loads of the batch are issued before the first MFMA
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                acc[mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[u], fa[u][mi], acc[mi], 0, 0, 0);
    }

    // acc[mi][i] <-> column 8*(i/4) + 4*g + (i%4), row mi*32 + l31
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<float4 *>(&wsum[wave][mi * 32 + l31][q * 8 + g * 4]) =
                make_float4(acc[mi][q * 4 + 0], acc[mi][q * 4 + 1], acc[mi][q * 4 + 2], acc[mi][q * 4 + 3]);
    __syncthreads();

    // thread t: row t/8, columns (t%8)*4 .. +3
    const int r = tid >> 3, c = (tid & 7) * 4;
    if (r < TMU) {
        float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float4 p0 = *reinterpret_cast<const float4 *>(&wsum[w][r][c]);
            v[0] += p0.x; v[1] += p0.y; v[2] += p0.z; v[3] += p0.w;
        }
        const int m = m0 + r, n = n0 + c;
        if (m < M && n < N) store_epilogue<EPI>(v, bias, resid, Cout, m, n, N);
    }
#endif
}

// The same for a 16-row tile (16 x 32 outputs, two 16x16x32 MFMA blocks side by side): for long K and
// few columns, where only narrow tiles give every compute unit one.  K is dealt in 32-wide slices.
template <int EPI>
__device__ inline void tile16(const uint16_t *__restrict__ A, const uint16_t *__restrict__ W,
                              const float *__restrict__ bias, const float *resid, void *Cout, int M, int N, int K,
                              int m0, int n0, float *lds)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    float (*wsum)[16][TN] = reinterpret_cast<float (*)[16][TN]>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l15 = lane & 15, g = lane >> 4;        // g: 8-element K group 0 .. 3 of a slice

    const __amdgpu_buffer_rsrc_t a_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(A), 0, (int)((size_t)M * K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(W), 0, (int)((size_t)N * K * 2), 0x00020000);
    constexpr int OOB = 0x7FFFFFF0;
    const int nsl = K / 32;                          // 32-wide slices; wave w takes w, w+8, ...
    const int my_nsl = (nsl - wave + NW - 1) / NW;
    const int am = m0 + l15;
    const int a_off = am < M ? (am * K + wave * 32 + g * 8) * 2 : OOB;
    int w_off[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int wn = n0 + j * 16 + l15;
        w_off[j] = wn < N ? (wn * K + wave * 32 + g * 8) * 2 : OOB;
    }

    f32x4 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[j][i] = 0.f;

    for (int s0 = 0; s0 < my_nsl; s0 += U) {
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 fa[U], fw[U][2];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool live = s0 + u < my_nsl;       // wave-uniform
            const int ko = (s0 + u) * NW * 64;       // bytes: my slices are NW * 32 elements apart
            fa[u] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(a_rs, live ? a_off + ko : OOB, 0, 0));
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fw[u][j] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(w_rs, live ? w_off[j] + ko : OOB, 0, 0));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[u][j], fa[u], acc[j], 0, 0, 0);
    }

    // acc[j][i] <-> column j*16 + 4*g + i, row l15
#pragma unroll
    for (int j = 0; j < 2; ++j)
        *reinterpret_cast<float4 *>(&wsum[wave][l15][j * 16 + g * 4]) = make_float4(acc[j][0], acc[j][1], acc[j][2], acc[j][3]);
    __syncthreads();

    const int r = tid >> 3, c = (tid & 7) * 4;       // thread t: row t/8, columns (t%8)*4 .. +3
    if (r < 16) {
        float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float4 p0 = *reinterpret_cast<const float4 *>(&wsum[w][r][c]);
            v[0] += p0.x; v[1] += p0.y; v[2] += p0.z; v[3] += p0.w;
        }
        const int m = m0 + r, n = n0 + c;
        if (m < M && n < N) store_epilogue<EPI>(v, bias, resid, Cout, m, n, N);
    }
#endif
}

}  // namespace ep_skinny
