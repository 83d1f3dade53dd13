// Persistent bf16 MFMA GEMM for the large dense layers of an encoder layer
// (paper section 2.1; section 5.1 attributes most of a layer's time to them).
//
//   C[M, N] = A[M, K] . W[N, K]^T + bias[N]   (+ erf GELU | + fp32 residual)
//
// One workgroup per compute unit stays resident and walks a static list of
// 256 x 256 output tiles; the K loop of consecutive tiles forms one continuous
// software pipeline, so the first K steps of the next tile are already in
// flight while the current tile is finished and stored.
//
// Pipeline (per workgroup, 8 waves laid out 2 x 4, wave tile 128 x 64):
//   - K advances in steps of 32.  A step's A and W panels (256 rows x 64 bytes
//     each) are brought from global memory straight into LDS with
//     buffer_load ... lds (no register staging), 4 stages deep: the loads of step
//     i+3 are issued while step i is multiplied.  Each wave issues 4 such loads
//     per step, interleaved one by one between MFMAs so that their issue cost is
//     hidden behind matrix-core time.
//   - LDS rows are 4 chunks of 16 bytes; chunk c of row r sits at slot
//     c ^ f(r), f(r) = ((r>>1)&3) ^ ((r>>3)&1), which makes the 16-byte fragment
//     reads of 32 consecutive rows conflict-free on the 64-bank LDS.
//   - Fragments are double-buffered in registers: the reads for the next
//     16-wide K slice are issued before the 8 MFMAs of the current slice.
//   - One barrier per K step, placed before the second slice's MFMAs: it
//     publishes step i+1 (its loads have landed: vmcnt) and retires step i's
//     stage for reuse.
// Epilogue: accumulators (+bias, GELU) are transposed through the LDS stage
// that has just been retired, one 32-row block per wave at a time, so that
// global stores (and residual loads) are full 128-byte row segments.
//
// Operand roles are swapped (MFMA A = W fragment, B = activation fragment) so
// that a lane owns 4 consecutive output columns of one row.
//
// Workgroup w runs on XCD w % 8 (round-robin dispatch); in every round the 32
// workgroups of an XCD take 32 consecutive tiles of an order that walks groups
// of 4 tile rows column by column, so that they share A and W panels in L2.
//
// Requirements: K % 32 == 0, N % 8 == 0; M*K*2, N*K*2 < 2^31; rows past M and
// columns past N are read as zeros (buffer bounds) and never stored.
#include "ep_kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 32, STAGES = 4;
constexpr int WM = 2, WN = 4, NW = WM * WN;          // 8 waves
constexpr int MI = 4, NI = 2;                        // 32x32 accumulators per wave: 128 (m) x 64 (n)
constexpr int CPR = BK / 8;                          // 4 chunks of 16 B per LDS row
constexpr int A_STAGE = BM * CPR, W_STAGE = BN * CPR;   // uint4 per stage and operand
constexpr int STAGE_U4 = A_STAGE + W_STAGE;          // 2048 uint4 = 32 KB
constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 4;
constexpr size_t SMEM_BYTES = (size_t)STAGES * STAGE_U4 * sizeof(uint4);   // 128 KB

__device__ inline float gelu_erf(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f)); }

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    const __bf16 a = (__bf16)lo, b = (__bf16)hi;   // round to nearest even
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

#define EP_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))
#define EP_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4) | (0x0 << 8))
#define EP_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

__device__ inline int swz(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }

template <int EPI>
__global__ __launch_bounds__(NW * 64, 1) void gemm_bf16_persistent_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, const float *__restrict__ bias,
    const float *resid, void *Cout, int M, int N, int K, int tiles_m, int tiles_n)
{
#if defined(__HIP_DEVICE_COMPILE__)
    extern __shared__ uint4 lds[];                   // [STAGES][A panel | W panel]
    typedef __attribute__((address_space(3))) void *lds_ptr;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WN) * (MI * 32), wn0 = (wave % WN) * (NI * 32);
    const int l31 = lane & 31, g = lane >> 5;

    // ---- this workgroup's tile list: tile j has logical id j*G + (w%8)*(G/8) + w/8
    const int G = gridDim.x;                         // multiple of 8
    const int total = tiles_m * tiles_n;
    const int first_id = (int)(blockIdx.x % NUM_XCD) * (G / NUM_XCD) + (int)(blockIdx.x / NUM_XCD);
    if (first_id >= total) return;
    const int n_my = (total - first_id + G - 1) / G;
    const int KT = K / BK;
    const int total_it = n_my * KT;

    auto tile_origin = [&](int seq, int &m0, int &n0) {
        const int id = seq * G + first_id;
        const int group_sz = GROUP_M * tiles_n;
        const int group = id / group_sz;
        const int fm = group * GROUP_M;
        const int rows = min(GROUP_M, tiles_m - fm);
        const int in_group = id - group * group_sz;
        m0 = (fm + in_group % rows) * BM;
        n0 = (in_group / rows) * BN;
    };

    // ---- load stream (runs STAGES-1 steps ahead of the multiply stream)
    const __amdgpu_buffer_rsrc_t a_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(A), 0, (int)((size_t)M * K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(W), 0, (int)((size_t)N * K * 2), 0x00020000);
    constexpr int OOB = 0x7FFFFFF0;
    int ld_seq = 0, ld_kt = 0, ld_stage = 0;
    int a_off[2], w_off[2];
    auto set_load_tile = [&](int seq) {
        int m0 = 0, n0 = 0;
        const bool live = seq < n_my;
        if (live) tile_origin(seq, m0, n0);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = (i * NW + wave) * 16 + (lane >> 2);       // row inside the 256-row panel
            const int c = (lane & 3) ^ swz(r);
            const int gm = m0 + r, gn = n0 + r;
            a_off[i] = (live && gm < M) ? (gm * K + c * 8) * 2 : OOB;
            w_off[i] = (live && gn < N) ? (gn * K + c * 8) * 2 : OOB;
        }
    };
    // which: 0,1 = A panel rows (which*128 + wave*16 ..), 2,3 = W panel likewise
    auto issue_one = [&](int which) {
        const int koff = ld_kt * (BK * 2);
        uint4 *dst = lds + ld_stage * STAGE_U4;
        if (which < 2)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rs, (lds_ptr)(dst + (which * NW + wave) * 64), 16,
                                                     a_off[which], koff, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rs, (lds_ptr)(dst + A_STAGE + ((which - 2) * NW + wave) * 64),
                                                     16, w_off[which - 2], koff, 0, 0);
    };
    auto advance_load = [&]() {
        ld_stage = (ld_stage + 1) & (STAGES - 1);
        if (++ld_kt == KT) {
            ld_kt = 0;
            set_load_tile(++ld_seq);
        }
    };

    // ---- fragment reads: offsets in uint4 inside a stage
    const int fsw = swz(l31);
    int a_rd[2], w_rd[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        a_rd[kk] = (wm0 + l31) * CPR + ((kk * 2 + g) ^ fsw);
        w_rd[kk] = A_STAGE + (wn0 + l31) * CPR + ((kk * 2 + g) ^ fsw);
    }
    bf16x8 fa[2][MI], fw[2][NI];
    auto read_frags = [&](int stage, int kk, int buf) {
        const uint4 *base = lds + stage * STAGE_U4;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) fw[buf][ni] = __builtin_bit_cast(bf16x8, base[w_rd[kk] + ni * 32 * CPR]);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) fa[buf][mi] = __builtin_bit_cast(bf16x8, base[a_rd[kk] + mi * 32 * CPR]);
    };

    f32x16 acc[NI][MI];
    auto zero_acc = [&]() {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[ni][mi][i] = 0.f;
    };
    // 8 MFMAs of one 16-wide K slice, with two global->LDS loads slipped in between
    auto mfma_slice = [&](int buf, int ld_a, int ld_b) {
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][0], fa[buf][0], acc[0][0], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][1], fa[buf][0], acc[1][0], 0, 0, 0);
        EP_SCHED_FENCE();
        issue_one(ld_a);
        EP_SCHED_FENCE();
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][0], fa[buf][1], acc[0][1], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][1], fa[buf][1], acc[1][1], 0, 0, 0);
        acc[0][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][0], fa[buf][2], acc[0][2], 0, 0, 0);
        acc[1][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][1], fa[buf][2], acc[1][2], 0, 0, 0);
        EP_SCHED_FENCE();
        issue_one(ld_b);
        EP_SCHED_FENCE();
        acc[0][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][0], fa[buf][3], acc[0][3], 0, 0, 0);
        acc[1][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][1], fa[buf][3], acc[1][3], 0, 0, 0);
    };

    // ---- epilogue of the tile at (m0, n0); `stage` is free LDS (32 KB, 4 KB per wave)
    auto epilogue = [&](int m0, int n0, int stage) {
        uint4 *stg = lds + stage * STAGE_U4 + wave * 256;          // 256 uint4 = 4 KB, rows of 128 B
        const int rrow = lane >> 3, rc = lane & 7;                  // read-back: 8 rows x 8 chunks per pass
        if (EPI == EPI_BIAS_RESID) {
            float *C = reinterpret_cast<float *>(Cout);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    // block [32 m][32 n] fp32: chunk = 4 floats, 8 chunks per row
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = n0 + wn0 + ni * 32 + q * 8 + g * 4;
                        float4 bb = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (n < N) bb = *reinterpret_cast<const float4 *>(bias + n);
                        float4 v = make_float4(acc[ni][mi][q * 4 + 0] + bb.x, acc[ni][mi][q * 4 + 1] + bb.y,
                                               acc[ni][mi][q * 4 + 2] + bb.z, acc[ni][mi][q * 4 + 3] + bb.w);
                        *reinterpret_cast<float4 *>(&stg[l31 * 8 + ((q * 2 + g) ^ (l31 & 7))]) = v;
                    }
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const int r = p * 8 + rrow;
                        const float4 v = *reinterpret_cast<const float4 *>(&stg[r * 8 + (rc ^ (r & 7))]);
                        const int m = m0 + wm0 + mi * 32 + r;
                        const int n = n0 + wn0 + ni * 32 + rc * 4;
                        if (m < M && n < N) {
                            const size_t off = (size_t)m * N + n;
                            const float4 x = *reinterpret_cast<const float4 *>(resid + off);
                            *reinterpret_cast<float4 *>(C + off) = make_float4(v.x + x.x, v.y + x.y, v.z + x.z, v.w + x.w);
                        }
                    }
                }
            }
        } else {
            uint16_t *C = reinterpret_cast<uint16_t *>(Cout);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                // block [32 m][64 n] bf16: chunk = 8 bf16, 8 chunks per row
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = n0 + wn0 + ni * 32 + q * 8 + g * 4;
                        float4 bb = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (n < N) bb = *reinterpret_cast<const float4 *>(bias + n);
                        float v0 = acc[ni][mi][q * 4 + 0] + bb.x, v1 = acc[ni][mi][q * 4 + 1] + bb.y;
                        float v2 = acc[ni][mi][q * 4 + 2] + bb.z, v3 = acc[ni][mi][q * 4 + 3] + bb.w;
                        if (EPI == EPI_BIAS_GELU) {
                            v0 = gelu_erf(v0); v1 = gelu_erf(v1); v2 = gelu_erf(v2); v3 = gelu_erf(v3);
                        }
                        uint2 o;
                        o.x = pack_bf16x2(v0, v1);
                        o.y = pack_bf16x2(v2, v3);
                        uint2 *dst = reinterpret_cast<uint2 *>(&stg[l31 * 8 + ((ni * 4 + q) ^ (l31 & 7))]) + g;
                        *dst = o;
                    }
                }
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int r = p * 8 + rrow;
                    const uint4 v = stg[r * 8 + (rc ^ (r & 7))];
                    const int m = m0 + wm0 + mi * 32 + r;
                    const int n = n0 + wn0 + rc * 8;
                    if (m < M && n < N) *reinterpret_cast<uint4 *>(C + (size_t)m * N + n) = v;
                }
            }
        }
    };

    // ---- prologue: fill STAGES-1 steps
    set_load_tile(0);
#pragma unroll
    for (int st = 0; st < STAGES - 1; ++st) {
#pragma unroll
        for (int q = 0; q < 4; ++q) issue_one(q);
        advance_load();
    }
    zero_acc();
    EP_WAIT_VMCNT(8);                               // step 0 landed (steps 1, 2 may be in flight)
    __builtin_amdgcn_s_barrier();
    read_frags(0, 0, 0);

    int c_seq = 0, c_kt = 0;
    bool after_store = false;
    for (int it = 0; it < total_it; ++it) {
        const int s = it & (STAGES - 1);
        // slice 0: prefetch slice 1 of this step, multiply slice 0, issue the A loads of step it+3
        read_frags(s, 1, 1);
        EP_SCHED_FENCE();
        mfma_slice(0, 0, 1);
        EP_SCHED_FENCE();
        // slice 1: publish step it+1, retire this step's stage
        EP_WAIT_LGKMCNT0();                         // my reads of stage s are done
        if (after_store) EP_WAIT_VMCNT(0); else EP_WAIT_VMCNT(6);   // step it+1 landed
        after_store = false;
        __builtin_amdgcn_s_barrier();
        read_frags((it + 1) & (STAGES - 1), 0, 0);
        EP_SCHED_FENCE();
        mfma_slice(1, 2, 3);
        EP_SCHED_FENCE();
        advance_load();
        if (++c_kt == KT) {
            int m0, n0;
            tile_origin(c_seq, m0, n0);
            epilogue(m0, n0, s);                    // stage s was retired by the barrier above
            zero_acc();
            c_kt = 0;
            ++c_seq;
            after_store = true;
            __builtin_amdgcn_s_barrier();           // staging reads done before stage s is refilled
        }
    }
    EP_WAIT_VMCNT(0);                               // drain the dummy tail loads before LDS is released
#endif
}

template <int EPI>
hipError_t launch_persistent(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                             void *C, int M, int N, int K, hipStream_t s)
{
    auto kern = gemm_bf16_persistent_kernel<EPI>;
    static bool attr_set = false;
    static int grid_cached = 0;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM_BYTES);
        if (e != hipSuccess) return e;
        int dev = 0, cus = 0;
        if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
        if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
        grid_cached = cus / NUM_XCD * NUM_XCD;
        if (grid_cached < NUM_XCD) grid_cached = NUM_XCD;
        attr_set = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(grid_cached), dim3(NW * 64), SMEM_BYTES, s, A, W, bias, resid, C, M, N, K,
                       tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

bool ep_bf16_gemm_persistent_supported(int64_t M, int N, int K)
{
    return M > 0 && N > 0 && K >= BK * STAGES && K % BK == 0 && N % 8 == 0 &&
           M * (int64_t)K * 2 < 0x7FFFFFF0ll && (int64_t)N * K * 2 < 0x7FFFFFF0ll && M * (int64_t)N < (1ll << 31);
}

hipError_t ep_bf16_gemm_persistent(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                                   void *C, int64_t M, int N, int K, int epi, hipStream_t s)
{
    if (!ep_bf16_gemm_persistent_supported(M, N, K)) return hipErrorInvalidValue;
    if (epi == EPI_BIAS_RESID && !resid) return hipErrorInvalidValue;
    switch (epi) {
    case EPI_BIAS: return launch_persistent<EPI_BIAS>(A, W, bias, resid, C, (int)M, N, K, s);
    case EPI_BIAS_GELU: return launch_persistent<EPI_BIAS_GELU>(A, W, bias, resid, C, (int)M, N, K, s);
    case EPI_BIAS_RESID: return launch_persistent<EPI_BIAS_RESID>(A, W, bias, resid, C, (int)M, N, K, s);
    }
    return hipErrorInvalidValue;
}
