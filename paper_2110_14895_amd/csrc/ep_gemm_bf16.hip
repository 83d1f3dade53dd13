// bf16 MFMA GEMM for the dense layers of a ViT encoder layer (paper section
// 2.1: q|k|v projection, attention output projection, the two MLP layers; the
// paper's per-layer timing in section 5.1 locates most of a layer's time here).
//
//   C[M, N] = A[M, K] . W[N, K]^T + bias[N]   (+ erf GELU | + fp32 residual)
//
// A: bf16 activations, W: bf16 weights [out, in], both K-contiguous, fp32
// accumulation on the matrix cores (v_mfma_f32_16x16x32_bf16).
//
// This file holds the one-tile-per-workgroup kernel used for problems too small
// for the persistent kernel (ep_gemm_bf16_persist.hip) and the dispatcher
// ep_bf16_gemm.
//
// Tiling.  A workgroup owns a BM x BN tile of C and walks K in steps of BK (128,
// 64 or 32).  Each K step's A and W panels live in LDS as rows of 16-byte chunks;
// chunk c of row r is stored at slot c ^ f(r) (f below), which makes the MFMA
// fragment reads bank-conflict free without padding.  The panels go from global
// memory straight into LDS (buffer_load ... lds), STAGES - 1 steps ahead of the
// MFMAs, with explicit s_waitcnt counts and one bare s_barrier per step.
// Waves are laid out WM x WN; each wave keeps (BN/WN/16) x (BM/WM/16)
// accumulators of 16x16 (the 16x16x32 form of the instruction draws less power
// per flop than 32x32x16, and power is what limits the clock in these loops).
//
// Operand roles are swapped with respect to C: the MFMA "A" operand is the W
// fragment (rows = output columns n) and the "B" operand is the activation
// fragment (columns = output rows m), so that a lane holds four consecutive
// n of one row m and the epilogue works on 8- or 16-byte vectors.
//
// Workgroup -> tile mapping: consecutive workgroup ids land on different XCDs
// (8 of them, each with its own L2), so ids are first regrouped per XCD, and
// inside an XCD tiles are visited in groups of GROUP_M tile rows so that
// concurrently running workgroups share A row panels and W column panels.
//
// Ragged edges: rows beyond M and columns beyond N are read as zeros (per-lane
// buffer offsets past the end of the buffer) and never stored.  K % 64 == 0 and
// N % 8 == 0 required.
//
// Dispatcher: when 256-row tiles fill the chip the persistent kernel takes the
// problem, its tile walk stopping up to two tile rows short of M when that saves
// a round of tiles (the remaining rows are computed by the tail phase of the same
// launch); everything else runs here.
#include <cstdint>
#include "ep_kernels.h"
#include "ep_device.h"
#include "ep_launch.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 4;


#if defined(__HIP_DEVICE_COMPILE__)   // buffer-resource builtins exist only in the device pass
// Buffer resource over a dense array: loads beyond `bytes` return zero, which is
// how rows past M (or N) and K tiles past the end are handled without branches.
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
#endif

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding)
#define EP_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

// Row-dependent XOR applied to the 16-byte chunk index inside an LDS row, for
// rows of 16 chunks (BK = 128), 8 chunks (BK = 64) or 4 chunks (BK = 32).  Chosen
// so that the MFMA fragment reads (16 consecutive rows, same logical chunk) spread
// over all banks whether the LDS serves 8 or 16 lanes of a 128-bit read per cycle.
template <int BK_>
__device__ inline int swz(int row)
{
    if (BK_ == 128) return row & 15;          // a row is 256 bytes, all the banks: 16 rows take 16 different chunks
    if (BK_ == 64) return (row & 7) ^ ((row >> 3) & 1);
    return ((row >> 1) & 3) ^ ((row >> 3) & 1);
}

template <int BM, int BN, int BK_, int STAGES, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM *WN * 64, (WM * WN <= 4 && STAGES * (BM + BN) * BK_ * 2 <= 80 * 1024) ? 2 : 1) void gemm_bf16_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, const float *__restrict__ bias,
    const float *resid, void *Cout, int M, int N, int K, int k_len, int tiles_m, int tiles_n)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int NW = WM * WN;                       // waves
    constexpr int WTM = BM / WM, WTN = BN / WN;       // wave tile
    constexpr int MI = WTM / 16, NI = WTN / 16;       // 16x16 accumulators per wave
    constexpr int CPR = BK_ / 8;                      // 16-byte chunks per LDS row
    constexpr int RPI = 64 / CPR;                     // rows covered by one wave-wide 16-byte load
    constexpr int A_LD = BM / RPI / NW, W_LD = BN / RPI / NW;   // load instructions per wave per tile
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "panel must split evenly over waves");
    static_assert(BK_ % 32 == 0 && WTM % 16 == 0 && WTN % 16 == 0, "16 x 16 x 32 fragments");
    constexpr int A_STAGE = BM * CPR, W_STAGE = BN * CPR;       // uint4 per stage

    extern __shared__ uint4 lds[];                    // [STAGES][A_STAGE] then [STAGES][W_STAGE]
    uint4 *As = lds;
    uint4 *Ws = lds + STAGES * A_STAGE;

    // ---- workgroup -> (K range, tile).  EPI_PARTIAL: K is cut into K / k_len ranges, range by range over
    // all tiles (the workgroups of a range share W panels and sit on neighbouring ids of one XCD).
    const int tiles = tiles_m * tiles_n;
    const int total = EPI == EPI_PARTIAL ? tiles * (K / k_len) : tiles;
    const int per_xcd = (total + NUM_XCD - 1) / NUM_XCD;
    int lid = (int)(blockIdx.x % NUM_XCD) * per_xcd + (int)(blockIdx.x / NUM_XCD);
    if (lid >= total) return;
    const int split = EPI == EPI_PARTIAL ? lid / tiles : 0;
    lid -= split * tiles;
    const int k0 = split * k_len;
    const int group_sz = GROUP_M * tiles_n;
    const int group = lid / group_sz;
    const int first_m = group * GROUP_M;
    const int rows_in_group = min(GROUP_M, tiles_m - first_m);
    const int in_group = lid - group * group_sz;
    const int tile_m = first_m + in_group % rows_in_group;
    const int tile_n = in_group / rows_in_group;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;
    const int l15 = lane & 15, g4 = lane >> 4;

    // ---- global -> LDS, asynchronous (buffer_load ... lds): instruction i of this wave
    // fills rows (i*NW + wave)*RPI .. +RPI-1 of the panel; lane l lands at row l/CPR,
    // slot l%CPR, and therefore fetches logical chunk slot ^ swz(row).
    const __amdgpu_buffer_rsrc_t a_rs = make_rsrc(A, (uint32_t)((size_t)M * K * 2));
    const __amdgpu_buffer_rsrc_t w_rs = make_rsrc(W, (uint32_t)((size_t)N * K * 2));
    int a_off[A_LD], w_off[W_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int r = (i * NW + wave) * RPI + lane / CPR;
        const int c = (lane % CPR) ^ swz<BK_>(r);
        const int gr = m0 + r;
        a_off[i] = gr < M ? (gr * K + k0 + c * 8) * 2 : 0x7FFFFFF0;     // beyond the buffer -> zeros
    }
#pragma unroll
    for (int i = 0; i < W_LD; ++i) {
        const int r = (i * NW + wave) * RPI + lane / CPR;
        const int c = (lane % CPR) ^ swz<BK_>(r);
        const int gr = n0 + r;
        w_off[i] = gr < N ? (gr * K + k0 + c * 8) * 2 : 0x7FFFFFF0;
    }
    const int KT = k_len / BK_;
    auto issue = [&](int kt) {
        const int stage = kt % STAGES;
        // past the last K step the per-lane offset points beyond the buffer: zeros, no traffic (the
        // load is still issued so that the count of loads in flight stays fixed)
        const bool live = kt < KT;
        const int koff = live ? kt * BK_ * 2 : 0;
        typedef __attribute__((address_space(3))) void *lds_ptr;
#pragma unroll
        for (int i = 0; i < A_LD; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rs, (lds_ptr)(As + stage * A_STAGE + (i * NW + wave) * 64), 16,
                                                     live ? a_off[i] : 0x7FFFFFF0, koff, 0, 0);
#pragma unroll
        for (int i = 0; i < W_LD; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rs, (lds_ptr)(Ws + stage * W_STAGE + (i * NW + wave) * 64), 16,
                                                     live ? w_off[i] : 0x7FFFFFF0, koff, 0, 0);
    };

    f32x4 acc[NI][MI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[ni][mi][i] = 0.f;

    // fragment read offsets (uint4 units) inside a stage; the swizzle depends on the lane only.  A
    // fragment is 16 rows by 32 of K: lane l reads row l % 16 and one 8-element K chunk per quarter
    // l / 16 of the wave, the chunks dealt 0, 2, 1, 3 (both operands alike), which keeps the 16-byte reads
    // of the four quarters off each other's banks.
    const int fsw = swz<BK_>(l15);
    const int kc4 = ((g4 & 1) << 1) | (g4 >> 1);
    int a_rd[BK_ / 32], w_rd[BK_ / 32];
#pragma unroll
    for (int kk = 0; kk < BK_ / 32; ++kk) {
        a_rd[kk] = (wm0 + l15) * CPR + ((kk * 4 + kc4) ^ fsw);
        w_rd[kk] = (wn0 + l15) * CPR + ((kk * 4 + kc4) ^ fsw);
    }

    // What the epilogue adds is fetched now, ahead of the first panel loads (loads return in order, so every
    // counted wait below covers it): a small launch is a handful of K steps long and would otherwise end with
    // one more trip to memory.  The residual only where it is a few registers (tiles of at most 64 rows).
    constexpr bool PRE_RES = EPI == EPI_BIAS_RESID && MI * NI <= 8;
    float4 bias_r[NI], res_r[PRE_RES ? NI : 1][PRE_RES ? MI : 1];
    if (EPI != EPI_PARTIAL) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int n = n0 + wn0 + ni * 16 + g4 * 4;
            bias_r[ni] = n < N ? *reinterpret_cast<const float4 *>(bias + n) : make_float4(0.f, 0.f, 0.f, 0.f);
            if (PRE_RES) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    const int m = m0 + wm0 + mi * 16 + l15;
                    res_r[ni][mi] = (m < M && n < N) ? *reinterpret_cast<const float4 *>(resid + (size_t)m * N + n)
                                                     : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        }
    }

#pragma unroll
    for (int st = 0; st < STAGES - 1; ++st) issue(st);

    for (int kt = 0; kt < KT; ++kt) {
        // tile kt has landed once at most the loads of the STAGES-2 younger tiles are in flight
        EP_WAIT_VMCNT((STAGES - 2) * (A_LD + W_LD));
        __builtin_amdgcn_s_barrier();          // everyone's part of tile kt has landed; stage of tile kt-1 is free
        issue(kt + STAGES - 1);
        const uint4 *Ab = As + (kt % STAGES) * A_STAGE;
        const uint4 *Wb = Ws + (kt % STAGES) * W_STAGE;
#pragma unroll
        for (int kk = 0; kk < BK_ / 32; ++kk) {
            bf16x8 wf[NI], af[MI];
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) wf[ni] = __builtin_bit_cast(bf16x8, Wb[w_rd[kk] + ni * 16 * CPR]);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) af[mi] = __builtin_bit_cast(bf16x8, Ab[a_rd[kk] + mi * 16 * CPR]);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    acc[ni][mi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[ni], af[mi], acc[ni][mi], 0, 0, 0);
        }
    }
    EP_WAIT_VMCNT(0);                          // drain the (empty) tail loads before LDS goes away

    // ---- epilogue.  acc[ni][mi][i]: n = ni*16 + 4*(lane/16) + i, m = mi*16 + lane%16
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int m = m0 + wm0 + mi * 16 + l15;
        if (m >= M) continue;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            {
                const int n = n0 + wn0 + ni * 16 + g4 * 4;
                if (n >= N) continue;
                if (EPI == EPI_PARTIAL) {          // the bare sum over this K range, fp32, range-major
                    const float4 o = make_float4(acc[ni][mi][0], acc[ni][mi][1], acc[ni][mi][2], acc[ni][mi][3]);
                    *reinterpret_cast<float4 *>(reinterpret_cast<float *>(Cout) + ((size_t)split * M + m) * N + n) = o;
                    continue;
                }
                const float4 bb = bias_r[ni];
                float v0 = acc[ni][mi][0] + bb.x;
                float v1 = acc[ni][mi][1] + bb.y;
                float v2 = acc[ni][mi][2] + bb.z;
                float v3 = acc[ni][mi][3] + bb.w;
                const size_t off = (size_t)m * N + n;
                if (EPI == EPI_BIAS_RESID) {
                    const float4 r = PRE_RES ? res_r[PRE_RES ? ni : 0][PRE_RES ? mi : 0]
                                             : *reinterpret_cast<const float4 *>(resid + off);
                    float4 o = make_float4(v0 + r.x, v1 + r.y, v2 + r.z, v3 + r.w);
                    *reinterpret_cast<float4 *>(reinterpret_cast<float *>(Cout) + off) = o;
                } else {
                    if (EPI == EPI_BIAS_GELU) {
                        v0 = gelu_erf(v0); v1 = gelu_erf(v1); v2 = gelu_erf(v2); v3 = gelu_erf(v3);
                    }
                    uint2 o;
                    o.x = pack_bf16x2(v0, v1);
                    o.y = pack_bf16x2(v2, v3);
                    *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(Cout) + off) = o;
                }
            }
        }
    }
#endif   // __HIP_DEVICE_COMPILE__
}

template <int BM, int BN, int BK_, int STAGES, int WM, int WN, int EPI>
hipError_t launch_cfg(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                      void *C, int M, int N, int K, int splits, hipStream_t s)
{
    auto kern = gemm_bf16_kernel<BM, BN, BK_, STAGES, WM, WN, EPI>;
    constexpr size_t smem = (size_t)STAGES * (BM + BN) * (BK_ / 8) * sizeof(uint4);
    static EpSmemLimit smem_limit;
    const hipError_t e = smem_limit.ensure(reinterpret_cast<const void *>(kern), (int)smem);
    if (e != hipSuccess) return e;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int total = tiles_m * tiles_n * splits;
    const int grid = (total + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), smem, s, A, W, bias, resid, C, M, N, K, K / splits,
                       tiles_m, tiles_n);
    return hipGetLastError();
}

template <int BM, int BN, int BK_, int STAGES, int WM, int WN>
hipError_t launch_epi(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                      void *C, int M, int N, int K, int epi, hipStream_t s)
{
    switch (epi) {
    case EPI_BIAS: return launch_cfg<BM, BN, BK_, STAGES, WM, WN, EPI_BIAS>(A, W, bias, resid, C, M, N, K, 1, s);
    case EPI_BIAS_GELU: return launch_cfg<BM, BN, BK_, STAGES, WM, WN, EPI_BIAS_GELU>(A, W, bias, resid, C, M, N, K, 1, s);
    case EPI_BIAS_RESID: return launch_cfg<BM, BN, BK_, STAGES, WM, WN, EPI_BIAS_RESID>(A, W, bias, resid, C, M, N, K, 1, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

// The small-problem kernel, one tile per workgroup, 4 waves, K step 64, in four shapes.  A launch that
// cannot fill the chip is bound by the latency of its loads, one K step after the other, so where 64 x 64
// tiles still give every compute unit at most one workgroup they are used with all of the unit's LDS in
// flight: four stages of K steps of 128 (half the barriers of a step of 64: ViT-Large at micro-batch 1
// 53.8 -> 50.2 us per layer), or eight stages of 64 when K is not a multiple of 128; ViT-Large at
// micro-batch 1, 107 -> 65 us per layer against 128 x 128 tiles only.  Up to two such
// workgroups per compute unit: four stages each.  Past that, 64 x 128 tiles with three stages while they
// fit two per compute unit (128 x 128 tiles would leave a third of the units idle there: ViT-Large at
// micro-batch 4, 80 -> 74 us per layer).  Everything else runs 128 x 128 tiles with two stages, two
// workgroups per compute unit (four stages and one workgroup per unit were slower there: the second
// workgroup hides more than the deeper prefetch).
hipError_t ep_bf16_gemm_small(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                              void *C, int64_t M, int N, int K, int epi, hipStream_t s)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    if (K <= 0 || K % 64 != 0 || N % 4 != 0) return hipErrorInvalidValue;
    // byte offsets inside the kernel are 32-bit
    if (M * (int64_t)K * 2 >= 0x7FFFFFF0ll || (int64_t)N * K * 2 >= 0x7FFFFFF0ll || M * (int64_t)N >= (1ll << 31))
        return hipErrorInvalidValue;
    if (epi == EPI_BIAS_RESID && !resid) return hipErrorInvalidValue;
    int cus = 0;
    const hipError_t e = ep_device_cu_count(&cus);
    if (e != hipSuccess) return e;
    const int64_t t64 = ((M + 63) / 64) * ((N + 63) / 64);
    if (t64 <= cus && K % 128 == 0) return launch_epi<64, 64, 128, 4, 2, 2>(A, W, bias, resid, C, (int)M, N, K, epi, s);
    if (t64 <= cus) return launch_epi<64, 64, 64, 8, 2, 2>(A, W, bias, resid, C, (int)M, N, K, epi, s);
    if (t64 <= 2 * cus) return launch_epi<64, 64, 64, 4, 2, 2>(A, W, bias, resid, C, (int)M, N, K, epi, s);
    const int64_t t64x128 = ((M + 63) / 64) * ((N + 127) / 128);
    if (t64x128 <= 2 * cus) return launch_epi<64, 128, 64, 3, 2, 2>(A, W, bias, resid, C, (int)M, N, K, epi, s);
    return launch_epi<128, 128, 64, 2, 2, 2>(A, W, bias, resid, C, (int)M, N, K, epi, s);
}

// The same kernel with K cut into `splits` ranges, one workgroup per (range, tile): part[r][m][n] is the
// bare fp32 sum over range r.  For dense layers with few tiles and a long K (the second MLP layer at small
// micro-batches: ViT-Large at micro-batch 1 is 64 tiles of 64 K steps), where the chain of K steps of a
// single workgroup is the whole launch time.  Whoever consumes `part` adds the ranges in index order, so
// the result does not depend on which workgroup finishes first.
hipError_t ep_bf16_gemm_partial(const uint16_t *A, const uint16_t *W, float *part, int64_t M, int N, int K,
                                int splits, hipStream_t s)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    if (splits < 1 || K <= 0 || K % (64 * splits) != 0 || N % 4 != 0) return hipErrorInvalidValue;
    if (M * (int64_t)K * 2 >= 0x7FFFFFF0ll || (int64_t)N * K * 2 >= 0x7FFFFFF0ll || M * (int64_t)N >= (1ll << 31))
        return hipErrorInvalidValue;
    int cus = 0;
    const hipError_t e = ep_device_cu_count(&cus);
    if (e != hipSuccess) return e;
    const int64_t w64 = ((M + 63) / 64) * ((N + 63) / 64) * splits;
    if (w64 <= cus && K % (128 * splits) == 0)
        return launch_cfg<64, 64, 128, 4, 2, 2, EPI_PARTIAL>(A, W, nullptr, nullptr, part, (int)M, N, K, splits, s);
    if (w64 <= cus)
        return launch_cfg<64, 64, 64, 8, 2, 2, EPI_PARTIAL>(A, W, nullptr, nullptr, part, (int)M, N, K, splits, s);
    if (w64 <= 2 * cus)
        return launch_cfg<64, 64, 64, 4, 2, 2, EPI_PARTIAL>(A, W, nullptr, nullptr, part, (int)M, N, K, splits, s);
    return launch_cfg<128, 128, 64, 2, 2, 2, EPI_PARTIAL>(A, W, nullptr, nullptr, part, (int)M, N, K, splits, s);
}

namespace {

// How ep_bf16_gemm cuts the problem: the persistent kernel with tile width bn walks the tiles
// of rows [0, m_main) and computes rows [m_main, M) in its tail phase (bn = 0: the
// one-tile-per-workgroup kernel takes all rows).  Either way a dense layer is one launch.
struct GemmPlan { int64_t m_main; int bn; };

// Cost of the tail phase in the units of ep_bf16_gemm_persistent_cost (a round of 256 x bn tiles
// costs bn): a round of 64 x 32 tiles over the compute units takes about a tenth of a round of
// 256 x 320 tiles of the same K (3-4 us against 36 us at K = 1280).
int64_t tail_cost(int64_t tail_rows, int N)
{
    const int64_t units = ((tail_rows + 63) / 64) * ((N + 31) / 32);
    return (units + 255) / 256 * 32;
}

GemmPlan plan_gemm(int64_t M, int N, int K)
{
    // The persistent kernel (256-row tiles, one workgroup per compute unit) when its tiles fill most of
    // the chip, or already from about a hundred tiles on when the alternative, 128x128 tiles at two
    // workgroups per compute unit, would need a second round (a launch of the persistent kernel takes
    // about as long for 128 tiles as for 256, and that is less than two rounds of the small tiles:
    // 130 against 153 us for the second MLP layer at 8224 rows).  The tile walk covers all rows, or stops
    // one or two tile rows short of M and leaves the rest (at most 511 rows) to the tail phase of the
    // same launch when that saves a round of tiles: a round of the narrow tail tiles is an order of
    // magnitude cheaper.  Otherwise the 128x128 tiles, which quantise better on small micro-batches.
    if (ep_bf16_gemm_persistent_supported(M, N, K)) {
        const int64_t small_tiles = ((M + 127) / 128) * ((N + 127) / 128);
        const int64_t min_tiles = small_tiles <= 2 * (int64_t)ep_bf16_gemm_persistent_workgroups() ? 192 : 96;
        int bn_all = 0;
        const int64_t cost_all = ep_bf16_gemm_persistent_cost(M, N, &bn_all);
        const int64_t tiles_all = ((M + 255) / 256) * ((N + bn_all - 1) / bn_all);
        GemmPlan best = {M, tiles_all >= min_tiles ? bn_all : 0};
        int64_t best_cost = tiles_all >= min_tiles ? cost_all : INT64_MAX;
        for (int64_t m_main = M / 256 * 256; m_main > 0 && M - m_main < 512; m_main -= 256) {
            const int64_t tail = M - m_main;
            if (tail == 0 || !ep_bf16_gemm_skinny_supported(tail, N, K)) continue;
            int bn_main = 0;
            const int64_t cost = ep_bf16_gemm_persistent_cost(m_main, N, &bn_main) + tail_cost(tail, N);
            const int64_t tiles_main = (m_main / 256) * ((N + bn_main - 1) / bn_main);
            if (tiles_main >= min_tiles && cost < best_cost) { best = {m_main, bn_main}; best_cost = cost; }
        }
        if (best.bn) return best;
    }
    return {M, 0};
}

}  // namespace

// Into how many K ranges a dense layer with fp32 output is cut (1: not at all).  Only problems that the
// one-tile-per-workgroup kernel runs.  Such a launch is a chain of K steps per workgroup, and what a step costs
// depends on the shape class the launch falls into (measured on ViT-Base/Large/Huge second MLP layers at
// micro-batches 1 to 16, microseconds per 64-deep step): 64 x 64 tiles with one workgroup per compute unit 0.28,
// with two 0.40; 128 x 128 tiles 0.7 while they leave compute units idle, 1.0 when they double up.  Cutting K
// into sp ranges divides the chain by sp, may move the launch to a dearer class, and makes the consumer of the
// sums read sp x M x N floats more (priced at 3 TB/s: they are spread over a few hundred waves).  The cheapest
// sp of 1, 2, 4, 8 wins; every range keeps at least eight K steps and the workgroups at most two per compute unit.
int ep_bf16_gemm_splits(int64_t M, int N, int K)
{
    if (M <= 0 || N <= 0 || K <= 0 || K % 64 != 0) return 1;
    if (plan_gemm(M, N, K).bn) return 1;
    int cus = 0;
    if (ep_device_cu_count(&cus) != hipSuccess) return 1;
    const int64_t t64 = ((M + 63) / 64) * ((N + 63) / 64), t128 = ((M + 127) / 128) * ((N + 127) / 128);
    const int steps = K / 64;
    auto cost_us = [&](int sp) -> double {
        double step;
        if (t64 * sp <= cus) step = 0.28;
        else if (t64 * sp <= 2 * cus) step = 0.40;
        else if (t128 * sp <= cus) step = 0.7;
        else if (t128 * sp <= 2 * cus) step = 1.0;
        else step = 1.0 * (double)((t128 * sp + 2 * cus - 1) / (2 * cus));      // rounds of workgroups (sp == 1 only)
        const double sums = sp > 1 ? (double)sp * (double)M * N * 4.0 / 3.0e6 : 0.0;
        return (double)(steps / sp) * step + sums;
    };
    int best = 1;
    double best_cost = cost_us(1);
    for (int sp = 2; sp <= 8; sp *= 2) {
        if (steps % sp != 0 || steps / sp < 8) break;
        if ((t64 * sp <= 2 * cus ? t64 : t128) * sp > 2 * cus) break;
        const double c = cost_us(sp);
        if (c < best_cost - 1.0) { best = sp; best_cost = c; }      // a microsecond is within the noise of the model
    }
    return best;
}

int64_t ep_bf16_gemm_main_rows(int64_t M, int N, int K)
{
    (void)N; (void)K;
    return M;                                        // a dense layer is one launch over all its rows
}

hipError_t ep_bf16_gemm(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                        void *C, int64_t M, int N, int K, int epi, hipEvent_t after_main, hipStream_t s)
{
    const GemmPlan p = plan_gemm(M, N, K);
    hipError_t e = p.bn ? ep_bf16_gemm_persistent(A, W, bias, resid, C, M, p.m_main, N, K, epi, p.bn, true, s)
                        : ep_bf16_gemm_small(A, W, bias, resid, C, M, N, K, epi, s);
    if (e != hipSuccess) return e;
    if (after_main) e = hipEventRecord(after_main, s);
    return e;
}
