// Persistent bf16 MFMA GEMM for the large dense layers of an encoder layer
// (paper section 2.1; section 5.1 attributes most of a layer's time to them).
//
//   C[M, N] = A[M, K] . W[N, K]^T + bias[N]   (+ erf GELU | + fp32 residual)
//
// One workgroup per compute unit stays resident and walks a static list of
// 256 x BN output tiles (BN = 256 or 320, chosen per problem so that the tile
// count is a multiple of the number of compute units where possible); the K
// loop of consecutive tiles forms one continuous software pipeline, so the
// first K step of the next tile is already in LDS when a tile is stored.
//
// Pipeline (per workgroup, 8 waves, two per SIMD):
//   - K advances in steps of 64 (rows of 128 bytes = whole cache lines, which the
//     L2 -> LDS path moves ~1.6x faster than half lines).  A step's A and W
//     panels go from global memory straight into LDS with buffer_load ... lds
//     (no register staging), two stages; the loads a wave issues per step are
//     slipped one by one between MFMAs, dealt over three quarters of a step:
//     the first right after the barrier that retires the stage they overwrite,
//     the rest in the first two quarters of the following step (a burst of all
//     of them holds every wave at the door of the memory pipeline at once); the
//     last of them still has half a step to land.
//   - LDS rows are 8 chunks of 16 bytes; chunk c of row r sits at slot
//     c ^ f(r), f(r) = (r & 7) ^ ((r >> 3) & 1): the 16-byte fragment reads of 16
//     consecutive rows are conflict-free on the 64-bank LDS (with the K chunks
//     dealt to the quarters of a wave in the order 0, 2, 1, 3).
//   - The matrix instruction is v_mfma_f32_16x16x32_bf16: at the power limit
//     the chip runs the same flops about 15 % faster in this form than as
//     32 x 32 x 16.  A 32-wide slice of the wave tile is multiplied in four
//     units of (half the activation fragments) x (half the weight fragments),
//     ordered so that consecutive units share one of their halves; the
//     registers of a retired half take the fragments needed two units later,
//     every LDS read is issued between two MFMAs at least a unit ahead of its
//     use, and a wave has no phase without matrix work except the one barrier
//     per step.
// Epilogue: 32 x 32 blocks of accumulators (+bias, GELU) are transposed through the
// W part of the LDS stage the tile's last step has just retired (4 KB per wave),
// so that global stores and residual loads are whole row segments; the refill of
// the stage's A part for the next tile is already under way meanwhile (issued
// before the epilogue, like after any other step), the rest follows it.  The
// tile's bias values wait in LDS (loaded there during the K loop).
//
// Operand roles are swapped (MFMA A = W fragment, B = activation fragment) so
// that a lane owns 4 consecutive output columns of one row.
//
// Workgroup w runs on XCD w % 8 (round-robin dispatch); in every round the 32
// workgroups of an XCD take 32 consecutive tiles of an order that walks groups
// of 4 tile rows column by column, so that they share A and W panels in L2.
//
// Requirements: K % 64 == 0, K >= 128, N % 8 == 0; M*K*2, N*K*2 < 2^31.  Rows
// past M and columns past N are read as zeros (per-lane buffer offsets beyond
// the end of the buffer) and never stored.  `m_rows` <= M limits the rows the
// tile walk computes.  The remaining rows are left to the caller, or, with
// `fuse_tail`, computed in the same launch: after its last tile a workgroup
// takes narrow tiles of rows [m_rows, M) (the short-M tile routine: 64, 32 or
// 16 rows by 32 columns, as narrow as it takes to give every workgroup one; K
// dealt to the 8 waves, fixed-order sum through LDS), which saves the launch and
// ramp of a second kernel when M is a few rows more than a multiple of 256.
#include "ep_kernels.h"
#include "ep_device.h"
#include "ep_gemm_bf16_skinny_tile.h"
#include "ep_launch.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BK = 64, STAGES = 2;
constexpr int NW = 8;                                // waves
constexpr int CPR = BK / 8;                          // 8 chunks of 16 B per LDS row
constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 4;

// Tile shape: BN columns, waves laid out WM x WN, wave tile (BM/WM) x (BN/WN).
template <int BN_, int WM_, int WN_>
struct Tile {
    static constexpr int BN = BN_, WM = WM_, WN = WN_;
    static constexpr int MI = BM / WM / 32, NI = BN / WN / 32;        // 32 x 32 blocks of the wave tile (epilogue)
    static constexpr int MI16 = 2 * MI, NI16 = 2 * NI;                // 16 x 16 accumulators per wave
    static constexpr int A_STAGE = BM * CPR, W_STAGE = BN * CPR;      // uint4 per stage and operand
    static constexpr int STAGE_U4 = A_STAGE + W_STAGE;
    static constexpr int LDA = BM / 8 / NW, LDW = BN / 8 / NW;        // loads per wave per step (8 rows each)
    static constexpr size_t SMEM = (size_t)(STAGES * STAGE_U4 + BN / 4) * sizeof(uint4);   // stages + the tile's bias
    static_assert(WM * WN == NW && BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BN % (8 * NW) == 0, "tile shape");
    // A step's loads are dealt over three groups (a burst of all of them holds every wave at the memory
    // pipeline's door at once): [0, P0) right after the barrier that retires the stage they fill, [P0, P1)
    // in the first unit of the next step and [P1, LDA+LDW) in its third unit - or, in the `early` variant
    // of the kernel, one load more in the first group and the last group in the second unit.  The early
    // variant serves launches of a single round of tiles, where every operand line is a first touch for
    // its L2 and takes longer to arrive (FC2 at 16448 rows: -5.8 us); where a workgroup walks several
    // tiles and finds the W panels of its earlier ones in L2, it costs time (FC1 at 65792 rows: +4.5 %).
    template <bool EARLY>
    struct Deal {
        static constexpr int P0 = EARLY ? 4 : 3, P1 = P0 + 3, LAST_UNIT = EARLY ? 1 : 2;
        static_assert(P1 < LDA + LDW, "three groups of loads");
        // the first group refills the A part of a retired stage while the epilogue stages through its W part
        static_assert(P0 <= LDA, "first loads: A panel only");
    };
    static_assert(W_STAGE >= NW * 256, "4 KB of epilogue staging per wave in the W part of a stage");
};
typedef Tile<256, 2, 4> Tile256;                     // wave tile 128 x 64
typedef Tile<320, 4, 2> Tile320;                     // wave tile 64 x 160

}  // namespace

// Measurement: the shader-cycle counter and the constant 100 MHz counter read by workgroup 0 at the
// start ([0], [1]) and at the end ([2], [3]) of the most recent launch on this device; their ratio
// is the shader clock that launch ran at (ep_gemm_clock_sample).
static __device__ unsigned long long g_clock_sample[4];

namespace {

#define EP_WAIT_VMCNT0() __builtin_amdgcn_s_waitcnt(0x0 | (0x0 << 14) | (0x7 << 4) | (0xF << 8))
#define EP_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4) | (0x0 << 8))
#define EP_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

__device__ inline int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <class T, int EPI, bool EARLY>
__global__ __launch_bounds__(NW * 64, 1) void gemm_bf16_persistent_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, const float *__restrict__ bias,
    const float *resid, void *Cout, int M, int m_rows, int N, int K, int tiles_m, int tiles_n, int tail_rows, int tail_tm)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int BN = T::BN, WN = T::WN, MI = T::MI, NI = T::NI;
    constexpr int A_STAGE = T::A_STAGE, STAGE_U4 = T::STAGE_U4, LDA = T::LDA, LDW = T::LDW;
    typedef typename T::template Deal<EARLY> Deal;
    constexpr int NLD = LDA + LDW, P0 = Deal::P0, P1 = Deal::P1, LAST_UNIT = Deal::LAST_UNIT;

    extern __shared__ uint4 lds[];                   // [STAGES][A panel | W panel]
    typedef __attribute__((address_space(3))) void *lds_ptr;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: wave-derived addressing stays scalar
    if (blockIdx.x == 0 && tid == 0) {
        g_clock_sample[0] = clock64();
        g_clock_sample[1] = wall_clock64();
    }
    const int wm0 = (wave / WN) * (MI * 32), wn0 = (wave % WN) * (NI * 32);

    // ---- this workgroup's tile list: tile j has logical id j*G + (w%8)*(G/8) + w/8
    const int G = gridDim.x;                         // multiple of 8
    const int total = tiles_m * tiles_n;
    const int first_id = (int)(blockIdx.x % NUM_XCD) * (G / NUM_XCD) + (int)(blockIdx.x / NUM_XCD);
    if (first_id >= total && tail_rows == 0) return;
    const int n_my = first_id < total ? (total - first_id + G - 1) / G : 0;
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

    // ---- load stream: one K step ahead of the multiply stream
    const __amdgpu_buffer_rsrc_t a_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(A), 0, (int)((size_t)M * K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(W), 0, (int)((size_t)N * K * 2), 0x00020000);
    constexpr int OOB = 0x7FFFFFF0;
    // load i of a wave fills panel rows (i*NW + wave)*8 .. +7; lane l lands at row l/8, slot l%8 and
    // fetches chunk slot ^ swz(row); swz sees the row only through l/8 and the parity of wave (NW
    // is even), so one per-lane offset serves every i.  Out-of-range handling relies on the per-lane
    // (VGPR) offset alone, which the buffer bounds check always covers.
    const int row_lane = wave * 8 + (lane >> 3);
    const int lane_off = (row_lane * K + ((lane & 7) ^ swz(row_lane)) * 8) * 2;
    const int istride = NW * 8 * K * 2;              // bytes between loads i and i+1
    int ld_seq = 0, ld_kt = 0, ld_stage = 0;
    int a_tile = OOB, w_tile = OOB;                  // byte offset of the tile's first A / W row, or OOB
    int a_rows = 0, w_rows = 0;                      // valid panel rows of the tile
    auto set_load_tile = [&](int seq) {
        int m0 = 0, n0 = 0;
        const bool live = seq < n_my;
        if (live) tile_origin(seq, m0, n0);
        a_tile = live ? m0 * K * 2 : OOB;
        w_tile = live ? n0 * K * 2 : OOB;
        a_rows = live ? M - m0 : 0;
        w_rows = live ? N - n0 : 0;
    };
    // which: 0 .. LDA-1 = A panel, LDA .. LDA+LDW-1 = W panel
    auto issue_one = [&](int which) {
        const int koff = ld_kt * (BK * 2);
        uint4 *dst = lds + ld_stage * STAGE_U4;
        if (which < LDA) {
            const bool ok = which * NW * 8 + row_lane < a_rows;
            const int vo = ok ? lane_off + a_tile + which * istride : OOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rs, (lds_ptr)(dst + (which * NW + wave) * 64), 16, vo, koff, 0, 0);
        } else {
            const int i = which - LDA;
            const bool ok = i * NW * 8 + row_lane < w_rows;
            const int vo = ok ? lane_off + w_tile + i * istride : OOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rs, (lds_ptr)(dst + A_STAGE + (i * NW + wave) * 64), 16, vo, koff, 0, 0);
        }
    };
    auto advance_load = [&]() {
        ld_stage ^= 1;
        if (++ld_kt == KT) {
            ld_kt = 0;
            set_load_tile(++ld_seq);
        }
    };

    // ---- fragments and accumulators (v_mfma_f32_16x16x32_bf16).  A fragment is 16 panel rows by 32 of K
    // (lane l: row l % 16, one 8-element K chunk per quarter l / 16 of the wave); accumulator (wi, ai) <->
    // columns wi*16 + 4*(l/16) + i, row ai*16 + l%16.  A 32-wide slice of the wave tile is multiplied in four
    // units (P half, H half): P is the side with fewer fragments, both sides are split in halves, and the
    // units run (a,0) (b,0) (b,1) (a,1) with a, b swapping from slice to slice, so that from one unit to the
    // next only one half changes and the registers of the half just retired take the fragments needed two
    // units later: one slice's worth of fragment registers in all, every read a unit or more ahead.
    constexpr int MI16 = T::MI16, NI16 = T::NI16;
    constexpr bool P_ACT = MI16 <= NI16;
    constexpr int PH = (P_ACT ? MI16 : NI16) / 2, HH = (P_ACT ? NI16 : MI16) / 2;
    constexpr int UM = PH * HH;                      // MFMAs per unit
    static_assert(PH + 2 * HH <= 2 * UM && 2 * HH <= UM && (UM + 1) / 2 >= P0 && (UM + 1) / 2 >= P1 - P0 &&
                      (UM + 1) / 2 >= NLD - P1,
                  "reads and loads fit between the MFMAs of their units");
    // quarter g4 of the wave multiplies K chunk kc4 of a slice (any assignment works as long as both
    // operands use it); 0, 2, 1, 3 keeps the 16-byte reads of the four quarters off each other's banks.
    // The offsets are derived again after every epilogue (from a lane index the compiler cannot see
    // through), so that they do not occupy registers while a tile is stored.
    int p_off[2], h_off[2];                          // per 32-wide slice
    auto derive_read_offsets = [&]() {
        int le = lane;
        asm volatile("" : "+v"(le));
        const int l15 = le & 15, g4 = le >> 4;
        const int fsw = swz(l15), kc4 = ((g4 & 1) << 1) | (g4 >> 1);
        const int p_row = P_ACT ? (wm0 + l15) * CPR : A_STAGE + (wn0 + l15) * CPR;
        const int h_row = P_ACT ? A_STAGE + (wn0 + l15) * CPR : (wm0 + l15) * CPR;
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            p_off[sl] = p_row + ((sl * 4 + kc4) ^ fsw);
            h_off[sl] = h_row + ((sl * 4 + kc4) ^ fsw);
        }
    };
    derive_read_offsets();
    bf16x8 fp[2][PH], fh[2][HH];
    f32x4 acc[NI16][MI16];
    auto read_p = [&](const uint4 *base, int slice, int half, int j) {
        fp[half][j] = __builtin_bit_cast(bf16x8, base[p_off[slice] + (half * PH + j) * 16 * CPR]);
    };
    auto read_h = [&](const uint4 *base, int slice, int half, int j) {
        fh[half][j] = __builtin_bit_cast(bf16x8, base[h_off[slice] + (half * HH + j) * 16 * CPR]);
    };
    auto zero_acc = [&]() {
#pragma unroll
        for (int wi = 0; wi < NI16; ++wi)
#pragma unroll
            for (int ai = 0; ai < MI16; ++ai)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[wi][ai][i] = 0.f;
    };
    // MFMA q of unit (hp, hh): the P fragments back and forth under each H fragment, so that consecutive
    // MFMAs share one operand (a little faster than changing both)
    auto mfma_one = [&](int hp, int hh, int q) {
        const int jh = q / PH, jp = (jh & 1) ? PH - 1 - q % PH : q % PH;
        const int ip = hp * PH + jp, ih = hh * HH + jh;
        if (P_ACT)
            acc[ih][ip] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fh[hh][jh], fp[hp][jp], acc[ih][ip], 0, 0, 0);
        else
            acc[ip][ih] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fp[hp][jp], fh[hh][jh], acc[ip][ih], 0, 0, 0);
    };

    // The BN bias values of a tile sit in LDS behind the stages, brought there with 4-byte
    // global -> LDS loads when the tile before it is stored (columns past N read as zeros), so the
    // epilogue gets its lane's four values with one LDS read and no select between the quarters of
    // the wave; the loads ride on the K loop's own waits.
    float *bias_lds = reinterpret_cast<float *>(lds + STAGES * STAGE_U4);
    const __amdgpu_buffer_rsrc_t b_rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(bias), 0, N * 4, 0x00020000);
    auto issue_bias = [&](int seq) {                 // wave w brings columns w*64 .. w*64+63 of tile seq
        if (wave < BN / 64 && seq < n_my) {
            int m0, n0;
            tile_origin(seq, m0, n0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rs, (lds_ptr)(bias_lds + wave * 64), 4, (n0 + wave * 64 + lane) * 4, 0,
                                                     0, 0);
        }
    };
    auto bias4 = [&](int col, int g4) {              // col: column inside the tile, a multiple of 16; g4 = lane / 16
        return *reinterpret_cast<const float4 *>(bias_lds + col + 4 * g4);
    };

    // ---- epilogue of the tile at (m0, n0); `stage` has just been retired and is free LDS.
    // It goes by 32 x 32 blocks: four accumulators (wj, aj) each.
    auto epilogue = [&](int m0, int n0, int stage) {
        // the lane-dependent addressing of the epilogue is derived afresh for every tile from a lane index
        // the compiler cannot see through: otherwise it computes all of it ahead of the K loop, where the
        // values do not fit in registers next to the accumulators and come back from scratch memory
        int le = lane;
        asm volatile("" : "+v"(le));
        const int l15 = le & 15, g4 = le >> 4, lane = le;
        uint4 *stg = lds + stage * STAGE_U4 + A_STAGE + wave * 256; // 4 KB of the W panel's part
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int nblk = n0 + wn0 + ni * 32, mblk = m0 + wm0 + mi * 32;
                if (EPI == EPI_BIAS_RESID) {
                    // block [32 m][32 n] fp32: rows of 128 B = 8 chunks of 4 floats
                    float *C = reinterpret_cast<float *>(Cout);
                    float4 bq[2];
#pragma unroll
                    for (int wj = 0; wj < 2; ++wj) bq[wj] = bias4(wn0 + ni * 32 + wj * 16, g4);
#pragma unroll
                    for (int aj = 0; aj < 2; ++aj)
#pragma unroll
                        for (int wj = 0; wj < 2; ++wj) {
                            const f32x4 c = acc[ni * 2 + wj][mi * 2 + aj];
                            const float4 bb = bq[wj];
                            const int r = aj * 16 + l15;
                            *reinterpret_cast<float4 *>(&stg[r * 8 + ((wj * 4 + g4) ^ (r & 7))]) =
                                make_float4(c[0] + bb.x, c[1] + bb.y, c[2] + bb.z, c[3] + bb.w);
                        }
                    const int rrow = lane >> 3, rc = lane & 7;      // read-back: 8 rows x 8 chunks per pass
                    float4 v[4], x[4];
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const int r = p * 8 + rrow, m = mblk + r, n = nblk + rc * 4;
                        x[p] = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (m < m_rows && n < N) x[p] = *reinterpret_cast<const float4 *>(resid + (size_t)m * N + n);
                        v[p] = *reinterpret_cast<const float4 *>(&stg[r * 8 + (rc ^ (r & 7))]);
                    }
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const int r = p * 8 + rrow, m = mblk + r, n = nblk + rc * 4;
                        if (m < m_rows && n < N)
                            *reinterpret_cast<float4 *>(C + (size_t)m * N + n) =
                                make_float4(v[p].x + x[p].x, v[p].y + x[p].y, v[p].z + x[p].z, v[p].w + x[p].w);
                    }
                } else {
                    // block [32 m][32 n] bf16: rows of 64 B = 4 chunks of 8 bf16; chunk c of row r sits at slot
                    // c ^ ((r >> 2) & 3): four rows span the 64 banks, so the 8-byte writes of 32 rows meet two to
                    // a bank (the best a 64-byte row stride allows) and the 16-byte reads of 4 rows not at all
                    uint16_t *C = reinterpret_cast<uint16_t *>(Cout);
                    float4 bq[2];
#pragma unroll
                    for (int wj = 0; wj < 2; ++wj) bq[wj] = bias4(wn0 + ni * 32 + wj * 16, g4);
#pragma unroll
                    for (int aj = 0; aj < 2; ++aj)
#pragma unroll
                        for (int wj = 0; wj < 2; ++wj) {
                            const f32x4 c = acc[ni * 2 + wj][mi * 2 + aj];
                            const float4 bb = bq[wj];
                            float v0 = c[0] + bb.x, v1 = c[1] + bb.y, v2 = c[2] + bb.z, v3 = c[3] + bb.w;
                            if (EPI == EPI_BIAS_GELU) {
                                v0 = gelu_erf(v0); v1 = gelu_erf(v1); v2 = gelu_erf(v2); v3 = gelu_erf(v3);
                            }
                            uint2 o;
                            o.x = pack_bf16x2(v0, v1);
                            o.y = pack_bf16x2(v2, v3);
                            const int r = aj * 16 + l15;
                            reinterpret_cast<uint2 *>(&stg[r * 4 + ((wj * 2 + (g4 >> 1)) ^ ((r >> 2) & 3))])[g4 & 1] = o;
                        }
                    const int rrow = lane >> 2, rc = lane & 3;      // read-back: 16 rows x 4 chunks per pass
#pragma unroll
                    for (int p = 0; p < 2; ++p) {
                        const int r = p * 16 + rrow, m = mblk + r, n = nblk + rc * 8;
                        const uint4 v = stg[r * 4 + (rc ^ ((r >> 2) & 3))];
                        if (m < m_rows && n < N) *reinterpret_cast<uint4 *>(C + (size_t)m * N + n) = v;
                    }
                }
            }
        }
    };

    // ---- prologue: step 0 into stage 0, wait, first fragments; then the first loads of step 1 into stage 1
    set_load_tile(0);
#pragma unroll
    for (int q = 0; q < LDA + LDW; ++q) issue_one(q);
    advance_load();
    issue_bias(0);
    zero_acc();
    EP_WAIT_VMCNT0();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int j = 0; j < PH; ++j) read_p(lds, 0, 0, j);
#pragma unroll
    for (int j = 0; j < HH; ++j) read_h(lds, 0, 0, j);
#pragma unroll
    for (int q = 0; q < P0; ++q) issue_one(q);

    int c_seq = 0, c_kt = 0;
    for (int it = 0; it < total_it; ++it) {
        const uint4 *cur = lds + (it & 1) * STAGE_U4;
        const uint4 *nxt = lds + ((it + 1) & 1) * STAGE_U4;
        const bool tile_end = c_kt == KT - 1;
        // two 32-wide slices of four units; the stage swap sits before the last two units of the step
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int pa = s, pb = s ^ 1;                   // P half of units 0, 3 and of units 1, 2
                const int hp = (u == 0 || u == 3) ? pa : pb, hh = u >> 1;
                const bool post = s == 1 && u >= 2;
                if (s == 1 && u == 2) {
                    advance_load();
                    // all my reads of this stage are done; the next step has landed; swap
                    EP_WAIT_LGKMCNT0();
                    EP_WAIT_VMCNT0();
                    __builtin_amdgcn_s_barrier();
                }
                const uint4 *src = post ? nxt : cur;            // units 2, 3 read the slice after this one
                const int rs = u < 2 ? s : (s ^ 1);
#pragma unroll
                for (int q = 0; q < UM; ++q) {
                    mfma_one(hp, hh, q);
                    if (s == 0 && u == 0 && q == 0) EP_SCHED_FENCE();   // the step's first MFMA waits for old reads only
                    // fragment reads: the P half of unit 1 first, the H half of units 2, 3 at every other
                    // MFMA of units 0, 1; the next slice's H half at every other MFMA of unit 2 and its P half
                    // at the start of unit 3 (the loads below take the MFMA slots in between)
                    if (u == 0 && q < PH) read_p(src, rs, pb, q);
                    if (u < 2) {
                        const int t = u * UM + q - PH;          // slots after the P reads
                        if (t >= 0 && (t & 1) && (t >> 1) < HH) read_h(src, rs, 1, t >> 1);
                    }
                    if (u == 2 && (q & 1) && (q >> 1) < HH) read_h(src, rs, 0, q >> 1);
                    if (u == 3 && q < PH) read_p(src, rs, pb, q);
                    if ((q & 1) == 0) {                         // the loads keep their spacing of two MFMA slots
                        const int k = q >> 1;
                        if (s == 0 && u == 0 && P0 + k < P1) issue_one(P0 + k);
                        if (s == 0 && u == LAST_UNIT && P1 + k < NLD) issue_one(P1 + k);
                        if (post && u == 2 && k < P0) issue_one(k);
                    }
                    EP_SCHED_FENCE();
                }
            }
        }
        if (tile_end) {
            int m0, n0;
            tile_origin(c_seq, m0, n0);
            epilogue(m0, n0, it & 1);
            zero_acc();
            c_kt = 0;
            ++c_seq;
            EP_WAIT_LGKMCNT0();
            __builtin_amdgcn_s_barrier();           // every wave is done with the staging area and the bias
            issue_bias(c_seq);
            derive_read_offsets();
        } else {
            ++c_kt;
        }
    }
    EP_WAIT_VMCNT0();                               // drain the tail loads before LDS is released
    // ---- rows [m_rows, m_rows + tail_rows): tail_tm x 32 tiles, dealt to the workgroups from the end
    // of the tile order backwards (those are the ones with a tile less when the tiles do not divide)
    if (tail_rows > 0) {
        __syncthreads();
        const int tn = (N + ep_skinny::TN - 1) / ep_skinny::TN;
        const int units = tn * ((tail_rows + tail_tm - 1) / tail_tm);
        float *scratch = reinterpret_cast<float *>(lds);
        for (int u = G - 1 - first_id; u < units; u += G) {
            const int tm0 = m_rows + (u / tn) * tail_tm, tn0 = (u % tn) * ep_skinny::TN;
            if (tail_tm == 64)
                ep_skinny::tile<EPI, 64>(A, W, bias, resid, Cout, m_rows + tail_rows, N, K, tm0, tn0, scratch);
            else if (tail_tm == 32)
                ep_skinny::tile<EPI, 32>(A, W, bias, resid, Cout, m_rows + tail_rows, N, K, tm0, tn0, scratch);
            else
                ep_skinny::tile16<EPI>(A, W, bias, resid, Cout, m_rows + tail_rows, N, K, tm0, tn0, scratch);
            __syncthreads();
        }
    }
    if (blockIdx.x == 0 && tid == 0) {
        g_clock_sample[2] = clock64();
        g_clock_sample[3] = wall_clock64();
    }
#endif
}

// Rows per tile (64, 32 or 16; all 32 columns wide) for the tail phase: the fewest rounds over the
// workgroups, then the fewest bytes a workgroup pulls per tile (rows + 32 panel rows of K elements).
int pick_tail_rows(int tail_rows, int N, int wgs)
{
    const int tn = (N + 31) / 32;
    int best = 64;
    int64_t best_cost = -1;
    for (int tm : {64, 32, 16}) {
        const int units = tn * ((tail_rows + tm - 1) / tm);
        const int64_t cost = (int64_t)((units + wgs - 1) / wgs) * (tm + 32);
        if (best_cost < 0 || cost < best_cost) { best = tm; best_cost = cost; }
    }
    return best;
}

// one resident workgroup per compute unit of the current device, a multiple of the number of XCDs
hipError_t resident_grid(int *grid)
{
    int cus = 0;
    const hipError_t e = ep_device_cu_count(&cus);
    if (e != hipSuccess) return e;
    *grid = cus / NUM_XCD * NUM_XCD;
    if (*grid < NUM_XCD) *grid = NUM_XCD;
    return hipSuccess;
}

template <class T, int EPI, bool EARLY>
hipError_t launch_persistent(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                             void *C, int M, int m_rows, int N, int K, int tail_rows, int g_grid, hipStream_t s)
{
    auto kern = gemm_bf16_persistent_kernel<T, EPI, EARLY>;
    static EpSmemLimit smem_limit;
    const hipError_t e = smem_limit.ensure(reinterpret_cast<const void *>(kern), (int)T::SMEM);
    if (e != hipSuccess) return e;
    const int tiles_m = (m_rows + BM - 1) / BM, tiles_n = (N + T::BN - 1) / T::BN;
    hipLaunchKernelGGL(kern, dim3(g_grid), dim3(NW * 64), T::SMEM, s, A, W, bias, resid, C, M, m_rows, N, K,
                       tiles_m, tiles_n, tail_rows, tail_rows ? pick_tail_rows(tail_rows, N, g_grid) : 0);
    return hipGetLastError();
}

template <class T>
hipError_t launch_tile(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid, void *C,
                       int M, int m_rows, int N, int K, int epi, int tail_rows, hipStream_t s)
{
    int g_grid = 0;
    const hipError_t e = resident_grid(&g_grid);
    if (e != hipSuccess) return e;
    // a single round of tiles: the variant that sends a step's loads out earlier
    const bool early = (int64_t)((m_rows + BM - 1) / BM) * ((N + T::BN - 1) / T::BN) <= g_grid;
    switch (epi * 2 + (early ? 1 : 0)) {
    case EPI_BIAS * 2: return launch_persistent<T, EPI_BIAS, false>(A, W, bias, resid, C, M, m_rows, N, K, tail_rows, g_grid, s);
    case EPI_BIAS * 2 + 1: return launch_persistent<T, EPI_BIAS, true>(A, W, bias, resid, C, M, m_rows, N, K, tail_rows, g_grid, s);
    case EPI_BIAS_GELU * 2: return launch_persistent<T, EPI_BIAS_GELU, false>(A, W, bias, resid, C, M, m_rows, N, K, tail_rows, g_grid, s);
    case EPI_BIAS_GELU * 2 + 1: return launch_persistent<T, EPI_BIAS_GELU, true>(A, W, bias, resid, C, M, m_rows, N, K, tail_rows, g_grid, s);
    case EPI_BIAS_RESID * 2: return launch_persistent<T, EPI_BIAS_RESID, false>(A, W, bias, resid, C, M, m_rows, N, K, tail_rows, g_grid, s);
    case EPI_BIAS_RESID * 2 + 1: return launch_persistent<T, EPI_BIAS_RESID, true>(A, W, bias, resid, C, M, m_rows, N, K, tail_rows, g_grid, s);
    }
    return hipErrorInvalidValue;
}

// Rounds of tiles over `cus` compute units, weighted by the tile width: the cost of a tile
// shape for this problem.
int64_t tile_cost(int64_t rows, int N, int bn, int cus)
{
    const int64_t tiles = ((rows + BM - 1) / BM) * ((N + bn - 1) / bn);
    return (tiles + cus - 1) / cus * bn;
}

}  // namespace

hipError_t ep_bf16_gemm_persistent_clock(double *shader_mhz, double *seconds)
{
    unsigned long long h[4] = {0, 0, 0, 0};
    const hipError_t e = hipMemcpyFromSymbol(h, HIP_SYMBOL(g_clock_sample), sizeof(h));
    if (e != hipSuccess) return e;
    const double cycles = (double)(h[2] - h[0]), ticks = (double)(h[3] - h[1]);     // ticks of 10 ns
    if (h[3] <= h[1] || h[2] <= h[0]) return hipErrorNotReady;      // no launch has finished on this device yet
    *shader_mhz = cycles / ticks * 100.0;
    *seconds = ticks * 1e-8;
    return hipSuccess;
}

bool ep_bf16_gemm_persistent_supported(int64_t M, int N, int K)
{
    return M > 0 && N > 0 && K >= 2 * BK && K % BK == 0 && N % 8 == 0 &&
           M * (int64_t)K * 2 < 0x7FFFFFF0ll && (int64_t)N * K * 2 < 0x7FFFFFF0ll && M * (int64_t)N < (1ll << 31);
}

int ep_bf16_gemm_persistent_workgroups()
{
    int g = 0;
    return resident_grid(&g) == hipSuccess ? g : 256;
}

int64_t ep_bf16_gemm_persistent_cost(int64_t rows, int N, int *tile_bn)
{
    const int cus = ep_bf16_gemm_persistent_workgroups();
    const int64_t c256 = tile_cost(rows, N, 256, cus), c320 = tile_cost(rows, N, 320, cus);
    if (tile_bn) *tile_bn = c320 <= c256 ? 320 : 256;      // a tie goes to the wider tile (fewer bytes loaded per flop)
    return c320 <= c256 ? c320 : c256;
}

// tile_bn: 0 = choose, else 256 or 320.  m_rows <= M: the tile walk covers rows [0, m_rows);
// fuse_tail: rows [m_rows, M) are computed by the same launch as 64 x 32 tiles.
hipError_t ep_bf16_gemm_persistent(const uint16_t *A, const uint16_t *W, const float *bias, const float *resid,
                                   void *C, int64_t M, int64_t m_rows, int N, int K, int epi, int tile_bn,
                                   bool fuse_tail, hipStream_t s)
{
    if (!ep_bf16_gemm_persistent_supported(M, N, K) || m_rows < 0 || m_rows > M) return hipErrorInvalidValue;
    if (epi == EPI_BIAS_RESID && !resid) return hipErrorInvalidValue;
    if (m_rows == 0) return hipSuccess;
    const int tail = fuse_tail ? (int)(M - m_rows) : 0;
    if (tile_bn == 0) (void)ep_bf16_gemm_persistent_cost(m_rows, N, &tile_bn);
    if (tile_bn == 320) return launch_tile<Tile320>(A, W, bias, resid, C, (int)M, (int)m_rows, N, K, epi, tail, s);
    if (tile_bn == 256) return launch_tile<Tile256>(A, W, bias, resid, C, (int)M, (int)m_rows, N, K, epi, tail, s);
    return hipErrorInvalidValue;
}
