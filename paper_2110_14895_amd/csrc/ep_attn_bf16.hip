// Multi-head self-attention of the bf16 path (paper section 2.1: attention
// scores of the token sequence through dot products; every output token
// independent).  qkv[b*T + t, :] = [q | k | v], each block head-major.
//
// Persistent workgroups, one per compute unit (the LDS footprint allows no
// more), each walking a list of (image, head) pairs; one wavefront per tile of
// 32 query tokens (at most 9, T <= 288) plus three producer waves.  K
// (row-major) and V (transposed: [component][token]) of the head are staged in
// LDS and shared by all query tiles; the producer waves load the next pair's K
// and V into registers while the query waves work on the current pair, and
// write them to LDS (transposing V) once the pair is retired, so the memory
// latency of a pair hides behind the arithmetic of the one before.  A query
// wave walks the keys in chunks of 96 and computes the transposed score tile
// S^T = K . Q^T with v_mfma_f32_32x32x16_bf16: the accumulator layout then
// puts one query per lane column and the keys inside the lane, so
//   - the chunk maximum is an in-lane reduction plus one exchange between the
//     two half-waves; the reference maximum of the exponentials follows the
//     true maximum lazily (the accumulated output is rescaled only when some
//     query's maximum grew by more than 2^6, which keeps exp2 far from
//     overflow and costs nothing in accuracy: bf16 keeps 8 bits at any scale),
//   - the probabilities, rounded to bf16, already are the B operand of the
//     second product O^T = V^T . P^T (the order of the contraction index is
//     free as long as both operands agree, and V^T is read from LDS in the
//     order the accumulator registers hold the keys),
//   - O^T again has one query per lane column, so the division by the softmax
//     sum is a per-lane scale.  When the head width leaves spare rows in the
//     last 32-row tile of V^T (80 -> 96), two of them hold ones, so the MFMA
//     also delivers the softmax denominator (the sum of the rounded
//     probabilities, i.e. of the weights that were actually applied); otherwise
//     the sum is accumulated on the vector ALU from the unrounded values.
// Softmax is fp32: exp2 of (score - reference) * scale * log2 e, keys beyond T
// masked to -inf.  The chunking bounds the registers of a wave (<= 168), so
// that 12 waves fit a compute unit and the lone last query of T = 257 does not
// cost a second pass; LDS fragments are fetched one step ahead of the MFMAs
// using them.
//
// Template: DH = head width (multiple of 16), NKT = number of 32-key tiles the
// LDS buffers hold (T <= 32*NKT, NKT a multiple of 3).
#include "ep_kernels.h"
#include "ep_device.h"
#include "ep_launch.h"
#include <algorithm>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));


constexpr int CH = 3;                              // 32-key tiles per chunk
constexpr int NPROD = 3;                           // producer waves (staging only)

template <int DH, int NKT>
struct AttnShape {
    static constexpr int TP = NKT * 32;            // padded token count
    static constexpr int KS = DH + 8;              // K row stride (elements): conflict-free b128 reads
    static constexpr int ET = (DH + 31) / 32;      // 32-row tiles of O^T
    static constexpr int VS = TP + 4;              // V^T row stride (elements): conflict-free b64 reads
    static constexpr bool SUM_MFMA = ET * 32 - DH >= 8;   // rows DH and DH+4 of V^T are free for ones
    static constexpr size_t k_bytes = (size_t)TP * KS * 2;
    static constexpr size_t v_bytes = (size_t)ET * 32 * VS * 2;
    static constexpr size_t smem = k_bytes + v_bytes;
};

template <int DH, int NKT>
__global__ __launch_bounds__((NKT + NPROD) * 64) void attn_bf16_kernel(const uint16_t *__restrict__ qkv,
                                                             uint16_t *__restrict__ o, int T, int D,
                                                             int H, int n_pairs, float scale_log2e)
{
    using S = AttnShape<DH, NKT>;
    constexpr int TP = S::TP, KS = S::KS, ET = S::ET, VS = S::VS;
    constexpr int KSTEPS = DH / 16;
    static_assert(DH % 16 == 0, "head width must be a multiple of 16");
    static_assert(NKT % CH == 0, "the LDS buffers hold whole chunks");

    extern __shared__ uint4 smem_raw[];
    uint16_t *Ks = reinterpret_cast<uint16_t *>(smem_raw);          // [TP][KS]
    uint16_t *Vt = Ks + TP * KS;                                    // [ET*32][VS]

    const int tid = threadIdx.x, nthr = blockDim.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, g = lane >> 5;
    const size_t ld = (size_t)3 * D;
    // waves [0, nq) own one tile of 32 queries each; the NPROD waves after them only stage K and V
    const int nq = (int)(blockDim.x >> 6) - NPROD;
    const bool producer = wave >= nq;                               // wave-uniform
    const int q0 = wave * 32;

    // Persistent workgroups: workgroup w sits on XCD w % 8 (round-robin dispatch).  Each XCD gets
    // a contiguous range of (image, head) pairs, so that the heads of an image, which share
    // cache lines of the qkv rows, meet in one L2; the workgroups of an XCD stride through it.
    int pair, pair_end, pair_step;
    if (gridDim.x % 8 == 0) {
        const int x = blockIdx.x % 8;
        pair = (int)((int64_t)n_pairs * x / 8) + blockIdx.x / 8;
        pair_end = (int)((int64_t)n_pairs * (x + 1) / 8);
        pair_step = gridDim.x / 8;
    } else {
        pair = blockIdx.x; pair_end = n_pairs; pair_step = gridDim.x;
    }
    if (pair >= pair_end) return;                                   // whole workgroup

    // ---- staging: K row-major, V transposed (unit = 4 tokens x 8 components).  A round of the
    // producer threads covers RPR token rows (K) or RPR groups of 4 tokens (V), 16 bytes per
    // thread and row; consecutive threads take consecutive 16-byte chunks of a row.  Tokens >= T
    // lie past the end of the buffer descriptors and read as zeros.  The producer waves issue
    // the loads of the next pair's K and V when the query waves start on the current pair, hold
    // them in registers, and write them to LDS after the barrier that retires the current pair.
    constexpr int ST = NPROD * 64;
    constexpr int CPR = DH / 8, RPR = ST / CPR;
    constexpr int KB = (TP + RPR - 1) / RPR, VB = (TP / 4 + RPR - 1) / RPR;
    constexpr int OOB = 0x7FFFFFF0;
    const int ptid = tid - nq * 64;                                 // thread index among the producers
    uint4 kv[KB], vv[VB][4];
    bf16x8 qf[KSTEPS];
    const int row_bytes = (int)ld * 2;
    const int seg_bytes = (T - 1) * row_bytes + DH * 2;             // first to last byte of a head's q, k or v

    // Q fragments of pair p (B operand: column = query l31, 8 consecutive components at 16*ks + 8*g)
    auto fetch_q = [&](int p) {
        const uint16_t *img = qkv + (size_t)(p / H) * T * ld + (size_t)(p % H) * DH;
        const __amdgpu_buffer_rsrc_t q_rs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(img), 0, seg_bytes, 0x00020000);
        const int qrow = min(q0 + l31, T - 1);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
            qf[ks] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(
                                                    q_rs, qrow * row_bytes + g * 16 + ks * 32, 0, 0));
    };
    auto fetch_kv = [&](int p) {
        const uint16_t *img = qkv + (size_t)(p / H) * T * ld + (size_t)(p % H) * DH;
        const __amdgpu_buffer_rsrc_t k_rs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(img + D), 0, seg_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t v_rs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(img + 2 * D), 0, seg_bytes, 0x00020000);
        const int r0 = ptid / CPR, c = ptid % CPR;
        const int off0 = ptid < RPR * CPR ? r0 * row_bytes + c * 16 : OOB;
#pragma unroll
        for (int i = 0; i < KB; ++i)
            kv[i] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(
                                                  k_rs, (int)((unsigned)off0 + (unsigned)(i * RPR * row_bytes)), 0, 0));
        const int voff0 = ptid < RPR * CPR ? 4 * r0 * row_bytes + c * 16 : OOB;
#pragma unroll
        for (int i = 0; i < VB; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                vv[i][j] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(
                                                         v_rs, (int)((unsigned)voff0 + (unsigned)((4 * i * RPR + j) * row_bytes)), 0, 0));
    };
    auto deposit = [&]() {
        if (ptid >= RPR * CPR) return;
        const int r0 = ptid / CPR, c = ptid % CPR;
#pragma unroll
        for (int i = 0; i < KB; ++i)
            if ((i + 1) * RPR <= TP || r0 + i * RPR < TP)
                *reinterpret_cast<uint4 *>(Ks + (r0 + i * RPR) * KS + c * 8) = kv[i];
#pragma unroll
        for (int i = 0; i < VB; ++i) {
            const int u4 = r0 + i * RPR;
            if ((i + 1) * RPR > TP / 4 && u4 >= TP / 4) continue;
            const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&vv[i][0]);
            const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&vv[i][1]);
            const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&vv[i][2]);
            const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&vv[i][3]);
#pragma unroll
            for (int p = 0; p < 4; ++p) {     // component pair (2p, 2p+1) of the chunk
                uint2 lo, hi;
                lo.x = (w0[p] & 0xFFFFu) | (w1[p] << 16);
                lo.y = (w2[p] & 0xFFFFu) | (w3[p] << 16);
                hi.x = (w0[p] >> 16) | (w1[p] & 0xFFFF0000u);
                hi.y = (w2[p] >> 16) | (w3[p] & 0xFFFF0000u);
                *reinterpret_cast<uint2 *>(Vt + (c * 8 + 2 * p) * VS + u4 * 4) = lo;
                *reinterpret_cast<uint2 *>(Vt + (c * 8 + 2 * p + 1) * VS + u4 * 4) = hi;
            }
        }
    };

    if (producer) fetch_kv(pair); else fetch_q(pair);
    // rows DH .. ET*32-1 of V^T feed accumulator rows that are never stored: zeros, except that
    // rows DH and DH+4 hold ones when the MFMA is to deliver the softmax sum.  Written once.
    for (int id = tid; id < (ET * 32 - DH) * (TP / 4); id += nthr) {
        const int e = DH + id / (TP / 4), u4 = id % (TP / 4);
        const uint32_t w = S::SUM_MFMA && (e == DH || e == DH + 4) ? 0x3F803F80u : 0u;
        *reinterpret_cast<uint2 *>(Vt + e * VS + u4 * 4) = make_uint2(w, w);
    }

    if (producer) deposit();
    __syncthreads();

    // Both roles run the same sequence of barriers: two per pair but the last.
    if (producer) {
        for (;;) {
            const int next = pair + pair_step;
            if (next >= pair_end) break;         // uniform over the workgroup
            fetch_kv(next);                      // in flight while the query waves work on this pair
            __syncthreads();                     // every query wave is done with this pair's K and V^T
            deposit();
            __syncthreads();
            pair = next;
        }
        return;
    }
    for (;;) {
    const int b = pair / H, h = pair % H;
    const int next = pair + pair_step;
    const bool more = next < pair_end;           // uniform over the workgroup

    f32x16 ot[ET];
#pragma unroll
    for (int et = 0; et < ET; ++et)
#pragma unroll
        for (int i = 0; i < 16; ++i) ot[et][i] = 0.f;
    float m = 0.f, l = 0.f;              // reference maximum (raw score), running sum (this half-wave's keys)

    const int nch = (T + 32 * CH - 1) / (32 * CH);
#pragma unroll 1
    for (int c = 0; c < nch; ++c) {
        const int kbase = c * 32 * CH;

        // ---- S^T = K . Q^T : st[kt][i] <-> key kbase + kt*32 + 8*(i/4) + 4*g + (i%4), query q0 + l31
        constexpr int NS = CH * KSTEPS, W = KSTEPS + 1;      // fragments in flight ahead of the MFMAs
        const uint16_t *kp = Ks + (kbase + l31) * KS + g * 8;
        f32x16 st[CH];
        bf16x8 kf[NS];
#pragma unroll
        for (int i = 0; i < W; ++i)
            kf[i] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const uint4 *>(kp + (i / KSTEPS) * 32 * KS + (i % KSTEPS) * 16));
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int kt = i / KSTEPS, ks = i % KSTEPS;
            if (ks == 0) {
#pragma unroll
                for (int r = 0; r < 16; ++r) st[kt][r] = 0.f;
            }
            st[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[ks], st[kt], 0, 0, 0);
            if (i + W < NS)
                kf[i + W] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const uint4 *>(kp + ((i + W) / KSTEPS) * 32 * KS + ((i + W) % KSTEPS) * 16));
            __builtin_amdgcn_sched_barrier(0);   // keeps the window of fragments (and the registers) bounded
        }

        // ---- chunk maximum, rescale of what has been accumulated so far
        if (kbase + 32 * CH > T) {               // wave-uniform: only the last chunk has keys to mask
            const int lim = T - kbase - 4 * g;
#pragma unroll
            for (int kt = 0; kt < CH; ++kt)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (kt * 32 + 8 * (i / 4) + (i % 4) >= lim) st[kt][i] = -INFINITY;
        }
        float cm = st[0][0];
#pragma unroll
        for (int kt = 0; kt < CH; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) cm = fmaxf(cm, st[kt][i]);
        cm = fmaxf(cm, __shfl_xor(cm, 32, 64));
        // The reference maximum m only has to keep exp2 in range, so it follows the true maximum
        // lazily: what has been accumulated is rescaled only when some query's maximum grew by
        // more than 2^6 (bf16 and fp32 have exponent range to spare).
        if (c == 0) {
            m = cm;                              // finite: every chunk visited has at least one key < T
        } else if (__builtin_amdgcn_ballot_w64((cm - m) * scale_log2e > 6.0f) != 0) {
            const float m_new = fmaxf(m, cm);
            const float alpha = __builtin_amdgcn_exp2f((m - m_new) * scale_log2e);
            m = m_new;
#pragma unroll
            for (int et = 0; et < ET; ++et)
#pragma unroll
                for (int i = 0; i < 16; ++i) ot[et][i] *= alpha;
            l *= alpha;
        }
        const float mb = m * scale_log2e;

        // ---- probabilities, rounded to bf16 in the register order the second product consumes:
        // registers 8j..8j+7 of st[kt] hold keys kbase + kt*32 + 16j + {4g..4g+3} and + 8
        bf16x8 pf[2 * CH];
#pragma unroll
        for (int kt = 0; kt < CH; ++kt)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float p[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    p[r] = __builtin_amdgcn_exp2f(fmaf(st[kt][8 * j + r], scale_log2e, -mb));
                    if (!S::SUM_MFMA) l += p[r];
                }
                uint4 pw;
                pw.x = pack_bf16x2(p[0], p[1]);
                pw.y = pack_bf16x2(p[2], p[3]);
                pw.z = pack_bf16x2(p[4], p[5]);
                pw.w = pack_bf16x2(p[6], p[7]);
                pf[2 * kt + j] = __builtin_bit_cast(bf16x8, pw);
            }

        // ---- O^T += V^T . P^T over the chunk's six 16-key steps
        constexpr int NV = 2 * CH;
        const uint16_t *vp = Vt + l31 * VS + kbase + 4 * g;
        bf16x8 vf[NV][ET];
        auto load_v = [&](int jj, int et) {
            const uint16_t *p = vp + et * 32 * VS + 16 * jj;
            const uint2 lo = *reinterpret_cast<const uint2 *>(p);
            const uint2 hi = *reinterpret_cast<const uint2 *>(p + 8);
            return __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
        };
#pragma unroll
        for (int et = 0; et < ET; ++et) vf[0][et] = load_v(0, et);
#pragma unroll
        for (int jj = 0; jj < NV; ++jj) {
            if (jj + 1 < NV) {
#pragma unroll
                for (int et = 0; et < ET; ++et) vf[jj + 1][et] = load_v(jj + 1, et);
            }
#pragma unroll
            for (int et = 0; et < ET; ++et)
                ot[et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[jj][et], pf[jj], ot[et], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    float sum;
    if (S::SUM_MFMA) {
        sum = ot[ET - 1][(DH % 32) / 8 * 4];     // accumulator row DH (g = 0) or DH + 4 (g = 1)
    } else {
        sum = l + __shfl_xor(l, 32, 64);
    }
    const float inv = 1.0f / sum;

    // ---- store: ot[et][i] <-> component et*32 + 8*(i/4) + 4*g + (i%4), query q0 + l31
    const int q = q0 + l31;
    if (q < T) {
        uint16_t *op = o + ((size_t)b * T + q) * D + (size_t)h * DH;
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                const int e = et * 32 + c4 * 8 + g * 4;
                if (e < DH) {
                    uint2 w;
                    w.x = pack_bf16x2(ot[et][c4 * 4 + 0] * inv, ot[et][c4 * 4 + 1] * inv);
                    w.y = pack_bf16x2(ot[et][c4 * 4 + 2] * inv, ot[et][c4 * 4 + 3] * inv);
                    *reinterpret_cast<uint2 *>(op + e) = w;
                }
            }
    }
    if (!more) break;
    fetch_q(next);
    __syncthreads();
    __syncthreads();
    pair = next;
    }
}

template <int DH, int NKT>
hipError_t launch_attn(const uint16_t *qkv, uint16_t *o, int B, int T, int D, int H, hipStream_t s)
{
    using S = AttnShape<DH, NKT>;
    auto kern = attn_bf16_kernel<DH, NKT>;
    static EpSmemLimit smem_limit;
    hipError_t e = smem_limit.ensure(reinterpret_cast<const void *>(kern), (int)S::smem);
    if (e != hipSuccess) return e;
    const int nq = (T + 31) / 32;          // one wave per tile of 32 queries, <= NKT
    const int nw = nq + NPROD;             // ... and the producer waves
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)DH);
    // one persistent workgroup per compute unit (the LDS footprint allows no more); a multiple
    // of 8 keeps the XCD-aware pair ranges
    int n_cu = 0;
    if ((e = ep_device_cu_count(&n_cu)) != hipSuccess) return e;
    const int n_pairs = B * H;
    int grid = n_pairs;
    if (n_pairs > n_cu) grid = n_cu;
    if (grid >= 8) grid -= grid % 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(nw * 64), S::smem, s, qkv, o, T, D, H, n_pairs,
                       scale_log2e);
    return hipGetLastError();
}

template <int DH>
hipError_t launch_attn_dh(const uint16_t *qkv, uint16_t *o, int B, int T, int D, int H, hipStream_t s)
{
    const int nkt = (T + 31) / 32;
    if (nkt <= 3) return launch_attn<DH, 3>(qkv, o, B, T, D, H, s);
    if (nkt <= 6) return launch_attn<DH, 6>(qkv, o, B, T, D, H, s);
    if (nkt <= 9) return launch_attn<DH, 9>(qkv, o, B, T, D, H, s);
    return hipErrorInvalidValue;
}

}  // namespace

bool ep_bf16_attention_supported(int T, int d_head)
{
    return T >= 1 && T <= 288 && (d_head == 64 || d_head == 80);
}

hipError_t ep_bf16_attention(const uint16_t *qkv, uint16_t *o, int B, int T, int D, int H, hipStream_t s)
{
    if (B <= 0) return hipSuccess;
    if (H <= 0 || D % H != 0 || !ep_bf16_attention_supported(T, D / H)) return hipErrorInvalidValue;
    if ((int64_t)B * H > 0x7FFFFFFF) return hipErrorInvalidValue;
    switch (D / H) {
    case 64: return launch_attn_dh<64>(qkv, o, B, T, D, H, s);
    case 80: return launch_attn_dh<80>(qkv, o, B, T, D, H, s);
    }
    return hipErrorInvalidValue;
}
