// Multi-head self-attention of the bf16 path (paper section 2.1:
// attention scores of the token sequence through dot products; every output
// token independent).  qkv[b*T + t, :] = [q | k | v], each block head-major.
//
// Persistent workgroups, one per compute unit, each walking a list of (image,
// head) pairs.  The keys and values of a pair stream through LDS in chunks of 96
// tokens, K and V both row-major as they lie in memory: two loader waves bring
// chunk after chunk in with buffer_load ... lds (no register staging, no
// transposing copy) into a ring of five chunk buffers, up to four chunks - more
// than a whole pair at T = 257 - ahead of the query waves, so the memory latency
// of a pair hides behind the arithmetic of the one before, and any number of
// tokens passes through the same buffers.  One barrier per chunk both hands a
// landed chunk to the query waves and returns the buffer they have finished to
// the loaders.
//
// A query wave owns 32 queries (two 16-query blocks) and walks a chunk in three
// steps of 32 keys with v_mfma_f32_16x16x32_bf16:
//   S^T = K . Q^T   (A = K fragment: 16 keys x 32 components, one ds_read_b128
//                    per lane; B = Q fragment, held in registers for the pair):
//                   the accumulator puts one query per lane column (l % 16) and
//                   four consecutive keys per lane, so the row maximum is an
//                   in-lane reduction plus two exchanges across the quarters of
//                   the wave;
//   P = exp2((S - reference) * scale * log2 e), fp32, keys beyond T masked to
//                   -inf; the reference follows the true maximum lazily (what
//                   has been accumulated is rescaled only when some query's
//                   maximum grew by more than 2^6: bf16 and fp32 have exponent
//                   range to spare); rounded to bf16 the probabilities of two
//                   16-key blocks are, register for register, the B operand of
//   O^T += V^T . P^T (the order of the contraction index is free as long as both
//                   operands agree: slot 8g + m of the 32-key step is key
//                   4g + m of its first block for m < 4 and of its second block
//                   for m >= 4).  The A operand, 16 components x 32 keys of V^T,
//                   comes straight out of the row-major V with two
//                   ds_read_b64_tr_b16 per lane (within 16 lanes the instruction
//                   takes four rows of 16 elements and hands lane j column j);
//                   a fragment of ones as a further A operand makes the matrix
//                   pipe deliver the softmax denominator as well (the sum of the
//                   rounded probabilities, i.e. of the weights actually applied).
// The last 32-component step of a head width that is not a multiple of 32 (80)
// reads past the row into the next row (finite data) against zeros in Q.
// More than 320 tokens: the query tiles are taken in passes of ten waves, the
// keys streaming through once per pass.
#include "ep_kernels.h"
#include "ep_device.h"
#include "ep_launch.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int CK = 96;                               // keys per chunk
constexpr int SUBS = CK / 32;                        // 32-key steps per chunk
constexpr int NBUF = 5;                              // chunk buffers in the ring
constexpr int DEPTH = NBUF - 1;                      // chunks in flight ahead of the one being consumed
constexpr int NLOADER = 2;                           // loader waves
constexpr int MAXQW = 10;                            // query waves (32 queries each)

template <int DH>
struct StreamShape {
    static constexpr int ROWB = DH * 2;              // bytes of a K or V row in LDS
    static constexpr int PARTB = CK * ROWB;          // K part (then V part) of a chunk buffer
    static constexpr int BUFB = 2 * PARTB;
    static constexpr int LPW = PARTB / 1024;         // ... per loader wave: one takes the K parts, the other the V parts
    static constexpr int KS = (DH + 31) / 32;        // 32-component steps of the first product
    static constexpr int EB = DH / 16;               // 16-component blocks of the output
    static constexpr size_t smem = (size_t)NBUF * BUFB;
    static_assert(DH % 16 == 0 && PARTB % 1024 == 0 && NLOADER == 2, "chunk parts are whole loads, one loader per part");
    static_assert(DEPTH * LPW <= 63, "the loaders' counted wait fits the vmcnt field");
};

// maximum over lanes l, l ^ 16, l ^ 32, l ^ 48 (the four quarters of the wave hold the keys of one query):
// v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the even rows of its
// second, v_permlane32_swap the upper half of the first with the lower half of the second; fed the
// same value twice, a maximum of the two results folds rows 0|1 and 2|3, then the two halves.
__device__ inline float quarter_max(float v)
{
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const float w = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    const unsigned x = __float_as_uint(w);
    const auto q = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}

#define EP_ATTN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

// Q fragments of NQB 16-query blocks starting at query q0 of a pair (B operand: column = query l15 of the
// block, 8 consecutive components at 32 ks + 8 g; components past the head width read as zeros: an offset
// past the descriptor's end).  The loads are issued here and NOT waited for: they are written as assembly
// so that the compiler neither tracks them nor sinks them to their use, a whole pair later.  Whoever
// consumes qf first calls q_landed on it.
template <int DH, int NQB>
__device__ __forceinline__ void issue_q(const uint16_t *__restrict__ qkv, int T, int D, int H, int pair, int q0,
                                        u32x4 (&qf)[NQB][StreamShape<DH>::KS])
{
    constexpr int KS = StreamShape<DH>::KS;
    const int lane = threadIdx.x & 63;
    const int l15 = lane & 15, g = lane >> 4;
    const int row_bytes = 3 * D * 2;
    const int seg_bytes = (T - 1) * row_bytes + DH * 2;
    const uint64_t base = reinterpret_cast<uint64_t>(qkv + (size_t)(pair / H) * T * 3 * D + (size_t)(pair % H) * DH);
    u32x4 rs;                                                       // raw buffer descriptor: base, no stride, size, flags
    rs[0] = __builtin_amdgcn_readfirstlane((uint32_t)base);
    rs[1] = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xFFFFu);
    rs[2] = __builtin_amdgcn_readfirstlane((uint32_t)seg_bytes);
    rs[3] = 0x00020000u;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        const int qrow = min(q0 + qb * 16 + l15, T - 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bool in_row = ks * 32 + g * 8 < DH;
            const int voff = in_row ? qrow * row_bytes + ks * 64 + g * 16 : 0x7FFFFFF0;
            asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(qf[qb][ks]) : "v"(voff), "s"(rs) : "memory");
        }
    }
}

// every vector-memory operation this wave has issued has completed, the fragments of issue_q among them
template <int NQB, int KS>
__device__ __forceinline__ void q_landed(u32x4 (&qf)[NQB][KS])
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[qb][ks]));   // uses of qf stay below the wait
}

// One pass of a query wave over the keys of a pair: NQB 16-query blocks starting at query q0 (the second
// block only where it holds a query), their Q fragments in qf, chunk steps j0 .. j0 + nch - 1 of the
// workgroup's barrier sequence.  mid() is called once, at the start of the pass's second chunk (of its only
// one): the place for the caller's fetch of the next pair's fragments, away from the burst of output stores
// at the end of a pair.
template <int DH, int NQB, class Mid>
__device__ __forceinline__ void attn_pass(const u32x4 (&qf)[NQB][StreamShape<DH>::KS], char *lds, int T, int q0, int nch, int j0,
                                          float scale_log2e, f32x4 (&acc_o)[StreamShape<DH>::EB][NQB], f32x4 (&acc_sum)[NQB],
                                          Mid mid)
{
    using S = StreamShape<DH>;
    constexpr int ROWB = S::ROWB, PARTB = S::PARTB, BUFB = S::BUFB, KS = S::KS, EB = S::EB;
    const int lane = threadIdx.x & 63;
    const int l15 = lane & 15, g = lane >> 4;
    bf16x8 ones;
#pragma unroll
    for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;
    // lane's part of the V^T fragment addressing: source lane s = l % 16 of quarter g supplies row 4g + s/4,
    // elements 4 (s % 4) .. + 3 of the 16-component block
    const int v_lane = (4 * g + (l15 >> 2)) * ROWB + (l15 & 3) * 8;
    const int k_lane = l15 * ROWB + g * 16;

    float mref[NQB];                                                // reference maximum, in scaled log2 units
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        mref[qb] = -INFINITY;
        acc_sum[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) acc_o[eb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int c = 0; c < nch; ++c) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();              // chunk j0 + c has landed; the buffer of the chunk before goes back to the loaders
        asm volatile("" ::: "memory");
        const char *Kb = lds + ((j0 + c) % NBUF) * BUFB;
        const char *Vb = Kb + PARTB;
        if (c == (nch > 1 ? 1 : 0)) mid();
#pragma unroll
        for (int sub = 0; sub < SUBS; ++sub) {
            const int key0 = c * CK + sub * 32;
            if (key0 >= T) break;                           // wave-uniform: nothing but padding from here on
            // ---- S^T = K . Q^T: s[kb][qb][i] <-> key key0 + kb*16 + 4g + i, query q0 + qb*16 + l15
            f32x4 s[2][NQB];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb) s[kb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const bf16x8 kf = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const uint4 *>(Kb + k_lane + (sub * 32 + kb * 16) * ROWB + ks * 64));
#pragma unroll
                    for (int qb = 0; qb < NQB; ++qb)
                        s[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, __builtin_bit_cast(bf16x8, qf[qb][ks]), s[kb][qb], 0, 0, 0);
                }
            if (key0 + 32 > T) {                            // wave-uniform: keys to mask in the last step only
                const int lim = T - key0 - 4 * g;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (kb * 16 + i >= lim) {
#pragma unroll
                            for (int qb = 0; qb < NQB; ++qb) s[kb][qb][i] = -INFINITY;
                        }
            }
            // ---- softmax numerators of the step, as B fragments of the second product
            bf16x8 pf[NQB];
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) {
                float mx = fmaxf(fmaxf(fmaxf(s[0][qb][0], s[0][qb][1]), fmaxf(s[0][qb][2], s[0][qb][3])),
                                 fmaxf(fmaxf(s[1][qb][0], s[1][qb][1]), fmaxf(s[1][qb][2], s[1][qb][3])));
                mx = quarter_max(mx);
                const float t = mx * scale_log2e;           // finite: a step visited has a key < T
                if (__builtin_amdgcn_ballot_w64(t > mref[qb] + 6.0f) != 0) {
                    const float nref = fmaxf(mref[qb], t);
                    const float alpha = __builtin_amdgcn_exp2f(mref[qb] - nref);
                    mref[qb] = nref;
#pragma unroll
                    for (int eb = 0; eb < EB; ++eb) acc_o[eb][qb] *= alpha;
                    acc_sum[qb] *= alpha;
                }
                const float mb = mref[qb];
                float p[8];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        p[kb * 4 + i] = __builtin_amdgcn_exp2f(fmaf(s[kb][qb][i], scale_log2e, -mb));
                u32x4 pw;
                pw[0] = pack_bf16x2(p[0], p[1]);
                pw[1] = pack_bf16x2(p[2], p[3]);
                pw[2] = pack_bf16x2(p[4], p[5]);
                pw[3] = pack_bf16x2(p[6], p[7]);
                pf[qb] = __builtin_bit_cast(bf16x8, pw);
            }
            // ---- O^T += V^T . P^T and the denominators
#pragma unroll
            for (int eb = 0; eb < EB; ++eb) {
                typedef __attribute__((address_space(3))) s16x4 *tr_ptr;
                const char *vp = Vb + v_lane + (sub * 32) * ROWB + eb * 32;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(vp));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(vp + 16 * ROWB));
                typedef short s16x8 __attribute__((ext_vector_type(8)));
                const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb)
                    acc_o[eb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[qb], acc_o[eb][qb], 0, 0, 0);
            }
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb)
                acc_sum[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf[qb], acc_sum[qb], 0, 0, 0);
        }
    }

}

// Normalise and store a pass's output: acc_o[eb][qb][i] <-> component eb*16 + 4g + i, query q0 + qb*16 + l15;
// every row of acc_sum's block holds the query's softmax denominator.  A lane's four components of a block
// are 8 bytes of bf16; for a pair of blocks (eb, eb + 1) v_permlane16_swap trades them between the even and
// odd quarters of the wave so that an even quarter ends up with components 4g .. 4g + 7 of block eb and an
// odd one with 4(g-1) .. 4(g-1) + 7 of block eb + 1: 16 contiguous bytes per lane, half the store
// instructions.  A last unpaired block goes out in 8-byte pieces.
template <int DH, int NQB>
__device__ __forceinline__ void store_pass(const f32x4 (&acc_o)[StreamShape<DH>::EB][NQB], const f32x4 (&acc_sum)[NQB],
                                           uint16_t *__restrict__ o, int T, int D, int H, int pair, int q0)
{
    constexpr int EB = StreamShape<DH>::EB;
    const int lane = threadIdx.x & 63;
    const int l15 = lane & 15, g = lane >> 4;
    const int b = pair / H, h = pair % H;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        const int q = q0 + qb * 16 + l15;
        const float inv = 1.0f / acc_sum[qb][0];
        uint16_t *row = o + ((size_t)b * T + q) * D + (size_t)h * DH;
        auto packed = [&](int eb, int half) {
            return pack_bf16x2(acc_o[eb][qb][2 * half] * inv, acc_o[eb][qb][2 * half + 1] * inv);
        };
#pragma unroll
        for (int eb = 0; eb + 1 < EB; eb += 2) {
            // after the swaps: even quarters hold (own block eb | block eb of quarter g + 1), odd quarters
            // (block eb + 1 of quarter g - 1 | own block eb + 1)
            const auto lo = __builtin_amdgcn_permlane16_swap(packed(eb, 0), packed(eb + 1, 0), false, false);
            const auto hi = __builtin_amdgcn_permlane16_swap(packed(eb, 1), packed(eb + 1, 1), false, false);
            const uint4 w = make_uint4(lo[0], hi[0], lo[1], hi[1]);
            const int e = (eb + (g & 1)) * 16 + 4 * (g & 2);
            if (q < T) *reinterpret_cast<uint4 *>(row + e) = w;
        }
        if (EB & 1) {
            uint2 w;
            w.x = packed(EB - 1, 0);
            w.y = packed(EB - 1, 1);
            if (q < T) *reinterpret_cast<uint2 *>(row + (EB - 1) * 16 + 4 * g) = w;
        }
    }
}

// All the tiles of a query wave.  With one pass per pair (T <= 32 * query waves) the wave's tile is the
// same 32 queries in every pair, and the Q fragments of the next pair are fetched before the current
// pair is worked on, so their latency hides behind it; with several passes they are fetched per pass.
template <int DH, int NQB>
__device__ __forceinline__ void attn_wave_single_pass(const uint16_t *__restrict__ qkv, uint16_t *__restrict__ o, char *lds,
                                                      int T, int D, int H, int pair, int pair_step, int my_pairs, int q0,
                                                      int nch, float scale_log2e)
{
    constexpr int KS = StreamShape<DH>::KS;
    u32x4 qf[NQB][KS], qn[NQB][KS];
    issue_q<DH, NQB>(qkv, T, D, H, pair, q0, qf);
    q_landed<NQB, KS>(qf);
    for (int pi = 0; pi < my_pairs; ++pi, pair += pair_step) {
        const bool more = pi + 1 < my_pairs;
        f32x4 acc_o[StreamShape<DH>::EB][NQB], acc_sum[NQB];
        attn_pass<DH, NQB>(qf, lds, T, q0, nch, pi * nch, scale_log2e, acc_o, acc_sum,
                           [&]() { if (more) issue_q<DH, NQB>(qkv, T, D, H, pair + pair_step, q0, qn); });
        if (more) q_landed<NQB, KS>(qn);    // issued a pair ago; ahead of the stores, so that it does not wait for them
        store_pass<DH, NQB>(acc_o, acc_sum, o, T, D, H, pair, q0);
        if (more) {
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = qn[qb][ks];
        }
    }
}

template <int DH>
__global__ __launch_bounds__((MAXQW + NLOADER) * 64) void attn_stream_kernel(const uint16_t *__restrict__ qkv,
                                                                             uint16_t *__restrict__ o, int T, int D, int H,
                                                                             int n_pairs, float scale_log2e)
{
#if defined(__HIP_DEVICE_COMPILE__)
    using S = StreamShape<DH>;
    constexpr int ROWB = S::ROWB, PARTB = S::PARTB, BUFB = S::BUFB, LPW = S::LPW, KS = S::KS, EB = S::EB;
    extern __shared__ uint4 smem_raw[];
    char *lds = reinterpret_cast<char *>(smem_raw);
    typedef __attribute__((address_space(3))) void *lds_ptr;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l15 = lane & 15, g = lane >> 4;
    const int nqw = (int)(blockDim.x >> 6) - NLOADER;              // query waves of this launch
    const bool loader = wave >= nqw;                               // wave-uniform
    const int row_bytes = 3 * D * 2;
    const int seg_bytes = (T - 1) * row_bytes + DH * 2;            // first to last byte of a head's q, k or v
    const int nch = (T + CK - 1) / CK;                             // chunks per pass
    const int nqt = (T + 31) / 32;                                 // query tiles
    const int npass = (nqt + nqw - 1) / nqw;

    // Workgroup w sits on XCD w % 8 (round-robin dispatch).  Each XCD gets a contiguous range of
    // (image, head) pairs, as long as its share of the workgroups, so that the heads of an image, which
    // share cache lines of the qkv rows, meet in one L2; the workgroups of an XCD stride through it.
    int pair, pair_end, pair_step;
    {
        const int x = blockIdx.x % 8, g8 = gridDim.x / 8, r8 = gridDim.x % 8;
        const int before = x * g8 + min(x, r8);                    // workgroups on the XCDs in front of this one
        pair_step = g8 + (x < r8 ? 1 : 0);                         // workgroups on this one
        pair = (int)((int64_t)n_pairs * before / gridDim.x) + blockIdx.x / 8;
        pair_end = (int)((int64_t)n_pairs * (before + pair_step) / gridDim.x);
    }
    if (pair >= pair_end) return;                                  // whole workgroup
    const int my_pairs = (pair_end - pair + pair_step - 1) / pair_step;
    const int total = my_pairs * npass * nch;                      // chunk steps = barriers, the same for every wave

    if (loader) {
        // ---- loader waves: loader 0 brings the K part of every chunk, loader 1 the V part, LPW loads of
        // 1 KB each (64 lanes x 16 bytes, contiguous in LDS); lane l of load s fetches the 16 bytes at linear
        // byte s*1024 + 16 l of the part, i.e. row lin / ROWB, byte lin % ROWB of the row.  Rows at or past T
        // lie past the end of the buffer descriptor (per-lane offset, which the bounds check covers) and read
        // as zeros.
        const int lw = wave - nqw;
        int goff[LPW];
#pragma unroll
        for (int s = 0; s < LPW; ++s) {
            const int lin = s * 1024 + lane * 16;
            goff[s] = (lin / ROWB) * row_bytes + lin % ROWB;
        }
        int pf_pair = pair, pf_pass = 0, pf_chunk = 0;               // the next chunk to fetch
        auto issue = [&](int buf) {
            const uint16_t *part = qkv + (size_t)(pf_pair / H) * T * 3 * D + (size_t)(pf_pair % H) * DH + (size_t)(1 + lw) * D;
            const __amdgpu_buffer_rsrc_t rs =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(part), 0, seg_bytes, 0x00020000);
            const int base = pf_chunk * CK * row_bytes;
            char *dst = lds + buf * BUFB + lw * PARTB;
#pragma unroll
            for (int s = 0; s < LPW; ++s)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr)(dst + s * 1024), 16, base + goff[s], 0, 0, 0);
            if (++pf_chunk == nch) {
                pf_chunk = 0;
                if (++pf_pass == npass) { pf_pass = 0; pf_pair += pair_step; }
            }
        };
        // Chunk 0 and its successor go out first, alone (everyone waits for them); from then on the loader
        // tops the ring up to DEPTH chunks ahead right after each barrier, which is where a buffer comes free.
        int issued = 0;
        for (int j = 0; j < total; ++j) {
            while (issued < total && issued < j + 2) issue(issued++ % NBUF);
            // chunk j has landed once at most the loads of the chunks issued after it are outstanding
            switch (issued - 1 - j) {
            case 0: EP_ATTN_WAIT_VMCNT(0); break;
            case 1: EP_ATTN_WAIT_VMCNT(1 * LPW); break;
            case 2: EP_ATTN_WAIT_VMCNT(2 * LPW); break;
            case 3: EP_ATTN_WAIT_VMCNT(3 * LPW); break;
            default: EP_ATTN_WAIT_VMCNT(4 * LPW); break;
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();          // chunk j is there; the query waves are done with chunk j - 1
            asm volatile("" ::: "memory");
            while (issued < total && issued < j + 1 + DEPTH) issue(issued++ % NBUF);   // ... whose buffer comes free here
        }
        return;
    }

    // ---- query waves
    auto idle_pass = [&]() {                                        // no tile in this pass: keep the barrier count
        for (int c = 0; c < nch; ++c) {
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
    };
    if (npass == 1) {
        const int q0 = wave * 32;                                   // < T: the launch has no more query waves than tiles
        if (q0 + 16 < T)
            attn_wave_single_pass<DH, 2>(qkv, o, lds, T, D, H, pair, pair_step, my_pairs, q0, nch, scale_log2e);
        else
            attn_wave_single_pass<DH, 1>(qkv, o, lds, T, D, H, pair, pair_step, my_pairs, q0, nch, scale_log2e);
        return;
    }
    int j = 0;                                                      // chunk step
    for (int pi = 0; pi < my_pairs; ++pi, pair += pair_step) {
        for (int pass = 0; pass < npass; ++pass, j += nch) {
            const int q0 = (pass * nqw + wave) * 32;
            // wave-uniform: the tile's 16-query blocks with a query in them pick the code path once per pass
            if (q0 + 16 < T) {
                u32x4 qf[2][KS];
                issue_q<DH, 2>(qkv, T, D, H, pair, q0, qf);
                q_landed<2, KS>(qf);
                f32x4 acc_o[EB][2], acc_sum[2];
                attn_pass<DH, 2>(qf, lds, T, q0, nch, j, scale_log2e, acc_o, acc_sum, []() {});
                store_pass<DH, 2>(acc_o, acc_sum, o, T, D, H, pair, q0);
            } else if (q0 < T) {
                u32x4 qf[1][KS];
                issue_q<DH, 1>(qkv, T, D, H, pair, q0, qf);
                q_landed<1, KS>(qf);
                f32x4 acc_o[EB][1], acc_sum[1];
                attn_pass<DH, 1>(qf, lds, T, q0, nch, j, scale_log2e, acc_o, acc_sum, []() {});
                store_pass<DH, 1>(acc_o, acc_sum, o, T, D, H, pair, q0);
            } else {
                idle_pass();
            }
        }
    }
#endif
}

template <int DH>
hipError_t launch_stream(const uint16_t *qkv, uint16_t *o, int B, int T, int D, int H, hipStream_t s)
{
    using S = StreamShape<DH>;
    auto kern = attn_stream_kernel<DH>;
    static EpSmemLimit smem_limit;
    hipError_t e = smem_limit.ensure(reinterpret_cast<const void *>(kern), (int)S::smem);
    if (e != hipSuccess) return e;
    const int nqt = (T + 31) / 32;
    const int nqw = nqt < MAXQW ? nqt : MAXQW;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)DH);
    int n_cu = 0;
    if ((e = ep_device_cu_count(&n_cu)) != hipSuccess) return e;
    const int n_pairs = B * H;
    const int grid = n_pairs < n_cu ? n_pairs : n_cu;      // one workgroup per compute unit, or per pair if there are fewer
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3((nqw + NLOADER) * 64), S::smem, s, qkv, o, T, D, H, n_pairs,
                       scale_log2e);
    return hipGetLastError();
}

}  // namespace

bool ep_bf16_attention_supported(int T, int d_head)
{
    return T >= 1 && T <= 4096 && (d_head == 64 || d_head == 80);
}

hipError_t ep_bf16_attention(const uint16_t *qkv, uint16_t *o, int B, int T, int D, int H, hipStream_t s)
{
    if (B <= 0) return hipSuccess;
    if (H <= 0 || D % H != 0 || !ep_bf16_attention_supported(T, D / H)) return hipErrorInvalidValue;
    if ((int64_t)B * H > 0x7FFFFFFF || (int64_t)T * 3 * D * 2 >= 0x7FFFFFF0ll) return hipErrorInvalidValue;
    switch (D / H) {
    case 64: return launch_stream<64>(qkv, o, B, T, D, H, s);
    case 80: return launch_stream<80>(qkv, o, B, T, D, H, s);
    }
    return hipErrorInvalidValue;
}
