// Multi-head self-attention of the bf16 path (paper section 2.1: attention
// scores of the token sequence through dot products; every output token
// independent).  qkv[b*T + t, :] = [q | k | v], each block head-major.
//
// One workgroup per (image, head); its wavefronts (at most 8, so that each may
// use 256 registers) take the tiles of 32 query tokens round-robin.
// K (row-major) and V (transposed: [component][token]) of the head are staged
// once in LDS and shared by all query tiles.  A wave computes the transposed
// score tile S^T = K . Q^T with v_mfma_f32_32x32x16_bf16: the accumulator
// layout then puts one query per lane column and the keys inside the lane,
// so
//   - the whole score row of a query (all T keys, T x T never leaves the CU)
//     sits in registers: softmax max and sum are in-lane reductions plus one
//     exchange between the two half-waves; no running rescale is needed,
//   - the probabilities, rounded to bf16, already are the B operand of the
//     second product O^T = V^T . P^T (the order of the contraction index is
//     free as long as both operands agree, and V^T is read from LDS in the
//     order the accumulator registers hold the keys),
//   - O^T again has one query per lane column, so the division by the softmax
//     sum is a per-lane scale.
// Softmax is fp32: exp2 of (score * scale * log2 e - max), keys beyond T masked
// to -inf, sum over the unrounded probabilities.
//
// Template: DH = head width (multiple of 16), NKT = number of 32-key tiles
// (T <= 32*NKT).
#include "ep_kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    const __bf16 a = (__bf16)lo, b = (__bf16)hi;
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

template <int DH, int NKT>
struct AttnShape {
    static constexpr int TP = NKT * 32;            // padded token count
    static constexpr int KS = DH + 8;              // K row stride (elements): conflict-free b128 reads
    static constexpr int ET = (DH + 31) / 32;      // 32-row tiles of O^T
    static constexpr int VS = TP + 8;              // V^T row stride (elements)
    static constexpr size_t k_bytes = (size_t)TP * KS * 2;
    static constexpr size_t v_bytes = (size_t)ET * 32 * VS * 2;
    static constexpr size_t smem = k_bytes + v_bytes;
};

template <int DH, int NKT>
__global__ __launch_bounds__((NKT < 8 ? NKT : 8) * 64) void attn_bf16_kernel(const uint16_t *__restrict__ qkv,
                                                             uint16_t *__restrict__ o, int T, int D,
                                                             int H, float scale_log2e)
{
    using S = AttnShape<DH, NKT>;
    constexpr int TP = S::TP, KS = S::KS, ET = S::ET, VS = S::VS;
    constexpr int KSTEPS = DH / 16;
    static_assert(DH % 16 == 0, "head width must be a multiple of 16");

    extern __shared__ uint4 smem_raw[];
    uint16_t *Ks = reinterpret_cast<uint16_t *>(smem_raw);          // [TP][KS]
    uint16_t *Vt = Ks + TP * KS;                                    // [ET*32][VS]

    const int b = blockIdx.x / H, h = blockIdx.x % H;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l31 = lane & 31, g = lane >> 5;
    const size_t ld = (size_t)3 * D;
    const uint16_t *base = qkv + (size_t)b * T * ld + (size_t)h * DH;

    // ---- stage K: TP rows x DH/8 chunks of 16 bytes; rows >= T are zero
    for (int id = tid; id < TP * (DH / 8); id += nthr) {
        const int r = id / (DH / 8), c = id % (DH / 8);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < T) v = *reinterpret_cast<const uint4 *>(base + (size_t)r * ld + D + c * 8);
        *reinterpret_cast<uint4 *>(Ks + r * KS + c * 8) = v;
    }
    // ---- stage V transposed: unit = 4 tokens x 8 components; tokens >= T are zero
    for (int id = tid; id < (TP / 4) * (DH / 8); id += nthr) {
        const int u4 = id % (TP / 4), c = id / (TP / 4);
        uint4 r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int u = u4 * 4 + j;
            r[j] = make_uint4(0, 0, 0, 0);
            if (u < T) r[j] = *reinterpret_cast<const uint4 *>(base + (size_t)u * ld + 2 * D + c * 8);
        }
        const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&r[0]);
        const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&r[1]);
        const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&r[2]);
        const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&r[3]);
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
    // rows DH .. ET*32-1 of V^T feed accumulator rows that are never stored; give them zeros
    for (int id = tid; id < (ET * 32 - DH) * (TP / 4); id += nthr) {
        const int e = DH + id / (TP / 4), u4 = id % (TP / 4);
        *reinterpret_cast<uint2 *>(Vt + e * VS + u4 * 4) = make_uint2(0, 0);
    }
    __syncthreads();

    const int nwaves = nthr >> 6;
    for (int q0 = wave * 32; q0 < T; q0 += nwaves * 32) {   // no barrier inside this loop

    // ---- Q fragments (B operand: column = query l31, 8 consecutive components at 16*ks + 8*g)
    bf16x8 qf[KSTEPS];
    {
        const int qrow = min(q0 + l31, T - 1);
        const uint16_t *qp = base + (size_t)qrow * ld + g * 8;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
            qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(qp + ks * 16));
    }

    // ---- S^T = K . Q^T : st[kt][i] <-> key kt*32 + 8*(i/4) + 4*g + (i%4), query q0 + l31
    f32x16 st[NKT];
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) {
#pragma unroll
        for (int i = 0; i < 16; ++i) st[kt][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const bf16x8 kf = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const uint4 *>(Ks + (kt * 32 + l31) * KS + ks * 16 + g * 8));
            st[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], st[kt], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads of later tiles from piling up in registers
    }

    // ---- softmax over keys (in-lane + the other half-wave)
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = kt * 32 + 8 * (i / 4) + 4 * g + (i % 4);
            const float s = key < T ? st[kt][i] * scale_log2e : -INFINITY;
            st[kt][i] = s;
            mx = fmaxf(mx, s);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = __builtin_amdgcn_exp2f(st[kt][i] - mx);
            st[kt][i] = p;
            sum += p;
        }
    sum += __shfl_xor(sum, 32, 64);
    const float inv = 1.0f / sum;

    // ---- O^T = V^T . P^T
    f32x16 ot[ET];
#pragma unroll
    for (int et = 0; et < ET; ++et)
#pragma unroll
        for (int i = 0; i < 16; ++i) ot[et][i] = 0.f;
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {      // two 16-key steps per 32-key tile
            // registers 8j..8j+7 of st[kt] hold keys kt*32 + 16j + {4g..4g+3} and + 8
            uint4 pw;
            pw.x = pack_bf16x2(st[kt][8 * j + 0], st[kt][8 * j + 1]);
            pw.y = pack_bf16x2(st[kt][8 * j + 2], st[kt][8 * j + 3]);
            pw.z = pack_bf16x2(st[kt][8 * j + 4], st[kt][8 * j + 5]);
            pw.w = pack_bf16x2(st[kt][8 * j + 6], st[kt][8 * j + 7]);
            const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
            const int key0 = kt * 32 + 16 * j + 4 * g;
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                const uint16_t *vp = Vt + (et * 32 + l31) * VS + key0;
                const uint2 lo = *reinterpret_cast<const uint2 *>(vp);
                const uint2 hi = *reinterpret_cast<const uint2 *>(vp + 8);
                const bf16x8 vf = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
                ot[et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, ot[et], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

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
    }   // query tiles
}

template <int DH, int NKT>
hipError_t launch_attn(const uint16_t *qkv, uint16_t *o, int B, int T, int D, int H, hipStream_t s)
{
    using S = AttnShape<DH, NKT>;
    auto kern = attn_bf16_kernel<DH, NKT>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int nq = min((T + 31) / 32, 8);  // waves; query tiles are dealt round-robin
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)DH);
    hipLaunchKernelGGL(kern, dim3((unsigned)(B * H)), dim3(nq * 64), S::smem, s, qkv, o, T, D, H,
                       scale_log2e);
    return hipGetLastError();
}

template <int DH>
hipError_t launch_attn_dh(const uint16_t *qkv, uint16_t *o, int B, int T, int D, int H, hipStream_t s)
{
    const int nkt = (T + 31) / 32;
    if (nkt <= 3) return launch_attn<DH, 3>(qkv, o, B, T, D, H, s);
    if (nkt <= 7) return launch_attn<DH, 7>(qkv, o, B, T, D, H, s);
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
