// What stands before the first and after the last encoder layer (the paper,
// section 4 "Deep Learning Models", keeps the embedding outside the transformer
// layers it partitions; the model definition is the original ViT):
//
//   embedding : x[b, 0, :]   = cls + pos[0]
//               x[b, 1+p, :] = patch_p(image b) . W_patch^T + b_patch + pos[1+p]
//               patch_p = the P x P x C pixels of patch p, flattened (channel, row, column)
//   head      : logits[b, :] = LayerNorm(x[b, 0, :]; g, beta) . W_head^T + b_head
//
// Embedding: a gather kernel writes the patches as GEMM rows (bf16 or fp32, K
// padded with zeros to a multiple of 64); the dense-layer dispatcher multiplies
// them with the projection and adds bias and the position rows in its fp32
// residual epilogue (the position rows are laid out once, at create time, as a
// [max_batch * patches, D] matrix); a second small kernel moves the result to
// the [B, T, D] token layout, inserts the class-token row and rounds once to
// the output dtype.  Head: gather of the class-token rows, LayerNorm, and the
// short-M GEMM with an fp32 store.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "edgepipe.h"
#include "ep_device.h"
#include "ep_error.h"
#include "ep_kernels.h"

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline float bf16_bits_to_float(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// host parameter vector of n elements in `dtype` -> fp32 host vector
void widen(const void *src, size_t n, int32_t dtype, std::vector<float> &dst)
{
    dst.resize(n);
    if (dtype == EP_BF16) {
        const uint16_t *s = (const uint16_t *)src;
        for (size_t i = 0; i < n; ++i) dst[i] = bf16_bits_to_float(s[i]);
    } else {
        std::memcpy(dst.data(), src, n * 4);
    }
}

// patches as GEMM rows: out[(b*NP + p), k], k = (c, iy, ix) < K, zeros for K <= k < Kp
template <typename OutT>
__global__ __launch_bounds__(256) void embed_gather_kernel(const float *__restrict__ img, OutT *__restrict__ out,
                                                           int64_t total, int C, int HW, int P, int G, int K, int Kp)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int k = (int)(i % Kp);
    const int64_t row = i / Kp;
    const int p = (int)(row % ((int64_t)G * G));
    const int64_t b = row / ((int64_t)G * G);
    float v = 0.f;
    if (k < K) {
        const int c = k / (P * P), iy = (k / P) % P, ix = k % P;
        const int y = (p / G) * P + iy, x = (p % G) * P + ix;
        v = img[((b * C + c) * HW + y) * HW + x];
    }
    if (sizeof(OutT) == 2) {
        const __bf16 h = (__bf16)v;
        reinterpret_cast<uint16_t *>(out)[i] = __builtin_bit_cast(uint16_t, h);
    } else {
        reinterpret_cast<float *>(out)[i] = v;
    }
}

// posb[(b*NP + p), :] = pos[1 + p, :]
__global__ __launch_bounds__(256) void embed_pos_rows_kernel(const float *__restrict__ pos, float *__restrict__ posb,
                                                             int64_t total, int NP, int D)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int d = (int)(i % D);
    const int p = (int)((i / D) % NP);
    posb[i] = pos[(size_t)(1 + p) * D + d];
}

// tmp [B*NP, D] fp32 -> x [B, 1 + NP, D] (row 0 = cls + pos[0]), rounded once to OutT
template <typename OutT>
__global__ __launch_bounds__(256) void embed_assemble_kernel(const float *__restrict__ tmp, const float *__restrict__ cls,
                                                             const float *__restrict__ pos, OutT *__restrict__ x,
                                                             int64_t total, int NP, int D)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int d = (int)(i % D);
    const int t = (int)((i / D) % (NP + 1));
    const int64_t b = i / ((int64_t)D * (NP + 1));
    const float v = t == 0 ? cls[d] + pos[d] : tmp[((size_t)b * NP + (t - 1)) * D + d];
    if (sizeof(OutT) == 2) {
        const __bf16 h = (__bf16)v;
        reinterpret_cast<uint16_t *>(x)[i] = __builtin_bit_cast(uint16_t, h);
    } else {
        reinterpret_cast<float *>(x)[i] = v;
    }
}

// cls_rows[b, :] = x[b, 0, :]
__global__ __launch_bounds__(256) void head_gather_kernel(const float *__restrict__ x, float *__restrict__ rows,
                                                          int64_t total, int T, int D)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    rows[i] = x[(i / D) * (size_t)T * D + (i % D)];
}

inline unsigned blocks_for(int64_t total) { return (unsigned)((total + 255) / 256); }

}  // namespace

#define EP_HIP(call)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            return ep_fail(EP_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));       \
    } while (0)

// --------------------------------------------------------------------- embedding
struct ep_embed {
    ep_embed_config cfg;
    int32_t max_batch, device;
    int G, NP, T, K, Kp;
    bool bf16;
    char *mem = nullptr;
    size_t mem_bytes = 0;
    void *w = nullptr;          // [D, Kp] param dtype
    float *b = nullptr, *cls = nullptr, *pos = nullptr, *posb = nullptr, *tmp = nullptr;
    void *rows = nullptr;       // [max_batch*NP, Kp] param dtype
};

extern "C" void ep_embed_destroy(ep_embed_t *e)
{
    if (!e) return;
    if (e->mem) (void)hipFree(e->mem);
    delete e;
}

extern "C" ep_status ep_embed_create(const ep_embed_config *cfg, const void *w_patch, const void *b_patch,
                                     const void *cls, const void *pos, int32_t max_batch, ep_embed_t **out)
{
    if (!out) return ep_fail(EP_ERR_INVALID_ARG, "ep_embed_create: null output");
    *out = nullptr;
    if (!cfg || !w_patch || !b_patch || !cls || !pos)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_embed_create: null argument");
    if (cfg->image_size < 1 || cfg->patch < 1 || cfg->channels < 1 || cfg->d_model < 1 || max_batch < 1 ||
        cfg->image_size % cfg->patch)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_embed_create: bad shape (image %d, patch %d, channels %d, width %d)",
                       cfg->image_size, cfg->patch, cfg->channels, cfg->d_model);
    auto is_dt = [](int32_t d) { return d == EP_F32 || d == EP_BF16; };
    if (!is_dt(cfg->param_dtype) || !is_dt(cfg->out_dtype))
        return ep_fail(EP_ERR_INVALID_ARG, "ep_embed_create: unknown dtype");
    const bool bf16 = cfg->param_dtype == EP_BF16;
    if (!bf16 && cfg->out_dtype != EP_F32)
        return ep_fail(EP_ERR_UNSUPPORTED, "fp32 parameters require fp32 output");
    if (bf16 && cfg->d_model % 64)
        return ep_fail(EP_ERR_UNSUPPORTED, "bf16 path needs d_model divisible by 64");
    ep_embed *e = new (std::nothrow) ep_embed;
    if (!e) return ep_fail(EP_ERR_OOM, "ep_embed_create: out of host memory");
    auto fail = [&](ep_status rc) { ep_embed_destroy(e); return rc; };
    e->cfg = *cfg;
    e->max_batch = max_batch;
    e->bf16 = bf16;
    e->G = cfg->image_size / cfg->patch;
    e->NP = e->G * e->G;
    e->T = e->NP + 1;
    e->K = cfg->channels * cfg->patch * cfg->patch;
    e->Kp = (e->K + 63) / 64 * 64;
    if (hipGetDevice(&e->device) != hipSuccess) return fail(ep_fail(EP_ERR_HIP, "hipGetDevice failed"));
    const int D = cfg->d_model;
    const size_t psz = bf16 ? 2 : 4;
    const size_t R = (size_t)max_batch * e->NP;
    if (R * (size_t)(e->Kp > D ? e->Kp : D) >= (1ull << 31))
        return fail(ep_fail(EP_ERR_UNSUPPORTED, "ep_embed_create: max_batch %d is too large for this image size", max_batch));

    const size_t w_bytes = align_up((size_t)D * e->Kp * psz, 256), v_bytes = align_up((size_t)D * 4, 256);
    const size_t pos_bytes = align_up((size_t)e->T * D * 4, 256), big = align_up(R * D * 4, 256);
    const size_t rows_bytes = align_up(R * e->Kp * psz, 256);
    e->mem_bytes = w_bytes + 2 * v_bytes + pos_bytes + 2 * big + rows_bytes;
    hipError_t he = hipMalloc((void **)&e->mem, e->mem_bytes);
    if (he != hipSuccess) {
        e->mem = nullptr;
        return fail(ep_fail(EP_ERR_OOM, "hipMalloc of %zu bytes failed: %s", e->mem_bytes, hipGetErrorString(he)));
    }
    char *m = e->mem;
    e->w = m; m += w_bytes;
    e->b = (float *)m; m += v_bytes;
    e->cls = (float *)m; m += v_bytes;
    e->pos = (float *)m; m += pos_bytes;
    e->posb = (float *)m; m += big;
    e->tmp = (float *)m; m += big;
    e->rows = m;

    // weight rows padded to Kp; vectors widened to fp32
    try {
        std::vector<char> wp((size_t)D * e->Kp * psz, 0);
        for (int d = 0; d < D; ++d)
            std::memcpy(wp.data() + (size_t)d * e->Kp * psz, (const char *)w_patch + (size_t)d * e->K * psz, (size_t)e->K * psz);
        std::vector<float> v;
        if ((he = hipMemcpy(e->w, wp.data(), wp.size(), hipMemcpyHostToDevice)) != hipSuccess)
            return fail(ep_fail(EP_ERR_HIP, "upload failed: %s", hipGetErrorString(he)));
        widen(b_patch, D, cfg->param_dtype, v);
        if ((he = hipMemcpy(e->b, v.data(), (size_t)D * 4, hipMemcpyHostToDevice)) != hipSuccess)
            return fail(ep_fail(EP_ERR_HIP, "upload failed: %s", hipGetErrorString(he)));
        widen(cls, D, cfg->param_dtype, v);
        if ((he = hipMemcpy(e->cls, v.data(), (size_t)D * 4, hipMemcpyHostToDevice)) != hipSuccess)
            return fail(ep_fail(EP_ERR_HIP, "upload failed: %s", hipGetErrorString(he)));
        widen(pos, (size_t)e->T * D, cfg->param_dtype, v);
        if ((he = hipMemcpy(e->pos, v.data(), (size_t)e->T * D * 4, hipMemcpyHostToDevice)) != hipSuccess)
            return fail(ep_fail(EP_ERR_HIP, "upload failed: %s", hipGetErrorString(he)));
    } catch (...) {
        return fail(ep_fail(EP_ERR_OOM, "ep_embed_create: out of host memory"));
    }
    const int64_t total = (int64_t)R * D;
    hipLaunchKernelGGL(embed_pos_rows_kernel, dim3(blocks_for(total)), dim3(256), 0, 0, e->pos, e->posb, total, e->NP, D);
    if ((he = hipGetLastError()) != hipSuccess || (he = hipDeviceSynchronize()) != hipSuccess)
        return fail(ep_fail(EP_ERR_HIP, "laying out the position rows failed: %s", hipGetErrorString(he)));
    *out = e;
    return EP_OK;
}

extern "C" ep_status ep_embed_forward(ep_embed_t *e, const void *images, int32_t B, void *x_out, void *stream)
{
    if (!e || !images || !x_out) return ep_fail(EP_ERR_INVALID_ARG, "ep_embed_forward: null argument");
    if (B < 1 || B > e->max_batch)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_embed_forward: B=%d outside [1, max_batch=%d]", B, e->max_batch);
    int dev = -1;
    EP_HIP(hipGetDevice(&dev));
    if (dev != e->device)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_embed_forward: created on device %d, current device is %d", e->device, dev);
    hipStream_t s = (hipStream_t)stream;
    const ep_embed_config &c = e->cfg;
    const int D = c.d_model;
    const int64_t R = (int64_t)B * e->NP;
    const int64_t n_rows = R * e->Kp;
    if (e->bf16) {
        hipLaunchKernelGGL(embed_gather_kernel<uint16_t>, dim3(blocks_for(n_rows)), dim3(256), 0, s, (const float *)images,
                           (uint16_t *)e->rows, n_rows, c.channels, c.image_size, c.patch, e->G, e->K, e->Kp);
        EP_HIP(hipGetLastError());
        EP_HIP(ep_bf16_gemm((const uint16_t *)e->rows, (const uint16_t *)e->w, e->b, e->posb, e->tmp, R, D, e->Kp,
                            EPI_BIAS_RESID, nullptr, s));
    } else {
        hipLaunchKernelGGL(embed_gather_kernel<float>, dim3(blocks_for(n_rows)), dim3(256), 0, s, (const float *)images,
                           (float *)e->rows, n_rows, c.channels, c.image_size, c.patch, e->G, e->K, e->Kp);
        EP_HIP(hipGetLastError());
        EP_HIP(ep_f32_gemm((const float *)e->rows, (const float *)e->w, e->b, e->posb, e->tmp, R, D, e->Kp, EPI_BIAS_RESID, s));
    }
    const int64_t n_out = (int64_t)B * e->T * D;
    if (c.out_dtype == EP_BF16)
        hipLaunchKernelGGL(embed_assemble_kernel<uint16_t>, dim3(blocks_for(n_out)), dim3(256), 0, s, e->tmp, e->cls, e->pos,
                           (uint16_t *)x_out, n_out, e->NP, D);
    else
        hipLaunchKernelGGL(embed_assemble_kernel<float>, dim3(blocks_for(n_out)), dim3(256), 0, s, e->tmp, e->cls, e->pos,
                           (float *)x_out, n_out, e->NP, D);
    EP_HIP(hipGetLastError());
    return EP_OK;
}

// --------------------------------------------------------------------------- head
struct ep_head {
    ep_head_config cfg;
    int32_t max_batch, device;
    bool bf16;
    char *mem = nullptr;
    size_t mem_bytes = 0;
    void *w = nullptr;          // [n_classes, D] param dtype
    float *b = nullptr, *g = nullptr, *beta = nullptr, *rows = nullptr;
    void *z = nullptr;          // [max_batch, D] LayerNorm output, param dtype
};

extern "C" void ep_head_destroy(ep_head_t *h)
{
    if (!h) return;
    if (h->mem) (void)hipFree(h->mem);
    delete h;
}

extern "C" ep_status ep_head_create(const ep_head_config *cfg, const void *ln_g, const void *ln_b, const void *w_head,
                                    const void *b_head, int32_t max_batch, ep_head_t **out)
{
    if (!out) return ep_fail(EP_ERR_INVALID_ARG, "ep_head_create: null output");
    *out = nullptr;
    if (!cfg || !ln_g || !ln_b || !w_head || !b_head) return ep_fail(EP_ERR_INVALID_ARG, "ep_head_create: null argument");
    if (cfg->d_model < 1 || cfg->n_tokens < 1 || cfg->n_classes < 1 || max_batch < 1 || !(cfg->ln_eps >= 0.f))
        return ep_fail(EP_ERR_INVALID_ARG, "ep_head_create: bad shape or ln_eps");
    if (cfg->param_dtype != EP_F32 && cfg->param_dtype != EP_BF16)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_head_create: unknown dtype");
    const bool bf16 = cfg->param_dtype == EP_BF16;
    if (bf16 && !ep_bf16_gemm_skinny_supported(max_batch, cfg->n_classes, cfg->d_model))
        return ep_fail(EP_ERR_UNSUPPORTED, "bf16 head needs n_classes %% 8 == 0, d_model %% 16 == 0 and max_batch <= 4096");
    if (cfg->d_model % 4 || cfg->d_model > 2048) return ep_fail(EP_ERR_UNSUPPORTED, "head needs d_model %% 4 == 0 and <= 2048");
    ep_head *h = new (std::nothrow) ep_head;
    if (!h) return ep_fail(EP_ERR_OOM, "ep_head_create: out of host memory");
    auto fail = [&](ep_status rc) { ep_head_destroy(h); return rc; };
    h->cfg = *cfg;
    h->max_batch = max_batch;
    h->bf16 = bf16;
    if (hipGetDevice(&h->device) != hipSuccess) return fail(ep_fail(EP_ERR_HIP, "hipGetDevice failed"));
    const int D = cfg->d_model, NC = cfg->n_classes;
    const size_t psz = bf16 ? 2 : 4;
    const size_t w_bytes = align_up((size_t)NC * D * psz, 256), b_bytes = align_up((size_t)NC * 4, 256);
    const size_t v_bytes = align_up((size_t)D * 4, 256), rows_bytes = align_up((size_t)max_batch * D * 4, 256);
    const size_t z_bytes = align_up((size_t)max_batch * D * psz, 256);
    h->mem_bytes = w_bytes + b_bytes + 2 * v_bytes + rows_bytes + z_bytes;
    hipError_t he = hipMalloc((void **)&h->mem, h->mem_bytes);
    if (he != hipSuccess) {
        h->mem = nullptr;
        return fail(ep_fail(EP_ERR_OOM, "hipMalloc of %zu bytes failed: %s", h->mem_bytes, hipGetErrorString(he)));
    }
    char *m = h->mem;
    h->w = m; m += w_bytes;
    h->b = (float *)m; m += b_bytes;
    h->g = (float *)m; m += v_bytes;
    h->beta = (float *)m; m += v_bytes;
    h->rows = (float *)m; m += rows_bytes;
    h->z = m;
    try {
        std::vector<float> v;
        if ((he = hipMemcpy(h->w, w_head, (size_t)NC * D * psz, hipMemcpyHostToDevice)) != hipSuccess)
            return fail(ep_fail(EP_ERR_HIP, "upload failed: %s", hipGetErrorString(he)));
        widen(b_head, NC, cfg->param_dtype, v);
        if ((he = hipMemcpy(h->b, v.data(), (size_t)NC * 4, hipMemcpyHostToDevice)) != hipSuccess)
            return fail(ep_fail(EP_ERR_HIP, "upload failed: %s", hipGetErrorString(he)));
        widen(ln_g, D, cfg->param_dtype, v);
        if ((he = hipMemcpy(h->g, v.data(), (size_t)D * 4, hipMemcpyHostToDevice)) != hipSuccess)
            return fail(ep_fail(EP_ERR_HIP, "upload failed: %s", hipGetErrorString(he)));
        widen(ln_b, D, cfg->param_dtype, v);
        if ((he = hipMemcpy(h->beta, v.data(), (size_t)D * 4, hipMemcpyHostToDevice)) != hipSuccess)
            return fail(ep_fail(EP_ERR_HIP, "upload failed: %s", hipGetErrorString(he)));
    } catch (...) {
        return fail(ep_fail(EP_ERR_OOM, "ep_head_create: out of host memory"));
    }
    *out = h;
    return EP_OK;
}

extern "C" ep_status ep_head_forward(ep_head_t *h, const void *x, int32_t B, void *logits, void *stream)
{
    if (!h || !x || !logits) return ep_fail(EP_ERR_INVALID_ARG, "ep_head_forward: null argument");
    if (B < 1 || B > h->max_batch)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_head_forward: B=%d outside [1, max_batch=%d]", B, h->max_batch);
    int dev = -1;
    EP_HIP(hipGetDevice(&dev));
    if (dev != h->device)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_head_forward: created on device %d, current device is %d", h->device, dev);
    hipStream_t s = (hipStream_t)stream;
    const ep_head_config &c = h->cfg;
    const int D = c.d_model, NC = c.n_classes;
    const int64_t n = (int64_t)B * D;
    hipLaunchKernelGGL(head_gather_kernel, dim3(blocks_for(n)), dim3(256), 0, s, (const float *)x, h->rows, n, c.n_tokens, D);
    EP_HIP(hipGetLastError());
    if (h->bf16) {
        EP_HIP(ep_bf16_layernorm(h->rows, h->g, h->beta, c.ln_eps, (uint16_t *)h->z, B, D, s));
        EP_HIP(ep_bf16_gemm_skinny((const uint16_t *)h->z, (const uint16_t *)h->w, h->b, nullptr, logits, B, NC, D,
                                   EPI_BIAS_F32, s));
    } else {
        EP_HIP(ep_f32_layernorm(h->rows, h->g, h->beta, c.ln_eps, (float *)h->z, B, D, s));
        EP_HIP(ep_f32_gemm((const float *)h->z, (const float *)h->w, h->b, nullptr, (float *)logits, B, NC, D, EPI_BIAS, s));
    }
    return EP_OK;
}
