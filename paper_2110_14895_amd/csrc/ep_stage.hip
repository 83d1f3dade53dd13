// Stage handle and launch sequencing: a pipeline stage T_i is a run of
// consecutive encoder layers applied to one micro-batch (paper section 3.1);
// each layer is LayerNorm -> q|k|v projection -> multi-head attention ->
// output projection + residual -> LayerNorm -> MLP with GELU + residual
// (section 2.1).  ep_stage_forward only enqueues kernels on the caller's
// stream; all device memory is obtained in ep_stage_create.
//
// Workspace per stage (R = max_batch * T rows):
//   x    fp32 [R, D]            residual stream
//   a    act  [R, D]            LayerNorm output, later the attention output
//   big  act  [R, max(3D, M)]   q|k|v, later the MLP hidden activations
//   part fp32 [S, R, D]         bf16 path, small R only: the second MLP layer's sums over S ranges of K
// where act is bf16 on the bf16 path and fp32 on the fp32 path.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "edgepipe.h"
#include "ep_error.h"
#include "ep_kernels.h"
#include "ep_launch.h"

namespace {

struct LayerDev {
    const void *w_qkv, *w_o, *w_fc1, *w_fc2;                       // param dtype
    const float *ln1_g, *ln1_b, *b_qkv, *b_o, *ln2_g, *ln2_b, *b_fc1, *b_fc2;   // always fp32
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline float bf16_bits_to_float(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

}  // namespace

// where a forward keeps its intermediates (see the file header)
struct Workspace {
    float *x;
    void *a;
    void *big;
    float *part;
    size_t part_bytes;
};

struct ep_stage {
    ep_vit_config cfg;
    int32_t begin, end, max_batch;
    int device;
    bool bf16;
    char *params = nullptr;
    size_t params_bytes = 0;
    char *ws = nullptr;
    size_t ws_bytes = 0;
    Workspace own = {nullptr, nullptr, nullptr, nullptr, 0};   // inside ws
    std::vector<LayerDev> layers;
    // per-kernel timing (ep_stage_trace_begin / _end)
    int trace_kernel = -1;
    size_t trace_used = 0;
    std::vector<hipEvent_t> trace_ev;      // pairs: start, stop
};

#define EP_HIP(call)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            return ep_fail(EP_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));       \
    } while (0)

namespace {

ep_status check_config(const ep_vit_config *c)
{
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_mlp < 1 || c->n_tokens < 1)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_create: non-positive shape in config");
    if (c->d_model % c->n_heads)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_create: d_model %d not divisible by n_heads %d",
                       c->d_model, c->n_heads);
    if (!(c->ln_eps >= 0.f))
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_create: ln_eps must be >= 0");
    auto is_dt = [](int32_t d) { return d == EP_F32 || d == EP_BF16; };
    if (!is_dt(c->param_dtype) || !is_dt(c->in_dtype) || !is_dt(c->out_dtype))
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_create: unknown dtype");
    if (c->param_dtype == EP_F32) {
        if (c->in_dtype != EP_F32 || c->out_dtype != EP_F32)
            return ep_fail(EP_ERR_UNSUPPORTED, "fp32 parameters require fp32 input and output");
        if (c->n_tokens > 8192)
            return ep_fail(EP_ERR_UNSUPPORTED, "fp32 path supports at most 8192 tokens");
    } else {
        const int dh = c->d_model / c->n_heads;
        if (c->d_model % 64 || c->d_mlp % 64)
            return ep_fail(EP_ERR_UNSUPPORTED, "bf16 path needs d_model and d_mlp divisible by 64");
        if (c->d_model > 2048)
            return ep_fail(EP_ERR_UNSUPPORTED, "bf16 path supports d_model <= 2048");
        if (!ep_bf16_attention_supported(c->n_tokens, dh))
            return ep_fail(EP_ERR_UNSUPPORTED,
                           "bf16 attention supports d_head in {64, 80} and n_tokens <= 4096 (got %d, %d)",
                           dh, c->n_tokens);
    }
    return EP_OK;
}

// K ranges of the second MLP layer at `batch` images (1: the layer runs uncut) and the bytes their sums take
int fc2_splits(const ep_vit_config &c, int64_t batch)
{
    return c.param_dtype == EP_BF16 ? ep_bf16_gemm_splits(batch * c.n_tokens, c.d_model, c.d_mlp) : 1;
}

size_t part_bytes(const ep_vit_config &c, int64_t batch)
{
    const int sp = fc2_splits(c, batch);
    return sp > 1 ? align_up((size_t)sp * batch * c.n_tokens * c.d_model * 4, 256) : 0;
}

// Workspace of a forward: x | a | big for `batch` images, then `part_b` bytes for the sums over K ranges;
// each part 256-byte aligned.
struct WorkspaceLayout { size_t x_bytes, a_bytes, big_bytes, part_b; };

WorkspaceLayout workspace_layout(const ep_vit_config &c, int64_t batch, size_t part_b)
{
    const size_t asz = c.param_dtype == EP_BF16 ? 2 : 4;     // bytes per activation-operand element
    const size_t R = (size_t)batch * c.n_tokens, D = c.d_model, M = c.d_mlp;
    const size_t wide = 3 * D > M ? 3 * D : M;
    return {align_up(R * D * 4, 256), align_up(R * D * asz, 256), align_up(R * wide * asz, 256), part_b};
}

size_t workspace_bytes(const ep_vit_config &c, int64_t batch, size_t part_b)
{
    const WorkspaceLayout l = workspace_layout(c, batch, part_b);
    return l.x_bytes + l.a_bytes + l.big_bytes + l.part_b;
}

Workspace carve_workspace(char *base, const ep_vit_config &c, int64_t batch, size_t part_b)
{
    const WorkspaceLayout l = workspace_layout(c, batch, part_b);
    char *part = base + l.x_bytes + l.a_bytes + l.big_bytes;
    return {(float *)base, base + l.x_bytes, base + l.x_bytes + l.a_bytes, part_b ? (float *)part : nullptr, part_b};
}

// Brackets one kernel of the layer with an event pair when that kernel is traced.  For a dense
// layer traced under its _MAIN id the closing event is handed to the GEMM dispatcher, which
// records it right after its first launch.
struct TraceScope {
    ep_stage *st; hipStream_t s; bool on, main_only;
    TraceScope(ep_stage *st_, int kernel, int main_id, hipStream_t s_) : st(st_), s(s_), on(false), main_only(false)
    {
        const bool hit = st->trace_kernel == kernel || (main_id >= 0 && st->trace_kernel == main_id);
        if (hit && st->trace_used + 2 <= st->trace_ev.size()) {
            on = hipEventRecord(st->trace_ev[st->trace_used], s) == hipSuccess;
            main_only = on && st->trace_kernel == main_id;
        }
    }
    hipEvent_t after_main() const { return main_only ? st->trace_ev[st->trace_used + 1] : nullptr; }
    ~TraceScope()
    {
        if (on) {
            if (!main_only) (void)hipEventRecord(st->trace_ev[st->trace_used + 1], s);
            st->trace_used += 2;
        }
    }
};
#define EP_TRACED(kernel, call) do { TraceScope ts_(st, kernel, -1, s); EP_HIP(call); } while (0)
// `call` may use ts_.after_main()
#define EP_TRACED_GEMM(kernel, main_id, call) do { TraceScope ts_(st, kernel, main_id, s); EP_HIP(call); } while (0)

// What a layer whose second MLP layer ran cut into K ranges has left for its successor: the residual stream
// in w.x still lacks ((part[0] + ... + part[splits-1]) + bias).
struct PendingSum { int splits; const float *bias; };

// One layer on R = B*T rows.  `xin` is the residual stream read by this layer
// (may be the caller's fp32 input), the layer leaves its result in `xout`.
// `before`: the layer in front left its sums over K ranges in w.part (xin is w.x then); this layer's first
// LayerNorm adds them.  `after`: if non-null the layer may leave its own in the same way (then xout must be
// w.x, and *after says so with splits > 1); if null it finishes its output itself.
ep_status run_layer(ep_stage *st, const Workspace &w, const LayerDev &L, const float *xin, float *xout, int B,
                    hipStream_t s, const PendingSum *before, PendingSum *after)
{
    const ep_vit_config &c = st->cfg;
    const int T = c.n_tokens, D = c.d_model, M = c.d_mlp, H = c.n_heads;
    const int64_t R = (int64_t)B * T;
    if (after) *after = {1, nullptr};
    if (st->bf16) {
        uint16_t *a = (uint16_t *)w.a, *big = (uint16_t *)w.big;
        if (before && before->splits > 1)
            EP_TRACED(EP_K_LN1, ep_bf16_layernorm_sum(w.x, w.part, before->splits, before->bias, L.ln1_g, L.ln1_b,
                                                      c.ln_eps, a, R, D, s));
        else
            EP_TRACED(EP_K_LN1, ep_bf16_layernorm(xin, L.ln1_g, L.ln1_b, c.ln_eps, a, R, D, s));
        EP_TRACED_GEMM(EP_K_QKV, EP_K_QKV_MAIN,
                       ep_bf16_gemm(a, (const uint16_t *)L.w_qkv, L.b_qkv, nullptr, big, R, 3 * D, D, EPI_BIAS,
                                    ts_.after_main(), s));
        EP_TRACED(EP_K_ATTN, ep_bf16_attention(big, a, B, T, D, H, s));
        EP_TRACED_GEMM(EP_K_PROJ, EP_K_PROJ_MAIN,
                       ep_bf16_gemm(a, (const uint16_t *)L.w_o, L.b_o, xin, w.x, R, D, D, EPI_BIAS_RESID,
                                    ts_.after_main(), s));
        EP_TRACED(EP_K_LN2, ep_bf16_layernorm(w.x, L.ln2_g, L.ln2_b, c.ln_eps, a, R, D, s));
        EP_TRACED_GEMM(EP_K_FC1, EP_K_FC1_MAIN,
                       ep_bf16_gemm(a, (const uint16_t *)L.w_fc1, L.b_fc1, nullptr, big, R, M, D, EPI_BIAS_GELU,
                                    ts_.after_main(), s));
        int sp = w.part ? fc2_splits(c, B) : 1;
        if ((size_t)sp * R * D * 4 > w.part_bytes) sp = 1;      // never beyond what the workspace holds
        if (sp > 1) {
            // few tiles and a long K: one workgroup per (K range, tile); the sums are added by the next
            // layer's first LayerNorm, or here when nobody follows
            TraceScope ts_(st, EP_K_FC2, EP_K_FC2_MAIN, s);
            EP_HIP(ep_bf16_gemm_partial(big, (const uint16_t *)L.w_fc2, w.part, R, D, M, sp, s));
            if (ts_.after_main()) EP_HIP(hipEventRecord(ts_.after_main(), s));
            if (after && xout == w.x)
                *after = {sp, L.b_fc2};
            else
                EP_HIP(ep_f32_residual_sum(w.x, w.part, sp, L.b_fc2, xout, R, D, s));
        } else {
            EP_TRACED_GEMM(EP_K_FC2, EP_K_FC2_MAIN,
                           ep_bf16_gemm(big, (const uint16_t *)L.w_fc2, L.b_fc2, w.x, xout, R, D, M, EPI_BIAS_RESID,
                                        ts_.after_main(), s));
        }
    } else {
        float *a = (float *)w.a, *big = (float *)w.big;
        EP_TRACED(EP_K_LN1, ep_f32_layernorm(xin, L.ln1_g, L.ln1_b, c.ln_eps, a, R, D, s));
        EP_TRACED(EP_K_QKV, ep_f32_gemm(a, (const float *)L.w_qkv, L.b_qkv, nullptr, big, R, 3 * D, D, EPI_BIAS, s));
        EP_TRACED(EP_K_ATTN, ep_f32_attention(big, a, B, T, D, H, s));
        EP_TRACED(EP_K_PROJ, ep_f32_gemm(a, (const float *)L.w_o, L.b_o, xin, w.x, R, D, D, EPI_BIAS_RESID, s));
        EP_TRACED(EP_K_LN2, ep_f32_layernorm(w.x, L.ln2_g, L.ln2_b, c.ln_eps, a, R, D, s));
        EP_TRACED(EP_K_FC1, ep_f32_gemm(a, (const float *)L.w_fc1, L.b_fc1, nullptr, big, R, M, D, EPI_BIAS_GELU, s));
        EP_TRACED(EP_K_FC2, ep_f32_gemm(big, (const float *)L.w_fc2, L.b_fc2, w.x, xout, R, D, M, EPI_BIAS_RESID, s));
    }
    return EP_OK;
}

}  // namespace

// ---- the library's own workspace for callers that cannot allocate -------------------------------
// One array per device, part of the loaded code object, held until the process ends.  In host code
// the array's name stands for the symbol, not for device memory: its device address is looked up
// once per device (with that device current) and only that address is handed to kernels.
static __device__ __align__(256) unsigned char scratch[EP_STATIC_SCRATCH_BYTES];

namespace {

std::atomic<unsigned char *> g_scratch_ptr[EP_MAX_DEVICES];      // zero-initialised

// device address of `scratch` on the current device `dev`
ep_status static_scratch(int dev, unsigned char **out)
{
    if (dev < 0 || dev >= EP_MAX_DEVICES)
        return ep_fail(EP_ERR_UNSUPPORTED, "device index %d outside the %d the library keeps a workspace for", dev,
                       EP_MAX_DEVICES);
    unsigned char *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        EP_HIP(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
        if (!p) return ep_fail(EP_ERR_HIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev].store(p, std::memory_order_release);    // every thread stores the same address
    }
    *out = p;
    return EP_OK;
}

}  // namespace

extern "C" ep_status ep_stage_create(const ep_vit_config *cfg, int32_t layer_begin, int32_t layer_end,
                                     const ep_layer_weights *layers, int32_t max_batch, ep_stage_t **out)
{
    ep_clear_error();
    if (!cfg || !layers || !out) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_create: null argument");
    *out = nullptr;
    ep_status rc = check_config(cfg);
    if (rc != EP_OK) return rc;
    if (layer_begin < 0 || layer_end <= layer_begin || layer_end > cfg->n_layers)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_create: layer range [%d, %d) not inside [0, %d)",
                       layer_begin, layer_end, cfg->n_layers);
    if (max_batch < 1) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_create: max_batch must be >= 1");
    const int nl = layer_end - layer_begin;
    const int64_t D = cfg->d_model, M = cfg->d_mlp, T = cfg->n_tokens;
    if ((int64_t)max_batch * T > (1ll << 24))
        return ep_fail(EP_ERR_UNSUPPORTED, "ep_stage_create: max_batch * n_tokens exceeds 2^24 rows");
    {
        // what the kernels of a forward over max_batch images index with 32 bits (or a 16-bit grid
        // dimension): refuse here rather than in the middle of a forward
        const int64_t R = (int64_t)max_batch * T, wide = 3 * D > M ? 3 * D : M, deep = D > M ? D : M;
        bool fits;
        if (cfg->param_dtype == EP_BF16)
            fits = R * wide < (1ll << 31) && R * deep * 2 < 0x7FFFFFF0ll && wide * deep * 2 < 0x7FFFFFF0ll;
        else
            fits = (R + 63) / 64 <= 65535 && max_batch <= 65535 && cfg->n_heads <= 65535;
        if (!fits)
            return ep_fail(EP_ERR_UNSUPPORTED,
                           "ep_stage_create: max_batch %d gives %lld rows, more than the dense layers of this "
                           "width can index", max_batch, (long long)R);
    }
    for (int l = 0; l < nl; ++l) {
        const ep_layer_weights &w = layers[l];
        if (!w.ln1_g || !w.ln1_b || !w.w_qkv || !w.b_qkv || !w.w_o || !w.b_o || !w.ln2_g || !w.ln2_b ||
            !w.w_fc1 || !w.b_fc1 || !w.w_fc2 || !w.b_fc2)
            return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_create: null parameter pointer in layer %d", l);
    }

    ep_stage *st = new (std::nothrow) ep_stage();
    if (!st) return ep_fail(EP_ERR_OOM, "ep_stage_create: host allocation failed");
    st->cfg = *cfg;
    st->begin = layer_begin; st->end = layer_end; st->max_batch = max_batch;
    st->bf16 = cfg->param_dtype == EP_BF16;
    const size_t wsz = st->bf16 ? 2 : 4;     // bytes per dense-weight element

    auto fail = [&](ep_status s) { ep_stage_destroy(st); return s; };
    hipError_t e = hipGetDevice(&st->device);
    if (e != hipSuccess) return fail(ep_fail(EP_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e)));
    {
        // set-up for ep_stage_forward_static on this device: the address of the library's own workspace
        unsigned char *unused = nullptr;
        const ep_status src = static_scratch(st->device, &unused);
        if (src != EP_OK) return fail(src);
    }

    // ---- parameter block layout (per layer): dense weights, then fp32 vectors
    const size_t n_w[4] = {(size_t)(3 * D * D), (size_t)(D * D), (size_t)(M * D), (size_t)(D * M)};
    const size_t n_v[8] = {(size_t)D, (size_t)D, (size_t)(3 * D), (size_t)D,
                           (size_t)D, (size_t)D, (size_t)M, (size_t)D};
    size_t layer_bytes = 0;
    size_t off_w[4], off_v[8];
    for (int i = 0; i < 4; ++i) { off_w[i] = layer_bytes; layer_bytes += align_up(n_w[i] * wsz, 256); }
    for (int i = 0; i < 8; ++i) { off_v[i] = layer_bytes; layer_bytes += align_up(n_v[i] * 4, 256); }
    st->params_bytes = layer_bytes * nl;
    e = hipMalloc((void **)&st->params, st->params_bytes);
    if (e != hipSuccess) {
        st->params = nullptr;
        return fail(ep_fail(EP_ERR_OOM, "hipMalloc of %zu parameter bytes failed: %s", st->params_bytes,
                            hipGetErrorString(e)));
    }

    // ---- workspace; the sums over K ranges only exist at small micro-batches (at most 2^15 rows), sized
    // for the micro-batch that needs most
    size_t part_max = 0;
    for (int64_t b = 1; b <= max_batch && (b - 1) * T <= (1 << 15); ++b) {
        const size_t pb = part_bytes(st->cfg, b);
        if (pb > part_max) part_max = pb;
    }
    st->ws_bytes = workspace_bytes(st->cfg, max_batch, part_max);
    e = hipMalloc((void **)&st->ws, st->ws_bytes);
    if (e != hipSuccess) {
        st->ws = nullptr;
        return fail(ep_fail(EP_ERR_OOM, "hipMalloc of %zu workspace bytes failed: %s", st->ws_bytes,
                            hipGetErrorString(e)));
    }
    st->own = carve_workspace(st->ws, st->cfg, max_batch, part_max);

    // ---- upload, one layer at a time through a host staging block
    std::vector<char> stage_buf;
    try {
        stage_buf.resize(layer_bytes);
    } catch (...) {
        return fail(ep_fail(EP_ERR_OOM, "ep_stage_create: host staging allocation failed"));
    }
    st->layers.resize(nl);
    for (int l = 0; l < nl; ++l) {
        const ep_layer_weights &w = layers[l];
        const void *src_w[4] = {w.w_qkv, w.w_o, w.w_fc1, w.w_fc2};
        const void *src_v[8] = {w.ln1_g, w.ln1_b, w.b_qkv, w.b_o, w.ln2_g, w.ln2_b, w.b_fc1, w.b_fc2};
        std::memset(stage_buf.data(), 0, layer_bytes);
        for (int i = 0; i < 4; ++i) std::memcpy(stage_buf.data() + off_w[i], src_w[i], n_w[i] * wsz);
        for (int i = 0; i < 8; ++i) {
            float *dst = reinterpret_cast<float *>(stage_buf.data() + off_v[i]);
            if (st->bf16) {
                const uint16_t *sv = static_cast<const uint16_t *>(src_v[i]);
                for (size_t k = 0; k < n_v[i]; ++k) dst[k] = bf16_bits_to_float(sv[k]);   // exact widening
            } else {
                std::memcpy(dst, src_v[i], n_v[i] * 4);
            }
        }
        char *base = st->params + (size_t)l * layer_bytes;
        e = hipMemcpy(base, stage_buf.data(), layer_bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess)
            return fail(ep_fail(EP_ERR_HIP, "parameter upload failed: %s", hipGetErrorString(e)));
        LayerDev &d = st->layers[l];
        d.w_qkv = base + off_w[0]; d.w_o = base + off_w[1]; d.w_fc1 = base + off_w[2]; d.w_fc2 = base + off_w[3];
        d.ln1_g = (const float *)(base + off_v[0]); d.ln1_b = (const float *)(base + off_v[1]);
        d.b_qkv = (const float *)(base + off_v[2]); d.b_o = (const float *)(base + off_v[3]);
        d.ln2_g = (const float *)(base + off_v[4]); d.ln2_b = (const float *)(base + off_v[5]);
        d.b_fc1 = (const float *)(base + off_v[6]); d.b_fc2 = (const float *)(base + off_v[7]);
    }
    *out = st;
    return EP_OK;
}

namespace {

// the launches of a forward over B images with the intermediates in `w`
ep_status forward_on(ep_stage *st, const Workspace &w, const void *x_in, int32_t B, void *x_out, hipStream_t s)
{
    const ep_vit_config &c = st->cfg;
    const int64_t n = (int64_t)B * c.n_tokens * c.d_model;
    const int nl = st->end - st->begin;

    const float *cur;
    if (c.in_dtype == EP_BF16) {
        EP_HIP(ep_bf16_to_f32((const uint16_t *)x_in, w.x, n, s));
        cur = w.x;
    } else {
        cur = (const float *)x_in;     // first layer reads the caller's buffer directly
    }
    PendingSum pending = {1, nullptr};
    for (int l = 0; l < nl; ++l) {
        const bool last = l + 1 == nl;
        float *dst = (last && c.out_dtype == EP_F32) ? (float *)x_out : w.x;
        const PendingSum before = pending;
        ep_status rc = run_layer(st, w, st->layers[l], cur, dst, B, s, &before, last ? nullptr : &pending);
        if (rc != EP_OK) return rc;
        cur = dst;
    }
    if (c.out_dtype == EP_BF16) EP_HIP(ep_f32_to_bf16(w.x, (uint16_t *)x_out, n, s));
    return EP_OK;
}

}  // namespace

extern "C" ep_status ep_stage_forward(ep_stage_t *st, const void *x_in, int32_t B, void *x_out, void *stream)
{
    if (!st || !x_in || !x_out) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_forward: null argument");
    if (B < 1 || B > st->max_batch)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_forward: B=%d outside [1, max_batch=%d]", B, st->max_batch);
    int dev = -1;
    EP_HIP(hipGetDevice(&dev));
    if (dev != st->device)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_forward: stage lives on device %d, current device is %d",
                       st->device, dev);
    return forward_on(st, st->own, x_in, B, x_out, (hipStream_t)stream);
}

extern "C" ep_status ep_stage_forward_static(ep_stage_t *st, const void *x_in, int32_t B, void *x_out, void *stream)
{
    if (!st || !x_in || !x_out) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_forward_static: null argument");
    if (B < 1) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_forward_static: B=%d, must be >= 1", B);
    // the sums over K ranges are an optimisation of small micro-batches: where they do not fit next to the rest,
    // the second MLP layer runs uncut (same result up to the order of the fp32 additions over K)
    const size_t need = workspace_bytes(st->cfg, B, 0);
    size_t part_b = part_bytes(st->cfg, B);
    if (need + part_b > (size_t)EP_STATIC_SCRATCH_BYTES) part_b = 0;
    if (need > (size_t)EP_STATIC_SCRATCH_BYTES)
        return ep_fail(EP_ERR_UNSUPPORTED,
                       "ep_stage_forward_static: a micro-batch of %d images needs %zu workspace bytes, the library's "
                       "own workspace holds %zu", B, need, (size_t)EP_STATIC_SCRATCH_BYTES);
    int dev = -1;
    EP_HIP(hipGetDevice(&dev));
    if (dev != st->device)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_forward_static: stage lives on device %d, current device is %d",
                       st->device, dev);
    unsigned char *base = nullptr;
    const ep_status rc = static_scratch(dev, &base);      // looked up when the stage was created: a table read
    if (rc != EP_OK) return rc;
    return forward_on(st, carve_workspace((char *)base, st->cfg, B, part_b), x_in, B, x_out, (hipStream_t)stream);
}

extern "C" ep_status ep_stage_profile(ep_stage_t *st, int32_t B, int32_t iters, void *stream,
                                      double *per_layer_seconds)
{
    if (!st || !per_layer_seconds) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_profile: null argument");
    if (B < 1 || B > st->max_batch || iters < 1)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_profile: need 1 <= B <= max_batch and iters >= 1");
    int dev = -1;
    EP_HIP(hipGetDevice(&dev));
    if (dev != st->device)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_profile: stage lives on device %d, current device is %d",
                       st->device, dev);
    hipStream_t s = (hipStream_t)stream;
    const ep_vit_config &c = st->cfg;
    const int64_t n = (int64_t)B * c.n_tokens * c.d_model;
    const int nl = st->end - st->begin;
    hipEvent_t t0, t1;
    EP_HIP(hipEventCreate(&t0));
    hipError_t e = hipEventCreate(&t1);
    if (e != hipSuccess) {
        (void)hipEventDestroy(t0);
        return ep_fail(EP_ERR_HIP, "hipEventCreate failed: %s", hipGetErrorString(e));
    }
    ep_status rc = EP_OK;
    for (int l = 0; l < nl && rc == EP_OK; ++l) {
        // fresh, bounded input for every layer so that repeated application cannot drift
        if ((e = ep_fill_pattern(st->own.x, n, s)) != hipSuccess) { rc = ep_fail(EP_ERR_HIP, "fill failed: %s", hipGetErrorString(e)); break; }
        rc = run_layer(st, st->own, st->layers[l], st->own.x, st->own.x, B, s, nullptr, nullptr);          // untimed
        if (rc != EP_OK) break;
        if ((e = ep_fill_pattern(st->own.x, n, s)) != hipSuccess) { rc = ep_fail(EP_ERR_HIP, "fill failed: %s", hipGetErrorString(e)); break; }
        if ((e = hipEventRecord(t0, s)) != hipSuccess) { rc = ep_fail(EP_ERR_HIP, "hipEventRecord failed: %s", hipGetErrorString(e)); break; }
        for (int it = 0; it < iters && rc == EP_OK; ++it) rc = run_layer(st, st->own, st->layers[l], st->own.x, st->own.x, B, s, nullptr, nullptr);
        if (rc != EP_OK) break;
        if ((e = hipEventRecord(t1, s)) != hipSuccess) { rc = ep_fail(EP_ERR_HIP, "hipEventRecord failed: %s", hipGetErrorString(e)); break; }
        if ((e = hipEventSynchronize(t1)) != hipSuccess) { rc = ep_fail(EP_ERR_HIP, "hipEventSynchronize failed: %s", hipGetErrorString(e)); break; }
        float ms = 0.f;
        if ((e = hipEventElapsedTime(&ms, t0, t1)) != hipSuccess) { rc = ep_fail(EP_ERR_HIP, "hipEventElapsedTime failed: %s", hipGetErrorString(e)); break; }
        per_layer_seconds[l] = (double)ms * 1e-3 / iters;
    }
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    return rc;
}

extern "C" ep_status ep_stage_trace_begin(ep_stage_t *st, int32_t kernel, int32_t max_launches)
{
    if (!st) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_trace_begin: null stage");
    if (kernel < 0 || kernel >= EP_K_TRACE_COUNT || max_launches < 1 || max_launches > (1 << 20))
        return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_trace_begin: bad kernel id or max_launches");
    if (kernel >= EP_K_COUNT && !st->bf16)
        return ep_fail(EP_ERR_UNSUPPORTED, "ep_stage_trace_begin: the _MAIN ids exist on the bf16 path only");
    if (st->trace_kernel >= 0) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_trace_begin: a trace is already active");
    st->trace_ev.clear();
    st->trace_ev.reserve((size_t)max_launches * 2);
    for (int i = 0; i < max_launches * 2; ++i) {
        hipEvent_t ev;
        hipError_t e = hipEventCreate(&ev);
        if (e != hipSuccess) {
            for (hipEvent_t x : st->trace_ev) (void)hipEventDestroy(x);
            st->trace_ev.clear();
            return ep_fail(EP_ERR_HIP, "hipEventCreate failed: %s", hipGetErrorString(e));
        }
        st->trace_ev.push_back(ev);
    }
    st->trace_used = 0;
    st->trace_kernel = kernel;
    return EP_OK;
}

extern "C" ep_status ep_stage_trace_end(ep_stage_t *st, int32_t *launches, double *seconds)
{
    if (!st || !launches || !seconds) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_trace_end: null argument");
    if (st->trace_kernel < 0) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_trace_end: no active trace");
    ep_status rc = EP_OK;
    double total = 0.0;
    for (size_t i = 0; i + 1 < st->trace_used && rc == EP_OK; i += 2) {
        hipError_t e = hipEventSynchronize(st->trace_ev[i + 1]);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, st->trace_ev[i], st->trace_ev[i + 1]);
        if (e != hipSuccess) rc = ep_fail(EP_ERR_HIP, "reading trace events failed: %s", hipGetErrorString(e));
        total += (double)ms * 1e-3;
    }
    for (hipEvent_t x : st->trace_ev) (void)hipEventDestroy(x);
    st->trace_ev.clear();
    if (rc == EP_OK) { *launches = (int32_t)(st->trace_used / 2); *seconds = total; }
    st->trace_used = 0;
    st->trace_kernel = -1;
    return rc;
}

extern "C" ep_status ep_stage_gemm_main_rows(const ep_stage_t *st, int32_t B, int32_t kernel, int64_t *rows)
{
    if (!st || !rows) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_gemm_main_rows: null argument");
    if (B < 0 || B > st->max_batch) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_gemm_main_rows: batch out of range");
    const ep_vit_config &c = st->cfg;
    const int64_t R = (int64_t)B * c.n_tokens;
    int N = 0, K = 0;
    switch (kernel) {
    case EP_K_QKV: case EP_K_QKV_MAIN: N = 3 * c.d_model; K = c.d_model; break;
    case EP_K_PROJ: case EP_K_PROJ_MAIN: N = c.d_model; K = c.d_model; break;
    case EP_K_FC1: case EP_K_FC1_MAIN: N = c.d_mlp; K = c.d_model; break;
    case EP_K_FC2: case EP_K_FC2_MAIN: N = c.d_model; K = c.d_mlp; break;
    default: return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_gemm_main_rows: kernel %d is not a dense layer", kernel);
    }
    *rows = st->bf16 && R > 0 ? ep_bf16_gemm_main_rows(R, N, K) : R;
    return EP_OK;
}

extern "C" ep_status ep_stage_info(const ep_stage_t *st, ep_vit_config *cfg, int32_t *layer_begin, int32_t *layer_end,
                                   int32_t *max_batch)
{
    if (!st) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_info: null stage");
    if (cfg) *cfg = st->cfg;
    if (layer_begin) *layer_begin = st->begin;
    if (layer_end) *layer_end = st->end;
    if (max_batch) *max_batch = st->max_batch;
    return EP_OK;
}

extern "C" ep_status ep_stage_device_bytes(const ep_stage_t *st, uint64_t *bytes)
{
    if (!st || !bytes) return ep_fail(EP_ERR_INVALID_ARG, "ep_stage_device_bytes: null argument");
    *bytes = (uint64_t)st->params_bytes + (uint64_t)st->ws_bytes;
    return EP_OK;
}

extern "C" void ep_stage_destroy(ep_stage_t *st)
{
    if (!st) return;
    if (st->params) (void)hipFree(st->params);
    if (st->ws) (void)hipFree(st->ws);
    for (hipEvent_t x : st->trace_ev) (void)hipEventDestroy(x);
    delete st;
}
