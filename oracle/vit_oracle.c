/*
 * CPU checker for the forward pass of one pipeline stage: a contiguous run of
 * ViT encoder layers applied to a micro-batch.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU
 * library's results can be compared against a plain statement of what a
 * stage computes.  Only the tests, the smoke check and the CPU-baseline leg of
 * the benchmark may call it.  It shares no source with the GPU library.
 *
 * What is computed (paper section 2.1, "Transformer-based Models": a layer is
 * multi-head self-attention, an MLP, two layer normalisations and residual
 * connections; section 3.1: a stage T_i is l_i consecutive layers and the
 * model is the composition T_k(...T_1(X)); section 2.1 "Pipeline Parallelism":
 * a micro-batch is a chunk of independent inputs).  The paper takes the layer
 * definition from the ViT architecture it cites; the specifics the paper does
 * not spell out are read as: pre-LN ordering, fused q|k|v projection with
 * head-major columns, softmax over all T tokens with scale 1/sqrt(d_head), no
 * mask, exact erf GELU, biased variance, biases on all four dense layers.
 *
 * Arithmetic: every intermediate is float64, loops are in the natural order of
 * the definitions, no blocking, no fusion, no library calls other than libm.
 * Parameters and inputs arrive as float32 values (what the GPU library is
 * handed, e.g. bf16-representable numbers) and are widened exactly.
 *
 * round_mode (diagnostic only, never the graded comparison): 0 = no rounding
 * anywhere; 1 = round-to-nearest-even to bf16 at the five points where a bf16
 * pipeline narrows a GEMM operand (both LayerNorm outputs, qkv, attention
 * probabilities, attention output, GELU output).  Mode 1 separates operand
 * quantisation noise from kernel defects.
 *
 * Parity pins: see tests/test_oracle_vit.py (closed forms, invariants,
 * hand-expanded attention on 2-4 tokens, library routines in float64).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t d_model;   /* D */
    int32_t n_heads;   /* H, d_head = D / H */
    int32_t d_mlp;     /* M */
    int32_t n_tokens;  /* T */
    double ln_eps;
    int32_t round_mode;
} epo_config;

typedef struct {
    const float *ln1_g, *ln1_b;   /* [D] */
    const float *w_qkv, *b_qkv;   /* [3D, D], [3D]; rows q | k | v, head-major */
    const float *w_o, *b_o;       /* [D, D], [D] */
    const float *ln2_g, *ln2_b;   /* [D] */
    const float *w_fc1, *b_fc1;   /* [M, D], [M] */
    const float *w_fc2, *b_fc2;   /* [D, M], [D] */
} epo_layer;

/* bf16 round-to-nearest-even of a double that is first narrowed to float32
 * (the GPU pipeline narrows from float32 accumulators).  Exported so that the
 * tests can pin it on its own: ties, double rounding, infinities, NaN. */
double epo_round_bf16(double v)
{
    float f = (float)v;
    uint32_t b;
    memcpy(&b, &f, 4);
    if ((b & 0x7F800000u) == 0x7F800000u) return (double)f; /* inf / nan pass */
    b += 0x7FFFu + ((b >> 16) & 1u);
    b &= 0xFFFF0000u;
    memcpy(&f, &b, 4);
    return (double)f;
}

static void maybe_round(double *a, size_t n, int mode)
{
    if (!mode) return;
    for (size_t i = 0; i < n; ++i) a[i] = epo_round_bf16(a[i]);
}

/* y[r, :] = (x[r, :] - mean) / sqrt(var + eps) * g + b, mean and biased
 * variance over the D entries of the row, two passes. */
void epo_layernorm(const double *x, int64_t rows, int32_t D, const float *g, const float *b,
                   double eps, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * D;
        double *yr = y + r * D;
        double mean = 0.0;
        for (int32_t d = 0; d < D; ++d) mean += xr[d];
        mean /= (double)D;
        double var = 0.0;
        for (int32_t d = 0; d < D; ++d) var += (xr[d] - mean) * (xr[d] - mean);
        var /= (double)D;
        double inv = 1.0 / sqrt(var + eps);
        for (int32_t d = 0; d < D; ++d) yr[d] = (xr[d] - mean) * inv * (double)g[d] + (double)b[d];
    }
}

/* y[r, n] = sum_k x[r, k] * W[n, k] + bias[n]   (W is [N, K], "out, in"). */
void epo_linear(const double *x, int64_t rows, int32_t K, const float *W, const float *bias,
                int32_t N, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * K;
        for (int32_t n = 0; n < N; ++n) {
            const float *wn = W + (int64_t)n * K;
            double acc = 0.0;
            for (int32_t k = 0; k < K; ++k) acc += xr[k] * (double)wn[k];
            y[r * N + n] = acc + (double)bias[n];
        }
    }
}

/* gelu(u) = u/2 * (1 + erf(u / sqrt 2)) */
void epo_gelu(const double *x, int64_t n, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) y[i] = 0.5 * x[i] * (1.0 + erf(x[i] / sqrt(2.0)));
}

/* Multi-head self-attention of ONE image.  qkv is [T, 3D]; column h*dh+e of
 * the first D columns is q of head h, the next D columns k, the last D
 * columns v.  For every head h and query t:
 *   s[u] = (sum_e q[t,e] k[u,e]) / sqrt(dh),  p = softmax_u(s),
 *   o[t, h*dh+e] = sum_u p[u] v[u,e].
 * If probs is not NULL it receives p as [H, T, T]. */
void epo_attention(const double *qkv, int32_t T, int32_t D, int32_t H, int round_mode,
                   double *o, double *probs)
{
    const int32_t dh = D / H;
    const double scale = 1.0 / sqrt((double)dh);
#pragma omp parallel for collapse(2) schedule(static)
    for (int32_t h = 0; h < H; ++h) {
        for (int32_t t = 0; t < T; ++t) {
            double *s = (double *)malloc(sizeof(double) * (size_t)T);
            const double *q = qkv + (int64_t)t * 3 * D + h * dh;
            double m = -INFINITY;
            for (int32_t u = 0; u < T; ++u) {
                const double *k = qkv + (int64_t)u * 3 * D + D + h * dh;
                double acc = 0.0;
                for (int32_t e = 0; e < dh; ++e) acc += q[e] * k[e];
                s[u] = acc * scale;
                if (s[u] > m) m = s[u];
            }
            double z = 0.0;
            for (int32_t u = 0; u < T; ++u) {
                s[u] = exp(s[u] - m);
                z += s[u];
            }
            for (int32_t u = 0; u < T; ++u) s[u] /= z;
            if (probs) memcpy(probs + ((int64_t)h * T + t) * T, s, sizeof(double) * (size_t)T);
            if (round_mode)
                for (int32_t u = 0; u < T; ++u) s[u] = epo_round_bf16(s[u]);
            for (int32_t e = 0; e < dh; ++e) {
                double acc = 0.0;
                for (int32_t u = 0; u < T; ++u)
                    acc += s[u] * qkv[(int64_t)u * 3 * D + 2 * D + h * dh + e];
                o[(int64_t)t * D + h * dh + e] = acc;
            }
            free(s);
        }
    }
}

/* One encoder layer on a micro-batch, in place: x is [B, T, D] float64. */
int epo_layer_forward(const epo_config *c, const epo_layer *w, int32_t B, double *x)
{
    const int32_t T = c->n_tokens, D = c->d_model, M = c->d_mlp, H = c->n_heads;
    if (T <= 0 || D <= 0 || M <= 0 || H <= 0 || D % H != 0 || B < 0) return 1;
    const int64_t R = (int64_t)B * T;
    const int rm = c->round_mode;
    double *y = (double *)malloc(sizeof(double) * (size_t)(R * D + 1));
    double *qkv = (double *)malloc(sizeof(double) * (size_t)(R * 3 * D + 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)(R * D + 1));
    double *hid = (double *)malloc(sizeof(double) * (size_t)(R * M + 1));
    if (!y || !qkv || !o || !hid) { free(y); free(qkv); free(o); free(hid); return 2; }

    /* attention block: x <- x + W_o . MHSA(LN1(x)) + b_o */
    epo_layernorm(x, R, D, w->ln1_g, w->ln1_b, c->ln_eps, y);
    maybe_round(y, (size_t)(R * D), rm);
    epo_linear(y, R, D, w->w_qkv, w->b_qkv, 3 * D, qkv);
    maybe_round(qkv, (size_t)(R * 3 * D), rm);
    for (int32_t b = 0; b < B; ++b)   /* images are independent */
        epo_attention(qkv + (int64_t)b * T * 3 * D, T, D, H, rm, o + (int64_t)b * T * D, NULL);
    maybe_round(o, (size_t)(R * D), rm);
    epo_linear(o, R, D, w->w_o, w->b_o, D, y);
    for (int64_t i = 0; i < R * D; ++i) x[i] = x[i] + y[i];

    /* MLP block: x <- x + W_2 . gelu(W_1 . LN2(x) + b_1) + b_2 */
    epo_layernorm(x, R, D, w->ln2_g, w->ln2_b, c->ln_eps, y);
    maybe_round(y, (size_t)(R * D), rm);
    epo_linear(y, R, D, w->w_fc1, w->b_fc1, M, hid);
    epo_gelu(hid, R * M, hid);
    maybe_round(hid, (size_t)(R * M), rm);
    epo_linear(hid, R, M, w->w_fc2, w->b_fc2, D, y);
    for (int64_t i = 0; i < R * D; ++i) x[i] = x[i] + y[i];

    free(y); free(qkv); free(o); free(hid);
    return 0;
}

/* A stage: n_layers consecutive layers applied in order.  x_in is float32
 * [B, T, D]; x_out is float64 [B, T, D]. */
int epo_stage_forward(const epo_config *c, int32_t n_layers, const epo_layer *layers,
                      const float *x_in, int32_t B, double *x_out)
{
    const int64_t n = (int64_t)B * c->n_tokens * c->d_model;
    for (int64_t i = 0; i < n; ++i) x_out[i] = (double)x_in[i];
    for (int32_t l = 0; l < n_layers; ++l) {
        int rc = epo_layer_forward(c, &layers[l], B, x_out);
        if (rc) return rc;
    }
    return 0;
}

#ifdef _OPENMP
#include <omp.h>
int epo_num_threads(void) { return omp_get_max_threads(); }
#else
int epo_num_threads(void) { return 1; }
#endif
