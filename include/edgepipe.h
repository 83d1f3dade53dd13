/*
 * edgepipe.h - C ABI of the MI355X pipeline-stage library.
 *
 * The library runs the forward pass of one pipeline stage of a partitioned
 * transformer encoder on one GPU, and plans the partition on the CPU.
 *
 *   - A model with L layers is cut into k parts T_1..T_k of consecutive layers;
 *     part T_i is one pipeline stage on one device and the model is the
 *     composition T_k(...T_2(T_1(X))) applied to one micro-batch X
 *     (paper section 3.1).  ep_stage_create / ep_stage_forward are one T_i.
 *   - A layer is multi-head self-attention, an MLP, two layer normalisations
 *     and residual connections (paper section 2.1, "Transformer-based Models").
 *   - Which layers go to which device is the partition problem of sections
 *     3.2-3.3 (Eq. 1-3, Algorithm 1): ep_partition.
 *   - The per-layer execution times the planner needs are measured on the
 *     device (section 5.1, per-layer execution time figure): ep_stage_profile.
 *
 * Conventions
 *   - All functions return an ep_status and never throw or abort; the text of
 *     the last error of the calling thread is ep_last_error().
 *   - "host" / "device" on a pointer says where the memory lives.  The library
 *     never takes ownership of a caller buffer.
 *   - A stage handle is not thread-safe; distinct handles are independent and
 *     may be driven from distinct host threads (the library's one-time launch
 *     set-up is kept per device and is safe against concurrent first calls).
 *   - One GPU: the device current at ep_stage_create is the stage's device.
 */
#ifndef EDGEPIPE_H
#define EDGEPIPE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ep_stage ep_stage_t; /* opaque, created and destroyed by the library */

typedef enum {
    EP_OK = 0,
    EP_ERR_INVALID_ARG = 1, /* null pointer, bad range, B > max_batch, ... */
    EP_ERR_UNSUPPORTED = 2, /* shape or dtype combination the kernels do not cover */
    EP_ERR_OOM = 3,         /* host or device allocation failed */
    EP_ERR_HIP = 4,         /* a HIP runtime call failed; see ep_last_error() */
    EP_ERR_INFEASIBLE = 5   /* ep_partition: no strategy satisfies the memory limits */
} ep_status;

typedef enum { EP_F32 = 0, EP_BF16 = 1 } ep_dtype;

/*
 * Encoder configuration.  Shapes of one layer: width D = d_model, H = n_heads
 * heads of d_head = D / H, MLP width M = d_mlp, T = n_tokens tokens per image
 * (patches plus the class token).  n_layers is L of the whole model; a stage
 * covers a sub-range of it.
 *
 * param_dtype selects the arithmetic path:
 *   EP_F32  - fp32 operands and accumulation everywhere; in_dtype and
 *             out_dtype must be EP_F32.
 *   EP_BF16 - parameters are bf16; GEMM and attention operands are bf16 on the
 *             matrix cores with fp32 accumulation; LayerNorm statistics,
 *             softmax, and the residual stream are fp32.  in_dtype / out_dtype
 *             choose bf16 or fp32 for the stage input / output (fp32 output
 *             keeps the residual stream un-rounded across stage boundaries).
 *             Requires D % 64 == 0, D <= 2048, M % 64 == 0, d_head in
 *             {64, 80}, T <= 4096.
 */
typedef struct {
    int32_t n_layers;    /* L */
    int32_t d_model;     /* D */
    int32_t n_heads;     /* H */
    int32_t d_mlp;       /* M */
    int32_t n_tokens;    /* T */
    float ln_eps;        /* added to the variance inside the square root */
    int32_t param_dtype; /* ep_dtype of every pointer in ep_layer_weights */
    int32_t in_dtype;    /* ep_dtype of x_in */
    int32_t out_dtype;   /* ep_dtype of x_out */
} ep_vit_config;

/*
 * Parameters of one layer, HOST pointers, element type param_dtype (bf16 is
 * the upper 16 bits of an IEEE float32).  Dense weights are [out, in]
 * row-major, y = x W^T + b:
 *   ln1_g, ln1_b [D]     LayerNorm before attention (gain, shift)
 *   w_qkv [3D, D], b_qkv [3D]   fused projection; rows 0..D-1 produce q,
 *                        D..2D-1 k, 2D..3D-1 v; inside each block row h*d_head+e
 *                        is component e of head h
 *   w_o [D, D], b_o [D]  attention output projection
 *   ln2_g, ln2_b [D]     LayerNorm before the MLP
 *   w_fc1 [M, D], b_fc1 [M]     first dense layer, followed by exact (erf) GELU
 *   w_fc2 [D, M], b_fc2 [D]     second dense layer
 */
typedef struct {
    const void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
    const void *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} ep_layer_weights;

/*
 * Build the stage T_i that holds layers layer_begin .. layer_end-1 of the model
 * (section 3.1).  `layers` has layer_end - layer_begin entries of host pointers;
 * the parameters are copied to the current device (the caller may free its
 * buffers afterwards).  A workspace for micro-batches of up to max_batch images
 * is allocated here; nothing is allocated later.  On success *out is the handle.
 * Errors: INVALID_ARG (null, empty or out-of-range layer range, max_batch < 1),
 * UNSUPPORTED (see ep_vit_config), OOM, HIP.
 */
ep_status ep_stage_create(const ep_vit_config *cfg, int32_t layer_begin, int32_t layer_end,
                          const ep_layer_weights *layers, int32_t max_batch, ep_stage_t **out);

/*
 * Y = T_i(X) for one micro-batch (section 3.1).  x_in and x_out are DEVICE
 * buffers [B, T, D] row-major (D contiguous) of in_dtype / out_dtype; they may
 * be the same buffer when the two dtypes have the same size.  For each layer of
 * the stage, with x the fp32 residual stream (section 2.1):
 *   x <- x + W_o . MHSA(LN1(x)) + b_o
 *   x <- x + W_2 . gelu(W_1 . LN2(x) + b_1) + b_2
 * MHSA: per head, softmax over all T tokens of q.k / sqrt(d_head), no mask.
 * All work is enqueued on `stream` (a hipStream_t; NULL is the default stream);
 * the call does not allocate and does not synchronise, so it may be recorded in
 * a stream capture once an earlier call on this device has run (the first call
 * of a kernel sets a function attribute); while a trace is armed it also records
 * events.  Calls on one stage share its workspace: do not overlap them.
 * 1 <= B <= max_batch.
 */
ep_status ep_stage_forward(ep_stage_t *stage, const void *x_in, int32_t B, void *x_out,
                           void *stream);

/*
 * ep_stage_forward for callers that cannot allocate device memory and want
 * stages that own none beyond their parameters: code under stream capture,
 * tight serving loops, harnesses that forbid allocation (such a caller creates
 * its stages with max_batch 1, whose own workspace is small, and runs them
 * through this call).  Same arguments, same kernels, same results as
 * ep_stage_forward, bit for bit; the intermediates (residual stream, GEMM
 * operands, q|k|v / hidden activations) live in a workspace of
 * EP_STATIC_SCRATCH_BYTES that is part of the library's code object - one per
 * GPU, held until the process ends - instead of in the stage's own.  The call
 * allocates nothing and frees nothing.  B is limited by that workspace, not by
 * max_batch: B * T * (4*D + e*D + e*max(3*D, M)) bytes (e = 2 on the bf16 path,
 * 4 on the fp32 path; each part rounded up to 256) must fit, else UNSUPPORTED
 * with the two sizes in ep_last_error() (ViT-Huge bf16: B <= 14; ViT-Base: B <= 31).
 * One exception to "bit for bit": at small micro-batches ep_stage_forward sums the
 * second MLP layer over ranges of K and keeps the range sums in its workspace; where
 * those do not fit next to the rest here, this call runs that layer uncut, and the
 * results differ in the order of the fp32 additions over K (the range sums take at most
 * 32 MiB, so never while the other intermediates stay under 32 MiB).
 * Every stage on a GPU shares that GPU's workspace and nothing in it is assumed
 * zero or kept between calls: calls that overlap in time on one GPU (two
 * streams, two threads) race; calls on one stream, or ordered by events, do not.
 * Other errors as ep_stage_forward.
 */
#define EP_STATIC_SCRATCH_BYTES (64u << 20)
ep_status ep_stage_forward_static(ep_stage_t *stage, const void *x_in, int32_t B, void *x_out,
                                  void *stream);

/*
 * Measure the execution time of each layer of the stage at micro-batch B on this
 * device: the T_comp(l, u) input of the planner (section 3.3; section 5.1
 * measures the same quantity per layer).  Each layer is run `iters` times
 * (after one untimed run) on the stage's own workspace, timed with events on
 * `stream`; per_layer_seconds (HOST, one double per layer of the stage) gets the
 * mean.  Synchronises `stream`.
 */
ep_status ep_stage_profile(ep_stage_t *stage, int32_t B, int32_t iters, void *stream,
                           double *per_layer_seconds);

/*
 * Per-kernel timing of the forward pass.  The kernels of one layer, in launch
 * order (section 2.1's parts of a layer):
 */
typedef enum {
    EP_K_LN1 = 0,  /* LayerNorm before attention */
    EP_K_QKV = 1,  /* fused q|k|v projection */
    EP_K_ATTN = 2, /* multi-head softmax attention */
    EP_K_PROJ = 3, /* output projection + residual */
    EP_K_LN2 = 4,  /* LayerNorm before the MLP */
    EP_K_FC1 = 5,  /* first dense layer + GELU */
    EP_K_FC2 = 6,  /* second dense layer + residual */
    EP_K_COUNT = 7,
    /*
     * The launch of a dense layer alone (bf16 path only), without the event
     * bracket's share of the neighbouring kernels' gaps that ids 2, 3, 5, 6 see;
     * ep_stage_gemm_main_rows gives the rows it covers (all rows of the layer: a
     * dense layer is one launch, the rows past the last whole 256-row tile are
     * computed in its last phase).
     */
    EP_K_QKV_MAIN = 7,
    EP_K_PROJ_MAIN = 8,
    EP_K_FC1_MAIN = 9,
    EP_K_FC2_MAIN = 10,
    EP_K_TRACE_COUNT = 11
} ep_kernel_id;

/*
 * Start timing one kernel of the layer: until ep_stage_trace_end, every launch
 * of `kernel` made by ep_stage_forward on this stage is bracketed by a pair of
 * events recorded on the forward's stream (at most max_launches pairs, created
 * here; later launches run untimed).  Tracing one kernel at a time keeps the
 * other kernels' launches back to back.
 */
ep_status ep_stage_trace_begin(ep_stage_t *stage, int32_t kernel, int32_t max_launches);
/*
 * Stop timing: waits for the recorded events, writes the number of timed
 * launches and the sum of their durations in seconds (HOST), frees the events.
 */
ep_status ep_stage_trace_end(ep_stage_t *stage, int32_t *launches, double *seconds);

/*
 * Rows of the B*T activation rows that the first launch of dense layer `kernel`
 * (EP_K_QKV, EP_K_PROJ, EP_K_FC1, EP_K_FC2 or their _MAIN ids) covers at
 * micro-batch B: what a roofline figure for that launch has to count.
 */
ep_status ep_stage_gemm_main_rows(const ep_stage_t *stage, int32_t B, int32_t kernel, int64_t *rows);

/*
 * Measurement hook: the rate this device sustains on a loop of nothing but
 * bf16 matrix instructions (no memory traffic), the yardstick a dense layer's
 * achieved rate is read against next to the published peak (the dense layers
 * are where a layer's time goes, section 5.1).  form 0: 16x16x32 (the form
 * the dense layers use), form 1: 32x32x16.  random_operands 0: every operand
 * value is 1.0; 1: random signs, mantissas and magnitudes in [0.5, 2) (the
 * chip lowers its clock under the switching activity of real data).  One
 * workgroup of 8 waves per compute unit runs 16 * iters instructions per wave,
 * timed with events on `stream` (a hipStream_t) after a short warm-up launch.
 * Outputs (HOST): *tflops; *shader_mhz (may be NULL) the shader clock the loop
 * ran at, from the ratio of the shader cycle counter to the 100 MHz counter.
 * Allocates and frees a small device buffer and synchronises `stream`.
 * Errors: INVALID_ARG (form, iters outside [1, 2^24], null), OOM, HIP.
 */
ep_status ep_mfma_peak(int32_t form, int32_t random_operands, int32_t iters, void *stream,
                       double *tflops, double *shader_mhz);

/*
 * Measurement hook: the shader clock the most recent large dense-layer launch
 * (one resident workgroup per compute unit; the launches ep_stage_forward makes
 * for micro-batches that fill the chip) ran at on the current device, and how
 * long its first workgroup ran: that workgroup reads the shader cycle counter
 * and the 100 MHz counter when it starts and when it ends.  Synchronise the
 * stream first.  Outputs HOST.  INVALID_ARG if no such launch has finished.
 */
ep_status ep_gemm_clock_sample(double *shader_mhz, double *seconds);

/* Configuration, layer range and max_batch the stage was created with (HOST outputs,
 * each may be NULL). */
ep_status ep_stage_info(const ep_stage_t *stage, ep_vit_config *cfg, int32_t *layer_begin,
                        int32_t *layer_end, int32_t *max_batch);

/* Device bytes held by the stage (parameters + workspace). */
ep_status ep_stage_device_bytes(const ep_stage_t *stage, uint64_t *bytes);

/* Free the stage's device memory.  The caller must have synchronised any stream
 * that still runs its work.  NULL is allowed. */
void ep_stage_destroy(ep_stage_t *stage);

/*
 * The parts around the encoder layers (section 4, "Deep Learning Models": the
 * embedding layer brings the images to the uniform input of the transformer
 * layers, which are what the paper partitions; model definition of the original
 * ViT).  With a stage that holds all layers they map images to logits.
 *
 * Embedding: x[b, 0, :] = cls + pos[0]; x[b, 1+p, :] = patch_p . w_patch^T +
 * b_patch + pos[1+p], patch p of the (image_size/patch)^2 grid in row-major
 * order, its pixels flattened (channel, row, column) as a convolution weight
 * [D, C, P, P] is.  T = 1 + (image_size/patch)^2 tokens.
 * ep_embed_create: w_patch [D, C*P*P], b_patch [D], cls [D], pos [T, D], HOST, in
 * param_dtype (bf16 bit patterns or fp32); copied.  param_dtype EP_BF16 runs the
 * projection on the matrix cores (d_model % 64 == 0), EP_F32 in fp32 (then
 * out_dtype must be EP_F32).  ep_embed_forward: images DEVICE fp32
 * [B, C, image_size, image_size]; x_out DEVICE [B, T, D] in out_dtype, rounded
 * once; enqueue only on `stream`.
 */
typedef struct {
    int32_t image_size;  /* pixels per side */
    int32_t patch;       /* P */
    int32_t channels;    /* C */
    int32_t d_model;     /* D */
    int32_t param_dtype; /* ep_dtype of the host parameters */
    int32_t out_dtype;   /* ep_dtype of x_out (the in_dtype of the first stage) */
} ep_embed_config;
typedef struct ep_embed ep_embed_t;
ep_status ep_embed_create(const ep_embed_config *cfg, const void *w_patch, const void *b_patch,
                          const void *cls, const void *pos, int32_t max_batch, ep_embed_t **out);
ep_status ep_embed_forward(ep_embed_t *embed, const void *images, int32_t B, void *x_out, void *stream);
void ep_embed_destroy(ep_embed_t *embed);

/*
 * Head: logits[b, :] = LayerNorm(x[b, 0, :]; ln_g, ln_b, ln_eps) . w_head^T +
 * b_head: the final LayerNorm and the classifier act on the class-token row
 * only.  ep_head_create: ln_g, ln_b [D], w_head [n_classes, D], b_head
 * [n_classes], HOST, in param_dtype; copied.  EP_BF16 needs n_classes % 8 == 0,
 * d_model % 16 == 0, max_batch <= 4096.  ep_head_forward: x DEVICE fp32
 * [B, n_tokens, D] (the fp32 output of the last stage); logits DEVICE fp32
 * [B, n_classes]; enqueue only on `stream`.
 */
typedef struct {
    int32_t d_model;
    int32_t n_tokens;
    int32_t n_classes;
    float ln_eps;
    int32_t param_dtype;
} ep_head_config;
typedef struct ep_head ep_head_t;
ep_status ep_head_create(const ep_head_config *cfg, const void *ln_g, const void *ln_b, const void *w_head,
                         const void *b_head, int32_t max_batch, ep_head_t **out);
ep_status ep_head_forward(ep_head_t *head, const void *x, int32_t B, void *logits, void *stream);
void ep_head_destroy(ep_head_t *head);

/*
 * Pipeline of stages on this device (section 3.1: parts T_1 .. T_n of consecutive
 * layers, micro-batches flowing through them; Eq. 2: the period is set by the
 * slowest part).  The runtime of the paper minus the network: one stream per
 * stage, two boundary buffers per stage boundary, events for "micro-batch m has
 * left stage k" and for the reuse of a boundary buffer.
 *
 * ep_pipeline_create: `stages` (HOST array of n_stages handles, 1..64) in pipeline
 * order; consecutive stages must cover consecutive layer ranges of the same
 * width and token count, and the out_dtype of a stage must be the in_dtype of the
 * next; every stage must have max_batch >= micro_batch.  The pipeline borrows the
 * handles (the caller destroys them after the pipeline) and owns its streams,
 * events and boundary buffers.
 *
 * ep_pipeline_run: x_in (DEVICE) holds n_micro micro-batches back to back,
 * [n_micro * micro_batch, T, D] in the first stage's in_dtype; x_out (DEVICE)
 * receives them in the last stage's out_dtype.  Enqueue only: the work is
 * ordered after what `stream` holds at the call, and `stream` is made to wait
 * for the last micro-batch; no host synchronisation.  Results are those of
 * running the stages one after the other on each micro-batch.  A stage must
 * not be used elsewhere while a run is in flight.  Streams have default priority.
 */
typedef struct ep_pipeline ep_pipeline_t;
ep_status ep_pipeline_create(int32_t n_stages, ep_stage_t *const *stages, int32_t micro_batch,
                             ep_pipeline_t **out);
ep_status ep_pipeline_run(ep_pipeline_t *pipeline, const void *x_in, int32_t n_micro, void *x_out,
                          void *stream);
/* Synchronise the device (or at least `stream` of the last run) first.  NULL is allowed. */
void ep_pipeline_destroy(ep_pipeline_t *pipeline);

/*
 * Heterogeneity-aware optimal partition (sections 3.2-3.3), CPU only,
 * deterministic, no global state.
 *
 * Inputs (HOST):
 *   L layers, D devices (1 <= D <= 20).
 *   t_comp[l*D + u]   seconds to run layer l on device u; T_comp of a run of
 *                     layers is their sum, added first layer to last.
 *   layer_mem[l]      M_j, memory a layer needs;  dev_mem[u]  m_u, capacity.
 *   xfer_bytes[l]     P_j, bytes sent to the next stage when a stage ends with
 *                     layer l.
 *   bw[u*D + v]       b_{u,v}, bytes/s from device u to device v.
 * A strategy selects S <= D distinct devices in pipeline order and gives each a
 * run of consecutive layers whose memory fits.  A stage's period is
 * max(T_comp, P_j / b_{u,v}) (Eq. 1, Eq. 2); the last stage sends nothing.
 * T_opt is the smallest achievable largest period (Eq. 3).
 *
 * Outputs (HOST): *t_opt; *n_stages = S; for stage s < S: stage_dev[s],
 * stage_first[s], stage_last[s] (0-based, inclusive); the three arrays must
 * have room for D entries.  Among all strategies that reach T_opt the one
 * returned has the lexicographically smallest sequence
 * (dev_0, last_0, dev_1, last_1, ...), so the answer is unique.
 * Errors: INVALID_ARG, OOM, INFEASIBLE (outputs untouched).
 */
ep_status ep_partition(int32_t L, int32_t D, const double *t_comp, const double *layer_mem,
                       const double *dev_mem, const double *xfer_bytes, const double *bw,
                       double *t_opt, int32_t *n_stages, int32_t *stage_dev,
                       int32_t *stage_first, int32_t *stage_last);

/*
 * The same problem, same inputs and the same answer, with identical devices
 * collapsed into categories (section 3.3, after Algorithm 1: N categories of
 * n_1 .. n_N identical devices shrink the search state from 2^D device subsets
 * to prod (n_c + 1) count vectors).  Devices u, v are identical when
 * t_comp[., u] == t_comp[., v], dev_mem[u] == dev_mem[v], bw[u][w] == bw[v][w]
 * and bw[w][u] == bw[w][v] for every third device w, and bw[u][v] == bw[v][u];
 * the categories are found from the inputs.  1 <= D <= 64; the table has
 * L * prod (n_c + 1) * N entries (EP_ERR_OOM above 2^31).  T_opt and the
 * strategy are bit for bit those of ep_partition on the same inputs.
 * n_categories (HOST, may be NULL) receives N.
 */
ep_status ep_partition_categories(int32_t L, int32_t D, const double *t_comp, const double *layer_mem,
                                  const double *dev_mem, const double *xfer_bytes, const double *bw,
                                  double *t_opt, int32_t *n_stages, int32_t *stage_dev,
                                  int32_t *stage_first, int32_t *stage_last, int32_t *n_categories);

const char *ep_status_string(ep_status s);
/* Text of the calling thread's most recent error ("" if none). */
const char *ep_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* EDGEPIPE_H */
