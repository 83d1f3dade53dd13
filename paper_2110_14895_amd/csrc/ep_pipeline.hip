// Pipeline of stages on one device (paper section 3.1: the model is cut into
// parts T_1 .. T_n of consecutive layers, the mini-batch into micro-batches that
// flow through the parts one after the other; Eq. 2: in steady state the period
// of the pipeline is set by its slowest part).
//
// This is the paper's runtime minus the network: every stage has a stream of its
// own, the activation of micro-batch m leaves stage k in one of two boundary
// buffers (m even / odd) and an event tells stage k+1 that it is there; a second
// wait keeps stage k from overwriting a boundary buffer before stage k+1 has
// consumed what it held two micro-batches earlier.  All of it is enqueued
// asynchronously; nothing here synchronises with the host.
//
// On one GPU the stages share the same compute units, so the measured period
// approaches the sum of the stage times rather than their maximum; what this
// component exercises is the schedule (order, overlap of independent work,
// hand-over of buffers), with results identical to running the stages in turn.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "edgepipe.h"
#include "ep_error.h"

struct ep_pipeline {
    std::vector<ep_stage_t *> stages;
    std::vector<hipStream_t> streams;
    std::vector<hipEvent_t> done;          // [stage][parity]: stage finished a micro-batch of that parity
    hipEvent_t start = nullptr;
    std::vector<char *> bound;             // [boundary][parity] device buffers
    std::vector<int32_t> bound_dtype;      // [boundary]
    int32_t micro_batch = 0;
    size_t elems = 0;                      // micro_batch * T * D
    size_t in_bytes = 0, out_bytes = 0;    // of one micro-batch
};

#define EP_HIP(call)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            return ep_fail(EP_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));       \
    } while (0)

extern "C" void ep_pipeline_destroy(ep_pipeline_t *p)
{
    if (!p) return;
    for (hipStream_t s : p->streams) (void)hipStreamDestroy(s);
    for (hipEvent_t e : p->done) (void)hipEventDestroy(e);
    if (p->start) (void)hipEventDestroy(p->start);
    for (char *b : p->bound) (void)hipFree(b);
    delete p;
}

extern "C" ep_status ep_pipeline_create(int32_t n_stages, ep_stage_t *const *stages, int32_t micro_batch,
                                        ep_pipeline_t **out)
{
    if (!out) return ep_fail(EP_ERR_INVALID_ARG, "ep_pipeline_create: null output");
    *out = nullptr;
    if (n_stages < 1 || n_stages > 64 || !stages || micro_batch < 1)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_pipeline_create: need 1 <= n_stages <= 64, stages and micro_batch >= 1");
    ep_pipeline *p = new (std::nothrow) ep_pipeline;
    if (!p) return ep_fail(EP_ERR_OOM, "ep_pipeline_create: out of host memory");
    auto fail = [&](ep_status rc) { ep_pipeline_destroy(p); return rc; };

    ep_vit_config prev{};
    int32_t prev_end = 0;
    for (int k = 0; k < n_stages; ++k) {
        if (!stages[k]) return fail(ep_fail(EP_ERR_INVALID_ARG, "ep_pipeline_create: stage %d is null", k));
        ep_vit_config c;
        int32_t begin, end, max_batch;
        ep_status rc = ep_stage_info(stages[k], &c, &begin, &end, &max_batch);
        if (rc != EP_OK) return fail(rc);
        if (max_batch < micro_batch)
            return fail(ep_fail(EP_ERR_INVALID_ARG, "ep_pipeline_create: stage %d holds at most %d images, micro_batch is %d",
                                k, max_batch, micro_batch));
        if (k > 0) {
            if (begin != prev_end)
                return fail(ep_fail(EP_ERR_INVALID_ARG, "ep_pipeline_create: stage %d starts at layer %d, stage %d ends at %d",
                                    k, begin, k - 1, prev_end));
            if (c.d_model != prev.d_model || c.n_tokens != prev.n_tokens)
                return fail(ep_fail(EP_ERR_INVALID_ARG, "ep_pipeline_create: stages %d and %d differ in width or tokens", k - 1, k));
            if (c.in_dtype != prev.out_dtype)
                return fail(ep_fail(EP_ERR_INVALID_ARG, "ep_pipeline_create: stage %d writes dtype %d, stage %d reads dtype %d",
                                    k - 1, prev.out_dtype, k, c.in_dtype));
        }
        const size_t elems = (size_t)micro_batch * c.n_tokens * c.d_model;
        p->elems = elems;
        if (k == 0) p->in_bytes = elems * (c.in_dtype == EP_BF16 ? 2 : 4);
        p->out_bytes = elems * (c.out_dtype == EP_BF16 ? 2 : 4);
        if (k + 1 < n_stages) p->bound_dtype.push_back(c.out_dtype);
        p->stages.push_back(stages[k]);
        prev = c;
        prev_end = end;
    }
    p->micro_batch = micro_batch;

    hipError_t e = hipEventCreateWithFlags(&p->start, hipEventDisableTiming);
    if (e != hipSuccess) { p->start = nullptr; return fail(ep_fail(EP_ERR_HIP, "hipEventCreate failed: %s", hipGetErrorString(e))); }
    for (int k = 0; k < n_stages; ++k) {
        hipStream_t s;
        e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);      // default priority
        if (e != hipSuccess) return fail(ep_fail(EP_ERR_HIP, "hipStreamCreate failed: %s", hipGetErrorString(e)));
        p->streams.push_back(s);
        for (int par = 0; par < 2; ++par) {
            hipEvent_t ev;
            e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
            if (e != hipSuccess) return fail(ep_fail(EP_ERR_HIP, "hipEventCreate failed: %s", hipGetErrorString(e)));
            p->done.push_back(ev);
        }
    }
    for (int k = 0; k + 1 < n_stages; ++k) {
        const size_t bytes = p->elems * (p->bound_dtype[k] == EP_BF16 ? 2 : 4);
        for (int par = 0; par < 2; ++par) {
            char *b = nullptr;
            e = hipMalloc((void **)&b, bytes);
            if (e != hipSuccess)
                return fail(ep_fail(EP_ERR_OOM, "hipMalloc of a %zu-byte boundary buffer failed: %s", bytes, hipGetErrorString(e)));
            p->bound.push_back(b);
        }
    }
    *out = p;
    return EP_OK;
}

extern "C" ep_status ep_pipeline_run(ep_pipeline_t *p, const void *x_in, int32_t n_micro, void *x_out, void *stream)
{
    if (!p || !x_in || !x_out) return ep_fail(EP_ERR_INVALID_ARG, "ep_pipeline_run: null argument");
    if (n_micro < 1) return ep_fail(EP_ERR_INVALID_ARG, "ep_pipeline_run: n_micro must be >= 1");
    hipStream_t caller = (hipStream_t)stream;
    const int S = (int)p->stages.size();

    // everything below comes after what the caller has enqueued so far
    EP_HIP(hipEventRecord(p->start, caller));
    for (int k = 0; k < S; ++k) EP_HIP(hipStreamWaitEvent(p->streams[k], p->start, 0));

    for (int m = 0; m < n_micro; ++m) {
        const int par = m & 1;
        for (int k = 0; k < S; ++k) {
            hipStream_t s = p->streams[k];
            // input of this stage for micro-batch m is there
            if (k > 0) EP_HIP(hipStreamWaitEvent(s, p->done[(k - 1) * 2 + par], 0));
            // the boundary buffer this stage writes is free: the next stage is done with micro-batch m-2
            if (k + 1 < S && m >= 2) EP_HIP(hipStreamWaitEvent(s, p->done[(k + 1) * 2 + par], 0));
            const void *in = k == 0 ? (const void *)((const char *)x_in + (size_t)m * p->in_bytes)
                                    : (const void *)p->bound[(k - 1) * 2 + par];
            void *outp = k + 1 == S ? (void *)((char *)x_out + (size_t)m * p->out_bytes) : (void *)p->bound[k * 2 + par];
            ep_status rc = ep_stage_forward(p->stages[k], in, p->micro_batch, outp, s);
            if (rc != EP_OK) return rc;
            EP_HIP(hipEventRecord(p->done[k * 2 + par], s));
        }
    }
    // the caller's stream continues after the last stage has delivered the last micro-batches
    // (stage S-1 runs its micro-batches in order, so its newest event covers all of them; the
    // other stages finished earlier along the dependency chain)
    EP_HIP(hipStreamWaitEvent(caller, p->done[(S - 1) * 2 + ((n_micro - 1) & 1)], 0));
    return EP_OK;
}
