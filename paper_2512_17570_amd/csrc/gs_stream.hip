// gs_stream.hip -- the step over states resident in pinned host memory.
//
// The paper's optimizer step walks parameter chunks: load a chunk's master parameters and
// optimizer states, step, write them back (Sec. 2.2), pipelined against the surrounding work
// (Sec. 4.3).  There the slow link is SSD<->host; here it is host<->HBM over PCIe, and the
// pipeline is the GPU's own: the step kernel runs IN PLACE on the pinned host arrays, so every
// wave loads its tile of p/m/v over the link, updates it and stores it back, thousands of waves
// at different stages at any time.  Nothing is staged in HBM and no copy engine is involved.
//
// Measured on MI355X (one GPT-65B-shaped layer and more, k = 8): 44-45 GB/s each way at once,
// the same on a stream confined to 16 of the 256 CUs, and the same whatever copy traffic the
// process ran before.  The staged alternative (copy-engine upload into HBM slots, kernel in
// HBM, copy back) reached 48 GB/s each way at best but depends on which engine the runtime
// picks per copy: the same code was seen at 28 GB/s after unrelated copies on other streams, and
// its device-to-host copies at a quarter of the link rate under the file tier's load.
//
// The kernel is the resident one, handed base pointers such that base[i] is element i of the
// layer, so its 4-element groups fall on the same absolute indices and the result is
// bit-identical to the device-resident step.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>

#include "gs_internal.h"
#include "gs_stream_internal.h"

using namespace gs;

static void destroy_partial(gs_stream_ctx *c)
{
    if (!c) return;
    if (c->ev_producer) (void)hipEventDestroy(c->ev_producer);
    if (c->s_comp) (void)hipStreamDestroy(c->s_comp);
    if (c->s_note) (void)hipStreamDestroy(c->s_note);
    delete c;
}

#define GS_TRY(call, what)                         \
    do {                                           \
        hipError_t e_ = (call);                    \
        if (e_ != hipSuccess) {                    \
            gs_status s_ = hip_fail(e_, what);     \
            return s_;                             \
        }                                          \
    } while (0)

namespace gs {

gs_status stream_validate(const gs_stream_ctx *c, const uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k,
                          int64_t n, const gs_adamw_hparams *hp, const double *d_sqnorm)
{
    if (!c || !d_w_bf16) return GS_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(d_w_bf16) & 15u) return GS_ERR_INVALID_ARG;
    gs_status st = validate_grads(d_grads, k);
    if (st != GS_OK) return st;
    if (n < 0) return GS_ERR_INVALID_ARG;
    st = validate_hparams(hp);
    if (st != GS_OK) return st;
    if (d_sqnorm && (reinterpret_cast<uintptr_t>(d_sqnorm) & 7u)) return GS_ERR_INVALID_ARG;
    return GS_OK;
}

gs_status stream_begin_layer(gs_stream_ctx *c, StepArgs &A, uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k,
                             const gs_adamw_hparams *hp, const double *d_sqnorm, void *producer_stream)
{
    int cur = -1;
    GS_TRY(hipGetDevice(&cur), "hipGetDevice");
    if (cur != c->device) return GS_ERR_INVALID_ARG;   // the context's streams live on another GPU

    // gradients and the norm come from the caller's stream
    GS_TRY(hipEventRecord(c->ev_producer, static_cast<hipStream_t>(producer_stream)), "hipEventRecord(producer)");
    GS_TRY(hipStreamWaitEvent(c->s_comp, c->ev_producer, 0), "hipStreamWaitEvent(producer)");

    memset(&A, 0, sizeof A);
    A.w = d_w_bf16;
    for (int j = 0; j < k; ++j) A.gt.g[j] = d_grads[j];
    A.k = k;
    A.c = make_consts(*hp);
    A.max_norm = hp->max_grad_norm;
    A.d_sqnorm = d_sqnorm;
    return GS_OK;
}

gs_status stream_range(gs_stream_ctx *c, StepArgs &A, float *host_p, float *host_m, float *host_v, int64_t b, int64_t e)
{
    // base pointers chosen so that base[i] is element i of the layer
    const intptr_t back = -(intptr_t)b * (intptr_t)sizeof(float);
    A.po = reinterpret_cast<float *>(reinterpret_cast<intptr_t>(host_p) + back);
    A.mo = reinterpret_cast<float *>(reinterpret_cast<intptr_t>(host_m) + back);
    A.vo = reinterpret_cast<float *>(reinterpret_cast<intptr_t>(host_v) + back);
    A.p = A.po;
    A.m = A.mo;
    A.v = A.vo;
    A.begin = b;
    A.end = e;
    hipError_t le = launch_accum_adamw(A, c->s_comp);
    if (le != hipSuccess) return hip_fail(le, "host-resident step launch");
    return GS_OK;
}

}  // namespace gs

extern "C" {

gs_status gs_stream_ctx_create(gs_stream_ctx **out, int num_cus)
{
    if (!out) return GS_ERR_INVALID_ARG;
    *out = nullptr;
    if (num_cus < 0) return GS_ERR_INVALID_ARG;

    gs_stream_ctx *c = new (std::nothrow) gs_stream_ctx();
    if (!c) return GS_ERR_NOMEM;
    c->num_cus = num_cus;
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) { destroy_partial(c); return hip_fail(e, "hipGetDevice"); }

    // default priority on every stream
    if (num_cus > 0) {
        void *s = nullptr;
        gs_status st = gs_cu_stream_create(&s, num_cus);
        if (st != GS_OK) { destroy_partial(c); return st; }
        c->s_comp = static_cast<hipStream_t>(s);
    } else if ((e = hipStreamCreateWithFlags(&c->s_comp, hipStreamNonBlocking)) != hipSuccess) {
        c->s_comp = nullptr;
        destroy_partial(c);
        return hip_fail(e, "hipStreamCreateWithFlags");
    }
    if ((e = hipStreamCreateWithFlags(&c->s_note, hipStreamNonBlocking)) != hipSuccess) {
        c->s_note = nullptr;
        destroy_partial(c);
        return hip_fail(e, "hipStreamCreateWithFlags");
    }
    if ((e = hipEventCreateWithFlags(&c->ev_producer, hipEventDisableTiming)) != hipSuccess) {
        c->ev_producer = nullptr;
        destroy_partial(c);
        return hip_fail(e, "hipEventCreateWithFlags");
    }
    *out = c;
    return GS_OK;
}

gs_status gs_stream_ctx_sync(gs_stream_ctx *c)
{
    if (!c) return GS_ERR_INVALID_ARG;
    GS_TRY(hipStreamSynchronize(c->s_comp), "hipStreamSynchronize(compute)");
    GS_TRY(hipStreamSynchronize(c->s_note), "hipStreamSynchronize(notify)");
    return GS_OK;
}

gs_status gs_stream_ctx_destroy(gs_stream_ctx *c)
{
    if (!c) return GS_ERR_INVALID_ARG;
    gs_status st = gs_stream_ctx_sync(c);
    destroy_partial(c);
    return st;
}

gs_status gs_stream_layer_step(gs_stream_ctx *c, float *h_p, float *h_m, float *h_v,
                               uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k, int64_t n,
                               const gs_adamw_hparams *hp, const double *d_sqnorm,
                               void *producer_stream)
{
    if (!c || !h_p || !h_m || !h_v) return GS_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(h_p) | reinterpret_cast<uintptr_t>(h_m) | reinterpret_cast<uintptr_t>(h_v)) & 15u)
        return GS_ERR_INVALID_ARG;
    gs_status st = stream_validate(c, d_w_bf16, d_grads, k, n, hp, d_sqnorm);
    if (st != GS_OK) return st;
    if (n == 0) return GS_OK;

    StepArgs A;
    st = stream_begin_layer(c, A, d_w_bf16, d_grads, k, hp, d_sqnorm, producer_stream);
    if (st != GS_OK) return st;
    return stream_range(c, A, h_p, h_m, h_v, 0, n);
}

}  // extern "C"
