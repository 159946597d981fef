// gs_defer.hip -- the deferred part of a layer's step, with its per-layer deadline.
//
// The paper delays a fraction alpha of every layer's optimizer step into the next iteration's
// forward pass; the only requirement is that a layer's delayed update has finished before that
// layer executes (Sec. 4.4).  A gs_defer_ctx is that schedule as a library object: one stream of
// its own (optionally confined to a budget of compute units, so that the bandwidth-bound step
// leaves the rest of the chip to the forward pass), on which the deferred ranges run in the order
// they are handed over, and one event per layer that the consumer -- the stream that runs the
// layer's forward, or the one that will overwrite its gradient buffers -- waits for.  The calls
// only enqueue; nothing here blocks the host except gs_defer_ctx_sync.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "gs_internal.h"

struct gs_defer_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    bool cu_masked = false;
    hipEvent_t ev_producer = nullptr;
    std::vector<hipEvent_t> done;      // per layer: recorded behind the layer's latest deferred step
    std::vector<char> pending;         // per layer: a deferred step has been enqueued and its event recorded
};

using namespace gs;

static void defer_free(gs_defer_ctx *c)
{
    if (!c) return;
    for (auto e : c->done)
        if (e) (void)hipEventDestroy(e);
    if (c->ev_producer) (void)hipEventDestroy(c->ev_producer);
    if (c->stream) (void)hipStreamDestroy(c->stream);
    delete c;
}

extern "C" {

gs_status gs_defer_ctx_create(gs_defer_ctx **out, int max_layers, int num_cus)
{
    if (!out) return GS_ERR_INVALID_ARG;
    *out = nullptr;
    if (max_layers < 1 || max_layers > 65536 || num_cus < 0) return GS_ERR_INVALID_ARG;
    gs_defer_ctx *c = new (std::nothrow) gs_defer_ctx();
    if (!c) return GS_ERR_NOMEM;
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) {
        defer_free(c);
        return hip_fail(e, "hipGetDevice");
    }
    if (num_cus > 0) {
        void *s = nullptr;
        gs_status st = gs_cu_stream_create(&s, num_cus);
        if (st != GS_OK) {
            defer_free(c);
            return st;
        }
        c->stream = static_cast<hipStream_t>(s);
        c->cu_masked = true;
    } else if ((e = hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking)) != hipSuccess) {
        c->stream = nullptr;
        defer_free(c);
        return hip_fail(e, "hipStreamCreateWithFlags");
    }
    if ((e = hipEventCreateWithFlags(&c->ev_producer, hipEventDisableTiming)) != hipSuccess) {
        c->ev_producer = nullptr;
        defer_free(c);
        return hip_fail(e, "hipEventCreateWithFlags");
    }
    c->done.assign(max_layers, nullptr);
    c->pending.assign(max_layers, 0);
    for (int i = 0; i < max_layers; ++i) {
        if ((e = hipEventCreateWithFlags(&c->done[i], hipEventDisableTiming)) != hipSuccess) {
            c->done[i] = nullptr;
            defer_free(c);
            return hip_fail(e, "hipEventCreateWithFlags");
        }
    }
    *out = c;
    return GS_OK;
}

gs_status gs_defer_ctx_sync(gs_defer_ctx *c)
{
    if (!c) return GS_ERR_INVALID_ARG;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize(deferred)");
    return GS_OK;
}

gs_status gs_defer_ctx_destroy(gs_defer_ctx *c)
{
    if (!c) return GS_ERR_INVALID_ARG;
    gs_status st = gs_defer_ctx_sync(c);
    defer_free(c);
    return st;
}

gs_status gs_defer_layer_step(gs_defer_ctx *c, int layer, float *p, float *m, float *v, uint16_t *w_bf16,
                              const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                              const gs_adamw_hparams *hp, const double *d_sqnorm, void *producer_stream)
{
    if (!c || layer < 0 || layer >= (int)c->done.size()) return GS_ERR_INVALID_ARG;
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (cur != c->device) return GS_ERR_INVALID_ARG;
    // the deferred range runs after whatever the producer stream holds now (gradients, norm, the
    // immediate part of the same layer need not be waited for: it touches other elements)
    if ((e = hipEventRecord(c->ev_producer, static_cast<hipStream_t>(producer_stream))) != hipSuccess)
        return hip_fail(e, "hipEventRecord(producer)");
    if ((e = hipStreamWaitEvent(c->stream, c->ev_producer, 0)) != hipSuccess)
        return hip_fail(e, "hipStreamWaitEvent(producer)");
    gs_status st = gs_accum_adamw(p, m, v, w_bf16, grads, k, begin, end, hp, d_sqnorm, c->stream);
    if (st != GS_OK) return st;
    if ((e = hipEventRecord(c->done[layer], c->stream)) != hipSuccess) return hip_fail(e, "hipEventRecord(layer done)");
    c->pending[layer] = 1;
    return GS_OK;
}

gs_status gs_defer_wait_layer(gs_defer_ctx *c, int layer, void *consumer_stream)
{
    if (!c || layer < 0 || layer >= (int)c->done.size()) return GS_ERR_INVALID_ARG;
    if (!c->pending[layer]) return GS_OK;      // nothing was deferred for this layer
    hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(consumer_stream), c->done[layer], 0);
    if (e != hipSuccess) return hip_fail(e, "hipStreamWaitEvent(layer done)");
    return GS_OK;
}

void *gs_defer_ctx_stream(gs_defer_ctx *c) { return c ? c->stream : nullptr; }

int gs_defer_layer_done(gs_defer_ctx *c, int layer)
{
    if (!c || layer < 0 || layer >= (int)c->done.size()) return -1;
    if (!c->pending[layer]) return 1;
    hipError_t e = hipEventQuery(c->done[layer]);
    if (e == hipSuccess) return 1;
    if (e == hipErrorNotReady) {
        (void)hipGetLastError();
        return 0;
    }
    hip_fail(e, "hipEventQuery(layer done)");
    return -1;
}

}  // extern "C"
