// gs_stream.hip -- streamed step over states resident in pinned host memory.
//
// The paper's optimizer step walks parameter chunks: load a chunk's master parameters and
// optimizer states, step, write them back (Sec. 2.2), pipelined against the surrounding work
// (Sec. 4.3).  There the slow link is SSD<->host; here it is host<->HBM over PCIe, so the
// pipeline is: upload stream (chunk c+1) | compute stream (chunk c) | download stream
// (chunk c-1), with `slots` staging slots in HBM rotating between the three.
//
// Staging keeps the absolute-index grouping of the kernel: chunk [b,e) is placed in its slot
// at offset (b mod 8), and the kernel is handed a base pointer such that element i of the
// layer sits at base[i].  The kernel's 4-element groups (and their 16-byte alignment)
// therefore fall exactly where they fall for device-resident states, which makes the streamed
// result bit-identical for any chunk size.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "gs_internal.h"
#include "gs_stream_internal.h"

using namespace gs;


static void destroy_partial(gs_stream_ctx *c)
{
    if (!c) return;
    for (auto e : c->ev_h2d) if (e) (void)hipEventDestroy(e);
    for (auto e : c->ev_comp) if (e) (void)hipEventDestroy(e);
    for (auto e : c->ev_d2h) if (e) (void)hipEventDestroy(e);
    if (c->ev_producer) (void)hipEventDestroy(c->ev_producer);
    if (c->pool) (void)hipFree(c->pool);
    if (c->s_h2d) (void)hipStreamDestroy(c->s_h2d);
    if (c->s_comp) (void)hipStreamDestroy(c->s_comp);
    if (c->s_d2h) (void)hipStreamDestroy(c->s_d2h);
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
    if (cur != c->device) return GS_ERR_INVALID_ARG;   // the context's streams and slots live on another GPU

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

gs_status stream_chunk(gs_stream_ctx *c, StepArgs &A, float *src_p, float *src_m, float *src_v, int64_t b, int64_t e,
                       int *slot_out)
{
    const int64_t len = e - b;
    const int slot = (int)(c->next_chunk % c->slots);
    c->next_chunk++;
    if (slot_out) *slot_out = slot;
    const int64_t pad = b & 7;
    float *sp = c->pool + (size_t)slot * 3u * (size_t)c->slot_elems;
    float *sm = sp + c->slot_elems;
    float *sv = sm + c->slot_elems;
    const size_t bytes = (size_t)len * sizeof(float);

    // upload: wait until the slot's previous download has drained
    if (c->used[slot]) GS_TRY(hipStreamWaitEvent(c->s_h2d, c->ev_d2h[slot], 0), "hipStreamWaitEvent(slot free)");
    GS_TRY(hipMemcpyAsync(sp + pad, src_p, bytes, hipMemcpyHostToDevice, c->s_h2d), "hipMemcpyAsync(H2D p)");
    GS_TRY(hipMemcpyAsync(sm + pad, src_m, bytes, hipMemcpyHostToDevice, c->s_h2d), "hipMemcpyAsync(H2D m)");
    GS_TRY(hipMemcpyAsync(sv + pad, src_v, bytes, hipMemcpyHostToDevice, c->s_h2d), "hipMemcpyAsync(H2D v)");
    GS_TRY(hipEventRecord(c->ev_h2d[slot], c->s_h2d), "hipEventRecord(h2d)");

    // compute: base pointers chosen so that base[i] is element i of the layer
    GS_TRY(hipStreamWaitEvent(c->s_comp, c->ev_h2d[slot], 0), "hipStreamWaitEvent(h2d)");
    const intptr_t shift = (intptr_t)(pad - b) * (intptr_t)sizeof(float);
    A.po = reinterpret_cast<float *>(reinterpret_cast<intptr_t>(sp) + shift);
    A.mo = reinterpret_cast<float *>(reinterpret_cast<intptr_t>(sm) + shift);
    A.vo = reinterpret_cast<float *>(reinterpret_cast<intptr_t>(sv) + shift);
    A.p = A.po;
    A.m = A.mo;
    A.v = A.vo;
    A.begin = b;
    A.end = e;
    hipError_t le = launch_accum_adamw(A, c->s_comp);
    if (le != hipSuccess) return hip_fail(le, "streamed step launch");
    GS_TRY(hipEventRecord(c->ev_comp[slot], c->s_comp), "hipEventRecord(compute)");

    // download
    GS_TRY(hipStreamWaitEvent(c->s_d2h, c->ev_comp[slot], 0), "hipStreamWaitEvent(compute)");
    GS_TRY(hipMemcpyAsync(src_p, sp + pad, bytes, hipMemcpyDeviceToHost, c->s_d2h), "hipMemcpyAsync(D2H p)");
    GS_TRY(hipMemcpyAsync(src_m, sm + pad, bytes, hipMemcpyDeviceToHost, c->s_d2h), "hipMemcpyAsync(D2H m)");
    GS_TRY(hipMemcpyAsync(src_v, sv + pad, bytes, hipMemcpyDeviceToHost, c->s_d2h), "hipMemcpyAsync(D2H v)");
    GS_TRY(hipEventRecord(c->ev_d2h[slot], c->s_d2h), "hipEventRecord(d2h)");
    c->used[slot] = 1;
    return GS_OK;
}

}  // namespace gs

extern "C" {

gs_status gs_stream_ctx_create(gs_stream_ctx **out, int64_t chunk_elems, int slots)
{
    if (!out) return GS_ERR_INVALID_ARG;
    *out = nullptr;
    if (chunk_elems < 1 || slots < 2 || slots > 64) return GS_ERR_INVALID_ARG;
    if (chunk_elems > ((int64_t)1 << 34)) return GS_ERR_INVALID_ARG;

    gs_stream_ctx *c = new (std::nothrow) gs_stream_ctx();
    if (!c) return GS_ERR_NOMEM;
    c->chunk = chunk_elems;
    c->slots = slots;
    c->slot_elems = ((chunk_elems + 8 + 63) / 64) * 64;   // keep every slot array 256-byte aligned
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) { destroy_partial(c); return hip_fail(e, "hipGetDevice"); }

    // default priority on every stream
    if ((e = hipStreamCreateWithFlags(&c->s_h2d, hipStreamNonBlocking)) != hipSuccess ||
        (e = hipStreamCreateWithFlags(&c->s_comp, hipStreamNonBlocking)) != hipSuccess ||
        (e = hipStreamCreateWithFlags(&c->s_d2h, hipStreamNonBlocking)) != hipSuccess) {
        destroy_partial(c);
        return hip_fail(e, "hipStreamCreateWithFlags");
    }
    const size_t bytes = (size_t)slots * 3u * (size_t)c->slot_elems * sizeof(float);
    e = hipMalloc(reinterpret_cast<void **>(&c->pool), bytes);
    if (e != hipSuccess) {
        hip_fail(e, "hipMalloc(staging slots)");
        (void)hipGetLastError();
        c->pool = nullptr;
        destroy_partial(c);
        return GS_ERR_NOMEM;
    }
    c->ev_h2d.assign(slots, nullptr);
    c->ev_comp.assign(slots, nullptr);
    c->ev_d2h.assign(slots, nullptr);
    c->used.assign(slots, 0);
    for (int i = 0; i < slots; ++i) {
        if ((e = hipEventCreateWithFlags(&c->ev_h2d[i], hipEventDisableTiming)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&c->ev_comp[i], hipEventDisableTiming)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&c->ev_d2h[i], hipEventDisableTiming)) != hipSuccess) {
            destroy_partial(c);
            return hip_fail(e, "hipEventCreateWithFlags");
        }
    }
    if ((e = hipEventCreateWithFlags(&c->ev_producer, hipEventDisableTiming)) != hipSuccess) {
        destroy_partial(c);
        return hip_fail(e, "hipEventCreateWithFlags");
    }
    *out = c;
    return GS_OK;
}

gs_status gs_stream_ctx_sync(gs_stream_ctx *c)
{
    if (!c) return GS_ERR_INVALID_ARG;
    GS_TRY(hipStreamSynchronize(c->s_h2d), "hipStreamSynchronize(h2d)");
    GS_TRY(hipStreamSynchronize(c->s_comp), "hipStreamSynchronize(compute)");
    GS_TRY(hipStreamSynchronize(c->s_d2h), "hipStreamSynchronize(d2h)");
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
    if ((reinterpret_cast<uintptr_t>(h_p) | reinterpret_cast<uintptr_t>(h_m) | reinterpret_cast<uintptr_t>(h_v)) & 3u)
        return GS_ERR_INVALID_ARG;
    gs_status st = stream_validate(c, d_w_bf16, d_grads, k, n, hp, d_sqnorm);
    if (st != GS_OK) return st;
    if (n == 0) return GS_OK;

    StepArgs A;
    st = stream_begin_layer(c, A, d_w_bf16, d_grads, k, hp, d_sqnorm, producer_stream);
    if (st != GS_OK) return st;
    for (int64_t b = 0; b < n; b += c->chunk) {
        const int64_t e = (b + c->chunk < n) ? b + c->chunk : n;
        st = stream_chunk(c, A, h_p + b, h_m + b, h_v + b, b, e, nullptr);
        if (st != GS_OK) return st;
    }
    return GS_OK;
}

}  // extern "C"
