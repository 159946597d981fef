// gs_stream.hip -- the step over states resident in pinned host memory.
//
// The paper's optimizer step walks parameter chunks: load a chunk's master parameters and
// optimizer states, step, write them back (Sec. 2.2), pipelined against the surrounding work
// (Sec. 4.3).  There the slow link is SSD<->host; here it is host<->HBM over PCIe.  Two ways:
//
// In place (gs_stream_ctx_create_inplace).  The step kernel runs on the pinned host arrays themselves, so every
// wave loads its tile of p/m/v over the link, updates it and stores it back, thousands of waves
// at different stages at any time.  Nothing is staged in HBM and no copy engine is involved.
// Measured on MI355X (GPT-65B-shaped layers, k = 8): 44-45 GB/s each way at once, the same on a
// stream confined to 16 of the 256 CUs, and the same whatever copy traffic the process ran
// before.
//
// Staged (gs_stream_ctx_create).  Chunk c+1 is uploaded by hipMemcpyAsync into one of `slots` staging slots in HBM while
// the kernel updates chunk c there and chunk c-1 is copied back: three streams, events per slot.
// It costs no CU time beyond the 0.5 ms kernel per chunk and reached 48 GB/s each way at its
// best, but its rate is in the runtime's hands: which copy path a copy takes (under the file
// tier's load its device-to-host copies were seen on the DMA engine at 12.8 GB/s) and which
// hardware queue a stream lands on (upload and download on one queue: 28 GB/s each way; the
// context checks for that when it is created and swaps the download stream until the two overlap).
//
// Either way the kernel is the resident one, handed base pointers such that base[i] is element i
// of the layer (staged: chunk [b,e) sits at offset (b mod 8) of its slot), so its 4-element
// groups fall on the same absolute indices and the result is bit-identical to the
// device-resident step.
#include <hip/hip_runtime.h>

#include <algorithm>
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
    if (c->s_d2h) (void)hipStreamDestroy(c->s_d2h);
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

// In-place contexts hand host addresses to a kernel: anything but page-locked, device-mapped host
// memory would fault the GPU, so the runtime is asked about the first and the last element of
// every array (a range that runs past its allocation fails on the last).
gs_status stream_check_mapped(const float *h, int64_t n)
{
    const float *probe[2] = {h, h + (n - 1)};
    for (const float *q : probe) {
        hipPointerAttribute_t a;
        memset(&a, 0, sizeof a);
        hipError_t e = hipPointerGetAttributes(&a, q);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return GS_ERR_INVALID_ARG;
        }
        if (a.type != hipMemoryTypeHost || a.devicePointer != static_cast<const void *>(q)) return GS_ERR_INVALID_ARG;
    }
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

// Staged mode: one chunk through upload -> kernel in its HBM slot -> download.
static gs_status staged_chunk(gs_stream_ctx *c, StepArgs &A, float *host_p, float *host_m, float *host_v, int64_t b,
                              int64_t e)
{
    const int64_t len = e - b;
    const int slot = (int)(c->next_chunk % c->slots);
    c->next_chunk++;
    const int64_t pad = b & 7;
    float *sp = c->pool + (size_t)slot * 3u * (size_t)c->slot_elems;
    float *sm = sp + c->slot_elems;
    float *sv = sm + c->slot_elems;
    const size_t bytes = (size_t)len * sizeof(float);

    // upload: wait until the slot's previous download has drained
    if (c->used[slot]) GS_TRY(hipStreamWaitEvent(c->s_h2d, c->ev_d2h[slot], 0), "hipStreamWaitEvent(slot free)");
    GS_TRY(hipMemcpyAsync(sp + pad, host_p, bytes, hipMemcpyHostToDevice, c->s_h2d), "hipMemcpyAsync(H2D p)");
    GS_TRY(hipMemcpyAsync(sm + pad, host_m, bytes, hipMemcpyHostToDevice, c->s_h2d), "hipMemcpyAsync(H2D m)");
    GS_TRY(hipMemcpyAsync(sv + pad, host_v, bytes, hipMemcpyHostToDevice, c->s_h2d), "hipMemcpyAsync(H2D v)");
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
    if (le != hipSuccess) return hip_fail(le, "staged step launch");
    GS_TRY(hipEventRecord(c->ev_comp[slot], c->s_comp), "hipEventRecord(compute)");

    // download
    GS_TRY(hipStreamWaitEvent(c->s_d2h, c->ev_comp[slot], 0), "hipStreamWaitEvent(compute)");
    GS_TRY(hipMemcpyAsync(host_p, sp + pad, bytes, hipMemcpyDeviceToHost, c->s_d2h), "hipMemcpyAsync(D2H p)");
    GS_TRY(hipMemcpyAsync(host_m, sm + pad, bytes, hipMemcpyDeviceToHost, c->s_d2h), "hipMemcpyAsync(D2H m)");
    GS_TRY(hipMemcpyAsync(host_v, sv + pad, bytes, hipMemcpyDeviceToHost, c->s_d2h), "hipMemcpyAsync(D2H v)");
    GS_TRY(hipEventRecord(c->ev_d2h[slot], c->s_d2h), "hipEventRecord(d2h)");
    c->used[slot] = 1;
    return GS_OK;
}

}  // namespace gs

// Staged mode lives on three streams that really run side by side.  HIP multiplexes a process's
// streams onto a few hardware queues, and a hardware queue takes its work in order: when the upload
// and the download stream share one, the two directions take turns; when the compute stream shares
// one with a copy stream, its wait for the next chunk's upload also holds back the previous chunk's
// download queued behind it.  Either way the pipeline runs at half its rate with nothing else to
// show for it.  Which queue a new stream gets depends on the streams the process already has, so
// the context checks each pair: `busy` is given a burst of copies of `bytes` each, and `other`,
// released by an event at the start of the burst, a 4 KB copy the other way.  If the small copy is
// done in under half the burst's time, the two streams run side by side.  Returns 1 (side by
// side, or too short to tell), 0 (in turns) or -1 (a HIP call failed; the error text is set).
static int overtakes(hipStream_t busy, hipStream_t other, bool busy_uploads, float *dev, float *host, size_t bytes)
{
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    int verdict = -1;
    float t_burst = 0.f, t_small = 0.f;
    char *d = reinterpret_cast<char *>(dev), *h = reinterpret_cast<char *>(host);
    const size_t small = 4096;
    const hipMemcpyKind burst_kind = busy_uploads ? hipMemcpyHostToDevice : hipMemcpyDeviceToHost;
    const hipMemcpyKind small_kind = busy_uploads ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice;
    void *burst_dst = busy_uploads ? static_cast<void *>(d) : static_cast<void *>(h);
    const void *burst_src = busy_uploads ? static_cast<const void *>(h) : static_cast<const void *>(d);
    void *small_dst = busy_uploads ? static_cast<void *>(h + bytes) : static_cast<void *>(d + bytes);
    const void *small_src = busy_uploads ? static_cast<const void *>(d + bytes) : static_cast<const void *>(h + bytes);
    hipError_t e = hipSuccess;
    auto fail = [&](const char *what) {
        hip_fail(e, what);
        return -1;
    };
    for (auto &x : ev)
        if ((e = hipEventCreateWithFlags(&x, 0)) != hipSuccess) {
            x = nullptr;
            verdict = fail("hipEventCreateWithFlags(stream check)");
            goto done;
        }
    // warm both paths
    if ((e = hipMemcpyAsync(burst_dst, burst_src, bytes, burst_kind, busy)) != hipSuccess ||
        (e = hipMemcpyAsync(small_dst, small_src, small, small_kind, other)) != hipSuccess ||
        (e = hipStreamSynchronize(busy)) != hipSuccess || (e = hipStreamSynchronize(other)) != hipSuccess) {
        verdict = fail("stream check (warm-up)");
        goto done;
    }
    if ((e = hipEventRecord(ev[0], busy)) != hipSuccess || (e = hipStreamWaitEvent(other, ev[0], 0)) != hipSuccess) {
        verdict = fail("stream check (start)");
        goto done;
    }
    for (int r = 0; r < 2; ++r)
        if ((e = hipMemcpyAsync(burst_dst, burst_src, bytes, burst_kind, busy)) != hipSuccess) {
            verdict = fail("hipMemcpyAsync(stream check)");
            goto done;
        }
    if ((e = hipEventRecord(ev[1], busy)) != hipSuccess ||
        (e = hipMemcpyAsync(small_dst, small_src, small, small_kind, other)) != hipSuccess ||
        (e = hipEventRecord(ev[2], other)) != hipSuccess || (e = hipStreamSynchronize(busy)) != hipSuccess ||
        (e = hipStreamSynchronize(other)) != hipSuccess || (e = hipEventElapsedTime(&t_burst, ev[0], ev[1])) != hipSuccess ||
        (e = hipEventElapsedTime(&t_small, ev[0], ev[2])) != hipSuccess) {
        verdict = fail("stream check (burst)");
        goto done;
    }
    // a burst too short to time (a runtime without a clock): take the streams as they are
    verdict = (t_burst < 0.05f) ? 1 : (t_small < 0.5f * t_burst ? 1 : 0);
done:
    for (auto x : ev)
        if (x) (void)hipEventDestroy(x);
    return verdict;
}

// the compute stream and the producer event, common to both modes
static gs_status create_common(gs_stream_ctx *c, int num_cus)
{
    hipError_t e;
    // default priority on every stream
    if (num_cus > 0) {
        void *s = nullptr;
        gs_status st = gs_cu_stream_create(&s, num_cus);
        if (st != GS_OK) return st;
        c->s_comp = static_cast<hipStream_t>(s);
    } else if ((e = hipStreamCreateWithFlags(&c->s_comp, hipStreamNonBlocking)) != hipSuccess) {
        c->s_comp = nullptr;
        return hip_fail(e, "hipStreamCreateWithFlags");
    }
    if ((e = hipEventCreateWithFlags(&c->ev_producer, hipEventDisableTiming)) != hipSuccess) {
        c->ev_producer = nullptr;
        return hip_fail(e, "hipEventCreateWithFlags");
    }
    return GS_OK;
}

extern "C" {

gs_status gs_stream_ctx_create_inplace(gs_stream_ctx **out, int num_cus)
{
    if (!out) return GS_ERR_INVALID_ARG;
    *out = nullptr;
    if (num_cus < 0) return GS_ERR_INVALID_ARG;

    gs_stream_ctx *c = new (std::nothrow) gs_stream_ctx();
    if (!c) return GS_ERR_NOMEM;
    c->num_cus = num_cus;
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) {
        destroy_partial(c);
        return hip_fail(e, "hipGetDevice");
    }
    gs_status st = create_common(c, num_cus);
    if (st != GS_OK) {
        destroy_partial(c);
        return st;
    }
    if ((e = hipStreamCreateWithFlags(&c->s_note, hipStreamNonBlocking)) != hipSuccess) {
        c->s_note = nullptr;
        destroy_partial(c);
        return hip_fail(e, "hipStreamCreateWithFlags");
    }
    *out = c;
    return GS_OK;
}

gs_status gs_stream_ctx_create(gs_stream_ctx **out, int64_t chunk_elems, int slots)
{
    if (!out) return GS_ERR_INVALID_ARG;
    *out = nullptr;
    if (chunk_elems < 1 || slots < 2 || slots > 64) return GS_ERR_INVALID_ARG;
    if (chunk_elems > ((int64_t)1 << 34)) return GS_ERR_INVALID_ARG;

    gs_stream_ctx *c = new (std::nothrow) gs_stream_ctx();
    if (!c) return GS_ERR_NOMEM;
    c->staged = true;
    c->chunk = chunk_elems;
    c->slots = slots;
    c->slot_elems = ((chunk_elems + 8 + 63) / 64) * 64;   // keep every slot array 256-byte aligned
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) {
        destroy_partial(c);
        return hip_fail(e, "hipGetDevice");
    }
    // Exactly three streams, created back to back: HIP multiplexes a process's streams onto a few
    // hardware queues (4 here), and two of these three landing on one queue serialises the two
    // copy directions (28 instead of 48 GB/s each way was measured when that happened).
    if ((e = hipStreamCreateWithFlags(&c->s_h2d, hipStreamNonBlocking)) != hipSuccess) {
        c->s_h2d = nullptr;
        destroy_partial(c);
        return hip_fail(e, "hipStreamCreateWithFlags");
    }
    gs_status st = create_common(c, 0);
    if (st != GS_OK) {
        destroy_partial(c);
        return st;
    }
    if ((e = hipStreamCreateWithFlags(&c->s_d2h, hipStreamNonBlocking)) != hipSuccess) {
        c->s_d2h = nullptr;
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
    // Make sure the three streams really run side by side; while a pair takes turns, swap one of the
    // two for a fresh stream (the rejected ones stay alive meanwhile, so each new one is handed another
    // hardware queue).
    const size_t probe_bytes = std::min<size_t>((size_t)64 << 20, bytes / 2) & ~(size_t)4095;
    if (probe_bytes >= ((size_t)1 << 20)) {
        void *host = nullptr;
        e = hipHostMalloc(&host, probe_bytes + 8192, hipHostMallocDefault);
        if (e != hipSuccess) {
            hip_fail(e, "hipHostMalloc(stream check)");
            (void)hipGetLastError();
            destroy_partial(c);
            return GS_ERR_NOMEM;
        }
        memset(host, 0, probe_bytes + 8192);
        float *hbuf = static_cast<float *>(host);
        std::vector<hipStream_t> rejected;
        int verdict = 0;
        for (int attempt = 0; attempt < 10; ++attempt) {
            const int ud = overtakes(c->s_h2d, c->s_d2h, true, c->pool, hbuf, probe_bytes);
            const int uc = ud < 0 ? -1 : overtakes(c->s_h2d, c->s_comp, true, c->pool, hbuf, probe_bytes);
            const int dc = uc < 0 ? -1 : overtakes(c->s_d2h, c->s_comp, false, c->pool, hbuf, probe_bytes);
            if (ud < 0 || uc < 0 || dc < 0) {
                verdict = -1;
                break;
            }
            verdict = (ud && uc && dc) ? 1 : 0;
            if (verdict == 1 || attempt == 9) break;
            hipStream_t cand = nullptr;
            if ((e = hipStreamCreateWithFlags(&cand, hipStreamNonBlocking)) != hipSuccess) {
                hip_fail(e, "hipStreamCreateWithFlags");
                verdict = -1;
                break;
            }
            hipStream_t &victim = !ud ? c->s_d2h : c->s_comp;      // the compute stream if it is the one that collides
            rejected.push_back(victim);
            victim = cand;
        }
        for (hipStream_t r : rejected) (void)hipStreamDestroy(r);
        (void)hipHostFree(host);
        if (verdict < 0) {
            destroy_partial(c);
            return GS_ERR_HIP;
        }
        c->copies_overlap = verdict;
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
    *out = c;
    return GS_OK;
}

int gs_stream_ctx_copies_overlap(const gs_stream_ctx *c) { return c ? c->copies_overlap : -1; }

gs_status gs_stream_ctx_sync(gs_stream_ctx *c)
{
    if (!c) return GS_ERR_INVALID_ARG;
    if (c->s_h2d) GS_TRY(hipStreamSynchronize(c->s_h2d), "hipStreamSynchronize(h2d)");
    GS_TRY(hipStreamSynchronize(c->s_comp), "hipStreamSynchronize(compute)");
    if (c->s_d2h) GS_TRY(hipStreamSynchronize(c->s_d2h), "hipStreamSynchronize(d2h)");
    if (c->s_note) GS_TRY(hipStreamSynchronize(c->s_note), "hipStreamSynchronize(notify)");
    return GS_OK;
}

gs_status gs_stream_ctx_destroy(gs_stream_ctx *c)
{
    if (!c) return GS_ERR_INVALID_ARG;
    gs_status st = gs_stream_ctx_sync(c);
    destroy_partial(c);
    return st;
}

gs_status gs_stream_layer_step_range(gs_stream_ctx *c, float *h_p, float *h_m, float *h_v,
                                     uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k,
                                     int64_t begin, int64_t end,
                                     const gs_adamw_hparams *hp, const double *d_sqnorm,
                                     void *producer_stream)
{
    if (!c || !h_p || !h_m || !h_v) return GS_ERR_INVALID_ARG;
    // in place the kernel's 16-byte accesses hit the host arrays; staged, only copies do
    const uintptr_t align_mask = c->staged ? 3u : 15u;
    if ((reinterpret_cast<uintptr_t>(h_p) | reinterpret_cast<uintptr_t>(h_m) | reinterpret_cast<uintptr_t>(h_v)) & align_mask)
        return GS_ERR_INVALID_ARG;
    if (begin < 0 || end < begin) return GS_ERR_INVALID_ARG;
    gs_status st = stream_validate(c, d_w_bf16, d_grads, k, end, hp, d_sqnorm);
    if (st != GS_OK) return st;
    if (begin == end) return GS_OK;
    if (!c->staged) {
        const int64_t len = end - begin;
        if ((st = stream_check_mapped(h_p + begin, len)) != GS_OK || (st = stream_check_mapped(h_m + begin, len)) != GS_OK ||
            (st = stream_check_mapped(h_v + begin, len)) != GS_OK)
            return st;
    }

    StepArgs A;
    st = stream_begin_layer(c, A, d_w_bf16, d_grads, k, hp, d_sqnorm, producer_stream);
    if (st != GS_OK) return st;
    if (!c->staged) return stream_range(c, A, h_p + begin, h_m + begin, h_v + begin, begin, end);
    for (int64_t b = begin; b < end; b += c->chunk) {
        const int64_t e = (b + c->chunk < end) ? b + c->chunk : end;
        st = staged_chunk(c, A, h_p + b, h_m + b, h_v + b, b, e);
        if (st != GS_OK) return st;
    }
    return GS_OK;
}

gs_status gs_stream_layer_step(gs_stream_ctx *c, float *h_p, float *h_m, float *h_v,
                               uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k, int64_t n,
                               const gs_adamw_hparams *hp, const double *d_sqnorm,
                               void *producer_stream)
{
    if (n < 0) return GS_ERR_INVALID_ARG;
    return gs_stream_layer_step_range(c, h_p, h_m, h_v, d_w_bf16, d_grads, k, 0, n, hp, d_sqnorm, producer_stream);
}

}  // extern "C"
