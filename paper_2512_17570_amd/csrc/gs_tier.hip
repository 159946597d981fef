// gs_tier.hip -- three-tier step: file (SSD) <-> pinned host <-> GPU.
//
// The paper keeps optimizer states on SSD and, per layer, runs: states SSD->CPU, step, states
// CPU->SSD, each stage overlapped with its neighbours (Sec. 4.3); a storage ratio decides which
// share of the states stays in CPU memory instead (Sec. 4.5).  Here a layer's fp32 p/m/v are
// split the same way: elements [0,n_host) in pinned host memory, elements [n_host,n) in files.
// The host share is stepped in place by the kernel, over the link.  The file share is walked in
// chunks, interleaved with launches over the host share: for file chunk c a reader thread reads
// p/m/v into a pinned bounce slot and enqueues the step kernel in place on that slot, and a
// writer thread, woken by a host function that follows the kernel, writes the slot back to the
// files.  Reading chunk c+1 overlaps the kernel of chunk c and the write-back of chunk c-1, and
// the caller is not held up by any of it: a call only checks its arguments, marks the producer
// stream and queues the layer.
//
// Every element goes through the same kernel with the same absolute-index grouping as the
// resident step, so the result is bit-identical for any n_host and chunk size.
#ifndef _GNU_SOURCE
#define _GNU_SOURCE   // O_DIRECT
#endif
#include <hip/hip_runtime.h>

#include <cerrno>
#include <condition_variable>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <deque>
#include <fcntl.h>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <unistd.h>
#include <vector>

#include "gs_internal.h"
#include "gs_stream_internal.h"

using namespace gs;

namespace {

struct WriteJob {
    int slot;
    int64_t len;            // elements
    int pad;                // the chunk starts this many elements into the slot's arrays
    bool direct;            // the descriptors are O_DIRECT: go through the slot's ordinary-memory twin
    int fd[3];
    int64_t off[3];         // byte offsets
};

// One queued call: everything the reader thread needs, copied at call time.
struct LayerJob {
    gs_tier_layer L;
    StepArgs A;             // w, gradient table, step constants, norm pointer
    int64_t h_lo, h_hi;     // the part of the range in the host share (empty if h_hi <= h_lo)
    int64_t f_lo, f_hi;     // the part of the range in the file share
    bool direct;
    hipEvent_t ev_producer; // recorded on the caller's producer stream at call time
};

// Whole-buffer pread / pwrite (short transfers are continued; EOF on read is an error).
bool read_all(int fd, void *buf, size_t bytes, int64_t off, int *err)
{
    char *p = static_cast<char *>(buf);
    while (bytes > 0) {
        ssize_t r = pread(fd, p, bytes, (off_t)off);
        if (r < 0) {
            if (errno == EINTR) continue;
            *err = errno;
            return false;
        }
        if (r == 0) {
            *err = ENODATA;   // file shorter than the layer
            return false;
        }
        p += r;
        off += r;
        bytes -= (size_t)r;
    }
    return true;
}

bool write_all(int fd, const void *buf, size_t bytes, int64_t off, int *err)
{
    const char *p = static_cast<const char *>(buf);
    while (bytes > 0) {
        ssize_t r = pwrite(fd, p, bytes, (off_t)off);
        if (r < 0) {
            if (errno == EINTR) continue;
            *err = errno;
            return false;
        }
        if (r == 0) {
            *err = EIO;
            return false;
        }
        p += r;
        off += r;
        bytes -= (size_t)r;
    }
    return true;
}

// p, m and v of one chunk move concurrently (two helper threads + the thread that asks); if a thread cannot
// be started its transfer runs on the asking thread instead.  via != nullptr: the file side of each
// transfer uses via[a] (ordinary page-aligned memory) and the data is copied between via[a] and
// buf[a] -- descriptors opened with O_DIRECT cannot transfer to or from page-locked memory that
// the GPU driver maps (EFAULT).  Returns the index of the first array that failed (errno in *err),
// or -1.
int move3(bool write, const int fd[3], float *const buf[3], float *const *via, size_t bytes, const int64_t off[3], int *err)
{
    int e[3] = {0, 0, 0};
    bool ok[3] = {true, true, true};
    auto one = [&](int a) {
        if (write) {
            if (via) memcpy(via[a], buf[a], bytes);
            ok[a] = write_all(fd[a], via ? via[a] : buf[a], bytes, off[a], &e[a]);
        } else {
            ok[a] = read_all(fd[a], via ? via[a] : buf[a], bytes, off[a], &e[a]);
            if (via && ok[a]) memcpy(buf[a], via[a], bytes);
        }
    };
    std::thread th[2];
    bool started[2] = {false, false};
    for (int a = 0; a < 2; ++a) {
        try {
            th[a] = std::thread(one, a + 1);
            started[a] = true;
        } catch (...) {
            started[a] = false;
        }
    }
    one(0);
    for (int a = 0; a < 2; ++a) {
        if (started[a]) th[a].join();
        else one(a + 1);
    }
    for (int a = 0; a < 3; ++a)
        if (!ok[a]) {
            *err = e[a];
            return a;
        }
    return -1;
}

}  // namespace

struct gs_tier_ctx {
    gs_stream_ctx *sc = nullptr;
    int device = 0;
    int slots = 0;
    int64_t chunk = 0;
    int64_t bounce_elems = 0;               // per-array stride of a bounce slot (multiple of 1024 floats)
    float *bounce = nullptr;                // pinned host: slots * 3 * bounce_elems floats
    float *plain = nullptr;                 // ordinary 4 KB-aligned memory of the same shape, made on first use
                                            // by a layer whose descriptors are O_DIRECT
    std::vector<hipEvent_t> ev_done;        // per bounce slot: its chunk's kernel has finished
    int64_t next_slot = 0;                  // running file-chunk counter across calls -> slot rotation
    struct Note {                           // argument of the host function that follows a chunk's kernel
        gs_tier_ctx *ctx;
        int slot;
    };
    std::vector<Note> notes;                // one per bounce slot, addresses stable after create
    std::vector<char> finished;           // the slot's chunk is back in the bounce slot (guarded by mu)

    std::mutex mu;
    std::condition_variable cv;
    std::deque<WriteJob> jobs;              // guarded by mu
    std::vector<char> busy;                 // bounce slot holds data not yet written back (guarded by mu)
    bool writer_active = false;             // the writer is inside a job (guarded by mu)
    bool stop = false;                      // guarded by mu
    gs_status err = GS_OK;                  // first failure of the file tier (guarded by mu)
    std::string err_text;                   // guarded by mu
    std::thread writer;
    bool writer_started = false;
    std::deque<LayerJob> layers;            // queued calls (guarded by mu)
    bool reader_active = false;             // the reader is inside a layer (guarded by mu)
    std::thread reader;
    bool reader_started = false;
    std::vector<hipEvent_t> spare_events;   // producer events not in use (guarded by mu)

    float *slot_ptr(int slot, int which) const
    {
        return bounce + ((size_t)slot * 3u + (size_t)which) * (size_t)bounce_elems;
    }
    float *plain_ptr(int slot, int which) const
    {
        return plain + ((size_t)slot * 3u + (size_t)which) * (size_t)bounce_elems;
    }
    // a failed HIP call on one of the context's threads: keep the runtime's own text too (the
    // per-thread text of gs_last_hip_error would stay behind on that thread)
    void fail_hip(gs_status st, const char *what)
    {
        std::string text = what;
        if (st == GS_ERR_HIP) {
            text += ": ";
            text += gs_last_hip_error();
        }
        fail(st, text.c_str(), 0);
    }
    void fail(gs_status st, const char *what, int err_no)
    {
        std::lock_guard<std::mutex> g(mu);
        if (err == GS_OK) {
            err = st;
            err_text = what;
            if (err_no) {
                err_text += ": ";
                err_text += strerror(err_no);
            }
        }
    }
};

// Runs on a runtime thread when the notification stream reaches it (the chunk's kernel has
// finished, its results are in the bounce slot): flag the slot and wake the writer.
static void on_chunk_done(void *arg)
{
    gs_tier_ctx::Note *note = static_cast<gs_tier_ctx::Note *>(arg);
    gs_tier_ctx *t = note->ctx;
    {
        std::lock_guard<std::mutex> g(t->mu);
        t->finished[note->slot] = 1;
    }
    t->cv.notify_all();
}

static void writer_main(gs_tier_ctx *t)
{
    for (;;) {
        WriteJob j;
        {
            std::unique_lock<std::mutex> lk(t->mu);
            t->cv.wait(lk, [&] { return t->stop || !t->jobs.empty(); });
            if (t->jobs.empty()) return;    // stop requested and nothing left
            j = t->jobs.front();
            t->jobs.pop_front();
            t->writer_active = true;
        }
        // The chunk's completion is announced by a host function enqueued behind its kernel;
        // this thread makes no HIP call, so it cannot get in the way of the reader thread's
        // (or the caller's own) enqueues.
        {
            std::unique_lock<std::mutex> lk(t->mu);
            t->cv.wait(lk, [&] { return t->finished[j.slot] != 0; });
            t->finished[j.slot] = 0;
        }
        {
            float *const buf[3] = {t->slot_ptr(j.slot, 0) + j.pad, t->slot_ptr(j.slot, 1) + j.pad,
                                   t->slot_ptr(j.slot, 2) + j.pad};
            float *const via[3] = {j.direct ? t->plain_ptr(j.slot, 0) : nullptr, j.direct ? t->plain_ptr(j.slot, 1) : nullptr,
                                   j.direct ? t->plain_ptr(j.slot, 2) : nullptr};
            int werr = 0;
            const int bad = move3(true, j.fd, buf, j.direct ? via : nullptr, (size_t)j.len * sizeof(float), j.off, &werr);
            static const char *const names[3] = {"pwrite(p)", "pwrite(m)", "pwrite(v)"};
            if (bad >= 0) t->fail(GS_ERR_IO, names[bad], werr);
        }
        {
            std::lock_guard<std::mutex> g(t->mu);
            t->busy[j.slot] = 0;
            t->writer_active = false;
        }
        t->cv.notify_all();
    }
}

static void tier_free(gs_tier_ctx *t)
{
    if (!t) return;
    {
        std::lock_guard<std::mutex> g(t->mu);
        t->stop = true;
    }
    t->cv.notify_all();
    if (t->reader_started) t->reader.join();
    if (t->writer_started) t->writer.join();
    if (t->sc) (void)gs_stream_ctx_destroy(t->sc);
    for (auto e : t->spare_events)
        if (e) (void)hipEventDestroy(e);
    for (auto e : t->ev_done)
        if (e) (void)hipEventDestroy(e);
    if (t->bounce) (void)hipHostFree(t->bounce);
    free(t->plain);
    delete t;
}

static void reader_main(gs_tier_ctx *t);

extern "C" {

gs_status gs_tier_ctx_create(gs_tier_ctx **out, int64_t chunk_elems, int slots, int num_cus)
{
    if (!out) return GS_ERR_INVALID_ARG;
    *out = nullptr;
    if (chunk_elems < 1 || slots < 2 || slots > 64) return GS_ERR_INVALID_ARG;
    if (chunk_elems > ((int64_t)1 << 34) || num_cus < 0) return GS_ERR_INVALID_ARG;

    gs_tier_ctx *t = new (std::nothrow) gs_tier_ctx();
    if (!t) return GS_ERR_NOMEM;
    gs_status st = gs_stream_ctx_create_inplace(&t->sc, num_cus);
    if (st != GS_OK) {
        t->sc = nullptr;
        tier_free(t);
        return st;
    }
    t->device = t->sc->device;
    t->slots = slots;
    t->chunk = chunk_elems;
    t->bounce_elems = ((chunk_elems + 3 + 1023) / 1024) * 1024;   // every array starts on a 4 KB boundary
    t->busy.assign(slots, 0);
    const size_t bytes = (size_t)slots * 3u * (size_t)t->bounce_elems * sizeof(float);
    t->bounce = static_cast<float *>(gs_pinned_alloc(bytes));
    if (!t->bounce) {
        tier_free(t);
        return GS_ERR_NOMEM;
    }
    t->ev_done.assign(slots, nullptr);
    for (int i = 0; i < slots; ++i) {
        hipError_t e = hipEventCreateWithFlags(&t->ev_done[i], hipEventDisableTiming);
        if (e != hipSuccess) {
            t->ev_done[i] = nullptr;
            tier_free(t);
            return hip_fail(e, "hipEventCreateWithFlags");
        }
    }
    t->finished.assign(slots, 0);
    t->notes.resize(slots);
    for (int i = 0; i < slots; ++i) t->notes[i] = gs_tier_ctx::Note{t, i};
    try {
        t->writer = std::thread(writer_main, t);
        t->writer_started = true;
        t->reader = std::thread(reader_main, t);
        t->reader_started = true;
    } catch (...) {
        tier_free(t);
        return GS_ERR_NOMEM;
    }
    *out = t;
    return GS_OK;
}

gs_status gs_tier_ctx_sync(gs_tier_ctx *t)
{
    if (!t) return GS_ERR_INVALID_ARG;
    {
        std::unique_lock<std::mutex> lk(t->mu);
        t->cv.wait(lk, [&] { return t->layers.empty() && !t->reader_active && t->jobs.empty() && !t->writer_active; });
    }
    gs_status st = gs_stream_ctx_sync(t->sc);
    std::lock_guard<std::mutex> g(t->mu);
    return t->err != GS_OK ? t->err : st;
}

gs_status gs_tier_ctx_destroy(gs_tier_ctx *t)
{
    if (!t) return GS_ERR_INVALID_ARG;
    gs_status st = gs_tier_ctx_sync(t);
    tier_free(t);
    return st;
}

const char *gs_tier_ctx_error(gs_tier_ctx *t)
{
    static thread_local std::string copy;
    if (!t) return "";
    std::lock_guard<std::mutex> g(t->mu);
    copy = t->err_text;
    return copy.c_str();
}

gs_status gs_tier_layer_step(gs_tier_ctx *t, const gs_tier_layer *L, uint16_t *d_w_bf16,
                             const uint16_t *const *d_grads, int k, int64_t n,
                             const gs_adamw_hparams *hp, const double *d_sqnorm, void *producer_stream)
{
    return gs_tier_layer_step_range(t, L, d_w_bf16, d_grads, k, n, 0, n, hp, d_sqnorm, producer_stream);
}

gs_status gs_tier_layer_step_range(gs_tier_ctx *t, const gs_tier_layer *L, uint16_t *d_w_bf16,
                                   const uint16_t *const *d_grads, int k, int64_t n, int64_t begin, int64_t end,
                                   const gs_adamw_hparams *hp, const double *d_sqnorm, void *producer_stream)
{
    if (!t || !L) return GS_ERR_INVALID_ARG;
    if (n < 0 || L->n_host < 0 || L->n_host > n) return GS_ERR_INVALID_ARG;
    if (begin < 0 || end < begin || end > n) return GS_ERR_INVALID_ARG;
    if (L->n_host > 0) {
        if (!L->h_p || !L->h_m || !L->h_v) return GS_ERR_INVALID_ARG;
        if ((reinterpret_cast<uintptr_t>(L->h_p) | reinterpret_cast<uintptr_t>(L->h_m) |
             reinterpret_cast<uintptr_t>(L->h_v)) & 15u)
            return GS_ERR_INVALID_ARG;
    }
    if (L->n_host < n) {
        if (L->fd_p < 0 || L->fd_m < 0 || L->fd_v < 0) return GS_ERR_INVALID_ARG;
        if (L->off_p < 0 || L->off_m < 0 || L->off_v < 0) return GS_ERR_INVALID_ARG;
    }
    gs_status st = stream_validate(t->sc, d_w_bf16, d_grads, k, n, hp, d_sqnorm);
    if (st != GS_OK) return st;
    {
        std::lock_guard<std::mutex> g(t->mu);
        if (t->err != GS_OK) return t->err;     // a failed context stays failed
    }
    if (begin == end) return GS_OK;
    // the parts of the range that fall into the host share and into the file share
    const int64_t h_lo = begin, h_hi = end < L->n_host ? end : L->n_host;          // empty if h_hi <= h_lo
    const int64_t f_lo = begin > L->n_host ? begin : L->n_host, f_hi = end;        // empty if f_hi <= f_lo
    if (h_hi > h_lo) {
        const int64_t len = h_hi - h_lo;
        if ((st = stream_check_mapped(L->h_p + h_lo, len)) != GS_OK || (st = stream_check_mapped(L->h_m + h_lo, len)) != GS_OK ||
            (st = stream_check_mapped(L->h_v + h_lo, len)) != GS_OK)
            return st;
    }

    bool direct = false;
    if (f_hi > f_lo) {
        const int fds[3] = {L->fd_p, L->fd_m, L->fd_v};
        for (int a = 0; a < 3; ++a) {
            const int fl = fcntl(fds[a], F_GETFL);
            if (fl < 0) return GS_ERR_INVALID_ARG;          // not an open descriptor
            if (fl & O_DIRECT) direct = true;
        }
        if (direct && !t->plain) {
            void *mem = nullptr;
            const size_t bytes = (size_t)t->slots * 3u * (size_t)t->bounce_elems * sizeof(float);
            if (posix_memalign(&mem, 4096, bytes) != 0) return GS_ERR_NOMEM;
            t->plain = static_cast<float *>(mem);
        }
    }

    gs_stream_ctx *c = t->sc;
    int cur = -1;
    hipError_t he = hipGetDevice(&cur);
    if (he != hipSuccess) return hip_fail(he, "hipGetDevice");
    if (cur != c->device) return GS_ERR_INVALID_ARG;   // the context lives on another GPU

    LayerJob job;
    memset(&job.A, 0, sizeof job.A);
    job.L = *L;
    job.A.w = d_w_bf16;
    for (int j = 0; j < k; ++j) job.A.gt.g[j] = d_grads[j];
    job.A.k = k;
    job.A.c = make_consts(*hp);
    job.A.max_norm = hp->max_grad_norm;
    job.A.d_sqnorm = d_sqnorm;
    job.h_lo = h_lo;
    job.h_hi = h_hi;
    job.f_lo = f_lo;
    job.f_hi = f_hi;
    job.direct = direct;
    // gradients and the norm come from the caller's stream: mark where it stands now
    job.ev_producer = nullptr;
    {
        std::lock_guard<std::mutex> g(t->mu);
        if (!t->spare_events.empty()) {
            job.ev_producer = t->spare_events.back();
            t->spare_events.pop_back();
        }
    }
    if (!job.ev_producer) {
        he = hipEventCreateWithFlags(&job.ev_producer, hipEventDisableTiming);
        if (he != hipSuccess) return hip_fail(he, "hipEventCreateWithFlags");
    }
    he = hipEventRecord(job.ev_producer, static_cast<hipStream_t>(producer_stream));
    if (he != hipSuccess) {
        std::lock_guard<std::mutex> g(t->mu);
        t->spare_events.push_back(job.ev_producer);
        return hip_fail(he, "hipEventRecord(producer)");
    }
    {
        std::lock_guard<std::mutex> g(t->mu);
        t->layers.push_back(job);
    }
    t->cv.notify_all();
    return GS_OK;
}

}  // extern "C"

// The reader thread's work for one queued call.  Failures are recorded in the context (the call
// that queued the layer has long returned).
static void run_layer(gs_tier_ctx *t, LayerJob &job)
{
    gs_stream_ctx *c = t->sc;
    StepArgs &A = job.A;
    const gs_tier_layer *L = &job.L;
    const int64_t h_lo = job.h_lo, h_hi = job.h_hi, f_lo = job.f_lo, f_hi = job.f_hi;
    const bool direct = job.direct;
    gs_status st = GS_OK;
    hipError_t we = hipStreamWaitEvent(c->s_comp, job.ev_producer, 0);
    {
        std::lock_guard<std::mutex> g(t->mu);
        t->spare_events.push_back(job.ev_producer);   // the wait has captured the record: free for reuse
    }
    if (we != hipSuccess) {
        t->fail_hip(hip_fail(we, "hipStreamWaitEvent(producer)"), "waiting for the producer stream failed");
        return;
    }

    // The two shares are walked together, each in proportion to its size, so that file reads and
    // write-backs run alongside the host share's PCIe traffic instead of after it.  (The update
    // is element-wise: the order of chunks does not change any result.)
    const int fd[3] = {L->fd_p, L->fd_m, L->fd_v};
    const int64_t base[3] = {L->off_p, L->off_m, L->off_v};
    const int64_t host_chunks = h_hi > h_lo ? (h_hi - h_lo + t->chunk - 1) / t->chunk : 0;
    const int64_t file_chunks = f_hi > f_lo ? (f_hi - f_lo + t->chunk - 1) / t->chunk : 0;
    int64_t hi = 0, fi = 0;
    while (hi < host_chunks || fi < file_chunks) {
        // next: the share that is further behind (fi/file_chunks < hi/host_chunks); ties go to the file share,
        // whose read takes host time
        const bool take_file = fi < file_chunks && (hi >= host_chunks || fi * host_chunks <= hi * file_chunks);
        if (!take_file) {
            const int64_t b = h_lo + hi * t->chunk;
            const int64_t e = (b + t->chunk < h_hi) ? b + t->chunk : h_hi;
            ++hi;
            st = stream_range(c, A, L->h_p + b, L->h_m + b, L->h_v + b, b, e);
            if (st != GS_OK) {
                t->fail_hip(st, "enqueue of a host chunk failed");
                return;
            }
            continue;
        }
        const int64_t b = f_lo + fi * t->chunk;
        const int64_t e = (b + t->chunk < f_hi) ? b + t->chunk : f_hi;
        ++fi;
        const int64_t len = e - b;
        const int slot = (int)(t->next_slot % t->slots);
        t->next_slot++;
        {
            std::unique_lock<std::mutex> lk(t->mu);
            t->cv.wait(lk, [&] { return !t->busy[slot]; });
            if (t->err != GS_OK) return;     // the writer failed: stop feeding it
        }
        int64_t off[3];
        for (int a = 0; a < 3; ++a) off[a] = base[a] + (b - L->n_host) * (int64_t)sizeof(float);
        // the chunk sits (b mod 4) elements into its bounce arrays, so that the kernel's 16-byte
        // accesses to absolute-index groups stay aligned
        const int64_t pad = b & 3;
        float *const buf[3] = {t->slot_ptr(slot, 0) + pad, t->slot_ptr(slot, 1) + pad, t->slot_ptr(slot, 2) + pad};
        float *const via[3] = {direct ? t->plain_ptr(slot, 0) : nullptr, direct ? t->plain_ptr(slot, 1) : nullptr,
                               direct ? t->plain_ptr(slot, 2) : nullptr};
        int rerr = 0;
        const int bad = move3(false, fd, buf, direct ? via : nullptr, (size_t)len * sizeof(float), off, &rerr);
        if (bad >= 0) {
            static const char *const names[3] = {"pread(p)", "pread(m)", "pread(v)"};
            t->fail(GS_ERR_IO, names[bad], rerr);
            return;
        }
        st = stream_range(c, A, buf[0], buf[1], buf[2], b, e);
        if (st == GS_OK) {
            // the notification rides on its own stream so that the compute stream never waits
            // for a host thread
            hipError_t he = hipEventRecord(t->ev_done[slot], c->s_comp);
            if (he == hipSuccess) he = hipStreamWaitEvent(c->s_note, t->ev_done[slot], 0);
            if (he == hipSuccess) he = hipLaunchHostFunc(c->s_note, on_chunk_done, &t->notes[slot]);
            if (he != hipSuccess) st = hip_fail(he, "hipLaunchHostFunc(chunk done)");
        }
        if (st != GS_OK) {
            t->fail_hip(st, "enqueue of a file chunk failed");
            return;
        }
        WriteJob j;
        j.slot = slot;
        j.len = len;
        j.pad = (int)pad;
        j.direct = direct;
        for (int a = 0; a < 3; ++a) {
            j.fd[a] = fd[a];
            j.off[a] = off[a];
        }
        {
            std::lock_guard<std::mutex> g(t->mu);
            t->busy[slot] = 1;
            t->jobs.push_back(j);
        }
        t->cv.notify_all();
    }
}

static void reader_main(gs_tier_ctx *t)
{
    const hipError_t de = hipSetDevice(t->device);
    if (de != hipSuccess) t->fail_hip(hip_fail(de, "hipSetDevice"), "the reader thread could not select the device");
    for (;;) {
        LayerJob job;
        bool skip;
        {
            std::unique_lock<std::mutex> lk(t->mu);
            t->cv.wait(lk, [&] { return t->stop || !t->layers.empty(); });
            if (t->layers.empty()) return;  // stop requested and nothing left
            job = t->layers.front();
            t->layers.pop_front();
            t->reader_active = true;
            skip = t->err != GS_OK;         // a failed context steps nothing further
            if (skip) t->spare_events.push_back(job.ev_producer);
        }
        if (!skip) run_layer(t, job);
        {
            std::lock_guard<std::mutex> g(t->mu);
            t->reader_active = false;
        }
        t->cv.notify_all();
    }
}
