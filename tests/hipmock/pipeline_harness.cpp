#ifndef _GNU_SOURCE
#define _GNU_SOURCE   // O_DIRECT
#endif
// Host-only exercise of the streaming and file-tier pipelines against the HIP stand-in.
// The step kernel is replaced by a trivial element-wise stand-in (the real arithmetic needs a GPU
// and is checked by the GPU parity tests); what is checked here is the plumbing: every element
// goes up, through the "kernel" exactly once and back to where it came from -- host array or file
// offset -- for any chunk size, slot count and host/file split, and failures of the file tier
// surface as GS_ERR_IO instead of a hang.  Built with -fsanitize=thread by the test that runs it.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fcntl.h>
#include <string>
#include <thread>
#include <unistd.h>
#include <atomic>
#include <vector>

#include "gs_internal.h"

namespace gs {

// planted launch failure: the nth launch from the moment it is armed fails (0: disarmed)
static std::atomic<int> g_launch_fault{0};

// stand-in "kernel": p' = p + 1, m' = 2 m, v' = v + g_0, w = low 16 bits of (i + k)
hipError_t launch_accum_adamw(const StepArgs &A, hipStream_t stream)
{
    if (g_launch_fault.load() > 0 && g_launch_fault.fetch_sub(1) == 1) return hipErrorUnknown;
    StepArgs a = A;
    hipmock_enqueue(stream, [a] {
        for (int64_t i = a.begin; i < a.end; ++i) {
            a.po[i] = a.p[i] + 1.0f;
            a.mo[i] = a.m[i] * 2.0f;
            a.vo[i] = a.v[i] + (float)a.gt.g[0][i];
            a.w[i] = (uint16_t)((i + a.k) & 0xffff);
        }
    });
    return hipSuccess;
}
hipError_t launch_accum_adamw_spec(const StepArgs &, double *, size_t, double *, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_grad_sqnorm(const SqnormArgs &, size_t, double *, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_accum_add(const AccumAddArgs &, int, size_t, double *, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_acc_sqnorm(const float *, int64_t, int64_t, double *, size_t, double *, int, hipStream_t) { return hipErrorUnknown; }

}  // namespace gs

static int g_fail = 0;
#define CHECK(cond, ...)                                   \
    do {                                                   \
        if (!(cond)) {                                     \
            printf("FAIL %s:%d: ", __FILE__, __LINE__);    \
            printf(__VA_ARGS__);                           \
            printf("\n");                                  \
            ++g_fail;                                      \
        }                                                  \
    } while (0)

static const gs_adamw_hparams HP = {1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 1.0f, 3};

struct Layer {
    int64_t n;
    std::vector<float> p0, m0, v0;          // initial states
    std::vector<uint16_t> g, w;
    explicit Layer(int64_t n_, unsigned seed) : n(n_), p0(n_), m0(n_), v0(n_), g(n_), w(n_, 0xdead)
    {
        srand(seed);
        for (int64_t i = 0; i < n; ++i) {
            p0[i] = (float)(rand() % 1000);
            m0[i] = (float)(rand() % 1000);
            v0[i] = (float)(rand() % 1000);
            g[i] = (uint16_t)(rand() & 0x3ff);
        }
    }
    // compares the states after `steps` applications of the stand-in
    void check(const float *p, const float *m, const float *v, int64_t lo, int64_t hi, int64_t src_off, int steps,
               const char *what) const
    {
        int64_t bad = 0;
        for (int64_t i = lo; i < hi; ++i) {
            float pe = p0[i], me = m0[i], ve = v0[i];
            for (int s = 0; s < steps; ++s) {
                pe += 1.0f;
                me *= 2.0f;
                ve += (float)g[i];
            }
            if (p[i - src_off] != pe || m[i - src_off] != me || v[i - src_off] != ve) ++bad;
        }
        CHECK(bad == 0, "%s: %lld of %lld elements wrong", what, (long long)bad, (long long)(hi - lo));
    }
    void check_w(int k, const char *what) const
    {
        int64_t bad = 0;
        for (int64_t i = 0; i < n; ++i)
            if (w[i] != (uint16_t)((i + k) & 0xffff)) ++bad;
        CHECK(bad == 0, "%s: %lld working weights wrong", what, (long long)bad);
    }
};

// chunk > 0: the staged copy-engine pipeline with that chunk size; else the in-place step
static void test_stream(int64_t n, int num_cus, int64_t chunk = 0, int slots = 0)
{
    Layer A(n, 1), B(n / 2 + 3, 2);
    gs_stream_ctx *ctx = nullptr;
    if (chunk > 0) CHECK(gs_stream_ctx_create(&ctx, chunk, slots) == GS_OK, "create staged");
    else CHECK(gs_stream_ctx_create_inplace(&ctx, num_cus) == GS_OK, "create");
    float *hp_[2][3];
    Layer *Ls[2] = {&A, &B};
    for (int l = 0; l < 2; ++l) {
        const std::vector<float> *src[3] = {&Ls[l]->p0, &Ls[l]->m0, &Ls[l]->v0};
        for (int a = 0; a < 3; ++a) {
            hp_[l][a] = (float *)gs_pinned_alloc((size_t)Ls[l]->n * 4);
            memcpy(hp_[l][a], src[a]->data(), (size_t)Ls[l]->n * 4);
        }
    }
    // the gradients are "produced" late on a stream of the caller's: the step has to wait for them
    hipStream_t producer = nullptr;
    CHECK(hipStreamCreateWithFlags(&producer, hipStreamNonBlocking) == hipSuccess, "producer stream");
    for (int step = 1; step <= 2; ++step) {
        for (int l = 0; l < 2; ++l) {
            std::vector<uint16_t> *g = &Ls[l]->g;
            std::vector<uint16_t> real = *g;
            std::fill(g->begin(), g->end(), (uint16_t)0x7777);
            hipmock_enqueue(producer, [g, real] {
                std::this_thread::sleep_for(std::chrono::milliseconds(20));
                *g = real;
            });
            const uint16_t *gt[1] = {g->data()};
            if (step == 1) {
                CHECK(gs_stream_layer_step(ctx, hp_[l][0], hp_[l][1], hp_[l][2], Ls[l]->w.data(), gt, 1, Ls[l]->n, &HP, nullptr,
                                           producer) == GS_OK, "layer step");
            } else {
                // the second step in three unaligned pieces, the last one first
                const int64_t cut[4] = {0, Ls[l]->n / 5 + 1, 3 * Ls[l]->n / 4 + 2, Ls[l]->n};
                for (int piece = 2; piece >= 0; --piece)
                    CHECK(gs_stream_layer_step_range(ctx, hp_[l][0], hp_[l][1], hp_[l][2], Ls[l]->w.data(), gt, 1, cut[piece],
                                                     cut[piece + 1], &HP, nullptr, producer) == GS_OK, "layer step range");
                CHECK(gs_stream_layer_step_range(ctx, hp_[l][0], hp_[l][1], hp_[l][2], Ls[l]->w.data(), gt, 1, 7, 7, &HP, nullptr,
                                                 producer) == GS_OK, "empty range");
                CHECK(gs_stream_layer_step_range(ctx, hp_[l][0], hp_[l][1], hp_[l][2], Ls[l]->w.data(), gt, 1, 9, 3, &HP, nullptr,
                                                 producer) == GS_ERR_INVALID_ARG, "reversed range accepted");
            }
        }
        CHECK(gs_stream_ctx_sync(ctx) == GS_OK, "sync");
        for (int l = 0; l < 2; ++l) {
            Ls[l]->check(hp_[l][0], hp_[l][1], hp_[l][2], 0, Ls[l]->n, 0, step, "host-resident");
            Ls[l]->check_w(1, "host-resident");
        }
    }
    // a host array that is not 16-byte aligned is refused in place (staged: only copies touch it)
    const uint16_t *gt[1] = {A.g.data()};
    if (chunk == 0) {
        CHECK(gs_stream_layer_step(ctx, hp_[0][0] + 1, hp_[0][1], hp_[0][2], A.w.data(), gt, 1, 16, &HP, nullptr, nullptr) ==
                  GS_ERR_INVALID_ARG, "misaligned host array accepted");
        // ... and so is pageable memory, and a range that runs past the end of a pinned array
        std::vector<float> pageable(64 + 4);
        float *pg = reinterpret_cast<float *>((reinterpret_cast<uintptr_t>(pageable.data()) + 15) & ~(uintptr_t)15);
        CHECK(gs_stream_layer_step(ctx, hp_[0][0], pg, hp_[0][2], A.w.data(), gt, 1, 16, &HP, nullptr, nullptr) ==
                  GS_ERR_INVALID_ARG, "pageable host array accepted");
        CHECK(gs_stream_layer_step(ctx, hp_[0][0], hp_[0][1], hp_[0][2], A.w.data(), gt, 1, A.n + 4096, &HP, nullptr,
                                   nullptr) == GS_ERR_INVALID_ARG, "range past the end of the pinned arrays accepted");
    }
    CHECK(gs_stream_ctx_destroy(ctx) == GS_OK, "destroy");
    CHECK(hipStreamDestroy(producer) == hipSuccess, "producer stream destroy");
    for (int l = 0; l < 2; ++l)
        for (int a = 0; a < 3; ++a) gs_pinned_free(hp_[l][a]);
}

struct Files {
    std::string path[3];
    int fd[3];
    Files(const std::string &dir, const char *tag, const Layer &L, int64_t n_host, int64_t header_bytes, int flags = O_RDWR)
    {
        const std::vector<float> *src[3] = {&L.p0, &L.m0, &L.v0};
        for (int a = 0; a < 3; ++a) {
            path[a] = dir + "/" + tag + "_" + "pmv"[a] + ".bin";
            FILE *f = fopen(path[a].c_str(), "wb");
            std::vector<char> hdr((size_t)header_bytes, (char)0x5a);
            if (!hdr.empty()) fwrite(hdr.data(), 1, hdr.size(), f);
            fwrite(src[a]->data() + n_host, 4, (size_t)(L.n - n_host), f);
            fwrite("TAIL", 1, 4, f);
            fclose(f);
            fd[a] = open(path[a].c_str(), flags);
        }
    }
    ~Files()
    {
        for (int a = 0; a < 3; ++a) {
            if (fd[a] >= 0) close(fd[a]);
            unlink(path[a].c_str());
        }
    }
    std::vector<float> load(int a, int64_t header_bytes, int64_t count, bool *frame_ok) const
    {
        std::vector<char> raw;
        FILE *f = fopen(path[a].c_str(), "rb");
        fseek(f, 0, SEEK_END);
        raw.resize((size_t)ftell(f));
        fseek(f, 0, SEEK_SET);
        size_t got = fread(raw.data(), 1, raw.size(), f);
        fclose(f);
        *frame_ok = got == (size_t)(header_bytes + count * 4 + 4);
        for (int64_t i = 0; i < header_bytes && *frame_ok; ++i) *frame_ok = raw[(size_t)i] == (char)0x5a;
        if (*frame_ok) *frame_ok = memcmp(raw.data() + header_bytes + count * 4, "TAIL", 4) == 0;
        std::vector<float> out((size_t)count);
        if (*frame_ok && count > 0) memcpy(out.data(), raw.data() + header_bytes, (size_t)count * 4);
        return out;
    }
};

static void test_tier(const std::string &dir, int64_t n, int64_t n_host, int64_t chunk, int slots)
{
    const int64_t header = 12;     // files start with bytes that must survive
    Layer A(n, 11), B(n / 3 + 5, 12);
    Layer *Ls[2] = {&A, &B};
    int64_t nh[2] = {n_host, n_host > B.n ? B.n : n_host / 2};
    gs_tier_ctx *ctx = nullptr;
    CHECK(gs_tier_ctx_create(&ctx, chunk, slots, 0) == GS_OK, "tier create");
    hipStream_t producer = nullptr;
    CHECK(hipStreamCreateWithFlags(&producer, hipStreamNonBlocking) == hipSuccess, "producer stream");
    float *host[2][3] = {{nullptr, nullptr, nullptr}, {nullptr, nullptr, nullptr}};
    Files *files[2];
    gs_tier_layer desc[2];
    for (int l = 0; l < 2; ++l) {
        const std::vector<float> *src[3] = {&Ls[l]->p0, &Ls[l]->m0, &Ls[l]->v0};
        for (int a = 0; a < 3 && nh[l] > 0; ++a) {
            host[l][a] = (float *)gs_pinned_alloc((size_t)nh[l] * 4);
            memcpy(host[l][a], src[a]->data(), (size_t)nh[l] * 4);
        }
        files[l] = new Files(dir, l ? "B" : "A", *Ls[l], nh[l], header);
        desc[l] = gs_tier_layer{host[l][0], host[l][1], host[l][2], nh[l], files[l]->fd[0], files[l]->fd[1],
                                files[l]->fd[2], header, header, header};
    }
    for (int step = 1; step <= 2; ++step) {
        for (int l = 0; l < 2; ++l) {
            const uint16_t *gt[2] = {Ls[l]->g.data(), Ls[l]->g.data()};
            if (step == 1) {
                // the call copies what it was handed: the descriptor, the pointer table and the
                // hyper-parameters may change as soon as it returns, long before the layer is read
                gs_tier_layer d = desc[l];
                gs_adamw_hparams hp = HP;
                // ... and the gradients are "produced" late on the caller's stream: the reader thread's
                // launches have to wait for the point that stream had reached at call time
                std::vector<uint16_t> *g = &Ls[l]->g;
                std::vector<uint16_t> real = *g;
                std::fill(g->begin(), g->end(), (uint16_t)0x7777);
                hipmock_enqueue(producer, [g, real] {
                    std::this_thread::sleep_for(std::chrono::milliseconds(20));
                    *g = real;
                });
                CHECK(gs_tier_layer_step(ctx, &d, Ls[l]->w.data(), gt, 2, Ls[l]->n, &hp, nullptr, producer) == GS_OK,
                      "tier layer step: %s", gs_tier_ctx_error(ctx));
                memset(&d, 0xff, sizeof d);
                memset(&hp, 0xff, sizeof hp);
                gt[0] = gt[1] = nullptr;
            } else {
                // the second step in three unaligned pieces (the cuts fall into either share, depending on n_host)
                const int64_t cut[4] = {0, Ls[l]->n / 5 + 1, 3 * Ls[l]->n / 4 + 2, Ls[l]->n};
                for (int piece = 2; piece >= 0; --piece)
                    CHECK(gs_tier_layer_step_range(ctx, &desc[l], Ls[l]->w.data(), gt, 2, Ls[l]->n, cut[piece], cut[piece + 1],
                                                   &HP, nullptr, nullptr) == GS_OK, "tier range: %s", gs_tier_ctx_error(ctx));
                CHECK(gs_tier_layer_step_range(ctx, &desc[l], Ls[l]->w.data(), gt, 2, Ls[l]->n, 5, Ls[l]->n + 1, &HP, nullptr,
                                               nullptr) == GS_ERR_INVALID_ARG, "range past the layer accepted");
            }
        }
        CHECK(gs_tier_ctx_sync(ctx) == GS_OK, "tier sync: %s", gs_tier_ctx_error(ctx));
        for (int l = 0; l < 2; ++l) {
            if (nh[l] > 0) Ls[l]->check(host[l][0], host[l][1], host[l][2], 0, nh[l], 0, step, "tier host share");
            bool ok[3];
            std::vector<float> fp = files[l]->load(0, header, Ls[l]->n - nh[l], &ok[0]);
            std::vector<float> fm = files[l]->load(1, header, Ls[l]->n - nh[l], &ok[1]);
            std::vector<float> fv = files[l]->load(2, header, Ls[l]->n - nh[l], &ok[2]);
            CHECK(ok[0] && ok[1] && ok[2], "file framing (header / length / trailer) damaged");
            if (ok[0] && ok[1] && ok[2])
                Ls[l]->check(fp.data(), fm.data(), fv.data(), nh[l], Ls[l]->n, nh[l], step, "tier file share");
            Ls[l]->check_w(2, "tier");
        }
    }
    CHECK(gs_tier_ctx_destroy(ctx) == GS_OK, "tier destroy");
    CHECK(hipStreamDestroy(producer) == hipSuccess, "producer stream destroy");
    for (int l = 0; l < 2; ++l) {
        delete files[l];
        for (int a = 0; a < 3; ++a) gs_pinned_free(host[l][a]);
    }
}

// Descriptors opened with O_DIRECT (the way a real SSD tier is read): every offset, length and
// buffer address the file tier uses must then be block-aligned, which holds when n_host, the chunk
// and the file share are multiples of 1024 elements.  Skipped where the file system refuses O_DIRECT.
static void test_tier_direct_io(const std::string &dir)
{
    const int64_t n = 64 * 1024, n_host = 16 * 1024, chunk = 8 * 1024, header = 4096;
    Layer A(n, 31);
    Files f(dir, "direct", A, n_host, header);
    int dfd[3];
    for (int a = 0; a < 3; ++a) {
        // the framing trailer makes the file length unaligned; cut it off for this case
        if (truncate(f.path[a].c_str(), header + (n - n_host) * 4) != 0) return;
        dfd[a] = open(f.path[a].c_str(), O_RDWR | O_DIRECT);
        if (dfd[a] < 0) {
            printf("O_DIRECT not available on %s: direct-I/O case skipped\n", dir.c_str());
            for (int b = 0; b < a; ++b) close(dfd[b]);
            return;
        }
    }
    float *host[3];
    const std::vector<float> *src[3] = {&A.p0, &A.m0, &A.v0};
    for (int a = 0; a < 3; ++a) {
        host[a] = (float *)gs_pinned_alloc((size_t)n_host * 4);
        memcpy(host[a], src[a]->data(), (size_t)n_host * 4);
    }
    gs_tier_ctx *ctx = nullptr;
    CHECK(gs_tier_ctx_create(&ctx, chunk, 3, 0) == GS_OK, "tier create");
    gs_tier_layer d{host[0], host[1], host[2], n_host, dfd[0], dfd[1], dfd[2], header, header, header};
    const uint16_t *gt[1] = {A.g.data()};
    CHECK(gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, n, &HP, nullptr, nullptr) == GS_OK, "direct-I/O step: %s",
          gs_tier_ctx_error(ctx));
    CHECK(gs_tier_ctx_destroy(ctx) == GS_OK, "direct-I/O destroy");
    for (int a = 0; a < 3; ++a) close(dfd[a]);
    A.check(host[0], host[1], host[2], 0, n_host, 0, 1, "direct-I/O host share");
    std::vector<float> got[3];
    for (int a = 0; a < 3; ++a) {
        got[a].resize((size_t)(n - n_host));
        FILE *fp = fopen(f.path[a].c_str(), "rb");
        fseek(fp, header, SEEK_SET);
        size_t r = fread(got[a].data(), 4, got[a].size(), fp);
        fclose(fp);
        CHECK(r == got[a].size(), "direct-I/O file length");
    }
    A.check(got[0].data(), got[1].data(), got[2].data(), n_host, n, n_host, 1, "direct-I/O file share");
    for (int a = 0; a < 3; ++a) gs_pinned_free(host[a]);
}

// The call only queues the layer: with the gradients still 300 ms away on the producer stream (so that
// no kernel can finish and no bounce slot can be handed back) it must return long before that.
static void test_tier_call_does_not_wait(const std::string &dir)
{
    Layer A(6000, 41);
    Files f(dir, "nowait", A, 0, 0);
    gs_tier_ctx *ctx = nullptr;
    CHECK(gs_tier_ctx_create(&ctx, 1024, 2, 0) == GS_OK, "tier create");
    hipStream_t producer = nullptr;
    CHECK(hipStreamCreateWithFlags(&producer, hipStreamNonBlocking) == hipSuccess, "producer stream");
    std::vector<uint16_t> *g = &A.g;
    std::vector<uint16_t> real = *g;
    std::fill(g->begin(), g->end(), (uint16_t)0x7777);
    hipmock_enqueue(producer, [g, real] {
        std::this_thread::sleep_for(std::chrono::milliseconds(300));
        *g = real;
    });
    const uint16_t *gt[1] = {g->data()};
    gs_tier_layer d{nullptr, nullptr, nullptr, 0, f.fd[0], f.fd[1], f.fd[2], 0, 0, 0};
    const auto t0 = std::chrono::steady_clock::now();
    CHECK(gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, A.n, &HP, nullptr, producer) == GS_OK, "tier layer step");
    const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    CHECK(ms < 150.0, "the call took %.1f ms: it waited for the pipeline", ms);
    CHECK(gs_tier_ctx_sync(ctx) == GS_OK, "sync: %s", gs_tier_ctx_error(ctx));
    bool ok[3];
    std::vector<float> fp = f.load(0, 0, A.n, &ok[0]), fm = f.load(1, 0, A.n, &ok[1]), fv = f.load(2, 0, A.n, &ok[2]);
    CHECK(ok[0] && ok[1] && ok[2], "file framing damaged");
    if (ok[0] && ok[1] && ok[2]) A.check(fp.data(), fm.data(), fv.data(), 0, A.n, 0, 1, "queued layer");
    A.check_w(1, "queued layer");
    CHECK(gs_tier_ctx_destroy(ctx) == GS_OK, "destroy");
    CHECK(hipStreamDestroy(producer) == hipSuccess, "producer stream destroy");
}

static void test_tier_failures(const std::string &dir)
{
    Layer A(5000, 21);
    const uint16_t *gt[1] = {A.g.data()};
    // a file shorter than the layer: the read fails, nothing hangs, the context stays failed
    {
        Layer shortL(3000, 21);
        Files f(dir, "short", shortL, 0, 0);
        gs_tier_ctx *ctx = nullptr;
        CHECK(gs_tier_ctx_create(&ctx, 1024, 2, 0) == GS_OK, "create");
        gs_tier_layer d{nullptr, nullptr, nullptr, 0, f.fd[0], f.fd[1], f.fd[2], 0, 0, 0};
        // the call only queues the layer; the reader thread meets the short read
        CHECK(gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_OK, "queueing failed");
        CHECK(gs_tier_ctx_sync(ctx) == GS_ERR_IO, "short file accepted");
        CHECK(strstr(gs_tier_ctx_error(ctx), "pread") != nullptr, "error text: '%s'", gs_tier_ctx_error(ctx));
        CHECK(gs_tier_ctx_sync(ctx) == GS_ERR_IO, "sync after failure");
        CHECK(gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, 10, &HP, nullptr, nullptr) == GS_ERR_IO, "failed context reused");
        CHECK(gs_tier_ctx_destroy(ctx) == GS_ERR_IO, "destroy after failure");
    }
    // descriptors that cannot be written: the writer thread reports it through sync
    {
        Files f(dir, "ro", A, 0, 0, O_RDONLY);
        gs_tier_ctx *ctx = nullptr;
        CHECK(gs_tier_ctx_create(&ctx, 1024, 2, 0) == GS_OK, "create");
        gs_tier_layer d{nullptr, nullptr, nullptr, 0, f.fd[0], f.fd[1], f.fd[2], 0, 0, 0};
        gs_status st = gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr);
        CHECK(st == GS_OK || st == GS_ERR_IO, "unexpected status %d", (int)st);
        CHECK(gs_tier_ctx_sync(ctx) == GS_ERR_IO, "write failure not reported");
        CHECK(strstr(gs_tier_ctx_error(ctx), "pwrite") != nullptr, "error text: '%s'", gs_tier_ctx_error(ctx));
        CHECK(gs_tier_ctx_destroy(ctx) == GS_ERR_IO, "destroy after failure");
    }
    // argument checks that need a live context
    {
        Files f(dir, "args", A, 0, 0);
        gs_tier_ctx *ctx = nullptr;
        CHECK(gs_tier_ctx_create(&ctx, 1024, 2, 0) == GS_OK, "create");
        gs_tier_layer d{nullptr, nullptr, nullptr, 0, f.fd[0], f.fd[1], f.fd[2], 0, 0, 0};
        gs_tier_layer bad = d;
        bad.n_host = A.n + 1;
        CHECK(gs_tier_layer_step(ctx, &bad, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_ERR_INVALID_ARG, "n_host > n");
        bad = d;
        bad.n_host = 10;   // host share without host pointers
        CHECK(gs_tier_layer_step(ctx, &bad, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_ERR_INVALID_ARG, "null host");
        bad = d;
        bad.fd_m = -1;
        CHECK(gs_tier_layer_step(ctx, &bad, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_ERR_INVALID_ARG, "bad fd");
        bad = d;
        bad.off_v = -4;
        CHECK(gs_tier_layer_step(ctx, &bad, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_ERR_INVALID_ARG, "bad offset");
        CHECK(gs_tier_layer_step(ctx, &d, A.w.data(), gt, 0, A.n, &HP, nullptr, nullptr) == GS_ERR_INVALID_ARG, "k = 0");
        CHECK(gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, 0, &HP, nullptr, nullptr) == GS_OK, "n = 0");
        CHECK(gs_tier_ctx_sync(ctx) == GS_OK, "sync of an idle context");
        CHECK(gs_tier_ctx_destroy(ctx) == GS_OK, "destroy");
    }
}

// HIP calls that fail in the middle of a layer: the status comes back (from the call, or from sync
// for work done on the context's own threads), nothing hangs, everything can still be destroyed.
static void test_hip_failures(const std::string &dir)
{
    Layer A(5000, 31);
    const uint16_t *gt[1] = {A.g.data()};
    float *h[3];
    const std::vector<float> *src[3] = {&A.p0, &A.m0, &A.v0};
    for (int a = 0; a < 3; ++a) {
        h[a] = (float *)gs_pinned_alloc((size_t)A.n * 4);
        memcpy(h[a], src[a]->data(), (size_t)A.n * 4);
    }
    // staged pipeline: a copy in the middle of the layer fails
    {
        gs_stream_ctx *ctx = nullptr;
        CHECK(gs_stream_ctx_create(&ctx, 1000, 2) == GS_OK, "create staged");
        hipmock_fail_nth("hipMemcpyAsync", 8);
        CHECK(gs_stream_layer_step(ctx, h[0], h[1], h[2], A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_ERR_HIP,
              "failed copy not reported");
        hipmock_fail_nth(nullptr, 0);
        CHECK(strstr(gs_last_hip_error(), "hipMemcpyAsync") != nullptr, "error text: '%s'", gs_last_hip_error());
        CHECK(gs_stream_ctx_sync(ctx) == GS_OK, "sync after a failed enqueue");
        CHECK(gs_stream_ctx_destroy(ctx) == GS_OK, "destroy after a failed enqueue");
    }
    // in place: the launch itself fails
    {
        gs_stream_ctx *ctx = nullptr;
        CHECK(gs_stream_ctx_create_inplace(&ctx, 0) == GS_OK, "create in place");
        gs::g_launch_fault.store(1);
        CHECK(gs_stream_layer_step(ctx, h[0], h[1], h[2], A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_ERR_HIP,
              "failed launch not reported");
        gs::g_launch_fault.store(0);
        CHECK(gs_stream_ctx_destroy(ctx) == GS_OK, "destroy after a failed launch");
    }
    // file tier: each of these fails on the reader thread, after the call has returned
    struct Case {
        const char *api;   // nullptr: the kernel launch
        int nth;
        int64_t n_host;
    };
    const Case cases[] = {{"hipLaunchHostFunc", 2, 0}, {"hipStreamWaitEvent", 1, 0}, {"hipStreamWaitEvent", 3, 0},
                          {"hipEventRecord", 3, 0},    {nullptr, 1, 2048},           {nullptr, 3, 0}};
    for (const Case &cs : cases) {
        Files f(dir, "hipfail", A, cs.n_host, 0);
        gs_tier_ctx *ctx = nullptr;
        CHECK(gs_tier_ctx_create(&ctx, 1024, 2, 0) == GS_OK, "tier create");
        gs_tier_layer d{h[0], h[1], h[2], cs.n_host, f.fd[0], f.fd[1], f.fd[2], 0, 0, 0};
        // armed after the call's own event record, so that the failure falls on the reader thread
        gs_status st = GS_OK;
        if (cs.api && strcmp(cs.api, "hipEventRecord") == 0) {
            hipmock_fail_nth(cs.api, cs.nth);      // 1st record: the call's; later ones: the reader's per chunk
            st = gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr);
        } else {
            if (cs.api) hipmock_fail_nth(cs.api, cs.nth);
            else gs::g_launch_fault.store(cs.nth);
            st = gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr);
        }
        CHECK(st == GS_OK, "queueing failed (%s #%d)", cs.api ? cs.api : "launch", cs.nth);
        CHECK(gs_tier_ctx_sync(ctx) == GS_ERR_HIP, "%s #%d failing on the reader thread was not reported", cs.api ? cs.api : "launch", cs.nth);
        hipmock_fail_nth(nullptr, 0);
        gs::g_launch_fault.store(0);
        // the text names what failed and carries the runtime's own message
        CHECK(strstr(gs_tier_ctx_error(ctx), "mock error") != nullptr, "error text: '%s'", gs_tier_ctx_error(ctx));
        CHECK(gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_ERR_HIP, "failed context reused");
        CHECK(gs_tier_ctx_destroy(ctx) == GS_ERR_HIP, "destroy after failure");
    }
    // the call's own event record fails: reported by the call, the context stays usable
    {
        Files f(dir, "hipfail2", A, 0, 0);
        gs_tier_ctx *ctx = nullptr;
        CHECK(gs_tier_ctx_create(&ctx, 1024, 2, 0) == GS_OK, "tier create");
        gs_tier_layer d{nullptr, nullptr, nullptr, 0, f.fd[0], f.fd[1], f.fd[2], 0, 0, 0};
        hipmock_fail_nth("hipEventRecord", 1);
        CHECK(gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_ERR_HIP, "failed record not reported");
        hipmock_fail_nth(nullptr, 0);
        CHECK(gs_tier_layer_step(ctx, &d, A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_OK, "context unusable after a rejected call");
        CHECK(gs_tier_ctx_sync(ctx) == GS_OK, "sync: %s", gs_tier_ctx_error(ctx));
        bool ok[3];
        std::vector<float> fp = f.load(0, 0, A.n, &ok[0]), fm = f.load(1, 0, A.n, &ok[1]), fv = f.load(2, 0, A.n, &ok[2]);
        if (ok[0] && ok[1] && ok[2]) A.check(fp.data(), fm.data(), fv.data(), 0, A.n, 0, 1, "after a rejected call");
        CHECK(gs_tier_ctx_destroy(ctx) == GS_OK, "destroy");
    }
    for (int a = 0; a < 3; ++a) gs_pinned_free(h[a]);
}

// The staged context's creation-time check that its three streams run side by side, driven by scripted
// clock readings: a pair that takes turns has its colliding stream swapped for a fresh one (and the
// rejected stream destroyed), a context whose streams never get apart still works and says so.
static void test_stream_check(bool ever_apart)
{
    const int before = hipmock_live_streams();
    std::vector<float> script;
    auto pair = [&](bool apart) { script.push_back(2.0f); script.push_back(apart ? 0.1f : 1.9f); };
    if (ever_apart) {
        pair(true); pair(false); pair(true);      // attempt 1: upload/compute collide -> the compute stream is swapped
        pair(false); pair(true); pair(true);      // attempt 2: upload/download collide -> the download stream is swapped
        pair(true); pair(true); pair(true);       // attempt 3: all three side by side
    } else {
        for (int i = 0; i < 40; ++i) pair(false);
    }
    hipmock_script_elapsed_ms(script.data(), (int)script.size());
    gs_stream_ctx *ctx = nullptr;
    CHECK(gs_stream_ctx_create(&ctx, 200000, 2) == GS_OK, "create staged (stream check)");
    hipmock_script_elapsed_ms(nullptr, 0);
    CHECK(gs_stream_ctx_copies_overlap(ctx) == (ever_apart ? 1 : 0), "copies_overlap = %d", gs_stream_ctx_copies_overlap(ctx));
    CHECK(hipmock_live_streams() == before + 3, "%d streams alive beside the context's three", hipmock_live_streams() - before - 3);
    Layer A(300000, 7);
    float *h[3];
    const std::vector<float> *src[3] = {&A.p0, &A.m0, &A.v0};
    for (int a = 0; a < 3; ++a) {
        h[a] = (float *)gs_pinned_alloc((size_t)A.n * 4);
        memcpy(h[a], src[a]->data(), (size_t)A.n * 4);
    }
    const uint16_t *gt[1] = {A.g.data()};
    CHECK(gs_stream_layer_step(ctx, h[0], h[1], h[2], A.w.data(), gt, 1, A.n, &HP, nullptr, nullptr) == GS_OK, "step");
    CHECK(gs_stream_ctx_sync(ctx) == GS_OK, "sync");
    A.check(h[0], h[1], h[2], 0, A.n, 0, 1, "after the stream check");
    A.check_w(1, "after the stream check");
    CHECK(gs_stream_ctx_destroy(ctx) == GS_OK, "destroy");
    CHECK(hipmock_live_streams() == before, "streams leaked: %d", hipmock_live_streams() - before);
    for (int a = 0; a < 3; ++a) gs_pinned_free(h[a]);
    CHECK(gs_stream_ctx_copies_overlap(nullptr) == -1, "copies_overlap(NULL)");
}

// The deferred part of each layer's step with its deadline: the immediate part [0,s) runs on the
// caller's stream, the deferred part [s,n) on the context's stream behind late-produced gradients,
// and a consumer stream (the layer's "forward") that waited for the layer must find every element of
// the layer stepped exactly once.
static void test_defer(int layers, int64_t n, int num_cus)
{
    gs_defer_ctx *ctx = nullptr;
    CHECK(gs_defer_ctx_create(&ctx, layers, num_cus) == GS_OK, "defer create");
    hipStream_t mainstream = nullptr, fwd = nullptr;
    CHECK(hipStreamCreateWithFlags(&mainstream, hipStreamNonBlocking) == hipSuccess, "main stream");
    CHECK(hipStreamCreateWithFlags(&fwd, hipStreamNonBlocking) == hipSuccess, "forward stream");
    std::vector<Layer *> Ls;
    std::vector<std::vector<float>> P, M, V;
    std::vector<std::atomic<int>> bad_seen(layers);
    const int64_t s = n * 2 / 5 + 3;
    for (int l = 0; l < layers; ++l) {
        Ls.push_back(new Layer(n, 100 + l));
        P.push_back(Ls[l]->p0); M.push_back(Ls[l]->m0); V.push_back(Ls[l]->v0);
        bad_seen[l].store(-1);
    }
    CHECK(gs_defer_layer_done(ctx, 0) == 1 && gs_defer_layer_done(ctx, layers) == -1, "done before any step");
    CHECK(gs_defer_wait_layer(ctx, 1, fwd) == GS_OK, "wait on a layer with nothing deferred");
    for (int l = 0; l < layers; ++l) {
        std::vector<uint16_t> *g = &Ls[l]->g;
        std::vector<uint16_t> real = *g;
        std::fill(g->begin(), g->end(), (uint16_t)0x7777);
        hipmock_enqueue(mainstream, [g, real] {
            std::this_thread::sleep_for(std::chrono::milliseconds(15));
            *g = real;
        });
        const uint16_t *gt[1] = {g->data()};
        CHECK(gs_accum_adamw(P[l].data(), M[l].data(), V[l].data(), Ls[l]->w.data(), gt, 1, 0, s, &HP, nullptr, mainstream) == GS_OK,
              "immediate part");
        CHECK(gs_defer_layer_step(ctx, l, P[l].data(), M[l].data(), V[l].data(), Ls[l]->w.data(), gt, 1, s, n, &HP, nullptr,
                                  mainstream) == GS_OK, "deferred part");
    }
    // the forward of layer l: waits for the immediate part (an event on the caller's stream) and for the
    // layer's deadline, then looks at the whole layer.  Last layer first: its deferred step is the last to
    // finish, so a deadline tied to the wrong layer's event lets this forward run early.
    for (int l = layers - 1; l >= 0; --l) {
        hipEvent_t imm = nullptr;
        CHECK(hipEventCreateWithFlags(&imm, hipEventDisableTiming) == hipSuccess, "event");
        CHECK(hipEventRecord(imm, mainstream) == hipSuccess && hipStreamWaitEvent(fwd, imm, 0) == hipSuccess, "immediate done");
        CHECK(gs_defer_wait_layer(ctx, l, fwd) == GS_OK, "deadline");
        Layer *L = Ls[l];
        const float *p = P[l].data(), *m = M[l].data(), *v = V[l].data();
        std::atomic<int> *out = &bad_seen[l];
        hipmock_enqueue(fwd, [L, p, m, v, out, n] {
            int bad = 0;
            for (int64_t i = 0; i < n; ++i) {
                if (p[i] != L->p0[i] + 1.0f || m[i] != L->m0[i] * 2.0f || v[i] != L->v0[i] + (float)L->g[i]) ++bad;
                if (L->w[i] != (uint16_t)((i + 1) & 0xffff)) ++bad;
            }
            out->store(bad);
        });
        CHECK(hipStreamSynchronize(fwd) == hipSuccess, "forward sync");
        CHECK(hipEventDestroy(imm) == hipSuccess, "event destroy");
        CHECK(bad_seen[l].load() == 0, "forward of layer %d saw %d elements not stepped exactly once", l, bad_seen[l].load());
    }
    CHECK(gs_defer_ctx_sync(ctx) == GS_OK, "defer sync");
    for (int l = 0; l < layers; ++l) CHECK(gs_defer_layer_done(ctx, l) == 1, "layer %d done after sync", l);
    CHECK(gs_defer_layer_step(ctx, layers, P[0].data(), M[0].data(), V[0].data(), Ls[0]->w.data(), nullptr, 1, 0, 1, &HP, nullptr,
                              mainstream) == GS_ERR_INVALID_ARG, "layer out of range");
    CHECK(gs_defer_ctx_destroy(ctx) == GS_OK, "defer destroy");
    CHECK(hipStreamDestroy(mainstream) == hipSuccess && hipStreamDestroy(fwd) == hipSuccess, "streams");
    for (Layer *L : Ls) delete L;
}

int main(int argc, char **argv)
{
    if (argc < 2) {
        printf("usage: %s <scratch dir>\n", argv[0]);
        return 2;
    }
    const std::string dir = argv[1];
    hipmock_set_copy_delay_us(50);
    test_stream(20000, 0);
    test_stream(777, 16);
    test_stream(20000, 0, 4096, 2);
    test_stream(20000, 0, 3001, 3);
    test_stream(777, 0, 100000, 2);
    test_tier(dir, 30000, 0, 4096, 2);
    test_tier(dir, 30000, 9999, 3001, 3);
    test_tier(dir, 30000, 30000, 4096, 2);
    test_tier(dir, 5000, 1, 100000, 2);
    test_tier(dir, 30000, 29999, 1024, 4);
    test_tier_direct_io(dir);
    test_tier_call_does_not_wait(dir);
    test_tier_failures(dir);
    test_hip_failures(dir);
    test_stream_check(true);
    test_stream_check(false);
    test_defer(4, 5000, 0);
    test_defer(3, 777, 64);
    printf(g_fail ? "FAILED (%d)\n" : "PIPELINE OK\n", g_fail);
    return g_fail ? 1 : 0;
}
