// Implementation of the host-only HIP stand-in (see hip/hip_runtime_api.h in this folder).
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <map>
#include <memory>
#include <mutex>
#include <set>
#include <string>
#include <thread>
#include <vector>

struct hipmock_stream {
    std::mutex mu;
    std::condition_variable cv;
    std::deque<std::function<void()>> q;
    bool running = false, stop = false;
    std::thread th;

    hipmock_stream() : th([this] { loop(); }) {}
    ~hipmock_stream()
    {
        {
            std::lock_guard<std::mutex> g(mu);
            stop = true;
        }
        cv.notify_all();
        th.join();
    }
    void loop()
    {
        for (;;) {
            std::function<void()> fn;
            {
                std::unique_lock<std::mutex> lk(mu);
                cv.wait(lk, [&] { return stop || !q.empty(); });
                if (q.empty()) return;
                fn = std::move(q.front());
                q.pop_front();
                running = true;
            }
            fn();
            {
                std::lock_guard<std::mutex> g(mu);
                running = false;
            }
            cv.notify_all();
        }
    }
    void push(std::function<void()> fn)
    {
        {
            std::lock_guard<std::mutex> g(mu);
            q.push_back(std::move(fn));
        }
        cv.notify_all();
    }
    void drain()
    {
        std::unique_lock<std::mutex> lk(mu);
        cv.wait(lk, [&] { return q.empty() && !running; });
    }
};

struct hipmock_event {
    std::mutex mu;
    std::condition_variable cv;
    uint64_t recorded = 0, completed = 0;
    void wait_for(uint64_t target)
    {
        std::unique_lock<std::mutex> lk(mu);
        cv.wait(lk, [&] { return completed >= target; });
    }
};

static std::atomic<uint64_t> g_copies{0};
static std::atomic<int> g_delay_us{0};

// Planted failure: the nth call (counted from the moment it is armed) of one API returns an error
// and does nothing else.
static std::mutex g_fault_mu;
static std::string g_fault_api;
static int g_fault_countdown = 0;
static bool fault_now(const char *api)
{
    std::lock_guard<std::mutex> g(g_fault_mu);
    if (g_fault_countdown <= 0 || g_fault_api != api) return false;
    return --g_fault_countdown == 0;
}

// ---- legacy null-stream semantics (HIPMOCK_LEGACY_NULL=1 in the environment) --------------------
// As in HIP's default ("legacy") mode: the null stream is a queue of its own; work enqueued on it
// starts only after everything enqueued earlier on every BLOCKING stream (one created without
// hipStreamNonBlocking, or by hipExtStreamCreateWithCUMask) has finished, and work enqueued on a
// blocking stream starts only after everything enqueued earlier on the null stream.  Non-blocking
// streams take no part.  Without the variable the null stream runs its work in place, at the call.
struct hipmock_token {
    std::mutex mu;
    std::condition_variable cv;
    bool done = false;
    void set()
    {
        {
            std::lock_guard<std::mutex> g(mu);
            done = true;
        }
        cv.notify_all();
    }
    void wait()
    {
        std::unique_lock<std::mutex> lk(mu);
        cv.wait(lk, [&] { return done; });
    }
};

static bool legacy_null()
{
    static const bool on = getenv("HIPMOCK_LEGACY_NULL") != nullptr;
    return on;
}
static std::mutex g_streams_mu;
static std::set<hipmock_stream *> g_all_streams, g_blocking_streams;
static hipmock_stream *null_stream()
{
    static hipmock_stream *n = new hipmock_stream();   // lives until the process ends
    return n;
}

void hipmock_enqueue(hipStream_t s, std::function<void()> fn)
{
    if (!legacy_null()) {
        if (!s) {
            fn();   // the null stream runs in place
            return;
        }
        s->push(std::move(fn));
        return;
    }
    if (!s) {
        std::vector<std::shared_ptr<hipmock_token>> toks;
        {
            std::lock_guard<std::mutex> g(g_streams_mu);
            for (hipmock_stream *b : g_blocking_streams) {
                auto t = std::make_shared<hipmock_token>();
                b->push([t] { t->set(); });
                toks.push_back(t);
            }
        }
        null_stream()->push([toks, fn] {
            for (auto &t : toks) t->wait();
            fn();
        });
        return;
    }
    bool blocking;
    {
        std::lock_guard<std::mutex> g(g_streams_mu);
        blocking = g_blocking_streams.count(s) != 0;
    }
    if (!blocking) {
        s->push(std::move(fn));
        return;
    }
    auto t = std::make_shared<hipmock_token>();
    null_stream()->push([t] { t->set(); });
    s->push([t, fn] {
        t->wait();
        fn();
    });
}

extern "C" {

uint64_t hipmock_copy_count(void) { return g_copies.load(); }
void hipmock_set_copy_delay_us(int us) { g_delay_us.store(us); }
void hipmock_fail_nth(const char *api, int nth)
{
    std::lock_guard<std::mutex> g(g_fault_mu);
    g_fault_api = api ? api : "";
    g_fault_countdown = api ? nth : 0;
}

const char *hipGetErrorString(hipError_t e) { return e == hipSuccess ? "no error" : "mock error"; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipDeviceGetAttribute(int *value, hipDeviceAttribute_t, int) { *value = 256; return hipSuccess; }

// live allocations: base -> (bytes, type)
static std::mutex g_alloc_mu;
static std::map<uintptr_t, std::pair<size_t, hipMemoryType>> g_allocs;

static void remember(void *p, size_t bytes, hipMemoryType t)
{
    std::lock_guard<std::mutex> g(g_alloc_mu);
    g_allocs[reinterpret_cast<uintptr_t>(p)] = {bytes, t};
}
static void forget(void *p)
{
    std::lock_guard<std::mutex> g(g_alloc_mu);
    g_allocs.erase(reinterpret_cast<uintptr_t>(p));
}

hipError_t hipMalloc(void **ptr, size_t bytes)
{
    *ptr = aligned_alloc(256, (bytes + 255) / 256 * 256);
    if (*ptr) remember(*ptr, bytes, hipMemoryTypeDevice);
    return *ptr ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void *ptr) { forget(ptr); free(ptr); return hipSuccess; }
hipError_t hipHostMalloc(void **ptr, size_t bytes, unsigned)
{
    *ptr = aligned_alloc(4096, (bytes + 4095) / 4096 * 4096);
    if (*ptr) remember(*ptr, bytes, hipMemoryTypeHost);
    return *ptr ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipHostFree(void *ptr) { forget(ptr); free(ptr); return hipSuccess; }

hipError_t hipPointerGetAttributes(hipPointerAttribute_t *attr, const void *ptr)
{
    std::lock_guard<std::mutex> g(g_alloc_mu);
    const uintptr_t a = reinterpret_cast<uintptr_t>(ptr);
    memset(attr, 0, sizeof *attr);
    attr->device = -2;
    auto it = g_allocs.upper_bound(a);
    if (it != g_allocs.begin()) {
        --it;
        if (a < it->first + it->second.first) {
            attr->type = it->second.second;
            attr->device = 0;
            attr->devicePointer = const_cast<void *>(ptr);
            if (attr->type == hipMemoryTypeHost) attr->hostPointer = const_cast<void *>(ptr);
        }
    }
    return hipSuccess;
}

static hipmock_stream *new_stream(bool blocking)
{
    hipmock_stream *s = new hipmock_stream();
    std::lock_guard<std::mutex> g(g_streams_mu);
    g_all_streams.insert(s);
    if (blocking) g_blocking_streams.insert(s);
    return s;
}
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned flags)
{
    *s = new_stream(!(flags & hipStreamNonBlocking));
    return hipSuccess;
}
// a CU-masked stream is a blocking stream, as in HIP (the call takes no flags)
hipError_t hipExtStreamCreateWithCUMask(hipStream_t *s, uint32_t, const uint32_t *) { *s = new_stream(true); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s)
{
    s->drain();
    {
        std::lock_guard<std::mutex> g(g_streams_mu);
        g_all_streams.erase(s);
        g_blocking_streams.erase(s);
    }
    delete s;
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t s)
{
    if (s) {
        s->drain();
    } else if (legacy_null()) {
        hipmock_enqueue(nullptr, [] {});
        null_stream()->drain();
    }
    return hipSuccess;
}
hipError_t hipDeviceSynchronize(void)
{
    for (int pass = 0; pass < 2; ++pass) {
        std::vector<hipmock_stream *> all;
        {
            std::lock_guard<std::mutex> g(g_streams_mu);
            all.assign(g_all_streams.begin(), g_all_streams.end());
        }
        for (hipmock_stream *s : all) s->drain();
        if (legacy_null()) null_stream()->drain();
    }
    return hipSuccess;
}
hipError_t hipMemset(void *dst, int value, size_t bytes)
{
    hipmock_enqueue(nullptr, [=] { memset(dst, value, bytes); });
    if (legacy_null()) null_stream()->drain();
    return hipSuccess;
}
hipError_t hipMemcpy(void *dst, const void *src, size_t bytes, hipMemcpyKind)
{
    // synchronous copy on the null stream
    hipmock_enqueue(nullptr, [=] { memcpy(dst, src, bytes); });
    if (legacy_null()) null_stream()->drain();
    return hipSuccess;
}

hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = new hipmock_event(); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e)
{
    {
        std::lock_guard<std::mutex> g(e->mu);   // let a completing record leave the lock first
    }
    delete e;
    return hipSuccess;
}

hipError_t hipEventRecord(hipEvent_t e, hipStream_t s)
{
    if (fault_now("hipEventRecord")) return hipErrorUnknown;
    uint64_t seq;
    {
        std::lock_guard<std::mutex> g(e->mu);
        seq = ++e->recorded;
    }
    hipmock_enqueue(s, [e, seq] {
        // notified under the lock: once a waiter has seen the completion, this task no longer
        // touches the event, so the event may be destroyed (as HIP allows after completion)
        std::lock_guard<std::mutex> g(e->mu);
        if (e->completed < seq) e->completed = seq;
        e->cv.notify_all();
    });
    return hipSuccess;
}

hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned)
{
    if (fault_now("hipStreamWaitEvent")) return hipErrorUnknown;
    uint64_t target;
    {
        std::lock_guard<std::mutex> g(e->mu);
        target = e->recorded;   // the record that is current NOW, as HIP defines it
    }
    hipmock_enqueue(s, [e, target] { e->wait_for(target); });
    return hipSuccess;
}

hipError_t hipEventQuery(hipEvent_t e)
{
    std::lock_guard<std::mutex> g(e->mu);
    return e->completed >= e->recorded ? hipSuccess : hipErrorNotReady;
}

// The stand-in keeps no clock: an interval reads as zero ("too short to tell") unless a test has
// scripted the next readings with hipmock_script_elapsed_ms.
static std::mutex g_elapsed_mu;
static std::deque<float> g_elapsed_script;
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t)
{
    std::lock_guard<std::mutex> g(g_elapsed_mu);
    if (g_elapsed_script.empty()) {
        *ms = 0.0f;
    } else {
        *ms = g_elapsed_script.front();
        g_elapsed_script.pop_front();
    }
    return hipSuccess;
}
void hipmock_script_elapsed_ms(const float *values, int count)
{
    std::lock_guard<std::mutex> g(g_elapsed_mu);
    g_elapsed_script.assign(values, values + count);
}
int hipmock_live_streams(void)
{
    std::lock_guard<std::mutex> g(g_streams_mu);
    return (int)g_all_streams.size();
}

hipError_t hipEventSynchronize(hipEvent_t e)
{
    uint64_t target;
    {
        std::lock_guard<std::mutex> g(e->mu);
        target = e->recorded;
    }
    e->wait_for(target);
    return hipSuccess;
}

hipError_t hipLaunchHostFunc(hipStream_t s, hipHostFn_t fn, void *userData)
{
    if (fault_now("hipLaunchHostFunc")) return hipErrorUnknown;
    hipmock_enqueue(s, [fn, userData] { fn(userData); });
    return hipSuccess;
}

hipError_t hipMemcpyAsync(void *dst, const void *src, size_t bytes, hipMemcpyKind, hipStream_t s)
{
    if (fault_now("hipMemcpyAsync")) return hipErrorUnknown;
    hipmock_enqueue(s, [=] {
        int d = g_delay_us.load();
        if (d > 0) std::this_thread::sleep_for(std::chrono::microseconds(d));
        memcpy(dst, src, bytes);
        g_copies.fetch_add(1);
    });
    return hipSuccess;
}

}  // extern "C"
