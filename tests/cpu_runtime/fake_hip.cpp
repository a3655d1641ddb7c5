// CPU stand-in for the HIP runtime -- TEST INFRASTRUCTURE ONLY (see hip/hip_runtime.h).
#include <hip/hip_runtime.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <mutex>
#include <random>
#include <set>
#include <thread>

struct FakeStream {
    std::mutex mu;
    std::condition_variable cv_work, cv_idle;
    std::deque<FakeTask> q;
    bool busy = false, stop = false, capturing = false;
    std::vector<FakeTask> recorded;
    std::thread worker;
};

struct FakeEvent {
    std::mutex mu;
    std::condition_variable cv;
    uint64_t recorded = 0, done = 0;        // generations: the event is complete when done == recorded
};

namespace {

std::atomic<unsigned> g_jitter_us{0};
std::mutex g_reg_mu;
std::set<FakeStream *> g_streams;
FakeStream *g_default = nullptr;

void worker_loop(FakeStream *s)
{
    std::minstd_rand rng((unsigned)(uintptr_t)s);
    for (;;) {
        FakeTask t;
        {
            std::unique_lock<std::mutex> lk(s->mu);
            s->cv_work.wait(lk, [&] { return s->stop || !s->q.empty(); });
            if (s->q.empty()) return;
            t = std::move(s->q.front());
            s->q.pop_front();
            s->busy = true;
        }
        const unsigned j = g_jitter_us.load(std::memory_order_relaxed);
        if (j) std::this_thread::sleep_for(std::chrono::microseconds(rng() % (j + 1)));
        t();
        {
            std::lock_guard<std::mutex> lk(s->mu);
            s->busy = false;
            if (s->q.empty()) s->cv_idle.notify_all();
        }
    }
}

FakeStream *make_stream()
{
    FakeStream *s = new FakeStream;
    s->worker = std::thread(worker_loop, s);
    std::lock_guard<std::mutex> lk(g_reg_mu);
    g_streams.insert(s);
    return s;
}

FakeStream *resolve(hipStream_t s)
{
    if (s) return s;
    std::lock_guard<std::mutex> lk(g_reg_mu);
    if (!g_default) {
        g_default = new FakeStream;
        g_default->worker = std::thread(worker_loop, g_default);
        g_streams.insert(g_default);
    }
    return g_default;
}

void sync_stream(FakeStream *s)
{
    std::unique_lock<std::mutex> lk(s->mu);
    s->cv_idle.wait(lk, [&] { return s->q.empty() && !s->busy; });
}

}  // namespace

void fake_enqueue(hipStream_t hs, FakeTask task)
{
    FakeStream *s = resolve(hs);
    std::lock_guard<std::mutex> lk(s->mu);
    if (s->capturing) { s->recorded.push_back(std::move(task)); return; }
    s->q.push_back(std::move(task));
    s->cv_work.notify_one();
}

void fake_begin_capture(hipStream_t hs)
{
    FakeStream *s = resolve(hs);
    std::lock_guard<std::mutex> lk(s->mu);
    s->capturing = true;
    s->recorded.clear();
}

std::vector<FakeTask> fake_end_capture(hipStream_t hs)
{
    FakeStream *s = resolve(hs);
    std::lock_guard<std::mutex> lk(s->mu);
    s->capturing = false;
    return std::move(s->recorded);
}

void fake_graph_launch(const std::vector<FakeTask> &graph, hipStream_t s)
{
    for (const FakeTask &t : graph) fake_enqueue(s, t);
}

void fake_set_jitter_us(unsigned max_us) { g_jitter_us.store(max_us); }

const char *hipGetErrorString(hipError_t e)
{
    switch (e) {
    case hipSuccess: return "success";
    case hipErrorNotReady: return "not ready";
    case hipErrorOutOfMemory: return "out of memory";
    default: return "invalid value";
    }
}
hipError_t hipGetDeviceCount(int *n) { *n = 1; return hipSuccess; }
hipError_t hipSetDevice(int dev) { return dev == 0 ? hipSuccess : hipErrorInvalidValue; }
hipError_t hipDeviceSynchronize()
{
    std::vector<FakeStream *> all;
    {
        std::lock_guard<std::mutex> lk(g_reg_mu);
        all.assign(g_streams.begin(), g_streams.end());
    }
    for (FakeStream *s : all) sync_stream(s);
    return hipSuccess;
}
hipError_t hipMalloc(void **p, size_t n)
{
    *p = std::aligned_alloc(256, (n + 255) / 256 * 256);
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipHostMalloc(void **p, size_t n, unsigned) { return hipMalloc(p, n); }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipHostGetDevicePointer(void **dev, void *host, unsigned) { *dev = host; return hipSuccess; }
hipError_t hipMemcpy(void *dst, const void *src, size_t n, hipMemcpyKind)
{
    (void)hipDeviceSynchronize();
    std::memcpy(dst, src, n);
    return hipSuccess;
}
hipError_t hipMemcpyAsync(void *dst, const void *src, size_t n, hipMemcpyKind, hipStream_t s)
{
    fake_enqueue(s, [=] { std::memcpy(dst, src, n); });
    return hipSuccess;
}
hipError_t hipMemsetAsync(void *dst, int value, size_t n, hipStream_t s)
{
    fake_enqueue(s, [=] { std::memset(dst, value, n); });
    return hipSuccess;
}
hipError_t hipStreamCreate(hipStream_t *s) { *s = make_stream(); return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned) { *s = make_stream(); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s)
{
    if (!s) return hipErrorInvalidValue;
    sync_stream(s);
    {
        std::lock_guard<std::mutex> lk(s->mu);
        s->stop = true;
        s->cv_work.notify_all();
    }
    s->worker.join();
    {
        std::lock_guard<std::mutex> lk(g_reg_mu);
        g_streams.erase(s);
    }
    delete s;
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t s) { sync_stream(resolve(s)); return hipSuccess; }
hipError_t hipStreamQuery(hipStream_t hs)
{
    FakeStream *s = resolve(hs);
    std::lock_guard<std::mutex> lk(s->mu);
    return s->q.empty() && !s->busy ? hipSuccess : hipErrorNotReady;
}
hipError_t hipStreamIsCapturing(hipStream_t hs, hipStreamCaptureStatus *status)
{
    FakeStream *s = resolve(hs);
    std::lock_guard<std::mutex> lk(s->mu);
    *status = s->capturing ? hipStreamCaptureStatusActive : hipStreamCaptureStatusNone;
    return hipSuccess;
}
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = new FakeEvent; return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { delete e; return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s)
{
    uint64_t gen;
    {
        std::lock_guard<std::mutex> lk(e->mu);
        gen = ++e->recorded;
    }
    fake_enqueue(s, [e, gen] {
        std::lock_guard<std::mutex> lk(e->mu);
        if (e->done < gen) e->done = gen;
        e->cv.notify_all();
    });
    return hipSuccess;
}
hipError_t hipEventQuery(hipEvent_t e)
{
    std::lock_guard<std::mutex> lk(e->mu);
    return e->done == e->recorded ? hipSuccess : hipErrorNotReady;
}
hipError_t hipEventSynchronize(hipEvent_t e)
{
    std::unique_lock<std::mutex> lk(e->mu);
    e->cv.wait(lk, [&] { return e->done == e->recorded; });
    return hipSuccess;
}
