// CPU stand-in for the HIP runtime calls of libsaga's host code (see hip/hip_runtime.h).
//
// Streams are queues of deferred operations. An event remembers the stream it was last recorded on and how
// many operations had been enqueued there; a wait enqueued on another stream blocks that stream until the
// recorded one has executed that many. Nothing runs concurrently: "when" an operation runs is a choice among
// the orders the API allows, made by the mode (eager, lazy, seeded random). A missing wait between two
// streams therefore shows up as stale data or as a use of freed memory under one of the orders, where the
// GPU would show it once in thousands of runs.
//
// Misuse that the real runtime answers with undefined behaviour aborts here with a message: a destroyed
// stream or event handed back to the API, a free of an unknown pointer, a wait cycle.
#include <hip/hip_runtime.h>

#if defined(__SANITIZE_ADDRESS__)
#include <sanitizer/asan_interface.h>
#define STUB_POISON(p, n) __asan_poison_memory_region((p), (n))
#define STUB_UNPOISON(p, n) __asan_unpoison_memory_region((p), (n))
#else
#define STUB_POISON(p, n) ((void)0)
#define STUB_UNPOISON(p, n) ((void)0)
#endif

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <map>
#include <vector>

struct StubOp {
    std::function<void()> fn;   // empty: a wait
    StubStream* dep = nullptr;  // wait: the stream that has to reach dep_seq first
    uint64_t dep_seq = 0;
};
struct StubStream {
    std::deque<StubOp> q;
    uint64_t enq = 0, done = 0;
    bool alive = true, running = false;
};
struct StubEvent {
    StubStream* s = nullptr;
    uint64_t seq = 0;
    bool alive = true;
};

namespace {

std::vector<StubStream*> g_streams;  // never freed: a stale handle is recognised, not dereferenced as garbage
std::vector<StubEvent*> g_events;
std::map<void*, size_t> g_allocs;
// Device memory is out of bounds for host code: every device allocation (and every tensor the test driver declares to
// be device memory) is poisoned for AddressSanitizer except while a deferred operation, the stand-in for the GPU, runs.
// A host-side read or write of a device pointer, a segmentation fault on the real machine, is reported as such here.
std::map<void*, size_t> g_device;
int g_device_open = 0;
void device_open()
{
    if (g_device_open++ == 0)
        for (auto& kv : g_device) STUB_UNPOISON(kv.first, kv.second);
}
void device_close()
{
    if (--g_device_open == 0)
        for (auto& kv : g_device) STUB_POISON(kv.first, kv.second);
}
int g_mode = 0;
uint64_t g_rng = 0x9e3779b97f4a7c15ULL;
int64_t g_fail_in = 0;
int64_t g_allocator_calls = 0;

[[noreturn]] void die(const char* what)
{
    fprintf(stderr, "hoststub: %s\n", what);
    fflush(stderr);
    abort();
}

uint64_t rnd()
{
    g_rng += 0x9e3779b97f4a7c15ULL;
    uint64_t x = g_rng;
    x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ULL;
    x = (x ^ (x >> 27)) * 0x94d049bb133111ebULL;
    return x ^ (x >> 31);
}

void check(hipStream_t s)
{
    if (!s) die("null stream (the library creates its streams)");
    if (!s->alive) die("use of a destroyed stream");
}
void check(hipEvent_t e)
{
    if (!e) die("null event");
    if (!e->alive) die("use of a destroyed event");
}

void run_until(StubStream* s, uint64_t target)
{
    if (s->done >= target) return;
    if (s->running) die("wait cycle between streams");
    s->running = true;
    while (s->done < target) {
        if (s->q.empty()) die("stream asked to run past what was enqueued");
        StubOp op = std::move(s->q.front());
        s->q.pop_front();
        if (op.fn) {
            device_open();
            op.fn();
            device_close();
        } else if (op.dep)
            run_until(op.dep, op.dep_seq);
        ++s->done;
    }
    s->running = false;
}

void run_all()
{
    for (StubStream* s : g_streams) run_until(s, s->enq);
}

// after every enqueue: decide how much runs now
void after_enqueue(StubStream* s)
{
    if (g_mode == 0) {
        run_until(s, s->enq);
    } else if (g_mode == 2) {
        // a few random advances of random streams (each at most to what it has been given)
        const int rounds = (int)(rnd() % 3);
        for (int r = 0; r < rounds && !g_streams.empty(); ++r) {
            StubStream* t = g_streams[rnd() % g_streams.size()];
            const uint64_t pending = t->enq - t->done;
            if (pending == 0) continue;
            run_until(t, t->done + 1 + rnd() % pending);
        }
    }
}

void push(StubStream* s, StubOp op)
{
    s->q.push_back(std::move(op));
    ++s->enq;
    after_enqueue(s);
}

void* alloc_poisoned(size_t bytes)
{
    if (g_fail_in > 0 && --g_fail_in == 0) return nullptr;
    void* p = malloc(bytes ? bytes : 1);
    if (p) memset(p, 0xff, bytes);  // NaN for fp32 and bf16, -1 for ids: reading what was never written shows
    return p;
}

}  // namespace

void stub_enqueue(hipStream_t s, std::function<void()> fn)
{
    check(s);
    StubOp op;
    op.fn = std::move(fn);
    push(s, std::move(op));
}

extern "C" void stub_set_mode(int mode, uint64_t seed)
{
    run_all();
    g_mode = mode;
    g_rng = seed * 0x9e3779b97f4a7c15ULL + 12345;
}

extern "C" void stub_device_synchronize(void) { run_all(); }

extern "C" void stub_live_counts(int64_t* allocations, int64_t* bytes, int64_t* streams, int64_t* events)
{
    int64_t b = 0, ns = 0, ne = 0;
    for (auto& kv : g_allocs) b += (int64_t)kv.second;
    for (StubStream* s : g_streams) ns += s->alive;
    for (StubEvent* e : g_events) ne += e->alive;
    if (allocations) *allocations = (int64_t)g_allocs.size();
    if (bytes) *bytes = b;
    if (streams) *streams = ns;
    if (events) *events = ne;
}

extern "C" void stub_fail_allocation(int64_t nth) { g_fail_in = nth; }

const char* hipGetErrorString(hipError_t e)
{
    switch (e) {
        case hipSuccess: return "no error";
        case hipErrorInvalidValue: return "invalid argument";
        case hipErrorOutOfMemory: return "out of memory";
        case hipErrorNotReady: return "not ready";
        default: return "unknown error";
    }
}
hipError_t hipGetLastError() { return hipSuccess; }
hipError_t hipGetDeviceCount(int* n)
{
    *n = 1;
    return hipSuccess;
}
hipError_t hipGetDevice(int* d)
{
    *d = 0;
    return hipSuccess;
}
hipError_t hipSetDevice(int d) { return d == 0 ? hipSuccess : hipErrorInvalidValue; }

extern "C" int64_t stub_allocator_calls(void) { return g_allocator_calls; }

hipError_t hipGetSymbolAddress(void** p, const void* symbol, size_t bytes)
{
    *p = const_cast<void*>(symbol);
    if (!g_device.count(*p)) {
        g_device[*p] = bytes;
        if (g_device_open == 0) STUB_POISON(*p, bytes);
    }
    return hipSuccess;
}

static hipError_t alloc_any(void** p, size_t bytes, bool device)
{
    ++g_allocator_calls;
    *p = alloc_poisoned(bytes);
    if (!*p) return hipErrorOutOfMemory;
    g_allocs[*p] = bytes;
    if (device) {
        g_device[*p] = bytes;
        if (g_device_open == 0) STUB_POISON(*p, bytes);
    }
    return hipSuccess;
}
static hipError_t free_any(void* p, bool device)
{
    ++g_allocator_calls;
    if (!p) return hipSuccess;
    run_all();  // the real call waits for the device
    auto it = g_allocs.find(p);
    if (it == g_allocs.end()) die("free of a pointer that is not a live allocation");
    if (device != (g_device.count(p) != 0)) die("device memory freed as pinned host memory, or the other way round");
    if (device) {
        STUB_UNPOISON(p, it->second);
        g_device.erase(p);
    }
    g_allocs.erase(it);
    free(p);
    return hipSuccess;
}
hipError_t hipMalloc(void** p, size_t bytes) { return alloc_any(p, bytes, true); }
hipError_t hipFree(void* p) { return free_any(p, true); }
hipError_t hipHostMalloc(void** p, size_t bytes, unsigned) { return alloc_any(p, bytes, false); }
hipError_t hipHostFree(void* p) { return free_any(p, false); }

// tensors of the test driver that stand for device memory: off limits to host code between these two calls
extern "C" void stub_register_device(void* p, size_t bytes)
{
    if (!p || bytes == 0) return;
    g_device[p] = bytes;
    if (g_device_open == 0) STUB_POISON(p, bytes);
}
extern "C" void stub_unregister_device(void* p)
{
    auto it = g_device.find(p);
    if (it == g_device.end()) return;
    STUB_UNPOISON(it->first, it->second);
    g_device.erase(it);
}

hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned)
{
    ++g_allocator_calls;
    *s = new StubStream();
    g_streams.push_back(*s);
    return hipSuccess;
}
hipError_t hipStreamDestroy(hipStream_t s)
{
    check(s);
    run_until(s, s->enq);  // pending work completes before the stream's resources go
    s->alive = false;
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t s)
{
    check(s);
    run_until(s, s->enq);
    return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned)
{
    check(s);
    check(e);
    if (!e->s) return hipSuccess;  // never recorded: nothing to wait for
    if (!e->s->alive && e->s->done < e->seq) die("wait on an event whose stream was destroyed with the record pending");
    StubOp op;
    op.dep = e->s;
    op.dep_seq = e->seq;
    push(s, std::move(op));
    return hipSuccess;
}

hipError_t hipEventCreate(hipEvent_t* e)
{
    ++g_allocator_calls;
    *e = new StubEvent();
    g_events.push_back(*e);
    return hipSuccess;
}
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { return hipEventCreate(e); }
hipError_t hipEventDestroy(hipEvent_t e)
{
    check(e);
    e->alive = false;
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s)
{
    check(e);
    check(s);
    e->s = s;
    e->seq = s->enq;
    return hipSuccess;
}
hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b)
{
    check(a);
    check(b);
    if (!a->s || !b->s) return hipErrorInvalidValue;
    if (a->s->done < a->seq || b->s->done < b->seq) return hipErrorNotReady;
    *ms = 0.f;
    return hipSuccess;
}

hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind, hipStream_t s)
{
    check(s);
    if (bytes == 0) return hipSuccess;
    if (!dst || !src) return hipErrorInvalidValue;
    StubOp op;
    op.fn = [=] { memmove(dst, src, bytes); };
    push(s, std::move(op));
    return hipSuccess;
}
hipError_t hipMemcpy2DAsync(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width, size_t height, hipMemcpyKind,
                            hipStream_t s)
{
    check(s);
    if (width == 0 || height == 0) return hipSuccess;
    if (!dst || !src || dpitch < width || spitch < width) return hipErrorInvalidValue;
    StubOp op;
    op.fn = [=] {
        for (size_t r = 0; r < height; ++r) memmove(static_cast<char*>(dst) + r * dpitch, static_cast<const char*>(src) + r * spitch, width);
    };
    push(s, std::move(op));
    return hipSuccess;
}
