// Host-only stand-in for the part of the HIP runtime API that libsaga's host code uses.
// Test infrastructure: with this header first on the include path, the host translation units of the
// library (context, graph ingest, chunk schedule, backward pass) compile with g++ and run on the CPU,
// so that AddressSanitizer and UBSan see every allocation, copy and pointer the schedule handles.
//
// "Device" memory is ordinary heap memory (poisoned with NaN bytes on allocation). Streams are queues
// of deferred operations executed in stream order and honouring event waits; when they run is up to the
// mode set with stub_set_mode: at once, as late as the API allows, or at seeded random points. Kernels
// are CPU closures enqueued like any other operation (stub_kernels.cpp).
#pragma once

#include <cstddef>
#include <cstdint>
#include <functional>

typedef int hipError_t;
enum : int {
    hipSuccess = 0,
    hipErrorInvalidValue = 1,
    hipErrorOutOfMemory = 2,
    hipErrorNotReady = 600,
    hipErrorUnknown = 999,
};
enum hipMemcpyKind { hipMemcpyHostToHost = 0, hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2, hipMemcpyDeviceToDevice = 3, hipMemcpyDefault = 4 };

struct StubStream;
struct StubEvent;
typedef StubStream* hipStream_t;
typedef StubEvent* hipEvent_t;

constexpr unsigned hipStreamNonBlocking = 1u;
constexpr unsigned hipEventDisableTiming = 2u;
constexpr unsigned hipHostMallocDefault = 0u;

const char* hipGetErrorString(hipError_t e);
hipError_t hipGetLastError();
hipError_t hipGetDeviceCount(int* n);
hipError_t hipGetDevice(int* d);
hipError_t hipSetDevice(int d);

hipError_t hipMalloc(void** p, size_t bytes);
hipError_t hipFree(void* p);
hipError_t hipHostMalloc(void** p, size_t bytes, unsigned flags);
hipError_t hipHostFree(void* p);

hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned flags);
hipError_t hipStreamDestroy(hipStream_t s);
hipError_t hipStreamSynchronize(hipStream_t s);
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned flags);

hipError_t hipEventCreate(hipEvent_t* e);
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned flags);
hipError_t hipEventDestroy(hipEvent_t e);
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s);
hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b);

// a `static __device__` array of the library is an ordinary static array here; its "device address" is its address,
// and from the first request on it is device memory: out of bounds for host code
#define __device__
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (static_cast<const void*>(&(x))), sizeof(x)
hipError_t hipGetSymbolAddress(void** p, const void* symbol, size_t bytes);

hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind kind, hipStream_t s);
hipError_t hipMemcpy2DAsync(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width, size_t height, hipMemcpyKind kind,
                            hipStream_t s);

// ---- for the CPU kernels and the test driver ----
// Append a closure to stream s (the stand-in for a kernel launch).
void stub_enqueue(hipStream_t s, std::function<void()> fn);
extern "C" {
// 0: every operation runs when it is enqueued; 1: as late as the API allows (at a synchronisation, a free,
// a stream's destruction); 2: at random points chosen by a generator seeded with `seed`
void stub_set_mode(int mode, uint64_t seed);
void stub_device_synchronize(void);
// live allocations (device + pinned) and live streams / events, for leak checks at the end of a session
void stub_live_counts(int64_t* allocations, int64_t* bytes, int64_t* streams, int64_t* events);
// make the n-th allocation from now on fail once (0: never): error paths
void stub_fail_allocation(int64_t nth);
// calls of hipMalloc, hipFree, hipHostMalloc, hipHostFree, stream and event creation so far
int64_t stub_allocator_calls(void);
// memory of the test driver that stands for device memory during a library call: host code must not touch it
void stub_register_device(void* p, size_t bytes);
void stub_unregister_device(void* p);
}
