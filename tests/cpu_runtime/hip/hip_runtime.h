// A stand-in for the HIP runtime on the CPU -- TEST INFRASTRUCTURE ONLY.
//
// The host runtime of the library (rings, admission, commit discovery, drain thread, exporter,
// replayable steps) is ordinary multi-threaded C++ around a handful of HIP calls.  Built against
// this header instead of ROCm's, and with cpu_kernels.cpp in place of the device code, it runs in
// a container without a GPU, where ThreadSanitizer and AddressSanitizer can watch it.
// "Device memory" is host memory; a stream is a worker thread with a queue, so launches, copies
// and events complete asynchronously as they do on a GPU; a capture records tasks instead of
// running them.  Nothing here computes what the library computes.
#pragma once
#include <cstddef>
#include <cstdint>
#include <functional>
#include <vector>

typedef int hipError_t;
enum : int { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorOutOfMemory = 2, hipErrorNotReady = 600 };

struct FakeStream;
struct FakeEvent;
typedef FakeStream *hipStream_t;
typedef FakeEvent *hipEvent_t;

struct uint4 { uint32_t x, y, z, w; };

enum hipMemcpyKind { hipMemcpyHostToHost = 0, hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2,
                     hipMemcpyDeviceToDevice = 3, hipMemcpyDefault = 4 };
enum hipStreamCaptureStatus { hipStreamCaptureStatusNone = 0, hipStreamCaptureStatusActive = 1 };
enum : unsigned { hipHostMallocMapped = 2u, hipHostMallocCoherent = 0x40000000u, hipStreamNonBlocking = 1u,
                  hipEventDisableTiming = 2u };

const char *hipGetErrorString(hipError_t e);
hipError_t hipGetDeviceCount(int *n);
hipError_t hipSetDevice(int dev);
hipError_t hipDeviceSynchronize();
hipError_t hipMalloc(void **p, size_t n);
hipError_t hipFree(void *p);
hipError_t hipHostMalloc(void **p, size_t n, unsigned flags);
hipError_t hipHostFree(void *p);
hipError_t hipHostGetDevicePointer(void **dev, void *host, unsigned flags);
hipError_t hipMemcpy(void *dst, const void *src, size_t n, hipMemcpyKind kind);
hipError_t hipMemcpyAsync(void *dst, const void *src, size_t n, hipMemcpyKind kind, hipStream_t s);
hipError_t hipMemsetAsync(void *dst, int value, size_t n, hipStream_t s);
hipError_t hipStreamCreate(hipStream_t *s);
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned flags);
hipError_t hipStreamDestroy(hipStream_t s);
hipError_t hipStreamSynchronize(hipStream_t s);
hipError_t hipStreamQuery(hipStream_t s);
hipError_t hipStreamIsCapturing(hipStream_t s, hipStreamCaptureStatus *status);
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned flags);
hipError_t hipEventDestroy(hipEvent_t e);
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s);
hipError_t hipEventQuery(hipEvent_t e);
hipError_t hipEventSynchronize(hipEvent_t e);

// -- what the CPU "kernels" and the test driver use beyond the HIP names
typedef std::function<void()> FakeTask;
// run `task` on the stream's worker, after everything enqueued before it (NULL = the default stream)
void fake_enqueue(hipStream_t s, FakeTask task);
// stream capture: tasks enqueued on `s` are recorded, not run, until fake_end_capture returns them
void fake_begin_capture(hipStream_t s);
std::vector<FakeTask> fake_end_capture(hipStream_t s);
// a "graph launch": enqueue the recorded tasks again
void fake_graph_launch(const std::vector<FakeTask> &graph, hipStream_t s);
// each worker sleeps a random 0..max_us microseconds in front of every task (shakes interleavings)
void fake_set_jitter_us(unsigned max_us);
