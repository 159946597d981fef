/* Host-only stand-in for the parts of the HIP runtime API that the library's HOST code uses.
 * Test infrastructure: lets the streaming and file-tier pipelines (threads, queues, events,
 * staging slots) be built with g++ and run under ThreadSanitizer without a GPU.
 *
 * Streams are real FIFO queues, each drained by its own thread; events complete when the stream
 * reaches them; copies are memcpy tasks.  The null stream runs its work in place unless
 * HIPMOCK_LEGACY_NULL is set in the environment: then it is a queue with HIP's legacy ordering
 * against blocking streams (see hipmock.cpp).  Because every stream runs concurrently, an ordering
 * that the pipeline forgets to express with an event shows up as a data race on the staging
 * memory (ThreadSanitizer) or as a wrong result. */
#ifndef HIPMOCK_RUNTIME_API_H
#define HIPMOCK_RUNTIME_API_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorOutOfMemory = 2, hipErrorNotReady = 600, hipErrorUnknown = 999 } hipError_t;
typedef struct hipmock_stream *hipStream_t;
typedef struct hipmock_event *hipEvent_t;
typedef enum { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2 } hipMemcpyKind;
typedef enum { hipDeviceAttributeMultiprocessorCount = 63 } hipDeviceAttribute_t;

#define hipStreamNonBlocking 1u
#define hipEventDisableTiming 2u
#define hipHostMallocDefault 0u

const char *hipGetErrorString(hipError_t e);
hipError_t hipGetLastError(void);
hipError_t hipGetDevice(int *dev);
hipError_t hipSetDevice(int dev);
hipError_t hipDeviceGetAttribute(int *value, hipDeviceAttribute_t attr, int dev);
hipError_t hipMalloc(void **ptr, size_t bytes);
hipError_t hipFree(void *ptr);
hipError_t hipHostMalloc(void **ptr, size_t bytes, unsigned flags);
hipError_t hipHostFree(void *ptr);
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned flags);
hipError_t hipExtStreamCreateWithCUMask(hipStream_t *s, uint32_t words, const uint32_t *mask);
hipError_t hipStreamDestroy(hipStream_t s);
hipError_t hipStreamSynchronize(hipStream_t s);
hipError_t hipDeviceSynchronize(void);
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned flags);
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned flags);
hipError_t hipEventDestroy(hipEvent_t e);
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s);
hipError_t hipEventSynchronize(hipEvent_t e);
hipError_t hipEventQuery(hipEvent_t e);
hipError_t hipEventElapsedTime(float *ms, hipEvent_t start, hipEvent_t stop);
typedef enum { hipMemoryTypeUnregistered = 0, hipMemoryTypeHost = 1, hipMemoryTypeDevice = 2, hipMemoryTypeManaged = 3 } hipMemoryType;
typedef struct {
    hipMemoryType type;
    int device;
    void *devicePointer;
    void *hostPointer;
    int isManaged;
    unsigned allocationFlags;
} hipPointerAttribute_t;
/* knows the blocks handed out by hipHostMalloc (host type) and hipMalloc (device type) */
hipError_t hipPointerGetAttributes(hipPointerAttribute_t *attr, const void *ptr);
typedef void (*hipHostFn_t)(void *userData);
hipError_t hipLaunchHostFunc(hipStream_t s, hipHostFn_t fn, void *userData);
hipError_t hipMemcpyAsync(void *dst, const void *src, size_t bytes, hipMemcpyKind kind, hipStream_t s);
hipError_t hipMemcpy(void *dst, const void *src, size_t bytes, hipMemcpyKind kind);
hipError_t hipMemset(void *dst, int value, size_t bytes);

#ifdef __cplusplus
}
/* enqueue an arbitrary host task on a mock stream (what a kernel launch becomes) */
#include <functional>
void hipmock_enqueue(hipStream_t s, std::function<void()> fn);
/* copies issued / bytes moved since process start, and a per-copy delay to widen race windows */
extern "C" uint64_t hipmock_copy_count(void);
extern "C" void hipmock_set_copy_delay_us(int us);
/* the nth call from now of the named API (hipEventRecord, hipStreamWaitEvent, hipLaunchHostFunc,
 * hipMemcpyAsync) returns hipErrorUnknown and does nothing; api == NULL disarms */
extern "C" void hipmock_fail_nth(const char *api, int nth);
/* the next `count` calls of hipEventElapsedTime return these values (then zero again) */
extern "C" void hipmock_script_elapsed_ms(const float *values, int count);
/* streams created and not yet destroyed */
extern "C" int hipmock_live_streams(void);
#endif
#endif
