// A host-only stand-in for the part of the HIP runtime API that the engine's host code uses
// (streams, events, asynchronous copies, pointer attributes).  TEST INFRASTRUCTURE: it lets
// sp_host.hip, sp_engine.hip and sp_train.hip be compiled with g++ and run on the CPU under
// AddressSanitizer / UndefinedBehaviorSanitizer / ThreadSanitizer, with every stream a real
// thread, so that a missing fence between a layer copy and a layer compute is a data race the
// sanitizer reports, and with injectable failures of the i-th call of an API.
// Implementation: tests/mock_hip/mock_hip.cpp.
#pragma once
#include <stddef.h>
#include <stdint.h>

typedef enum {
    hipSuccess = 0,
    hipErrorInvalidValue = 1,
    hipErrorOutOfMemory = 2,
    hipErrorUnknown = 999
} hipError_t;

typedef struct mockStream* hipStream_t;
typedef struct mockEvent* hipEvent_t;

enum { hipEventDefault = 0, hipEventDisableTiming = 2 };
typedef enum { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2 } hipMemcpyKind;
typedef enum { hipMemoryTypeUnregistered = 0, hipMemoryTypeHost = 1, hipMemoryTypeDevice = 2 } hipMemoryType;
typedef struct { hipMemoryType type; } hipPointerAttribute_t;
typedef enum { hipFuncAttributeMaxDynamicSharedMemorySize = 8 } hipFuncAttribute;

hipError_t hipEventCreate(hipEvent_t* ev);
hipError_t hipEventCreateWithFlags(hipEvent_t* ev, unsigned flags);
hipError_t hipEventDestroy(hipEvent_t ev);
hipError_t hipEventRecord(hipEvent_t ev, hipStream_t st);
hipError_t hipEventSynchronize(hipEvent_t ev);
hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b);
hipError_t hipStreamWaitEvent(hipStream_t st, hipEvent_t ev, unsigned flags);
hipError_t hipStreamSynchronize(hipStream_t st);
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind kind, hipStream_t st);
hipError_t hipPointerGetAttributes(hipPointerAttribute_t* at, const void* p);
hipError_t hipFuncSetAttribute(const void* fn, hipFuncAttribute a, int v);
hipError_t hipGetLastError(void);
const char* hipGetErrorString(hipError_t e);

// ---- controls of the stand-in (not part of HIP) ----
hipStream_t mock_stream_create(void);
void mock_stream_destroy(hipStream_t st);
// memory that hipPointerGetAttributes reports as pinned host memory
void* mock_pinned_alloc(size_t bytes);
void mock_pinned_free(void* p);
// The n-th call from now (n >= 1) of the named API returns hipErrorUnknown; api is one of
// "hipMemcpyAsync", "hipEventCreateWithFlags", "hipEventRecord", "hipStreamWaitEvent", "launch"
// (any kernel launcher).  n = 0 clears.
void mock_fail_nth(const char* api, int n);
// how often the named API has been called since the last mock_count_reset
long mock_count(const char* api);
void mock_count_reset(void);
