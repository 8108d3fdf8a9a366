// TEST INFRASTRUCTURE: a stand-in for <hip/hip_runtime.h> that keeps "device" memory on the host heap, so that the
// host side of the C-ABI library (handles, contexts, argument checks, copies, scratch layout) can be compiled with
// g++ and run under AddressSanitizer / UndefinedBehaviorSanitizer on a machine without a GPU.  Only what
// csrc/lite_attn.cpp and csrc/lite_attn_host.cpp use is here.  Never on the include path of the product build.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorOutOfMemory = 2, hipErrorNoDevice = 100 };
typedef struct fake_hip_stream* hipStream_t;
typedef struct fake_hip_event { int recorded; } * hipEvent_t;
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2 };

template <class T>
inline hipError_t hipMalloc(T** p, size_t n) {
  *p = static_cast<T*>(malloc(n ? n : 1));
  return *p ? hipSuccess : hipErrorOutOfMemory;
}
inline hipError_t hipFree(void* p) {
  free(p);
  return hipSuccess;
}
inline hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t) {
  memcpy(dst, src, n);
  return hipSuccess;
}
inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
inline hipError_t hipGetDevice(int* d) {
  *d = 0;
  return hipSuccess;
}
inline hipError_t hipEventCreate(hipEvent_t* e) {
  *e = static_cast<hipEvent_t>(calloc(1, sizeof(fake_hip_event)));
  return *e ? hipSuccess : hipErrorOutOfMemory;
}
inline hipError_t hipEventDestroy(hipEvent_t e) {
  free(e);
  return hipSuccess;
}
inline hipError_t hipEventRecord(hipEvent_t e, hipStream_t) {
  e->recorded = 1;
  return hipSuccess;
}
inline hipError_t hipEventSynchronize(hipEvent_t e) { return e->recorded ? hipSuccess : hipErrorInvalidValue; }
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b) {
  *ms = 0.f;
  return a->recorded && b->recorded ? hipSuccess : hipErrorInvalidValue;
}
