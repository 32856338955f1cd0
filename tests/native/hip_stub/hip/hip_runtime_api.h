// Test-only stand-in for the HIP runtime API, used to build the update phase's
// host logic (piece/chunk bookkeeping, worker pool, upload ring, validation) for
// the CPU and run it under the sanitizers.  Every "device" pointer is plain host
// memory, every stream operation completes before the call returns, events are
// time stamps.  Never part of libdos.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <chrono>

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidDevice = 101, hipErrorLaunchFailure = 719 };
typedef struct stub_stream* hipStream_t;
struct stub_event {
  double t_ms;
};
typedef stub_event* hipEvent_t;
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2 };
enum { hipStreamNonBlocking = 1, hipEventDisableTiming = 2, hipEventBlockingSync = 1 };

inline double stub_now_ms() {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}
inline hipError_t hipSetDevice(int d) { return d == 0 ? hipSuccess : hipErrorInvalidDevice; }
inline hipError_t hipGetLastError() { return hipSuccess; }
enum hipDeviceAttribute_t { hipDeviceAttributeIsLargeBar = 1 };
// the stand-in device's memory is host memory: the host can always write it
inline hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t, int d) {
  if (d != 0) return hipErrorInvalidDevice;
  *v = 1;
  return hipSuccess;
}
inline const char* hipGetErrorString(hipError_t) { return "stub"; }
inline hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) {
  *s = reinterpret_cast<hipStream_t>(new int(0));
  return hipSuccess;
}
inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
inline hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
inline hipError_t hipEventCreate(hipEvent_t* e) {
  *e = new stub_event{0.0};
  return hipSuccess;
}
inline hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { return hipEventCreate(e); }
inline hipError_t hipEventDestroy(hipEvent_t e) {
  delete e;
  return hipSuccess;
}
inline hipError_t hipEventRecord(hipEvent_t e, hipStream_t) {
  e->t_ms = stub_now_ms();
  return hipSuccess;
}
inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b) {
  *ms = (float)(b->t_ms - a->t_ms);
  return hipSuccess;
}
inline hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t) {
  memcpy(dst, src, n);
  return hipSuccess;
}
inline hipError_t hipMemsetAsync(void* dst, int v, size_t n, hipStream_t) {
  memset(dst, v, n);
  return hipSuccess;
}
enum { hipHostMallocDefault = 0 };
inline hipError_t hipHostMalloc(void** p, size_t n, unsigned) {
  *p = aligned_alloc(4096, (n + 4095) / 4096 * 4096);
  return *p ? hipSuccess : 2;
}
inline hipError_t hipHostFree(void* p) {
  free(p);
  return hipSuccess;
}
