// A stand-in for the HIP runtime, for HOST-ONLY test builds of the library's C ABI (api.cpp)
// under AddressSanitizer: "device" memory is host memory, streams run at once, events are
// small heap objects (so a leaked one is reported).  Test infrastructure only: the product is
// never built against this header.
#pragma once
#include <cstdlib>
#include <cstring>

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorOutOfMemory = 2, hipErrorInvalidValue = 1 };
struct fakeStream { int id; };
struct fakeEvent { long recorded; };
typedef fakeStream *hipStream_t;
typedef fakeEvent *hipEvent_t;
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2, hipMemcpyDeviceToDevice = 3 };
enum { hipStreamNonBlocking = 1, hipEventDisableTiming = 2, hipHostMallocDefault = 0 };

extern long fake_hip_host_limit;   // bytes hipHostMalloc may hand out in total (-1 = no limit)
extern long fake_hip_host_bytes;   // bytes currently handed out
extern long fake_hip_copies;       // hipMemcpyAsync calls so far

inline const char *hipGetErrorString(hipError_t e) { return e == hipSuccess ? "no error" : "fake HIP error"; }
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned) { *s = new fakeStream{1}; return hipSuccess; }
inline hipError_t hipStreamDestroy(hipStream_t s) { delete s; return hipSuccess; }
enum hipStreamCaptureStatus { hipStreamCaptureStatusNone = 0, hipStreamCaptureStatusActive = 1 };
inline hipError_t hipStreamIsCapturing(hipStream_t, hipStreamCaptureStatus *st) { *st = hipStreamCaptureStatusNone; return hipSuccess; }
inline hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = new fakeEvent{0}; return hipSuccess; }
inline hipError_t hipEventDestroy(hipEvent_t e) { delete e; return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t e, hipStream_t) { ++e->recorded; return hipSuccess; }
inline hipError_t hipEventSynchronize(hipEvent_t e) { return e->recorded >= 0 ? hipSuccess : hipErrorInvalidValue; }
inline hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t e, unsigned) { return e->recorded >= 0 ? hipSuccess : hipErrorInvalidValue; }
inline hipError_t hipHostMalloc(void **p, size_t n, unsigned) {
    if (fake_hip_host_limit >= 0 && fake_hip_host_bytes + long(n) > fake_hip_host_limit) { *p = nullptr; return hipErrorOutOfMemory; }
    // the size sits in front of the block so that hipHostFree can keep the count
    char *raw = static_cast<char *>(std::malloc(n + 256));
    if (!raw) return hipErrorOutOfMemory;
    std::memcpy(raw, &n, sizeof n);
    fake_hip_host_bytes += long(n);
    *p = raw + 256;
    return hipSuccess;
}
inline hipError_t hipHostFree(void *p) {
    if (!p) return hipSuccess;
    char *raw = static_cast<char *>(p) - 256;
    size_t n;
    std::memcpy(&n, raw, sizeof n);
    fake_hip_host_bytes -= long(n);
    std::free(raw);
    return hipSuccess;
}
inline hipError_t hipFree(void *p) { std::free(p); return hipSuccess; }
inline hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, hipMemcpyKind, hipStream_t) {
    std::memcpy(d, s, n);
    ++fake_hip_copies;
    return hipSuccess;
}
