/* Stand-in for the HIP runtime header, for building the library's C ABI (argument checking, plan cache,
 * scratch bookkeeping) for the host alone.  "Device memory" is host memory; nothing is ever launched.
 * Test infrastructure: used only by tests/test_abi_host_sanitized.py. */
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef int hipError_t;
typedef struct hip_stream_standin* hipStream_t;
enum { hipSuccess = 0, hipErrorOutOfMemory = 2, hipErrorInvalidValue = 1 };
enum { hipMemcpyHostToDevice = 1 };
enum { hipDeviceAttributeMaxSharedMemoryPerBlock = 1 };

#define __device__
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (&(x))

extern size_t hip_standin_live_allocations;   /* allocations not yet freed */
extern size_t hip_standin_fail_after;          /* hipMalloc fails once this many more calls have been made */

static inline hipError_t hipGetDeviceCount(int* n) { *n = 1; return hipSuccess; }
static inline hipError_t hipSetDevice(int d) { return d == 0 ? hipSuccess : hipErrorInvalidValue; }
static inline hipError_t hipGetLastError(void) { return hipSuccess; }
static inline const char* hipGetErrorString(hipError_t e) { return e == hipSuccess ? "no error" : "stand-in error"; }
static inline hipError_t hipDeviceGetAttribute(int* v, int attr, int dev) { (void)attr; (void)dev; *v = 160 * 1024; return hipSuccess; }
static inline hipError_t hipStreamSynchronize(hipStream_t s) { (void)s; return hipSuccess; }
static inline hipError_t hipMalloc(void** p, size_t bytes) {
    if (hip_standin_fail_after != (size_t)-1) {
        if (hip_standin_fail_after == 0) { *p = NULL; return hipErrorOutOfMemory; }
        --hip_standin_fail_after;
    }
    /* large requests are not backed: the library never touches device memory from the host */
    *p = aligned_alloc(256, bytes < 4096 ? 4096 : 4096);
    if (!*p) return hipErrorOutOfMemory;
    ++hip_standin_live_allocations;
    return hipSuccess;
}
static inline hipError_t hipFree(void* p) { if (p) { free(p); --hip_standin_live_allocations; } return hipSuccess; }
static inline hipError_t hipMemcpy(void* dst, const void* src, size_t bytes, int kind) {
    (void)kind;
    memcpy(dst, src, bytes < 4096 ? bytes : 4096);
    return hipSuccess;
}
static inline hipError_t hipMemset(void* dst, int v, size_t bytes) { memset(dst, v, bytes < 4096 ? bytes : 4096); return hipSuccess; }
static inline hipError_t hipGetSymbolAddress(void** p, const void* symbol) { *p = (void*)symbol; return hipSuccess; }
#ifdef __cplusplus
template <class T> static inline hipError_t hipMalloc(T** p, size_t bytes) { return hipMalloc(reinterpret_cast<void**>(p), bytes); }
template <class T> static inline hipError_t hipGetSymbolAddress(void** p, T* symbol) { *p = (void*)symbol; return hipSuccess; }
#endif
