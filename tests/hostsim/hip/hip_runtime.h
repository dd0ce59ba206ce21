// Stand-in HIP runtime for a host build of the library under sanitizers: device memory
// is host memory, streams run synchronously, kernels run one thread at a time.
#pragma once
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <cstdio>
#include <algorithm>
typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1 };
typedef void *hipStream_t;
typedef void *hipEvent_t;
struct dim3 { unsigned x, y, z; dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {} };
extern thread_local dim3 threadIdx, blockIdx, blockDim, gridDim;
#define __global__
#define __device__
#define __forceinline__ inline
#define __launch_bounds__(...)
#define __restrict__
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (&(x))
static inline int hipGetSymbolAddress(void **p, const void *sym) { *p = const_cast<void *>(sym); return 0; }
#define __builtin_amdgcn_readfirstlane(v) (v)
static inline uint32_t __float_as_uint(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static inline float __uint_as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
enum hipMemcpyKind { hipMemcpyHostToDevice, hipMemcpyDeviceToHost, hipMemcpyDeviceToDevice };
enum { hipEventDisableTiming = 2, hipHostMallocMapped = 2, hipHostMallocPortable = 1, hipHostMallocNumaUser = 0x20000000 };
enum { hipDeviceAttributeMultiprocessorCount = 1 };
enum hipMemoryType { hipMemoryTypeHost = 1, hipMemoryTypeDevice = 2 };
struct hipPointerAttribute_t { hipMemoryType type; void *devicePointer; void *hostPointer; };
static inline const char *hipGetErrorString(hipError_t) { return "fake"; }
static inline hipError_t hipGetLastError() { return hipSuccess; }
static inline hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
static inline hipError_t hipSetDevice(int) { return hipSuccess; }
static inline hipError_t hipDeviceGetAttribute(int *v, int, int) { *v = 4; return hipSuccess; }
static inline hipError_t hipMalloc(void **p, size_t n) { *p = malloc(n); return hipSuccess; }
static inline hipError_t hipFree(void *p) { free(p); return hipSuccess; }
static inline hipError_t hipMemcpy(void *d, const void *s, size_t n, hipMemcpyKind) { memcpy(d, s, n); return hipSuccess; }
static inline hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, hipMemcpyKind, hipStream_t) { memcpy(d, s, n); return hipSuccess; }
static inline hipError_t hipHostMalloc(void **p, size_t n, unsigned) { *p = malloc(n); return hipSuccess; }
static inline hipError_t hipHostFree(void *p) { free(p); return hipSuccess; }
static inline hipError_t hipHostGetDevicePointer(void **d, void *h, unsigned) { *d = h; return hipSuccess; }
static inline hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = malloc(1); return hipSuccess; }
static inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
static inline hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
static inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
static inline hipError_t hipPointerGetAttributes(hipPointerAttribute_t *a, const void *p) { a->type = hipMemoryTypeHost; a->devicePointer = const_cast<void *>(p); return hipSuccess; }
#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...)                      \
    do {                                                                                  \
        dim3 g_ = (grid), b_ = (block);                                                   \
        gridDim = g_; blockDim = b_;                                                      \
        for (unsigned bx_ = 0; bx_ < g_.x; ++bx_)                                         \
            for (unsigned tx_ = 0; tx_ < b_.x; ++tx_) {                                   \
                blockIdx = dim3(bx_); threadIdx = dim3(tx_);                              \
                kernel(__VA_ARGS__);                                                      \
            }                                                                             \
    } while (0)
// x86 non-temporal vector loads demand 16-byte alignment; plain accesses here
#define __builtin_nontemporal_load(p) (*(p))
#define __builtin_nontemporal_store(v, p) (*(p) = (v))
static inline hipError_t hipEventCreate(hipEvent_t *e) { *e = malloc(1); return hipSuccess; }
static inline hipError_t hipEventDestroy(hipEvent_t e) { free(e); return hipSuccess; }
static inline hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 1.0f; return hipSuccess; }
static inline hipError_t hipEventQuery(hipEvent_t) { return hipSuccess; }
typedef void *hipDeviceptr_t;
// the stand-in runtime does not track allocations: "unknown pointer", which the library lets through
static inline hipError_t hipMemGetAddressRange(hipDeviceptr_t *, size_t *, hipDeviceptr_t) { return hipErrorInvalidValue; }
