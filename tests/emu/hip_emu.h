// CPU stand-in for the few HIP constructs the kernels use, for ONE purpose: running
// the kernel sources of the library through their indexing on the CPU (tiny shapes,
// guard pages behind every buffer) before they are ever launched on a GPU.  It is
// test scaffolding, lives under tests/, and is never part of the library build.
//
// Each "thread" of a block is a ucontext fiber; __syncthreads() yields to the
// block scheduler, which resumes the fibers round-robin.  "Device memory" is host
// memory with a PROT_NONE page directly behind it, so an overrun faults on the CPU.
#pragma once
#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <functional>

#define __global__
#define __device__
#define __host__
#define __shared__ static
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) x

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {}
};
struct double2 { double x, y; };
static inline double2 make_double2(double a, double b) { return double2{a, b}; }
struct ulonglong2 { unsigned long long x, y; };
static inline ulonglong2 make_ulonglong2(unsigned long long a, unsigned long long b) { return ulonglong2{a, b}; }

extern dim3 threadIdx, blockIdx, blockDim, gridDim;

typedef int hipError_t;
typedef void *hipStream_t;
#define hipSuccess 0
#define hipMemcpyHostToDevice 1
#define hipMemcpyDeviceToHost 2
#define hipMemcpyDeviceToDevice 3

namespace emu {
void launch(dim3 grid, dim3 block, const std::function<void()> &body);
void sync();
void *guarded_alloc(size_t bytes);
void guarded_free(void *p);
}  // namespace emu

static inline void __syncthreads() { emu::sync(); }
static inline hipError_t hipMalloc(void **p, size_t n) { *p = emu::guarded_alloc(n); return *p ? 0 : 2; }
static inline hipError_t hipFree(void *p) { emu::guarded_free(p); return 0; }
static inline hipError_t hipMemcpy(void *d, const void *s, size_t n, int) { memcpy(d, s, n); return 0; }
static inline hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, int, hipStream_t) { memcpy(d, s, n); return 0; }
static inline hipError_t hipMemsetAsync(void *d, int v, size_t n, hipStream_t) { memset(d, v, n); return 0; }
template <class Sym>
static inline hipError_t hipGetSymbolAddress(void **p, Sym &symbol) { *p = (void *)&symbol; return 0; }
static inline hipError_t hipSetDevice(int) { return 0; }
static inline hipError_t hipGetDevice(int *d) { *d = 0; return 0; }
static inline hipError_t hipGetLastError() { return 0; }
static inline hipError_t hipDeviceSynchronize() { return 0; }
static inline hipError_t hipStreamSynchronize(hipStream_t) { return 0; }

typedef void *hipEvent_t;
static inline hipError_t hipEventCreate(hipEvent_t *e) { *e = nullptr; return 0; }
static inline hipError_t hipEventDestroy(hipEvent_t) { return 0; }
static inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return 0; }
static inline hipError_t hipEventSynchronize(hipEvent_t) { return 0; }
static inline hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0; return 0; }

static inline double __longlong_as_double(long long v) { double d; memcpy(&d, &v, 8); return d; }
static inline long long __double_as_longlong(double d) { long long v; memcpy(&v, &d, 8); return v; }
static inline unsigned __brev(unsigned x) {
    unsigned r = 0;
    for (int i = 0; i < 32; i++) { r = (r << 1) | (x & 1); x >>= 1; }
    return r;
}

#define CKKSMI_LAUNCH(kern, grid, block, stream, ...) emu::launch(grid, block, [&]() { kern(__VA_ARGS__); })
static inline unsigned __umul24(unsigned a, unsigned b) { return (a & 0xffffffu) * (b & 0xffffffu); }
