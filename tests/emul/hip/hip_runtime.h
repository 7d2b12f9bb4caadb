// Host stand-in for <hip/hip_runtime.h>, used by tests/test_kernel_bounds.py only.
//
// It lets the kernel sources compile as plain C++ and runs a launch as nested loops:
// every thread of every workgroup runs to completion, one after the other.  There are
// no barrier or cross-lane semantics (values that travel through LDS, DPP or MFMA are
// meaningless), which is enough for what the test checks: with AddressSanitizer on,
// every global load and store and every LDS access of every thread is bounds checked
// on the CPU before the kernels ever touch a GPU.  LDS arrays become per-thread stack
// arrays of the same shape, dynamic LDS one global array of the hardware's size.
#pragma once
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <algorithm>

#define ST_NO_GPU_ASSEMBLY 1   // the one hand-written GPU instruction of the kernels falls back to its plain form
#define ST_PIN_VGPR(x) ((void)0)
#define ST_WAIT_STATES(n) ((void)0)
#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __shared__
#define __constant__
#define __launch_bounds__(...)
#define __restrict__
#define HIP_SYMBOL(x) x
#define __align__(n) __attribute__((aligned(n)))

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {}
};
struct float4 { float x, y, z, w; };
struct float2 { float x, y; };
static inline float4 make_float4(float a, float b, float c, float d) { return float4{a, b, c, d}; }
static inline float2 make_float2(float a, float b) { return float2{a, b}; }

static dim3 threadIdx, blockIdx, blockDim, gridDim;

static inline void __syncthreads() {}
static inline void __builtin_amdgcn_sched_barrier(int) {}
static inline void __builtin_amdgcn_s_barrier() {}
typedef float emu_f32x4 __attribute__((ext_vector_type(4)));
static inline emu_f32x4 __builtin_amdgcn_mfma_f32_16x16x4f32(float, float, emu_f32x4 c, int, int, int) { return c; }
static inline int __builtin_amdgcn_update_dpp(int, int src, int, int, int, bool) { return src; }
static inline int __builtin_amdgcn_readlane(int v, int) { return v; }
static inline int __builtin_amdgcn_readfirstlane(int v) { return v; }
static inline float __shfl_xor(float v, int) { return v; }

using std::max;
using std::min;
static inline uint32_t min(uint32_t a, uint32_t b) { return a < b ? a : b; }
static inline uint32_t max(uint32_t a, uint32_t b) { return a > b ? a : b; }

typedef void *hipStream_t;
typedef int hipError_t;
enum { hipSuccess = 0 };
enum { hipFuncAttributeMaxDynamicSharedMemorySize = 8, hipDeviceAttributeMultiprocessorCount = 63,
       hipDeviceAttributeMaxSharedMemoryPerBlock = 74 };
enum hipMemcpyKind { hipMemcpyHostToDevice = 1 };
static inline hipError_t hipMemcpyAsync(void *dst, const void *src, size_t bytes, hipMemcpyKind, hipStream_t)
{
    memcpy(dst, src, bytes);
    return hipSuccess;
}
static inline hipError_t hipGetLastError() { return hipSuccess; }
enum { hipHostMallocPortable = 1 };
static inline hipError_t hipHostMalloc(void **p, size_t bytes, unsigned) { *p = malloc(bytes); return *p ? hipSuccess : 1; }
static inline hipError_t hipGetSymbolAddress(void **p, const void *symbol) { *p = const_cast<void *>(symbol); return hipSuccess; }
static inline hipError_t hipFuncSetAttribute(const void *, int, int) { return hipSuccess; }
static inline hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
static inline hipError_t hipDeviceGetAttribute(int *v, int attr, int)
{
    *v = attr == hipDeviceAttributeMaxSharedMemoryPerBlock ? 160 * 1024 : 256;
    return hipSuccess;
}

namespace st { extern float lds[]; }   // dynamic LDS (declared `extern __shared__` in the kernels)

#define hipLaunchKernelGGL(K, G, B, LDS, S, ...)                                     \
    do {                                                                             \
        const dim3 g_ = (G), b_ = (B);                                               \
        gridDim = g_;                                                                \
        blockDim = b_;                                                               \
        for (unsigned by_ = 0; by_ < g_.y; ++by_)                                    \
            for (unsigned bx_ = 0; bx_ < g_.x; ++bx_)                                \
                for (unsigned t_ = 0; t_ < b_.x; ++t_) {                             \
                    blockIdx = dim3(bx_, by_);                                       \
                    threadIdx = dim3(t_);                                            \
                    K(__VA_ARGS__);                                                  \
                }                                                                    \
    } while (0)
