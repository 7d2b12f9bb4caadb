// Measurement support: the floors a kernel is judged against on this chip -- what an empty launch of a given
// shape costs, how long a plain streaming read of an operand takes in that shape, and the rate the
// single-precision MFMA reaches from registers, alone and with vector work mixed in -- so that a reported
// kernel time can be split into launch, memory, matrix-core time and the rest.  Nothing here is part of a computation.
#include "st_common.h"

namespace st {

__global__ void probe_empty_kernel(float *sink)
{
    if (sink != nullptr && threadIdx.x == 0xffffffffu) *sink = 0.f;      // never true: the kernel does nothing
}

// Every thread issues PER 16-byte loads (all in flight at once), a workgroup reads one contiguous slab; the
// values are added and stored only if the sum hits a value it cannot have, which keeps the loads alive.
template <int PER>
__global__ __launch_bounds__(1024) void probe_stream_kernel(const float4 *__restrict__ src, size_t n16,
                                                           float *__restrict__ sink)
{
    const size_t base = (size_t)blockIdx.x * blockDim.x * PER + threadIdx.x;
    float4 v[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const size_t e = base + (size_t)i * blockDim.x;
        v[i] = src[e < n16 ? e : 0];
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) s += v[i].x + v[i].y + v[i].z + v[i].w;
    if (s == 123.456f) sink[0] = s;
}

// The matrix-core floor of the single-precision kernels: every wave repeats a block of NV vector multiplies
// (cross-lane forms, as the moment kernels form their pair products) followed by 23 independent 16x16x4 MFMAs,
// two waves per SIMD, operands in registers.  On this chip the single-precision MFMA and the vector ALU do not
// run side by side, so the rate with NV > 0 is what a kernel with that instruction mix can reach at best.
typedef float probe_f32x4 __attribute__((ext_vector_type(4)));
constexpr int PROBE_MFMAS = 23;
template <int NV, int V = 0> __device__ __forceinline__ void probe_products(float (&p)[NV > 0 ? NV : 1], float a)
{
    if constexpr (V < NV) {
        // a times the value of the lane V+1 places to the left in its row of 16 (row rotate)
        p[V] = a * __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0x121 + V, 0xf, 0xf, false));
        probe_products<NV, V + 1>(p, a);
    }
}
template <int NV>
__global__ __launch_bounds__(512) void probe_mfma_kernel(float *__restrict__ sink, int iters)
{
    probe_f32x4 acc[PROBE_MFMAS];
#pragma unroll
    for (int i = 0; i < PROBE_MFMAS; ++i) acc[i] = (probe_f32x4){0.f, 0.f, 0.f, 0.f};
    float a = 1.f + 0.001f * (float)threadIdx.x, b = 0.5f;
    float p[NV > 0 ? NV : 1];
    p[0] = b;
    for (int it = 0; it < iters; ++it) {
        probe_products<NV>(p, a);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < PROBE_MFMAS; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, p[i % (NV > 0 ? NV : 1)], acc[i], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        a += 1e-9f;                                   // keeps the products inside the loop
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PROBE_MFMAS; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace st

using namespace st;

extern "C" {

__attribute__((visibility("default"))) st_status st_probe_empty(int grid, int block, void *stream)
{
    if (grid < 1 || block < 1 || block > 1024) return ST_ERR_SHAPE;
    hipLaunchKernelGGL(probe_empty_kernel, dim3((unsigned)grid), dim3((unsigned)block), 0, (hipStream_t)stream,
                       (float *)nullptr);
    return launch_status();
}

__attribute__((visibility("default"))) st_status st_probe_stream(const void *src, size_t bytes, int grid, int block,
                                                                 float *sink, void *stream)
{
    if (!src || !sink) return ST_ERR_NULL;
    if (grid < 1 || block < 1 || block > 1024 || bytes < 16) return ST_ERR_SHAPE;
    if (!aligned16(src)) return ST_ERR_ALIGN;
    const size_t n16 = bytes / 16, threads = (size_t)grid * (size_t)block, per = (n16 + threads - 1) / threads;
#define ST_PROBE_CASE(P)                                                                                     \
    if (per <= P) {                                                                                          \
        hipLaunchKernelGGL(probe_stream_kernel<P>, dim3((unsigned)grid), dim3((unsigned)block), 0,           \
                           (hipStream_t)stream, (const float4 *)src, n16, sink);                             \
        return launch_status();                                                                              \
    }
    ST_PROBE_CASE(1) ST_PROBE_CASE(2) ST_PROBE_CASE(3) ST_PROBE_CASE(4) ST_PROBE_CASE(6) ST_PROBE_CASE(8)
    ST_PROBE_CASE(12) ST_PROBE_CASE(16) ST_PROBE_CASE(24) ST_PROBE_CASE(32)
#undef ST_PROBE_CASE
    return ST_ERR_UNSUPPORTED;          /* more than 32 loads per thread: use a larger grid */
}

__attribute__((visibility("default"))) st_status st_probe_mfma_f32(int valu, int iters, float *sink, void *stream)
{
    if (!sink) return ST_ERR_NULL;
    if (iters < 1 || (valu != 0 && valu != 9 && valu != 13)) return ST_ERR_SHAPE;
    if (valu == 0) hipLaunchKernelGGL(probe_mfma_kernel<0>, dim3(256), dim3(512), 0, (hipStream_t)stream, sink, iters);
    else if (valu == 9) hipLaunchKernelGGL(probe_mfma_kernel<9>, dim3(256), dim3(512), 0, (hipStream_t)stream, sink, iters);
    else hipLaunchKernelGGL(probe_mfma_kernel<13>, dim3(256), dim3(512), 0, (hipStream_t)stream, sink, iters);
    return launch_status();
}

}  // extern "C"
