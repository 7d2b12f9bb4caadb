// Shared host-side helpers of the library: launch declarations and checks.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/structtensor.h"

// Two statements the kernels use to steer the compiler, as macros so that a build of the kernel sources for
// another target can give them its own meaning (the CPU bounds-check build of the tests defines both as nothing):
// ST_PIN_VGPR(x): an empty statement the compiler cannot see through, which pins x in a vector register here;
// ST_WAIT_STATES(n): n + 1 idle issue cycles.
#ifndef ST_PIN_VGPR
#define ST_PIN_VGPR(x) asm volatile("" : "+v"(x))
#endif
#ifndef ST_WAIT_STATES
#define ST_WAIT_STATES(n) asm volatile("s_nop " #n)
#endif

namespace st {

// Number of compute units of the current device (cached per device).
int num_cus();

// Raises the dynamic-LDS limit of `kernel` to `bytes` on the current device, once per device and kernel.
bool allow_dynamic_lds(const void *kernel, int bytes);

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool overlap(const void *a, size_t abytes, const void *b, size_t bbytes)
{
    uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}

inline st_status launch_status()
{
    return hipGetLastError() == hipSuccess ? ST_OK : ST_ERR_LAUNCH;
}

// Sum of a value over the 64 lanes of a wave, the same bits in every lane: four DPP steps inside the rows of 16,
// then the four row sums through scalar registers, in a fixed order.
template <int CTRL> __device__ __forceinline__ float wave_dpp(float v)
{
    return __builtin_bit_cast(float,
                              __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float wave_sum(float v)
{
    v += wave_dpp<0xB1>(v);     // quad_perm [1,0,3,2]
    v += wave_dpp<0x4E>(v);     // quad_perm [2,3,0,1]
    v += wave_dpp<0x141>(v);    // row_half_mirror
    v += wave_dpp<0x140>(v);    // row_mirror
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return (r0 + r1) + (r2 + r3);
}

// ---- launchers (one translation unit per kernel family) -------------------
st_status launch_unrank(int kind, int64_t n, int64_t w, int64_t p0, int64_t count, int32_t *out,
                        hipStream_t s);
st_status launch_expand(const float *Sc, float *S, int n, int order, hipStream_t s);

size_t batax_workspace(int n);
st_status launch_batax(const float *Ap, const float *x, float *y, int n, float beta, void *ws,
                       hipStream_t s);

// partial results in a static device array of the library (for callers that cannot allocate)
int batax_static_max_n();
st_status launch_batax_static(const float *Ap, const float *x, float *y, int n, float beta, hipStream_t s);

size_t ttm_workspace(int n, int w, int nl, int R);
st_status launch_ttm(const float *Tc, const float *U, float *Yc, int64_t rows, int nl, int R,
                     void *ws, hipStream_t s);

size_t moment3_workspace(int64_t N, int n);
st_status launch_moment3(const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws,
                         hipStream_t s);

size_t moment2_workspace(int64_t N, int n);
st_status launch_moment2(const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws,
                         hipStream_t s);

size_t moment4_workspace(int64_t N, int n);
st_status launch_moment4(const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws,
                         hipStream_t s);

// third / fourth moment on the matrix cores for up to 256 features (st_moment_mfma.hip)
bool moment_mfma_wins(int order, int n);
size_t moment_mfma_workspace(int order, int64_t N, int n);
st_status launch_moment_mfma(int order, const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws,
                             hipStream_t s);

// all three covariance terms in one pass for at most six features (st_covar_small.hip)
bool covar_small_applies(int n);
size_t covar_small_workspace(int64_t N, int n);
st_status launch_covar_small(const float *X, int64_t N, int n, float *S1, float *S2, float *S3, int accumulate,
                             void *ws, hipStream_t s);

size_t mttkrp_workspace(int n, int R);
st_status launch_mttkrp(const float *Tc, const float *B, float *M, int n, int R, void *ws,
                        hipStream_t s);

// the kernel table's sparsity structures (diagonal plane, fixed index, upper half cube)
st_status launch_thp(int structure, const float *Bc, const float *C, float *Ac, int64_t pairs, int nj, int nl,
                     int fixed, hipStream_t s);
size_t mttkrp_fixed_workspace(int kind, int ni, int nk, int nl, int R);
st_status launch_mttkrp_fixed(int kind, const float *Bc, const float *C, const float *D, float *A, int ni, int nk,
                              int nl, int R, int fixed_k, void *ws, hipStream_t s);
st_status launch_expand_band(const float *Tc, float *T, int n, int w, int nl, hipStream_t s);

}  // namespace st
