// Shared host-side helpers of the library: launch declarations and checks.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/structtensor.h"

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

// ---- launchers (one translation unit per kernel family) -------------------
st_status launch_unrank(int kind, int64_t n, int64_t w, int64_t p0, int64_t count, int32_t *out,
                        hipStream_t s);
st_status launch_expand(const float *Sc, float *S, int n, int order, hipStream_t s);

size_t batax_workspace(int n);
st_status launch_batax(const float *Ap, const float *x, float *y, int n, float beta, void *ws,
                       hipStream_t s);

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
