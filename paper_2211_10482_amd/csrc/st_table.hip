// The other sparsity structures of the paper's kernel table (TTM, THP, MTTKRP with a
// diagonal-plane, fixed-index or upper-half-cube operand B), on packed operands.
//
// In packed storage a structure on the index pair (i,j) of B(i,j,l) is nothing but an
// enumeration p -> (i(p), j(p)) of the non-zero fibres B(i,j,:), so
//   * TTM  A(i,j,k) = sum_l B(i,j,l) C(k,l)  is one dense [pairs x nl] . [nl x R]
//     contraction whatever the structure (st_ttm_pairs runs the kernels of st_ttm.hip);
//   * THP  A(i,j,k) = B(i,j,k) C(i,j,k)  streams the packed fibres of B once and gathers
//     the matching fibres of the dense C (HBM bound, 16-byte accesses along l);
//   * MTTKRP  A(i,r) = sum_{k,l} B(i,k,l) C(k,r) D(l,r)  with a fixed index of B
//     collapses to a contraction over l followed by a scaling or a weighted column sum:
//       k = K fixed :  A(i,r) = C(K,r) * sum_l B(i,K,l) D(l,r)         [ni x nl] . [nl x R]
//       i = I fixed :  A(I,r) = sum_k C(k,r) * (sum_l B(I,k,l) D(l,r)) [nk x nl] . [nl x R], then a
//                      weighted column sum in a fixed order
//       both fixed  :  A(I,r) = C(K,r) * sum_l B(I,K,l) D(l,r)
//     The contractions over l run on the matrix cores through the TTM kernels.
// Also here: the zero-filled dense form of a packed band tensor.
#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;

// (i, j) of packed pair p under structure `st` (the enum of structtensor.h)
__device__ __forceinline__ void pair_of(int st, u32 p, u32 nj, u32 fixed, u32 &i, u32 &j)
{
    if (st == ST_STRUCT_DIAG) { i = p; j = p; }
    else if (st == ST_STRUCT_FIXED_I) { i = fixed; j = p; }
    else if (st == ST_STRUCT_FIXED_J) { i = p; j = fixed; }
    else unrank_sym2<u32>(nj, p, i, j);          // upper half cube: sym2 order, square pair
}

// one thread per group of four l of one packed fibre (VEC) or per element
template <bool VEC>
__global__ __launch_bounds__(256) void thp_kernel(int st, const float *__restrict__ Bc,
                                                  const float *__restrict__ C, float *__restrict__ Ac,
                                                  u32 pairs, u32 nj, u32 nl, u32 fixed)
{
    const u32 per = VEC ? nl / 4u : nl;
    const uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (t >= (uint64_t)pairs * per) return;
    const u32 p = (u32)(t / per), q = (u32)(t - (uint64_t)p * per);
    u32 i, j;
    pair_of(st, p, nj, fixed, i, j);
    const size_t cbase = ((size_t)i * nj + j) * nl, bbase = (size_t)p * nl;
    if constexpr (VEC) {
        const float4 b = *reinterpret_cast<const float4 *>(Bc + bbase + 4u * q);
        const float4 c = *reinterpret_cast<const float4 *>(C + cbase + 4u * q);
        *reinterpret_cast<float4 *>(Ac + bbase + 4u * q) = make_float4(b.x * c.x, b.y * c.y, b.z * c.z, b.w * c.w);
    } else {
        Ac[bbase + q] = Bc[bbase + q] * C[cbase + q];
    }
}

st_status launch_thp(int st, const float *Bc, const float *C, float *Ac, int64_t pairs, int nj, int nl, int fixed,
                     hipStream_t s)
{
    if (pairs == 0) return ST_OK;
    const bool vec = nl % 4 == 0;
    const uint64_t threads = (uint64_t)pairs * (vec ? nl / 4 : nl);
    const uint64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffull) return ST_ERR_UNSUPPORTED;
    if (vec)
        hipLaunchKernelGGL(thp_kernel<true>, dim3((u32)blocks), dim3(256), 0, s, st, Bc, C, Ac, (u32)pairs, (u32)nj,
                           (u32)nl, (u32)fixed);
    else
        hipLaunchKernelGGL(thp_kernel<false>, dim3((u32)blocks), dim3(256), 0, s, st, Bc, C, Ac, (u32)pairs,
                           (u32)nj, (u32)nl, (u32)fixed);
    return launch_status();
}

// ---- MTTKRP with fixed indices of B ---------------------------------------------------------
// Dk(l,r) = D(l,r) * C(K,r)
__global__ __launch_bounds__(256) void scale_columns_kernel(const float *__restrict__ D, const float *__restrict__ crow,
                                                           float *__restrict__ out, u32 nl, u32 R)
{
    const u32 t = blockIdx.x * 256u + threadIdx.x;
    if (t >= nl * R) return;
    out[t] = D[t] * crow[t % R];
}

// a(r) = sum_k C(k,r) T(k,r): a block owns 32 columns and cuts k into 8 slices (k ascending
// inside a slice, slices ascending)
__global__ __launch_bounds__(256) void weighted_colsum_kernel(const float *__restrict__ T, const float *__restrict__ C,
                                                             float *__restrict__ a, u32 nk, u32 R)
{
    __shared__ float part[8][32];
    const u32 o = threadIdx.x & 31u, sl = threadIdx.x >> 5;
    const u32 r = blockIdx.x * 32u + o;
    float s = 0.f;
    if (r < R) {
        const u32 per = (nk + 7u) / 8u, k0 = min(nk, sl * per), k1 = min(nk, k0 + per);
        for (u32 k = k0; k < k1; ++k) s += C[(size_t)k * R + r] * T[(size_t)k * R + r];
    }
    part[sl][o] = s;
    __syncthreads();
    if (sl == 0 && r < R) {
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) v += part[q][o];
        a[r] = v;
    }
}

// a(r) = C(K,r) * sum_l b(l) D(l,r): one thread per column
__global__ __launch_bounds__(256) void fibre_kernel(const float *__restrict__ b, const float *__restrict__ crow,
                                                   const float *__restrict__ D, float *__restrict__ a, u32 nl, u32 R)
{
    const u32 r = blockIdx.x * 256u + threadIdx.x;
    if (r >= R) return;
    float s = 0.f;
    for (u32 l = 0; l < nl; ++l) s += b[l] * D[(size_t)l * R + r];
    a[r] = crow[r] * s;
}

size_t mttkrp_fixed_workspace(int kind, int ni, int nk, int nl, int R)
{
    (void)ni;
    if (kind == ST_MTTKRP_FIXED_K) return (size_t)nl * R * sizeof(float);       // D scaled by the row of C
    if (kind == ST_MTTKRP_FIXED_I) return (size_t)nk * R * sizeof(float);       // the contraction over l
    return 0;
}

st_status launch_mttkrp_fixed(int kind, const float *Bc, const float *C, const float *D, float *Ac, int ni, int nk,
                              int nl, int R, int fixed_k, void *ws, hipStream_t s)
{
    float *wsf = static_cast<float *>(ws);
    if (kind == ST_MTTKRP_FIXED_K) {
        const u32 total = (u32)nl * (u32)R;
        hipLaunchKernelGGL(scale_columns_kernel, dim3((total + 255u) / 256u), dim3(256), 0, s, D,
                           C + (size_t)fixed_k * R, wsf, (u32)nl, (u32)R);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        return launch_ttm(Bc, wsf, Ac, ni, nl, R, nullptr, s);
    }
    if (kind == ST_MTTKRP_FIXED_I) {
        st_status rc = launch_ttm(Bc, D, wsf, nk, nl, R, nullptr, s);
        if (rc != ST_OK) return rc;
        hipLaunchKernelGGL(weighted_colsum_kernel, dim3(((u32)R + 31u) / 32u), dim3(256), 0, s, wsf, C, Ac, (u32)nk,
                           (u32)R);
        return launch_status();
    }
    hipLaunchKernelGGL(fibre_kernel, dim3(((u32)R + 255u) / 256u), dim3(256), 0, s, Bc, C + (size_t)fixed_k * R, D, Ac,
                       (u32)nl, (u32)R);
    return launch_status();
}

// ---- zero-filled dense form of a packed band tensor -----------------------------------------
// one thread per group of four l (VEC) or per element of the dense n x n x nl output
template <bool VEC>
__global__ __launch_bounds__(256) void expand_band_kernel(const float *__restrict__ Tc, float *__restrict__ T, u32 n,
                                                          u32 w, u32 nl)
{
    const u32 per = VEC ? nl / 4u : nl;
    const uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (t >= (uint64_t)n * n * per) return;
    const u32 ij = (u32)(t / per), q = (u32)(t - (uint64_t)ij * per);
    const u32 i = ij / n, j = ij - i * n;
    const bool in = (i > j ? i - j : j - i) <= w;
    const size_t src = in ? (size_t)rank_band<u32>(n, w, i, j) * nl : 0;
    if constexpr (VEC) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (in) v = *reinterpret_cast<const float4 *>(Tc + src + 4u * q);
        *reinterpret_cast<float4 *>(T + (size_t)ij * nl + 4u * q) = v;
    } else {
        T[(size_t)ij * nl + q] = in ? Tc[src + q] : 0.f;
    }
}

st_status launch_expand_band(const float *Tc, float *T, int n, int w, int nl, hipStream_t s)
{
    const bool vec = nl % 4 == 0;
    const uint64_t threads = (uint64_t)n * n * (vec ? nl / 4 : nl);
    const uint64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffull) return ST_ERR_UNSUPPORTED;
    const u32 wc = (u32)(w > n - 1 ? n - 1 : w);
    if (vec)
        hipLaunchKernelGGL(expand_band_kernel<true>, dim3((u32)blocks), dim3(256), 0, s, Tc, T, (u32)n, wc, (u32)nl);
    else
        hipLaunchKernelGGL(expand_band_kernel<false>, dim3((u32)blocks), dim3(256), 0, s, Tc, T, (u32)n, wc, (u32)nl);
    return launch_status();
}

}  // namespace st
