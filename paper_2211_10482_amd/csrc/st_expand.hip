// Reconstruction through the redundancy map, and the device index-map check.
//
// expand: T(x) = T_C(x) + T_R(x,x') * T_C(x')  (Property 5).  For a symmetric
// structure the redundancy map sends an index tuple to its ascending sort
// (class S: i' = j, j' = i for j < i; order 3 likewise), so each thread owns
// four consecutive DENSE outputs (one 16-byte store), sorts the indices of
// each, ranks the sorted tuple in closed form and gathers from the packed
// array (which is small and cache resident).  HBM-bound on the dense write.
#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;

__device__ __forceinline__ void sort3(u32 &a, u32 &b, u32 &c)
{
    u32 lo = min(a, b), hi = max(a, b);
    u32 mn = min(lo, c), mx = max(hi, c);
    u32 md = max(lo, min(hi, c));
    a = mn; b = md; c = mx;
}

// order 3: grid.x covers (i*n+j) pairs x k-quads
__global__ __launch_bounds__(256) void expand3_kernel(const float *__restrict__ Sc,
                                                      float *__restrict__ S, u32 n, u32 kq)
{
    u32 t = blockIdx.x * 256u + threadIdx.x;
    u32 nn = n * n;
    if (t >= nn * kq) return;
    u32 ij = t / kq, k0 = (t - ij * kq) * 4u;
    u32 i = ij / n, j = ij - i * n;
    float v[4];
#pragma unroll
    for (u32 e = 0; e < 4; ++e) {
        u32 k = k0 + e;
        u32 a = i, b = j, c = k < n ? k : n - 1;
        sort3(a, b, c);
        v[e] = Sc[rank_sym3<u32>(n, a, b, c)];
    }
    size_t o = (size_t)ij * n + k0;
    if ((n & 3u) == 0) {
        *reinterpret_cast<float4 *>(S + o) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (u32 e = 0; e < 4; ++e)
            if (k0 + e < n) S[o + e] = v[e];
    }
}

// order 4: one thread per l-quad of an (i,j,k) fibre; the three leading indices are sorted
// once, the fourth is inserted per output
__global__ __launch_bounds__(256) void expand4_kernel(const float *__restrict__ Sc,
                                                      float *__restrict__ S, u32 n, u32 lq)
{
    const uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    const uint64_t nnn = (uint64_t)n * n * n;
    if (t >= nnn * lq) return;
    const u32 ijk = (u32)(t / lq), l0 = (u32)(t - (uint64_t)ijk * lq) * 4u;
    const u32 i = ijk / (n * n), jk = ijk - i * n * n, j = jk / n, k = jk - j * n;
    u32 a = i, b = j, c = k;
    sort3(a, b, c);
    float v[4];
#pragma unroll
    for (u32 e = 0; e < 4; ++e) {
        const u32 l = l0 + e < n ? l0 + e : n - 1;
        // insert l into a <= b <= c
        const u32 q0 = min(a, l), r0 = max(a, l);
        const u32 q1 = min(b, r0), r1 = max(b, r0);
        const u32 q2 = min(c, r1), q3 = max(c, r1);
        v[e] = Sc[rank_sym4<u32>(n, q0, q1, q2, q3)];
    }
    const size_t o = (size_t)ijk * n + l0;
    if ((n & 3u) == 0) {
        *reinterpret_cast<float4 *>(S + o) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (u32 e = 0; e < 4; ++e)
            if (l0 + e < n) S[o + e] = v[e];
    }
}

// order 2: one thread per j-quad of a row
__global__ __launch_bounds__(256) void expand2_kernel(const float *__restrict__ Sc,
                                                      float *__restrict__ S, u32 n, u32 jq)
{
    u32 t = blockIdx.x * 256u + threadIdx.x;
    if (t >= n * jq) return;
    u32 i = t / jq, j0 = (t - i * jq) * 4u;
    float v[4];
#pragma unroll
    for (u32 e = 0; e < 4; ++e) {
        u32 j = j0 + e < n ? j0 + e : n - 1;
        u32 a = min(i, j), b = max(i, j);
        v[e] = Sc[rank_sym2<u32>(n, a, b)];
    }
    size_t o = (size_t)i * n + j0;
    if ((n & 3u) == 0) {
        *reinterpret_cast<float4 *>(S + o) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (u32 e = 0; e < 4; ++e)
            if (j0 + e < n) S[o + e] = v[e];
    }
}

st_status launch_expand(const float *Sc, float *S, int n, int order, hipStream_t s)
{
    u32 un = (u32)n, q = (un + 3u) / 4u;
    if (order == 4) {
        // n <= 256: every packed position (< 2^28) and 4*pent fit 32 bits
        uint64_t threads = (uint64_t)un * un * un * q;
        uint64_t blocks = (threads + 255) / 256;
        if (blocks > 0x7fffffffull) return ST_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(expand4_kernel, dim3((u32)blocks), dim3(256), 0, s, Sc, S, un, q);
    } else if (order == 3) {
        // n <= 2000: n*n*q < 2^32 and every packed position fits 32 bits
        uint64_t threads = (uint64_t)un * un * q;
        u32 blocks = (u32)((threads + 255) / 256);
        hipLaunchKernelGGL(expand3_kernel, dim3(blocks), dim3(256), 0, s, Sc, S, un, q);
    } else {
        uint64_t threads = (uint64_t)un * q;
        u32 blocks = (u32)((threads + 255) / 256);
        hipLaunchKernelGGL(expand2_kernel, dim3(blocks), dim3(256), 0, s, Sc, S, un, q);
    }
    return launch_status();
}

// ---- device evaluation of the inverse index maps ------------------------------
template <typename I>
__global__ __launch_bounds__(256) void unrank_kernel(int kind, I n, I w, I p0, int64_t count,
                                                     int32_t *__restrict__ out)
{
    int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= count) return;
    I p = p0 + (I)t;
    if (kind == 3) {
        I i, j, k;
        unrank_sym3<I>(n, p, i, j, k);
        out[3 * t] = (int32_t)i; out[3 * t + 1] = (int32_t)j; out[3 * t + 2] = (int32_t)k;
    } else if (kind == 5) {
        I i, j, k, l;
        unrank_sym4<I>(n, p, i, j, k, l);
        out[4 * t] = (int32_t)i; out[4 * t + 1] = (int32_t)j; out[4 * t + 2] = (int32_t)k; out[4 * t + 3] = (int32_t)l;
    } else {
        I i, j;
        if (kind == 2) unrank_sym2<I>(n, p, i, j); else unrank_band<I>(n, w, p, i, j);
        out[2 * t] = (int32_t)i; out[2 * t + 1] = (int32_t)j;
    }
}

st_status launch_unrank(int kind, int64_t n, int64_t w, int64_t p0, int64_t count, int32_t *out,
                        hipStream_t s)
{
    if (count > ((int64_t)1 << 31) * 200) return ST_ERR_UNSUPPORTED;
    u32 blocks = (u32)((count + 255) / 256);
    // 32-bit index arithmetic is what the kernels use; it is valid while every
    // intermediate (8*count+1 for sym2, 6*count for sym3, 24*count in fp64 and 4*count
    // in integers for sym4) stays below 2^32.
    bool small = (kind == 2 && n <= 20000) || (kind == 3 && n <= 1000) || (kind == 4 && n <= 20000 && w <= 20000) ||
                 (kind == 5 && n <= 256);
    if (small)
        hipLaunchKernelGGL(unrank_kernel<u32>, dim3(blocks), dim3(256), 0, s, kind, (u32)n,
                           (u32)(w > n ? n : w), (u32)p0, count, out);
    else
        hipLaunchKernelGGL(unrank_kernel<int64_t>, dim3(blocks), dim3(256), 0, s, kind, n, w, p0,
                           count, out);
    return launch_status();
}

}  // namespace st
