// The three covariance terms of degree-2 polynomial regression in ONE pass over the samples,
// for at most six features (the smaller of the paper's two end-to-end data sets has six):
//     S1(i,j) (+)= sum_s x_i x_j,   S2(i,j,k) (+)= sum_s x_i x_j x_k,   S3(i,j,k,l) (+)= sum_s x_i x_j x_k x_l
// over the unique sets i <= j (<= k (<= l)).  All 21 + 56 + 126 unique entries of n = 6 fit a
// lane's registers, so a lane takes whole samples (a wave reads 64 consecutive rows, every byte
// of them used) and walks the nest  for i, for j = i, for k = j, for l = k  with the running
// products x_i x_j and x_i x_j x_k shared by the inner loops.  Nothing is shared between lanes
// until the end: the lanes of a wave, then the four waves of a workgroup, are added in a fixed
// order; workgroup partials -> reduce kernel (fixed order, no atomics).  Bound by the HBM stream.
#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;

constexpr int CS_NMAX = 6;
constexpr int CS_WGS = 512;                       // workgroups at most: one round at two waves per SIMD

template <int NP> struct CsCounts {
    static constexpr int A2 = NP * (NP + 1) / 2, A3 = NP * (NP + 1) * (NP + 2) / 6,
                         A4 = NP * (NP + 1) * (NP + 2) * (NP + 3) / 24, ALL = A2 + A3 + A4;
};

template <int NP>
__global__ __launch_bounds__(256) void covar_small_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                         float *__restrict__ ws)
{
    typedef CsCounts<NP> C;
    __shared__ float red[4][C::ALL];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    float acc[C::ALL];
#pragma unroll
    for (int a = 0; a < C::ALL; ++a) acc[a] = 0.f;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t s = (int64_t)blockIdx.x * 256 + tid; s < N; s += stride) {
        const float *row = X + s * (int64_t)n;
        float x[NP];
#pragma unroll
        for (int c = 0; c < NP; ++c) x[c] = (u32)c < n ? row[c] : 0.f;
        int a2 = 0, a3 = C::A2, a4 = C::A2 + C::A3;      // packed (lexicographic) order inside each term
#pragma unroll
        for (int i = 0; i < NP; ++i)
#pragma unroll
            for (int j = i; j < NP; ++j) {
                const float pij = x[i] * x[j];
                acc[a2++] += pij;
#pragma unroll
                for (int k = j; k < NP; ++k) {
                    const float pijk = pij * x[k];
                    acc[a3++] += pijk;
#pragma unroll
                    for (int l = k; l < NP; ++l) acc[a4++] += pijk * x[l];
                }
            }
    }
    // lanes of the wave (DPP steps, every lane ends with the sum), then the four waves
#pragma unroll
    for (int a = 0; a < C::ALL; ++a) {
        const float v = wave_sum(acc[a]);
        if (lane == 0u) red[wave][a] = v;
    }
    __syncthreads();
    for (u32 a = tid; a < (u32)C::ALL; a += 256u)
        ws[(size_t)blockIdx.x * C::ALL + a] = (red[0][a] + red[1][a]) + (red[2][a] + red[3][a]);
}

// 16 accumulators x 16 groups of workgroup partials per block; keeps the entries with every index < n
__global__ __launch_bounds__(256) void covar_small_reduce_kernel(const float *__restrict__ ws, u32 G, u32 n, u32 np,
                                                                float *__restrict__ S1, float *__restrict__ S2,
                                                                float *__restrict__ S3, int accumulate)
{
    __shared__ float part[16][16];
    const u32 a = threadIdx.x & 15u, g = threadIdx.x >> 4;
    const u32 a2 = count_sym2<u32>(np), a3 = count_sym3<u32>(np), a4 = count_sym4<u32>(np), all = a2 + a3 + a4;
    const u32 t = blockIdx.x * 16u + a;
    float s = 0.f;
    if (t < all) {
        const u32 per = (G + 15u) / 16u, y0 = min(G, g * per), y1 = min(G, y0 + per);
        for (u32 y = y0; y < y1; ++y) s += ws[(size_t)y * all + t];
    }
    part[g][a] = s;
    __syncthreads();
    if (g != 0u || t >= all) return;
    s = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) s += part[q][a];
    u32 i, j, k, l;
    if (t < a2) {
        unrank_sym2<u32>(np, t, i, j);
        if (j >= n) return;
        const u32 p = rank_sym2<u32>(n, i, j);
        S1[p] = accumulate ? S1[p] + s : s;
    } else if (t < a2 + a3) {
        unrank_sym3<u32>(np, t - a2, i, j, k);
        if (k >= n) return;
        const u32 p = rank_sym3<u32>(n, i, j, k);
        S2[p] = accumulate ? S2[p] + s : s;
    } else {
        unrank_sym4<u32>(np, t - a2 - a3, i, j, k, l);
        if (l >= n) return;
        const u32 p = rank_sym4<u32>(n, i, j, k, l);
        S3[p] = accumulate ? S3[p] + s : s;
    }
}

static inline u32 cs_groups(int64_t N)
{
    const int64_t g = (N + 255) / 256;
    return (u32)(g < 1 ? 1 : g > CS_WGS ? CS_WGS : g);
}
static inline u32 cs_np(int n) { return n <= 4 ? 4u : 6u; }

bool covar_small_applies(int n) { return n >= 1 && n <= CS_NMAX; }

size_t covar_small_workspace(int64_t N, int n)
{
    if (N <= 0) return 0;
    const u32 np = cs_np(n);
    return (size_t)cs_groups(N) * (count_sym2<u32>(np) + count_sym3<u32>(np) + count_sym4<u32>(np)) * sizeof(float);
}

// N >= 1
st_status launch_covar_small(const float *X, int64_t N, int n, float *S1, float *S2, float *S3, int accumulate,
                             void *ws, hipStream_t s)
{
    const u32 G = cs_groups(N), np = cs_np(n);
    float *wsf = static_cast<float *>(ws);
    if (np == 4u) hipLaunchKernelGGL(covar_small_kernel<4>, dim3(G), dim3(256), 0, s, X, N, (u32)n, wsf);
    else hipLaunchKernelGGL(covar_small_kernel<6>, dim3(G), dim3(256), 0, s, X, N, (u32)n, wsf);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    const u32 all = count_sym2<u32>(np) + count_sym3<u32>(np) + count_sym4<u32>(np);
    hipLaunchKernelGGL(covar_small_reduce_kernel, dim3((all + 15u) / 16u), dim3(256), 0, s, wsf, G, (u32)n, np, S1, S2,
                       S3, accumulate);
    return launch_status();
}

}  // namespace st
