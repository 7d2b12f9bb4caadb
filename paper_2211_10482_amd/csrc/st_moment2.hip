// Second-moment accumulation over N samples, unique entries only:
//     Sc(rank2(i,j)) (+)= sum_s X(s,i) X(s,j)      for i <= j
// (the M1 = f (x) f term of the degree-2 polynomial-regression covariance, summed
// over the data; the structure is plain symmetry, the upper half is kept).
//
// MFMA path (n <= 64).  The sample sum is the dense contraction S = X^T X on the fp32
// matrix cores (v_mfma_f32_16x16x4_f32).  The 64 indices are split into four groups
// g = i mod 4, so one 16-byte load per lane -- lane (m, q) reads X(s+q, 4m .. 4m+3),
// a wave reads four whole rows, 1 KB contiguous -- is at once the A operand of the
// row group and the B operand of the column group of every tile: tile (ga, gb),
// ga <= gb, holds S(4m+ga, 4m'+gb) for all m, m', and the 10 tiles cover every
// unordered pair exactly once (a tile with ga = gb holds its pairs twice, the copy
// with m > m' is dropped).  A wave owns all 10 tiles (40 accumulator registers) and
// streams its own samples straight from HBM with eight loads in flight; nothing goes
// through LDS until the end, when the 8 waves of a workgroup add their tiles in a
// fixed tree.  Workgroup partials -> second kernel adds them in a fixed order and
// scatters through rank2.  No float atomics.
//
// Algorithmic traffic: 4n bytes per sample, read once.  At n = 64 the matrix cores
// need 10 MFMAs per four samples, about the same time as the HBM stream.
//
// General path (n > 64): one thread per unique entry and sample slice.
#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;
typedef float f32x4 __attribute__((ext_vector_type(4)));

#ifndef ST_M2_WAVES
#define ST_M2_WAVES 8
#endif
constexpr int M2_WAVES = ST_M2_WAVES;             // 8 or 16
constexpr int M2_THREADS = M2_WAVES * 64;
constexpr int M2_TILES = 10;                      // group pairs ga <= gb
constexpr int M2_ACC = M2_TILES * 256;            // accumulators per wave / workgroup
#ifndef ST_M2_DEPTH
#define ST_M2_DEPTH 8
#endif
#ifndef ST_M2_GMAX
#define ST_M2_GMAX 256
#endif
constexpr int M2_DEPTH = ST_M2_DEPTH;             // loads in flight per lane
constexpr int M2_GMAX = ST_M2_GMAX;               // workgroups (one per CU measured best)

// tile t = 0..9 <-> (ga, gb), ga <= gb, row-major over the upper triangle of 4 x 4
__host__ __device__ constexpr int m2_ga(int t) { return t < 4 ? 0 : t < 7 ? 1 : t < 9 ? 2 : 3; }
__host__ __device__ constexpr int m2_gb(int t) { return t < 4 ? t : t < 7 ? t - 3 : t < 9 ? t - 5 : 3; }

// Four samples s .. s+3 for this lane's row q = lane/16, columns 4m .. 4m+3 (m = lane%16).
// Unconditional (row clamped); mask_quad zeroes what lies outside.
template <bool FULL>
__device__ __forceinline__ f32x4 load_quad(const float *__restrict__ X, int64_t s, int64_t N, u32 n, u32 lane)
{
    const u32 m = lane & 15u, q = lane >> 4;
    const int64_t r = s + q < N ? s + q : N - 1;
    if constexpr (FULL) {
        const float4 t = *reinterpret_cast<const float4 *>(X + r * 64 + 4u * m);
        return (f32x4){t.x, t.y, t.z, t.w};
    } else {
        const float *row = X + r * (int64_t)n;
        f32x4 v;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) v[g] = row[4u * m + g < n ? 4u * m + g : n - 1u];
        return v;
    }
}

template <bool FULL>
__device__ __forceinline__ f32x4 mask_quad(f32x4 v, int64_t s, int64_t N, u32 n, u32 lane)
{
    const u32 m = lane & 15u, q = lane >> 4;
    const bool row_ok = s + q < N;
#pragma unroll
    for (u32 g = 0; g < 4; ++g) {
        const bool ok = row_ok && (FULL || 4u * m + g < n);
        v[g] = ok ? v[g] : 0.f;
    }
    return v;
}

__device__ __forceinline__ void m2_step(f32x4 (&acc)[M2_TILES], const f32x4 &x)
{
#pragma unroll
    for (int t = 0; t < M2_TILES; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[m2_ga(t)], x[m2_gb(t)], acc[t], 0, 0, 0);
}

// Sample quads are dealt to the waves of the whole grid round-robin: quad index
// w + k * (waves in the grid), so neighbouring waves stream neighbouring kilobytes.
template <bool FULL>
__global__ __launch_bounds__(M2_THREADS) void moment2_mfma_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                                float *__restrict__ ws)
{
    __shared__ __attribute__((aligned(16))) float red[M2_WAVES / 2][M2_ACC];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const int64_t nquads = (N + 3) / 4;
    const int64_t stride = (int64_t)gridDim.x * M2_WAVES;
    const int64_t first = (int64_t)blockIdx.x * M2_WAVES + wave;
    const int64_t mine = first < nquads ? (nquads - first + stride - 1) / stride : 0;   // quads of this wave

    f32x4 acc[M2_TILES];
#pragma unroll
    for (int t = 0; t < M2_TILES; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // ring of M2_DEPTH loads: quads past the end are clamped loads of the last row and masked
    f32x4 ring[M2_DEPTH];
#pragma unroll
    for (int d = 0; d < M2_DEPTH; ++d) ring[d] = load_quad<FULL>(X, 4 * (first + d * stride), N, n, lane);
    for (int64_t k = 0; k < mine; k += M2_DEPTH) {
#pragma unroll
        for (int d = 0; d < M2_DEPTH; ++d) {
            const int64_t s = 4 * (first + (k + d) * stride);
            const f32x4 x = mask_quad<FULL>(ring[d], s, N, n, lane);
            ring[d] = load_quad<FULL>(X, s + 4 * M2_DEPTH * stride, N, n, lane);
            __builtin_amdgcn_sched_barrier(0);
            m2_step(acc, x);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // fixed tree over the waves: upper half -> lower half, repeatedly (8 waves: 4..7 -> 0..3,
    // then 2,3 -> 0,1, then 1 -> 0)
#pragma unroll
    for (u32 half = M2_WAVES / 2; half >= 1; half >>= 1) {
        if (wave >= half && wave < 2 * half) {
            float *dst = &red[wave - half][lane];
#pragma unroll
            for (int t = 0; t < M2_TILES; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) dst[(t * 4 + v) * 64] = acc[t][v];
        }
        __syncthreads();
        if (wave < half) {
            const float *src = &red[wave][lane];
#pragma unroll
            for (int t = 0; t < M2_TILES; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[t][v] += src[(t * 4 + v) * 64];
        }
        __syncthreads();
    }
    if (wave == 0) {
        float *dst = ws + (size_t)blockIdx.x * M2_ACC + lane;
#pragma unroll
        for (int t = 0; t < M2_TILES; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) dst[(t * 4 + v) * 64] = acc[t][v];
    }
}

// Adds the G workgroup partials and scatters the unique ones.  A block owns 64 raw
// accumulators and cuts the partials into 4 slices (g ascending inside a slice, slices
// ascending).
__global__ __launch_bounds__(256) void moment2_reduce_kernel(const float *__restrict__ ws, u32 G, u32 n,
                                                            float *__restrict__ Sc, int accumulate)
{
    __shared__ float accs[4][64];
    const u32 lane = threadIdx.x & 63u, sl = threadIdx.x >> 6;
    const u32 e = blockIdx.x * 64u + lane;        // raw accumulator id, < M2_ACC
    const u32 tile = e >> 8, v = (e >> 6) & 3u;
    const u32 ga = (u32)m2_ga((int)tile), gb = (u32)m2_gb((int)tile);
    // D layout of the 16x16 MFMA: lane holds column lane%16 of rows 4*(lane/16) + v
    const u32 mrow = 4u * (lane >> 4) + v, mcol = lane & 15u;
    const u32 i = 4u * mrow + ga, j = 4u * mcol + gb;
    const bool keep = (ga != gb || mrow <= mcol) && i < n && j < n;
    float s = 0.f;
    if (keep) {
        const u32 per = (G + 3u) / 4u, g0 = min(G, sl * per), g1 = min(G, g0 + per);
        const float *src = ws + e;
#pragma unroll 8
        for (u32 g = g0; g < g1; ++g) s += src[(size_t)g * M2_ACC];
    }
    accs[sl][lane] = s;
    __syncthreads();
    if (sl == 0 && keep) {
        s = (accs[0][lane] + accs[1][lane]) + (accs[2][lane] + accs[3][lane]);
        const u32 p = rank_sym2<u32>(n, min(i, j), max(i, j));
        Sc[p] = accumulate ? Sc[p] + s : s;
    }
}

// ---- general path -----------------------------------------------------------------
__global__ __launch_bounds__(256) void moment2_plain_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                           u32 count, int64_t slice,
                                                           float *__restrict__ part)
{
    u32 p = blockIdx.x * 256u + threadIdx.x;
    if (p >= count) return;
    u32 i, j;
    unrank_sym2<u32>(n, p, i, j);
    int64_t s0 = (int64_t)blockIdx.y * slice, s1 = s0 + slice < N ? s0 + slice : N;
    float s = 0.f;
    for (int64_t q = s0; q < s1; ++q) {
        const float *row = X + q * (int64_t)n;
        s += row[i] * row[j];
    }
    part[(size_t)blockIdx.y * count + p] = s;
}

__global__ __launch_bounds__(256) void moment2_plain_reduce_kernel(const float *__restrict__ part, u32 SY,
                                                                  u32 count, float *__restrict__ Sc,
                                                                  int accumulate)
{
    u32 p = blockIdx.x * 256u + threadIdx.x;
    if (p >= count) return;
    float s = 0.f;
    for (u32 y = 0; y < SY; ++y) s += part[(size_t)y * count + p];
    Sc[p] = accumulate ? Sc[p] + s : s;
}

__global__ __launch_bounds__(256) void moment2_zero_kernel(float *__restrict__ p, u32 count)
{
    u32 t = blockIdx.x * 256u + threadIdx.x;
    if (t < count) p[t] = 0.f;
}

static inline u32 m2_groups(int64_t N)
{
    // at least M2_DEPTH quads per wave, at most M2_GMAX workgroups
    int64_t quads = (N + 3) / 4, g = (quads + (int64_t)M2_WAVES * M2_DEPTH - 1) / ((int64_t)M2_WAVES * M2_DEPTH);
    return (u32)(g < 1 ? 1 : g > M2_GMAX ? M2_GMAX : g);
}
static inline u32 m2_plain_slices(int64_t N, int n)
{
    // up to 64 sample slices, fewer when the partials would exceed 64 M values
    int64_t s = (N + 1023) / 1024, cap = ((int64_t)64 << 20) / count_sym2<int64_t>(n);
    if (s > 64) s = 64;
    if (s > cap) s = cap;
    return (u32)(s < 1 ? 1 : s);
}

size_t moment2_workspace(int64_t N, int n)
{
    if (N == 0) return 0;
    if (n <= 64) return (size_t)m2_groups(N) * M2_ACC * sizeof(float);
    return (size_t)m2_plain_slices(N, n) * (size_t)count_sym2<int64_t>(n) * sizeof(float);
}

st_status launch_moment2(const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws, hipStream_t s)
{
    u32 count = (u32)count_sym2<int64_t>(n);
    if (N == 0) {
        if (!accumulate)
            hipLaunchKernelGGL(moment2_zero_kernel, dim3((count + 255u) / 256u), dim3(256), 0, s, Sc, count);
        return launch_status();
    }
    float *wsf = static_cast<float *>(ws);
    if (n <= 64) {
        u32 G = m2_groups(N);
        if (n == 64)
            hipLaunchKernelGGL(moment2_mfma_kernel<true>, dim3(G), dim3(M2_THREADS), 0, s, X, N, (u32)n, wsf);
        else
            hipLaunchKernelGGL(moment2_mfma_kernel<false>, dim3(G), dim3(M2_THREADS), 0, s, X, N, (u32)n, wsf);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment2_reduce_kernel, dim3(M2_ACC / 64), dim3(256), 0, s, wsf, G, (u32)n, Sc,
                           accumulate);
        return launch_status();
    }
    u32 SY = m2_plain_slices(N, n);
    int64_t slice = (N + SY - 1) / SY;
    hipLaunchKernelGGL(moment2_plain_kernel, dim3((count + 255u) / 256u, SY), dim3(256), 0, s, X, N, (u32)n, count,
                       slice, wsf);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    hipLaunchKernelGGL(moment2_plain_reduce_kernel, dim3((count + 255u) / 256u), dim3(256), 0, s, wsf, SY, count,
                       Sc, accumulate);
    return launch_status();
}

}  // namespace st
