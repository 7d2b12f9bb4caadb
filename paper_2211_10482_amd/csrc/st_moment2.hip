// Second-moment accumulation over N samples, unique entries only:
//     Sc(rank2(i,j)) (+)= sum_s X(s,i) X(s,j)      for i <= j
// (the M1 = f (x) f term of the degree-2 polynomial-regression covariance, summed
// over the data; the structure is plain symmetry, the upper half is kept).
//
// MFMA path (16 < n <= 64; n <= 16: one lane per sample, further down).  The sample sum is the dense contraction S = X^T X on the fp32
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
// 64 < n <= 1024: strips of 64 columns on the matrix cores (strip path below; 128 < n < 180: 8 x 8 register
// tiles per lane on the vector ALUs, the tile path); larger n: one thread per unique entry and sample slice.
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
// Unconditional (row clamped, columns >= n clamped to ones that exist); mask_quad zeroes the rows
// past N, and what columns >= n bring only reaches accumulators the reduce kernel drops.
// MODE 0: n == 64; 1: n % 4 == 0 (aligned 16-byte loads, a piece is wholly inside or outside);
// 2: any n (four 4-byte loads).
template <int MODE>
__device__ __forceinline__ f32x4 load_quad(const float *__restrict__ X, int64_t s, int64_t N, u32 n, u32 lane)
{
    const u32 m = lane & 15u, q = lane >> 4;
    const int64_t r = s + q < N ? s + q : N - 1;
    if constexpr (MODE == 0) {
        const float4 t = *reinterpret_cast<const float4 *>(X + r * 64 + 4u * m);
        return (f32x4){t.x, t.y, t.z, t.w};
    } else {
        const float *row = X + r * (int64_t)n;
        const u32 c0 = 4u * m;
        if constexpr (MODE == 1) {
            const float4 t = *reinterpret_cast<const float4 *>(row + (c0 < n ? c0 : 0u));
            return (f32x4){t.x, t.y, t.z, t.w};
        } else {
            // rows start at any multiple of four bytes: element by element (16-byte loads that only promise
            // 4-byte alignment measured 40 % slower here)
            f32x4 v;
#pragma unroll
            for (u32 g = 0; g < 4; ++g) v[g] = row[c0 + g < n ? c0 + g : n - 1u];
            return v;
        }
    }
}

__device__ __forceinline__ f32x4 mask_quad(f32x4 v, int64_t s, int64_t N, u32 lane)
{
    const bool row_ok = s + (lane >> 4) < N;
#pragma unroll
    for (u32 g = 0; g < 4; ++g) v[g] = row_ok ? v[g] : 0.f;
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
template <int MODE>
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
    for (int d = 0; d < M2_DEPTH; ++d) ring[d] = load_quad<MODE>(X, 4 * (first + d * stride), N, n, lane);
    for (int64_t k = 0; k < mine; k += M2_DEPTH) {
#pragma unroll
        for (int d = 0; d < M2_DEPTH; ++d) {
            const int64_t s = 4 * (first + (k + d) * stride);
            const f32x4 x = mask_quad(ring[d], s, N, lane);
            ring[d] = load_quad<MODE>(X, s + 4 * M2_DEPTH * stride, N, n, lane);
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

// ---- a handful of features (n <= 16): one lane per sample ---------------------------------
// The whole upper triangle fits a lane's registers (NP (NP + 1) / 2 accumulators for n padded to
// NP = 4, 8, 12 or 16), so a lane takes whole samples: it reads its row (a wave reads 64
// consecutive rows, every byte of them used) and adds the products; nothing is shared until the
// end, when the lanes of a wave and then the four waves of the workgroup are added in a fixed
// order.  Workgroup partials -> moment2_small_reduce_kernel.  Bound by the HBM stream.
constexpr int M2S_WGS = 1024;                     // workgroups at most (four per CU)
template <int NP>
__global__ __launch_bounds__(256) void moment2_small_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                           float *__restrict__ ws)
{
    constexpr int NA = NP * (NP + 1) / 2;
    __shared__ float red[4][NA];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    float acc[NA];
#pragma unroll
    for (int a = 0; a < NA; ++a) acc[a] = 0.f;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t s = (int64_t)blockIdx.x * 256 + tid; s < N; s += stride) {
        const float *row = X + s * (int64_t)n;
        float x[NP];
#pragma unroll
        for (int c = 0; c < NP; ++c) x[c] = (u32)c < n ? row[c] : 0.f;
        int a = 0;
#pragma unroll
        for (int i = 0; i < NP; ++i)
#pragma unroll
            for (int j = i; j < NP; ++j) acc[a++] += x[i] * x[j];
    }
    // lanes of the wave (DPP steps, every lane ends with the sum), then the four waves
#pragma unroll
    for (int a = 0; a < NA; ++a) {
        const float v = wave_sum(acc[a]);
        if (lane == 0u) red[wave][a] = v;
    }
    __syncthreads();
    for (u32 a = tid; a < (u32)NA; a += 256u)
        ws[(size_t)blockIdx.x * NA + a] = (red[0][a] + red[1][a]) + (red[2][a] + red[3][a]);
}

// 16 entries x 16 groups of workgroup partials per block; keeps i <= j < n of the padded triangle
__global__ __launch_bounds__(256) void moment2_small_reduce_kernel(const float *__restrict__ ws, u32 G, u32 n, u32 np,
                                                                  float *__restrict__ Sc, int accumulate)
{
    __shared__ float part[16][16];
    const u32 a = threadIdx.x & 15u, g = threadIdx.x >> 4;
    const u32 na = np * (np + 1u) / 2u, t = blockIdx.x * 16u + a;
    float s = 0.f;
    if (t < na) {
        const u32 per = (G + 15u) / 16u, y0 = min(G, g * per), y1 = min(G, y0 + per);
        for (u32 y = y0; y < y1; ++y) s += ws[(size_t)y * na + t];
    }
    part[g][a] = s;
    __syncthreads();
    if (g != 0u || t >= na) return;
    s = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) s += part[q][a];
    u32 i, j;
    unrank_sym2<u32>(np, t, i, j);                        // the kernel's accumulators are in packed order of np
    if (j >= n) return;
    const u32 p = rank_sym2<u32>(n, i, j);
    Sc[p] = accumulate ? Sc[p] + s : s;
}
constexpr int M2S_NMAX = 16;
static inline u32 m2s_groups(int64_t N)
{
    const int64_t g = (N + 255) / 256;
    return (u32)(g < 1 ? 1 : g > M2S_WGS ? M2S_WGS : g);
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

// ---- tile path: 128 < n < 180 (written for any n <= 1024), plain fp32 vector arithmetic -------
// Blocks of eight indices; a block pair I <= J is owned by one lane with its 8 x 8 accumulators in
// registers: per sample four 16-byte LDS reads and 64 multiply-adds.  Samples go through a
// double-buffered LDS chunk per workgroup (rows padded to 8*ceil(n/8) floats), the sample range is cut
// into slices (grid.y); slice partials -> second kernel adds them in a fixed order, keeps i <= j < n
// and scatters through rank2.  No atomics.
constexpr int M2T_THREADS = 256;
constexpr int M2T_LPT = 8;                         // 16-byte pieces of a chunk per thread
constexpr int M2T_NMAX = 1024;
constexpr int M2T_WGTARGET = 1024;

struct M2TPlan {
    u32 nb8, np, nbp, gx, ch, S;
    int64_t slice;
};
static inline M2TPlan m2t_plan(int64_t N, int n)
{
    M2TPlan p;
    p.nb8 = ((u32)n + 7u) / 8u;
    p.np = 8u * p.nb8;
    p.nbp = (u32)count_sym2<int64_t>(p.nb8);
    p.gx = (p.nbp + M2T_THREADS - 1u) / M2T_THREADS;
    u32 ch = (u32)(M2T_LPT * M2T_THREADS * 4) / p.np;        // samples whose pieces fit the threads' registers
    p.ch = ch > 64u ? 64u : ch & ~7u;                        // n <= 1024: at least 8
    int64_t S = (M2T_WGTARGET + p.gx - 1) / p.gx;
    const int64_t smax = (N + p.ch - 1) / p.ch;
    if (S > smax) S = smax;
    if (S > 512) S = 512;
    if (S < 1) S = 1;
    p.slice = ((N + S - 1) / S + p.ch - 1) / p.ch * p.ch;    // whole chunks
    p.S = (u32)((N + p.slice - 1) / p.slice);
    return p;
}

__device__ __forceinline__ void m2t_load_chunk(f32x4 (&r)[M2T_LPT], const float *__restrict__ X, int64_t s0,
                                               int64_t s_end, u32 n, u32 np4, u32 pieces, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M2T_LPT; ++k) {
        const u32 j = min(tid + (u32)M2T_THREADS * k, pieces - 1u), smp = j / np4, c0 = 4u * (j - smp * np4);
        const int64_t s = s0 + smp, sc = s < s_end ? s : s_end - 1;
        const float *row = X + sc * (int64_t)n;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) r[k][g] = row[c0 + g < n ? c0 + g : n - 1u];
    }
}

__device__ __forceinline__ void m2t_store_chunk(const f32x4 (&r)[M2T_LPT], float *__restrict__ buf, int64_t s0,
                                                int64_t s_end, u32 n, u32 np4, u32 pieces, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M2T_LPT; ++k) {
        const u32 j = tid + (u32)M2T_THREADS * k, smp = j / np4, c0 = 4u * (j - smp * np4);
        if (j >= pieces) continue;
        const bool row_ok = s0 + smp < s_end;
        f32x4 v;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) v[g] = (row_ok && c0 + g < n) ? r[k][g] : 0.f;
        *reinterpret_cast<f32x4 *>(buf + (size_t)j * 4u) = v;
    }
}

// grid.x = block pairs / 256, grid.y = sample slices; dynamic LDS: 2 chunks of ch x np floats
__global__ __launch_bounds__(M2T_THREADS) void moment2_tile_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                                u32 nb8, u32 nbp, u32 ch, int64_t slice,
                                                                float *__restrict__ ws)
{
    extern __shared__ float lds[];
    const u32 tid = threadIdx.x, np = 8u * nb8, np4 = 2u * nb8;
    const u32 pieces = ch * np4, chunk_f = ch * np;
    const u32 bp = blockIdx.x * (u32)M2T_THREADS + tid;
    u32 I, J;
    unrank_sym2<u32>(nb8, min(bp, nbp - 1u), I, J);
    const u32 oi = 8u * I, oj = 8u * J;

    const int64_t s_begin = (int64_t)blockIdx.y * slice;
    const int64_t s_end = s_begin + slice < N ? s_begin + slice : N;
    const int64_t nchunks = s_end > s_begin ? (s_end - s_begin + ch - 1) / ch : 0;

    float acc[64];
#pragma unroll
    for (int e = 0; e < 64; ++e) acc[e] = 0.f;

    if (nchunks > 0) {
        f32x4 r[M2T_LPT];
        m2t_load_chunk(r, X, s_begin, s_end, n, np4, pieces, tid);
        m2t_store_chunk(r, lds, s_begin, s_end, n, np4, pieces, tid);
        if (nchunks > 1) m2t_load_chunk(r, X, s_begin + ch, s_end, n, np4, pieces, tid);
        __syncthreads();
        for (int64_t c = 0; c < nchunks; ++c) {
            const u32 cb = (u32)(c & 1);
            if (c + 1 < nchunks) m2t_store_chunk(r, lds + (cb ^ 1u) * chunk_f, s_begin + (c + 1) * ch, s_end, n, np4, pieces, tid);
            if (c + 2 < nchunks) m2t_load_chunk(r, X, s_begin + (c + 2) * ch, s_end, n, np4, pieces, tid);
            __builtin_amdgcn_sched_barrier(0);
            const float *row = lds + cb * chunk_f;
#pragma unroll 2
            for (u32 smp = 0; smp < ch; ++smp, row += np) {
                const f32x4 a0 = *reinterpret_cast<const f32x4 *>(row + oi), a1 = *reinterpret_cast<const f32x4 *>(row + oi + 4u);
                const f32x4 b0 = *reinterpret_cast<const f32x4 *>(row + oj), b1 = *reinterpret_cast<const f32x4 *>(row + oj + 4u);
                const float xa[8] = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
                const float xb[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[i * 8 + j] += xa[i] * xb[j];
            }
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
        }
    }

    if (bp < nbp) {
        f32x4 *dst = reinterpret_cast<f32x4 *>(ws + ((size_t)blockIdx.y * nbp + bp) * 64u);
#pragma unroll
        for (int e = 0; e < 16; ++e) dst[e] = (f32x4){acc[4 * e], acc[4 * e + 1], acc[4 * e + 2], acc[4 * e + 3]};
    }
}

// A block owns 16 raw accumulators (block pair, i, j) and cuts the S slice partials into 16 groups
// (slices g, g+16, ... ascending inside a group, groups ascending); stores the entries of the unique set.
__global__ __launch_bounds__(256) void moment2_tile_reduce_kernel(const float *__restrict__ ws, u32 S, u32 n,
                                                                 u32 nb8, u32 nbp, float *__restrict__ Sc,
                                                                 int accumulate)
{
    __shared__ float part[16][16];
    const u32 a = threadIdx.x & 15u, g = threadIdx.x >> 4;
    const u32 t = blockIdx.x * 16u + a;                  // < nbp * 64
    const size_t stride = (size_t)nbp * 64u;
    float s = 0.f;
    if (t < nbp * 64u) {
#pragma unroll 4
        for (u32 y = g; y < S; y += 16u) s += ws[(size_t)y * stride + t];
    }
    part[g][a] = s;
    __syncthreads();
    if (g != 0u || t >= nbp * 64u) return;
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) v += part[q][a];
    const u32 bp = t >> 6, e = t & 63u;
    u32 I, J;
    unrank_sym2<u32>(nb8, bp, I, J);
    const u32 i = 8u * I + (e >> 3), j = 8u * J + (e & 7u);
    if (!(i <= j && j < n)) return;
    const u32 p = rank_sym2<u32>(n, i, j);
    Sc[p] = accumulate ? Sc[p] + v : v;
}

// ---- strip path: 64 < n <= 1024 on the matrix cores ------------------------------------------
// The columns are cut into strips of 64 and a strip is split into the four residue groups of the
// n <= 64 kernel, so one 16-byte load per lane is again four MFMA operands at once.  Two strips make
// a block (an odd strip count: strip 0 is a block of its own).  A workgroup owns one task and one
// sample slice; a task is either a whole diagonal block (strip pairs (a0,a0), (a0,a1), (a1,a1):
// 10 + 16 + 10 tiles, only ga <= gb inside a strip) or one strip against both strips of a later
// block (2 x 16 tiles).  The eight waves take the quads of the slice in turn: a wave loads its four
// rows of the (two or three) strips straight from memory, two register sets of M2W_DEPTH quads, one
// of them in flight, and feeds every tile of the task; nothing goes through LDS until the waves add
// their tiles at the end.  At n <= 128 there is one task and X is read once; beyond, a strip is read
// by every task that contains it, and the workgroups of one slice are launched next to each other on
// one XCD (block index -> XCD is round-robin) so that those re-reads meet in that XCD's L2.  Slice
// partials -> moment2_strip_reduce_kernel (fixed order, keeps i <= j < n, scatters through rank2).
// No atomics.
constexpr int M2W_NMAX = 1024;
constexpr int M2W_WAVES = 8;
constexpr int M2W_THREADS = M2W_WAVES * 64;
constexpr int M2W_BLKS = 3;                       // accumulator blocks of 16 tiles per task
constexpr int M2W_ACC = M2W_BLKS * 16 * 256;      // accumulators of a task
constexpr int M2W_DEPTH = 2;                      // quads per register set; two sets, one of them in flight
constexpr int M2W_WGTARGET = 1024;
constexpr int64_t M2W_SLICE_MAX = 131072;         // bounds the fp32 accumulation chain of a wave (16,384 samples)

// Three strips with one nearly empty (128 < n < 180) cost 2.9 times the matrix-core work of two; there the
// vector-ALU tile path measures faster.
static inline bool m2w_applies(int n)
{
    return n > 64 && n <= M2W_NMAX && !(n > 128 && n < 180);
}
// Blocks: two strips each; with an odd number of strips the FIRST block is the single strip 0, so that every
// column block of an off-diagonal task is whole.  first strip of block b:
__host__ __device__ inline u32 m2w_first(u32 nb, u32 b)
{
    return (nb & 1u) ? (b == 0u ? 0u : 2u * b - 1u) : 2u * b;
}
// tasks: the nbb diagonal blocks, then for every column block JB >= 1 the strips before it, one task each
struct M2WPlan {
    u32 nb, nbb, ntasks, S, S8;
    int64_t slice;
};
static inline M2WPlan m2w_plan(int64_t N, int n)
{
    M2WPlan p;
    p.nb = ((u32)n + 63u) / 64u;
    p.nbb = (p.nb + 1u) / 2u;
    p.ntasks = p.nbb;
    for (u32 JB = 1; JB < p.nbb; ++JB) p.ntasks += m2w_first(p.nb, JB);
    // Slices are dealt to the eight XCDs, so their number is a multiple of 8, and one workgroup fits a CU at a
    // time.  The tasks are of nearly equal length (36 or 32 MFMAs per quad): among the counts with at most
    // M2W_WGTARGET workgroups the one that fills its rounds of 256 best wins (ties: the smallest, every workgroup
    // ends with a reduction over its waves).
    int64_t S = 8;
    double best = 0.0;
    for (int64_t c = 8; c == 8 || c * p.ntasks <= M2W_WGTARGET; c += 8) {
        const int64_t wgs = c * p.ntasks, rounds = (wgs + 255) / 256;
        const double fill = (double)wgs / (double)(rounds * 256);
        if (fill > best + 1e-9) {
            best = fill;
            S = c;
        }
    }
    const int64_t smax = (N + 63) / 64, smin = (N + M2W_SLICE_MAX - 1) / M2W_SLICE_MAX;
    if (S > smax) S = smax;                       // at least two quads per wave
    if (S < smin) S = smin;
    if (S < 1) S = 1;
    p.slice = ((N + S - 1) / S + 31) / 32 * 32;   // whole rounds of the eight waves
    p.S = (u32)((N + p.slice - 1) / p.slice);
    p.S8 = (p.S + 7u) / 8u;
    return p;
}
// task -> row strip sa and first column strip sb; diag: the task is the diagonal block that starts at sb;
// single: that block is the single strip (accumulator blocks 1 and 2 then hold copies of block 0's pairs)
__host__ __device__ inline void m2w_task(u32 nb, u32 nbb, u32 task, u32 &sa, u32 &sb, bool &diag, bool &single)
{
    if (task < nbb) {
        sa = sb = m2w_first(nb, task);
        diag = true;
        single = (nb & 1u) && task == 0u;
        return;
    }
    u32 t = task - nbb, JB = 1u;
    while (t >= m2w_first(nb, JB)) {               // at most 8 blocks
        t -= m2w_first(nb, JB);
        ++JB;
    }
    sa = t;
    sb = m2w_first(nb, JB);
    diag = false;
    single = false;
}

// MODE 0 / 1: n % 4 == 0 (aligned 16-byte loads, a piece is wholly inside or outside; 0: n % 64 == 0, kept as
// an instance of its own); 2: any n (16-byte loads at 4-byte alignment: faster than 3 from three strips on,
// slower with two); 3: any n (four 4-byte loads).  Rows past the end of the slice and
// columns past n are clamped to ones that exist.
// roq = q * n: the lane's row offset inside a quad (it does not change from quad to quad)
template <int MODE>
__device__ __forceinline__ f32x4 m2w_load(const float *__restrict__ X, int64_t s, int64_t s_end, u32 n, u32 c0, u32 roq)
{
    // (32-bit on purpose: the scalar unit has no 64-bit ordered compare, so the same tests on an int64_t are made
    // by the vector ALU, about fifteen vector instructions per quad that the MFMAs then wait for; the launcher
    // admits fewer than 2^31 samples)
    const int rows = (int)(s_end - s);                                       // may be <= 0
    const float *base = X + (rows > 0 ? s : s_end - 1) * (int64_t)n;        // wave-uniform
    const u32 qm = rows >= 4 ? 3u : rows > 0 ? (u32)rows - 1u : 0u;          // last row of the quad that exists
    const u32 ro = min(roq, qm * n);
    if constexpr (MODE < 2) {
        const u32 c = c0 < n ? c0 : 0u;                                      // does not change from quad to quad
        const float4 t = *reinterpret_cast<const float4 *>(base + (ro + c));
        return (f32x4){t.x, t.y, t.z, t.w};
    } else if constexpr (MODE == 3) {
        f32x4 v;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) v[g] = base[ro + (c0 + g < n ? c0 + g : n - 1u)];
        return v;
    } else {
        // rows start at any multiple of four bytes: a 16-byte load that only promises that alignment (global
        // memory needs no more); the one piece that straddles column n goes element by element
        typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));
        f32x4 v;
        if (c0 + 4u <= n || c0 >= n) {
            v = *reinterpret_cast<const f32x4u *>(base + (ro + (c0 < n ? c0 : 0u)));
        } else {
#pragma unroll
            for (u32 g = 0; g < 4; ++g) v[g] = base[ro + (c0 + g < n ? c0 + g : n - 1u)];
        }
        return v;
    }
}
// Zeroes the rows past the end of the slice (both operands: a clamped row may hold a value that is not finite, and
// 0 * inf is not 0).  Columns >= n need no mask at all: they only reach accumulators that the reduce kernel drops.
__device__ __forceinline__ f32x4 m2w_mask(f32x4 v, int64_t s, int64_t s_end, u32 q)
{
    const int rows = (int)(s_end - s);
    if (rows < 4) {                                                          // wave-uniform, the end of a slice only
        ST_PIN_VGPR(v);                                                      // a branch, not four selects per quad
        const bool row_ok = (int)q < rows;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) v[g] = row_ok ? v[g] : 0.f;
    }
    return v;
}
template <int BLK>
__device__ __forceinline__ void m2w_full(f32x4 (&acc)[M2W_BLKS * 16], const f32x4 &xa, const f32x4 &xb)
{
#pragma unroll
    for (int ga = 0; ga < 4; ++ga)
#pragma unroll
        for (int gb = 0; gb < 4; ++gb)
            acc[BLK * 16 + ga * 4 + gb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[ga], xb[gb], acc[BLK * 16 + ga * 4 + gb], 0, 0, 0);
}
template <int BLK>
__device__ __forceinline__ void m2w_upper(f32x4 (&acc)[M2W_BLKS * 16], const f32x4 &x)
{
#pragma unroll
    for (int ga = 0; ga < 4; ++ga)
#pragma unroll
        for (int gb = ga; gb < 4; ++gb)
            acc[BLK * 16 + ga * 4 + gb] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[ga], x[gb], acc[BLK * 16 + ga * 4 + gb], 0, 0, 0);
}
// the sixteen tiles of accumulator block BLK: the eight waves' values meet in wave 0 (upper half -> lower half, repeatedly)
template <int BLK>
__device__ __forceinline__ void m2w_tree(f32x4 (&acc)[M2W_BLKS * 16], float (*red)[16 * 256], u32 wave, u32 lane)
{
#pragma unroll
    for (u32 half = M2W_WAVES / 2; half >= 1; half >>= 1) {
        if (wave >= half && wave < 2 * half) {
            float *dst = &red[wave - half][lane];
#pragma unroll
            for (int t = 0; t < 16; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) dst[(t * 4 + v) * 64] = acc[BLK * 16 + t][v];
        }
        __syncthreads();
        if (wave < half) {
            const float *src = &red[wave][lane];
#pragma unroll
            for (int t = 0; t < 16; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[BLK * 16 + t][v] += src[(t * 4 + v) * 64];
        }
        __syncthreads();
    }
}
template <int BLK>
__device__ __forceinline__ void m2w_emit(const f32x4 (&acc)[M2W_BLKS * 16], float *__restrict__ dst)
{
#pragma unroll
    for (int t = 0; t < 16; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) dst[((BLK * 16 + t) * 4 + v) * 64] = acc[BLK * 16 + t][v];
}

// Accumulator blocks of a task: diagonal block: 0 = (sb, sb), 1 = (sb, sb+1), 2 = (sb+1, sb+1); else 0 = (sa, sb), 1 = (sa, sb+1).
// grid.x = 8 * S8 * ntasks: block x works for slice 8 * (x / 8 / ntasks) + x % 8 and task (x / 8) % ntasks
template <int MODE>
__global__ __launch_bounds__(M2W_THREADS) void moment2_strip_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                                  u32 nb, u32 nbb, u32 ntasks, u32 S, int64_t slice,
                                                                  float *__restrict__ ws)
{
    __shared__ __attribute__((aligned(16))) float red[M2W_WAVES / 2][16 * 256];
    const u32 tid = threadIdx.x, lane = tid & 63u, q = lane >> 4;
    const u32 wave = (u32)__builtin_amdgcn_readfirstlane((int)(tid >> 6));
    const u32 xcd = blockIdx.x & 7u, rest = blockIdx.x >> 3, round = rest / ntasks, task = rest - round * ntasks;
    const u32 sl = round * 8u + xcd;
    if (sl >= S) return;                                                   // the whole workgroup
    u32 sa, sb;
    bool diag, single;
    m2w_task(nb, nbb, task, sa, sb, diag, single);
    const u32 m4 = 4u * (lane & 15u), roq = q * n;
    // the single strip stands in for its missing neighbour: the loops stay free of branches, and the reduce
    // kernel reads accumulator block 0 of that task only
    const u32 ca = 64u * sa + m4, cb0 = 64u * sb + m4, cb1 = single ? cb0 : cb0 + 64u;
    const int64_t s_begin = (int64_t)sl * slice, s_end = s_begin + slice < N ? s_begin + slice : N;
    const int64_t quads = (s_end - s_begin + 3) / 4;
    const int64_t mine = (int64_t)wave < quads ? (quads - wave + M2W_WAVES - 1) / M2W_WAVES : 0;
    const int64_t first = s_begin + 4 * (int64_t)wave;
    constexpr int64_t STEP = 4 * M2W_WAVES;                                 // samples from one quad of a wave to its next

    f32x4 acc[M2W_BLKS * 16];
#pragma unroll
    for (int t = 0; t < M2W_BLKS * 16; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // Two register sets of M2W_DEPTH quads each.  While one set is consumed the other one is in flight: its loads are
    // issued behind the MFMAs that last read it, a whole set of quads before its values are needed.
    f32x4 ra[M2W_DEPTH][3], rb[M2W_DEPTH][3];
#pragma unroll
    for (int d = 0; d < M2W_DEPTH; ++d)
#pragma unroll
        for (int k = 0; k < 3; ++k) ra[d][k] = rb[d][k] = (f32x4){0.f, 0.f, 0.f, 0.f};

    if (diag) {
        auto fetch = [&](f32x4 (&r)[M2W_DEPTH][3], int64_t kq) {
#pragma unroll
            for (int d = 0; d < M2W_DEPTH; ++d) {
                r[d][1] = m2w_load<MODE>(X, first + (kq + d) * STEP, s_end, n, cb0, roq);
                r[d][2] = m2w_load<MODE>(X, first + (kq + d) * STEP, s_end, n, cb1, roq);
            }
        };
        auto feed = [&](const f32x4 (&r)[M2W_DEPTH][3], int64_t kq) {
#pragma unroll
            for (int d = 0; d < M2W_DEPTH; ++d) {
                const int64_t s = first + (kq + d) * STEP;
                const f32x4 y0 = m2w_mask(r[d][1], s, s_end, q), y1 = m2w_mask(r[d][2], s, s_end, q);
                m2w_upper<0>(acc, y0);
                m2w_full<1>(acc, y0, y1);
                m2w_upper<2>(acc, y1);
            }
        };
        fetch(ra, 0);
        for (int64_t k = 0; k < mine; k += 2 * M2W_DEPTH) {
            fetch(rb, k + M2W_DEPTH);
            __builtin_amdgcn_sched_barrier(0);
            feed(ra, k);
            __builtin_amdgcn_sched_barrier(0);
            fetch(ra, k + 2 * M2W_DEPTH);
            __builtin_amdgcn_sched_barrier(0);
            feed(rb, k + M2W_DEPTH);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        auto fetch = [&](f32x4 (&r)[M2W_DEPTH][3], int64_t kq) {
#pragma unroll
            for (int d = 0; d < M2W_DEPTH; ++d) {
                r[d][0] = m2w_load<MODE>(X, first + (kq + d) * STEP, s_end, n, ca, roq);
                r[d][1] = m2w_load<MODE>(X, first + (kq + d) * STEP, s_end, n, cb0, roq);
                r[d][2] = m2w_load<MODE>(X, first + (kq + d) * STEP, s_end, n, cb1, roq);
            }
        };
        auto feed = [&](const f32x4 (&r)[M2W_DEPTH][3], int64_t kq) {
#pragma unroll
            for (int d = 0; d < M2W_DEPTH; ++d) {
                const int64_t s = first + (kq + d) * STEP;
                const f32x4 x = m2w_mask(r[d][0], s, s_end, q);
                const f32x4 y0 = m2w_mask(r[d][1], s, s_end, q), y1 = m2w_mask(r[d][2], s, s_end, q);
                m2w_full<0>(acc, x, y0);
                m2w_full<1>(acc, x, y1);
            }
        };
        fetch(ra, 0);
        for (int64_t k = 0; k < mine; k += 2 * M2W_DEPTH) {
            fetch(rb, k + M2W_DEPTH);
            __builtin_amdgcn_sched_barrier(0);
            feed(ra, k);
            __builtin_amdgcn_sched_barrier(0);
            fetch(ra, k + 2 * M2W_DEPTH);
            __builtin_amdgcn_sched_barrier(0);
            feed(rb, k + M2W_DEPTH);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // accumulator blocks in use (the same for all waves)
    const bool use1 = !single, use2 = diag && !single;
    float *dst = ws + ((size_t)sl * ntasks + task) * M2W_ACC + lane;
    m2w_tree<0>(acc, red, wave, lane);
    if (use1) m2w_tree<1>(acc, red, wave, lane);
    if (use2) m2w_tree<2>(acc, red, wave, lane);
    if (wave == 0) {
        m2w_emit<0>(acc, dst);
        if (use1) m2w_emit<1>(acc, dst);
        if (use2) m2w_emit<2>(acc, dst);
    }
}

// A block owns 32 raw accumulators of one task and cuts the S slice partials into 8 groups
// (slices g, g+8, ... ascending inside a group, groups ascending); stores the entries of the unique set.
__global__ __launch_bounds__(256) void moment2_strip_reduce_kernel(const float *__restrict__ ws, u32 S, u32 n,
                                                                  u32 nb, u32 nbb, u32 ntasks, float *__restrict__ Sc,
                                                                  int accumulate)
{
    __shared__ float part[8][32];
    const u32 a = threadIdx.x & 31u, g = threadIdx.x >> 5;
    const u32 id = blockIdx.x * 32u + a;                 // < ntasks * M2W_ACC
    const u32 task = id / (u32)M2W_ACC, e = id % (u32)M2W_ACC;
    const u32 blk = e >> 12, tile = (e >> 8) & 15u, v = (e >> 6) & 3u, lane = e & 63u;
    const u32 ga = tile >> 2, gb = tile & 3u;
    u32 sa, sb;
    bool diag, single;
    m2w_task(nb, nbb, task, sa, sb, diag, single);
    const u32 sI = diag ? sb + (blk >> 1) : sa, sJ = diag ? sb + ((blk + 1u) >> 1) : sb + blk;
    // D layout of the 16x16 MFMA: lane holds column lane%16 of rows 4*(lane/16) + v
    const u32 mrow = 4u * (lane >> 4) + v, mcol = lane & 15u;
    const u32 i = 64u * sI + 4u * mrow + ga, j = 64u * sJ + 4u * mcol + gb;
    const bool keep = (diag ? (!single || blk == 0u) : blk < 2u) && (sI != sJ || ga < gb || (ga == gb && mrow <= mcol)) &&
                      i < n && j < n;
    float s = 0.f;
    if (keep) {
        const size_t stride = (size_t)ntasks * M2W_ACC;
#pragma unroll 4
        for (u32 y = g; y < S; y += 8u) s += ws[(size_t)y * stride + id];
    }
    part[g][a] = s;
    __syncthreads();
    if (g != 0u || !keep) return;
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) t += part[k][a];
    const u32 p = rank_sym2<u32>(n, min(i, j), max(i, j));
    Sc[p] = accumulate ? Sc[p] + t : t;
}

size_t moment2_workspace(int64_t N, int n)
{
    if (N == 0) return 0;
    if (n <= M2S_NMAX) {
        const size_t np = ((size_t)n + 3u) / 4u * 4u;
        return (size_t)m2s_groups(N) * (np * (np + 1u) / 2u) * sizeof(float);
    }
    if (n <= 64) return (size_t)m2_groups(N) * M2_ACC * sizeof(float);
    if (m2w_applies(n)) {
        if (N > 0x7fffffff) return ST_ERR_UNSUPPORTED;        // the kernel counts the rows left in a slice in 32 bits
        const M2WPlan p = m2w_plan(N, n);
        return (size_t)p.S * p.ntasks * M2W_ACC * sizeof(float);
    }
    if (n <= M2T_NMAX) {
        const M2TPlan p = m2t_plan(N, n);
        return (size_t)p.S * p.nbp * 64u * sizeof(float);
    }
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
    if (n <= M2S_NMAX) {
        const u32 G = m2s_groups(N), np = ((u32)n + 3u) / 4u * 4u, na = np * (np + 1u) / 2u;
        switch (np) {
        case 4: hipLaunchKernelGGL(moment2_small_kernel<4>, dim3(G), dim3(256), 0, s, X, N, (u32)n, wsf); break;
        case 8: hipLaunchKernelGGL(moment2_small_kernel<8>, dim3(G), dim3(256), 0, s, X, N, (u32)n, wsf); break;
        case 12: hipLaunchKernelGGL(moment2_small_kernel<12>, dim3(G), dim3(256), 0, s, X, N, (u32)n, wsf); break;
        default: hipLaunchKernelGGL(moment2_small_kernel<16>, dim3(G), dim3(256), 0, s, X, N, (u32)n, wsf); break;
        }
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment2_small_reduce_kernel, dim3((na + 15u) / 16u), dim3(256), 0, s, wsf, G, (u32)n, np, Sc,
                           accumulate);
        return launch_status();
    }
    if (n <= 64) {
        u32 G = m2_groups(N);
        if (n == 64)
            hipLaunchKernelGGL(moment2_mfma_kernel<0>, dim3(G), dim3(M2_THREADS), 0, s, X, N, (u32)n, wsf);
        else if (n % 4 == 0)
            hipLaunchKernelGGL(moment2_mfma_kernel<1>, dim3(G), dim3(M2_THREADS), 0, s, X, N, (u32)n, wsf);
        else
            hipLaunchKernelGGL(moment2_mfma_kernel<2>, dim3(G), dim3(M2_THREADS), 0, s, X, N, (u32)n, wsf);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment2_reduce_kernel, dim3(M2_ACC / 64), dim3(256), 0, s, wsf, G, (u32)n, Sc,
                           accumulate);
        return launch_status();
    }
    if (m2w_applies(n)) {
        const M2WPlan p = m2w_plan(N, n);
        const dim3 grid(8u * p.S8 * p.ntasks), block(M2W_THREADS);
        if (n % 64 == 0)
            hipLaunchKernelGGL(moment2_strip_kernel<0>, grid, block, 0, s, X, N, (u32)n, p.nb, p.nbb, p.ntasks, p.S, p.slice, wsf);
        else if (n % 4 == 0)
            hipLaunchKernelGGL(moment2_strip_kernel<1>, grid, block, 0, s, X, N, (u32)n, p.nb, p.nbb, p.ntasks, p.S, p.slice, wsf);
        else if (p.nb > 2u)
            hipLaunchKernelGGL(moment2_strip_kernel<2>, grid, block, 0, s, X, N, (u32)n, p.nb, p.nbb, p.ntasks, p.S, p.slice, wsf);
        else
            hipLaunchKernelGGL(moment2_strip_kernel<3>, grid, block, 0, s, X, N, (u32)n, p.nb, p.nbb, p.ntasks, p.S, p.slice, wsf);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment2_strip_reduce_kernel, dim3(p.ntasks * (u32)M2W_ACC / 32u), dim3(256), 0, s, wsf, p.S,
                           (u32)n, p.nb, p.nbb, p.ntasks, Sc, accumulate);
        return launch_status();
    }
    if (n <= M2T_NMAX) {
        const M2TPlan p = m2t_plan(N, n);
        const size_t lds_bytes = (size_t)2u * p.ch * p.np * sizeof(float);          // at most 64 KB
        if (!allow_dynamic_lds(reinterpret_cast<const void *>(moment2_tile_kernel), 64 * 1024)) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment2_tile_kernel, dim3(p.gx, p.S), dim3(M2T_THREADS), lds_bytes, s, X, N, (u32)n, p.nb8,
                           p.nbp, p.ch, p.slice, wsf);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment2_tile_reduce_kernel, dim3((p.nbp * 64u + 15u) / 16u), dim3(256), 0, s, wsf, p.S,
                           (u32)n, p.nb8, p.nbp, Sc, accumulate);
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
