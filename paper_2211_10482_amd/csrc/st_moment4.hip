// Fourth-moment accumulation over N samples, unique entries only:
//     Sc(rank4(i,j,k,l)) (+)= sum_s X(s,i) X(s,j) X(s,k) X(s,l)      for i <= j <= k <= l
// (the M3 = vec(f (x) f) (x) vec(f (x) f) term of the degree-2 polynomial-regression
// covariance, summed over the data; about 23 of every 24 dense entries are redundant).
//
// Matrix cores (st_moment_mfma.hip) for 29..32, 41..48 and 53..256 features; lanes that take whole
// samples up to 16 features (st_covar_small.hip); fp32 vector arithmetic on register tiles, in this
// file, for the rest (where padding the indices to whole groups of 16 costs more than the matrix
// cores gain).
//
// Tile path, plain fp32 vector arithmetic: on the vector ALUs any set of entries
// can be owned by any thread, so nothing but the block
// diagonals is padded.  The indices are cut into blocks of four; a block quadruple
// I <= J <= K <= L (unranked with the same closed form as the entries themselves, on
// n/4 blocks) is owned by four neighbouring lanes, one per i in block I, each with the
// 4 x 4 x 4 accumulators of (j, k, l) in registers.  Per sample a lane reads x_i and the
// three 16-byte groups x_J, x_K, x_L from the staged sample row and does
// 4 + 16 + 64 multiply(-add)s:  a_j = x_i x_j,  b_jk = a_j x_k,  acc_jkl += b_jk x_l.
// Samples are staged through a double-buffered LDS chunk per workgroup (loads of chunk
// c+2 in flight while chunk c is consumed), and the sample range is cut into slices
// (grid.y) so that the grid fills the chip.  Slice partials -> second kernel adds them
// in a fixed order, keeps i <= j <= k <= l < n and scatters through rank4.  No atomics.
//
// Algorithmic work per sample: one multiply-add per unique quadruple (+ the pair
// products).  Bound by the fp32 vector rate.
#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int M4_THREADS = 256;                    // 64 block quadruples x 4 lanes
constexpr int M4_CH = 64;                          // samples per staged chunk
constexpr int M4_LPT = M4_CH * 16 / M4_THREADS;    // 16-byte pieces of a chunk per thread (4)
constexpr int M4_WGTARGET = 1024;                  // workgroups to aim for (four per CU)

// A chunk of M4_CH samples is staged as [sample][64 columns]; only the 4*nb4 columns the tiles
// read are loaded and written (columns >= n and samples past the end of the slice as zeros).
// load_chunk only issues the loads (row clamped into the slice), store_chunk masks and writes.
__device__ __forceinline__ void m4_load_chunk(f32x4 (&r)[M4_LPT], const float *__restrict__ X, int64_t s0,
                                              int64_t s_end, u32 n, u32 nb4, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M4_LPT; ++k) {
        const u32 j = tid + (u32)M4_THREADS * k, smp = j >> 4, c0 = 4u * (j & 15u);
        if ((j & 15u) >= nb4) continue;
        const int64_t s = s0 + smp, sc = s < s_end ? s : s_end - 1;
        const float *row = X + sc * (int64_t)n;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) r[k][g] = row[c0 + g < n ? c0 + g : n - 1];
    }
}

__device__ __forceinline__ void m4_store_chunk(const f32x4 (&r)[M4_LPT], float *__restrict__ buf, int64_t s0,
                                               int64_t s_end, u32 n, u32 nb4, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M4_LPT; ++k) {
        const u32 j = tid + (u32)M4_THREADS * k, smp = j >> 4, c0 = 4u * (j & 15u);
        if ((j & 15u) >= nb4) continue;
        const bool row_ok = s0 + smp < s_end;
        f32x4 v;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) v[g] = (row_ok && c0 + g < n) ? r[k][g] : 0.f;
        *reinterpret_cast<f32x4 *>(buf + smp * 64u + c0) = v;
    }
}

// grid.x = block quadruples / 64, grid.y = sample slices (17 <= n: at least 70 block quadruples)
__global__ __launch_bounds__(M4_THREADS) void moment4_tile_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                                u32 nb4, u32 nbq, int64_t slice,
                                                                float *__restrict__ ws)
{
    __shared__ __attribute__((aligned(16))) float xs[2][M4_CH * 64];
    const u32 tid = threadIdx.x, ii = tid & 3u;
    const u32 bq = blockIdx.x * 64u + (tid >> 2);
    const bool live = bq < nbq;
    u32 I, J, K, L;
    unrank_sym4<u32>(nb4, min(bq, nbq - 1u), I, J, K, L);
    const u32 oi = 4u * I + ii, oj = 4u * J, ok = 4u * K, ol = 4u * L;

    const int64_t s_begin = (int64_t)blockIdx.y * slice;
    const int64_t s_end = s_begin + slice < N ? s_begin + slice : N;
    const int64_t nchunks = s_end > s_begin ? (s_end - s_begin + M4_CH - 1) / M4_CH : 0;

    float acc[64];
#pragma unroll
    for (int e = 0; e < 64; ++e) acc[e] = 0.f;

    if (nchunks > 0) {
        f32x4 r[M4_LPT];
        m4_load_chunk(r, X, s_begin, s_end, n, nb4, tid);
        m4_store_chunk(r, xs[0], s_begin, s_end, n, nb4, tid);
        if (nchunks > 1) m4_load_chunk(r, X, s_begin + M4_CH, s_end, n, nb4, tid);
        __syncthreads();
        for (int64_t c = 0; c < nchunks; ++c) {
            const u32 cb = (u32)(c & 1);
            // registers hold chunk c+1: park it in the other buffer (its readers finished
            // before the barrier that ended the previous iteration), then put chunk c+2 in flight
            if (c + 1 < nchunks) m4_store_chunk(r, xs[cb ^ 1u], s_begin + (c + 1) * M4_CH, s_end, n, nb4, tid);
            if (c + 2 < nchunks) m4_load_chunk(r, X, s_begin + (c + 2) * M4_CH, s_end, n, nb4, tid);
            __builtin_amdgcn_sched_barrier(0);
            const float *row = xs[cb];
#pragma unroll 2
            for (int smp = 0; smp < M4_CH; ++smp, row += 64) {
                const float xi = row[oi];
                const f32x4 xj = *reinterpret_cast<const f32x4 *>(row + oj);
                const f32x4 xk = *reinterpret_cast<const f32x4 *>(row + ok);
                const f32x4 xl = *reinterpret_cast<const f32x4 *>(row + ol);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float a = xi * xj[j];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float b = a * xk[k];
#pragma unroll
                        for (int l = 0; l < 4; ++l) acc[(j * 4 + k) * 4 + l] += b * xl[l];
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
        }
    }

    if (live) {
        f32x4 *dst = reinterpret_cast<f32x4 *>(ws + (((size_t)blockIdx.y * nbq + bq) * 4u + ii) * 64u);
#pragma unroll
        for (int e = 0; e < 16; ++e) dst[e] = (f32x4){acc[4 * e], acc[4 * e + 1], acc[4 * e + 2], acc[4 * e + 3]};
    }
}

// Raw accumulators (block quadruple, lane, j, k, l) -> unique entries: a block owns 16 accumulators and cuts the
// S slice partials into 16 groups (ascending inside a group, groups ascending), then keeps i <= j <= k <= l < n.
__global__ __launch_bounds__(256) void moment4_reduce_kernel(const float *__restrict__ ws, u32 S, u32 n, u32 nb4,
                                                            u32 nbq, float *__restrict__ Sc, int accumulate)
{
    __shared__ float part[16][16];
    const u32 a = threadIdx.x & 15u, g = threadIdx.x >> 4;
    const u32 t = blockIdx.x * 16u + a;                  // < nbq * 256
    const size_t stride = (size_t)nbq * 256u;
    float s = 0.f;
    if (t < nbq * 256u) {
        const u32 per = (S + 15u) / 16u, y0 = min(S, g * per), y1 = min(S, y0 + per);
#pragma unroll 4
        for (u32 y = y0; y < y1; ++y) s += ws[(size_t)y * stride + t];
    }
    part[g][a] = s;
    __syncthreads();
    if (g != 0u || t >= nbq * 256u) return;
    s = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) s += part[q][a];
    const u32 bq = t >> 8, ii = (t >> 6) & 3u, e = t & 63u;
    u32 I, J, K, L;
    unrank_sym4<u32>(nb4, bq, I, J, K, L);
    const u32 i = 4u * I + ii, j = 4u * J + (e >> 4), k = 4u * K + ((e >> 2) & 3u), l = 4u * L + (e & 3u);
    if (!(i <= j && j <= k && k <= l && l < n)) return;
    const u32 p = rank_sym4<u32>(n, i, j, k, l);
    Sc[p] = accumulate ? Sc[p] + s : s;
}

__global__ __launch_bounds__(256) void moment4_zero_kernel(float *__restrict__ p, u32 count)
{
    u32 t = blockIdx.x * 256u + threadIdx.x;
    if (t < count) p[t] = 0.f;
}

struct M4Plan {
    u32 nb4, nbq, gx, S, ch;
    int64_t slice;
};
static inline M4Plan m4_plan(int64_t N, int n)
{
    M4Plan p;
    p.nb4 = ((u32)n + 3u) / 4u;
    p.nbq = (u32)count_sym4<int64_t>(p.nb4);
    p.gx = (p.nbq + 63u) / 64u;
    p.ch = (u32)M4_CH;
    int64_t S = (M4_WGTARGET + p.gx - 1) / p.gx;           // enough slices to fill the chip (four per CU) ...
    int64_t smax = (N + p.ch - 1) / p.ch;                  // ... each of at least one chunk
    const int64_t scap = p.gx >= 12u ? 64 : 768 / (int64_t)p.gx;     // (measured: more slices of many quadruples lose)
    if (S > scap) S = scap;
    if (S > smax) S = smax;
    if (S < 1) S = 1;
    p.slice = ((N + S - 1) / S + p.ch - 1) / p.ch * p.ch;      // whole chunks
    p.S = (u32)((N + p.slice - 1) / p.slice);
    return p;
}

size_t moment4_workspace(int64_t N, int n)
{
    if (N == 0) return 0;
    if (moment_mfma_wins(4, n)) return moment_mfma_workspace(4, N, n);
    if (covar_small_applies(n)) return covar_small_workspace(N, n);
    M4Plan p = m4_plan(N, n);
    return (size_t)p.S * p.nbq * 256u * sizeof(float);
}

st_status launch_moment4(const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws, hipStream_t s)
{
    const u32 count = (u32)count_sym4<int64_t>(n);         // n <= 256: below 2^28
    if (N == 0) {
        if (!accumulate)
            hipLaunchKernelGGL(moment4_zero_kernel, dim3((count + 255u) / 256u), dim3(256), 0, s, Sc, count);
        return launch_status();
    }
    if (moment_mfma_wins(4, n)) return launch_moment_mfma(4, X, N, n, Sc, accumulate, ws, s);
    // Up to 16 features the one-pass covariance kernel is the fastest way to the fourth
    // moment as well (every multiply-add a unique entry; the two smaller terms it also forms cost little)
    if (covar_small_applies(n)) return launch_covar_small(X, N, n, nullptr, nullptr, Sc, accumulate, ws, s);
    const M4Plan p = m4_plan(N, n);
    float *wsf = static_cast<float *>(ws);
    hipLaunchKernelGGL(moment4_tile_kernel, dim3(p.gx, p.S), dim3(M4_THREADS), 0, s, X, N, (u32)n, p.nb4, p.nbq,
                       p.slice, wsf);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    hipLaunchKernelGGL(moment4_reduce_kernel, dim3(p.nbq * 16u), dim3(256), 0, s, wsf, p.S, (u32)n, p.nb4, p.nbq, Sc,
                       accumulate);
    return launch_status();
}

}  // namespace st
