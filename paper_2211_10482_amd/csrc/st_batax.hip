// y = beta * A^T (A x) for a packed upper-triangular A (unique set 0<=i<=j<n).
//
// One-pass kernel (n <= 8192).  The packed matrix is streamed from HBM once:
// a row has to stay on chip between its use in t_i = A(i,:) x and its use in
// y += t_i A(i,:), so a workgroup of 1024 threads holds whole rows in
// registers.  Thread `tid` owns the fixed columns 4*(tid + 1024 v) .. +3, keeps
// x and its partial y for those columns in registers for the whole kernel, and
// rows are dealt to workgroups round-robin (row i -> workgroup i mod G), which
// balances the triangular row lengths.  Per batch of RB rows: every thread
// loads its (unaligned, 16-byte) pieces of the rows, a DPP wave reduction and
// one LDS exchange give the RB dot products t_i to every thread in a fixed
// summation order, and the same registers are reused for the rank-one update
// of y.  The next batch is already in flight while the current one is reduced.
// Each workgroup writes its partial y; a second small kernel adds the G
// partials in a fixed order and applies beta.  No float atomics anywhere.
//
// Algorithmic traffic: 4 bytes per stored entry, read once.
//
// General path (larger n): two plain passes (t = A x, then y = beta A^T t).
#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;

constexpr int BT = 1024;   // threads per workgroup (16 waves)
constexpr int RB = 4;      // rows per batch
constexpr int GMAX = 256;  // workgroups of the one-pass kernel (one per CU)

struct __attribute__((packed, aligned(4))) f4u { float x, y, z, w; };

template <int CTRL> __device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// Sum over the 64 lanes, same bits in every lane.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_f<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);   // row_half_mirror
    v += dpp_f<0x140>(v);   // row_mirror
    float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return (r0 + r1) + (r2 + r3);
}

template <int V>
__device__ __forceinline__ void load_batch(float4 (&a)[RB][V], const float *__restrict__ Ap, u32 n,
                                           u32 row0, u32 rstride, u32 tid)
{
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        u32 i = row0 + (u32)r * rstride;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            u32 c0 = 4u * (tid + (u32)BT * v);
            float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < n && c0 + 3u >= i && c0 < n) {
                const float *rowp = Ap + row_sym2<u32>(n, i);   // address of A(i,i)
                if (c0 >= i && c0 + 3u < n) {
                    f4u t = *reinterpret_cast<const f4u *>(rowp + (c0 - i));
                    val = make_float4(t.x, t.y, t.z, t.w);
                } else {
                    float e[4];
#pragma unroll
                    for (u32 q = 0; q < 4; ++q) {
                        u32 c = c0 + q;
                        e[q] = (c >= i && c < n) ? rowp[c - i] : 0.f;
                    }
                    val = make_float4(e[0], e[1], e[2], e[3]);
                }
            }
            a[r][v] = val;
        }
    }
}

template <int V>
__device__ __forceinline__ void process_batch(const float4 (&a)[RB][V], const float4 (&xs)[V],
                                              float4 (&ya)[V], float (*red)[RB][BT / 64], int pb,
                                              u32 lane, u32 wave)
{
    float p[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        float s = 0.f;
#pragma unroll
        for (int v = 0; v < V; ++v)
            s += a[r][v].x * xs[v].x + a[r][v].y * xs[v].y + a[r][v].z * xs[v].z + a[r][v].w * xs[v].w;
        p[r] = wave_sum(s);
    }
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < RB; ++r) red[pb][r][wave] = p[r];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < BT / 64; ++w) t += red[pb][r][w];   // same order in every thread
#pragma unroll
        for (int v = 0; v < V; ++v) {
            ya[v].x += t * a[r][v].x; ya[v].y += t * a[r][v].y;
            ya[v].z += t * a[r][v].z; ya[v].w += t * a[r][v].w;
        }
    }
}

template <int V>
__global__ __launch_bounds__(BT) void batax_onepass_kernel(const float *__restrict__ Ap,
                                                          const float *__restrict__ x,
                                                          float *__restrict__ part, u32 n, u32 npad,
                                                          u32 G)
{
    __shared__ float red[2][RB][BT / 64];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6, g = blockIdx.x;

    float4 xs[V], ya[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        u32 c0 = 4u * (tid + (u32)BT * v);
        float e[4];
#pragma unroll
        for (u32 q = 0; q < 4; ++q) e[q] = (c0 + q < n) ? x[c0 + q] : 0.f;
        xs[v] = make_float4(e[0], e[1], e[2], e[3]);
        ya[v] = make_float4(0.f, 0.f, 0.f, 0.f);
    }

    // rows g, g+G, g+2G, ...; batch b holds rows g + G*(RB*b + r)
    const u32 nrows = (n > g) ? (n - g + G - 1) / G : 0;
    const u32 nb = (nrows + RB - 1) / RB;
    float4 a0[RB][V], a1[RB][V];
    load_batch<V>(a0, Ap, n, g, G, tid);
    for (u32 b = 0; b < nb; b += 2) {
        load_batch<V>(a1, Ap, n, g + G * RB * (b + 1), G, tid);
        process_batch<V>(a0, xs, ya, red, 0, lane, wave);
        load_batch<V>(a0, Ap, n, g + G * RB * (b + 2), G, tid);
        process_batch<V>(a1, xs, ya, red, 1, lane, wave);
    }

    float *dst = part + (size_t)g * npad;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        u32 c0 = 4u * (tid + (u32)BT * v);
        if (c0 < npad) *reinterpret_cast<float4 *>(dst + c0) = ya[v];
    }
}

// y[j] = beta * sum_g part[g][j], g ascending inside 8 slices, slices ascending.
__global__ __launch_bounds__(256) void batax_reduce_kernel(const float *__restrict__ part,
                                                          float *__restrict__ y, u32 n, u32 npad, u32 G,
                                                          float beta)
{
    __shared__ float acc[8][32];
    u32 cx = threadIdx.x & 31u, sl = threadIdx.x >> 5;
    u32 j = blockIdx.x * 32u + cx;
    u32 per = (G + 7u) / 8u;
    u32 g0 = sl * per, g1 = min(G, g0 + per);
    float s = 0.f;
    if (j < n)
        for (u32 g = g0; g < g1; ++g) s += part[(size_t)g * npad + j];
    acc[sl][cx] = s;
    __syncthreads();
    if (sl == 0 && j < n) {
        float t = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) t += acc[q][cx];
        y[j] = beta * t;
    }
}

// ---- general path: two plain passes -------------------------------------------
__global__ __launch_bounds__(256) void batax_ax_kernel(const float *__restrict__ Ap,
                                                      const float *__restrict__ x, float *__restrict__ t,
                                                      u32 n)
{
    u32 lane = threadIdx.x & 63u;
    u32 i = blockIdx.x * 4u + (threadIdx.x >> 6);   // one wave per row
    if (i >= n) return;
    const float *rowp = Ap + row_sym2<u32>(n, i);
    float s = 0.f;
    for (u32 c = lane; c < n - i; c += 64u) s += rowp[c] * x[i + c];
    s = wave_sum(s);
    if (lane == 0) t[i] = s;
}

__global__ __launch_bounds__(256) void batax_aty_kernel(const float *__restrict__ Ap,
                                                       const float *__restrict__ t, float *__restrict__ y,
                                                       u32 n, float beta)
{
    u32 j = blockIdx.x * 256u + threadIdx.x;
    if (j >= n) return;
    float s = 0.f;
    for (u32 i = 0; i <= j; ++i) s += Ap[row_sym2<u32>(n, i) + (j - i)] * t[i];
    y[j] = beta * s;
}

static inline u32 onepass_grid(int n) { return (u32)(n < GMAX ? n : GMAX); }
static inline u32 pad4(int n) { return ((u32)n + 3u) & ~3u; }

size_t batax_workspace(int n)
{
    if (n <= 2 * 4 * BT) return (size_t)onepass_grid(n) * pad4(n) * sizeof(float);
    return (size_t)pad4(n) * sizeof(float);
}

st_status launch_batax(const float *Ap, const float *x, float *y, int n, float beta, void *ws,
                       hipStream_t s)
{
    u32 un = (u32)n;
    float *wsf = static_cast<float *>(ws);
    if (n <= 2 * 4 * BT) {
        u32 G = onepass_grid(n), npad = pad4(n);
        if (n <= 4 * BT)
            hipLaunchKernelGGL(batax_onepass_kernel<1>, dim3(G), dim3(BT), 0, s, Ap, x, wsf, un, npad, G);
        else
            hipLaunchKernelGGL(batax_onepass_kernel<2>, dim3(G), dim3(BT), 0, s, Ap, x, wsf, un, npad, G);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(batax_reduce_kernel, dim3((un + 31u) / 32u), dim3(256), 0, s, wsf, y, un, npad,
                           G, beta);
        return launch_status();
    }
    hipLaunchKernelGGL(batax_ax_kernel, dim3((un + 3u) / 4u), dim3(256), 0, s, Ap, x, wsf, un);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    hipLaunchKernelGGL(batax_aty_kernel, dim3((un + 255u) / 256u), dim3(256), 0, s, Ap, wsf, y, un, beta);
    return launch_status();
}

}  // namespace st
