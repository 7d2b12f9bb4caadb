// y = beta * A^T (A x) for a packed upper-triangular A (unique set 0<=i<=j<n).
//
// One-pass kernel (n <= 16384).  The packed matrix is streamed from HBM once:
// a row has to stay on chip between its use in t_i = A(i,:) x and its use in
// y += t_i A(i,:), so a workgroup of 1024 threads holds whole rows in
// registers.  Thread `tid` owns the fixed columns 4*(tid + 1024 v) .. +3, v < 4, keeps
// x and its partial y for those columns in registers for the whole kernel.
// Rows are dealt to workgroups round-robin AND folded: a workgroup alternates
// between a row i from the top half and its mirror image n-1-i from the bottom
// half, so that every pair of consecutive rows holds n+1 entries -- the bytes in
// flight per batch stay constant from the first batch to the last, instead of
// shrinking with the triangle until the short rows are latency bound.
// Per batch of RB rows: every thread
// loads its (unaligned, 16-byte) pieces of the rows, a DPP wave reduction and
// one LDS exchange give the RB dot products t_i to every thread in a fixed
// summation order, and the same registers are reused for the rank-one update
// of y.  The next batch is already in flight while the current one is reduced.
// Each workgroup writes its partial y; a second small kernel adds the G
// partials in a fixed order and applies beta.  No float atomics anywhere.
//
// Algorithmic traffic: 4 bytes per stored entry, read once.
//
// General path (larger n): two passes (t = A x, one wave per row; then y = beta A^T t in 64 row slices
// whose partials are added in a fixed order).
#include <mutex>

#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;

#ifndef ST_BATAX_BT
#define ST_BATAX_BT 1024
#endif
#ifndef ST_BATAX_RB
#define ST_BATAX_RB 4
#endif
constexpr int BT = ST_BATAX_BT;   // threads per workgroup
constexpr int RB_SHORT = ST_BATAX_RB;   // rows per batch while a thread holds at most two column groups of a row
constexpr int GMAX = 256;  // workgroups of the one-pass kernel (one per CU)

struct __attribute__((packed, aligned(4))) f4u { float x, y, z, w; };

// Row held by slot q of workgroup g: q even -> row g + G*(q/2) from the top, q odd ->
// its mirror image from the bottom; the middle row of an odd n is dealt once, as a
// top row.  Slots past the middle return n ("no row").
__device__ __forceinline__ u32 row_of_slot(u32 n, u32 g, u32 G, u32 q)
{
    const u32 it = g + G * (q >> 1);
    if (q & 1u) return (2u * it + 1u < n) ? n - 1u - it : n;
    return (2u * it + 1u <= n) ? it : n;
}

// Raw (unmasked) pieces of RB rows.  FAST (n % 4 == 0, n >= 4): branch free, so
// that all loads of a batch are in flight together -- a group of four columns
// that starts left of the diagonal is read from up to three entries before the
// row start (the tail of the previous row, always inside the array for i >= 1),
// groups entirely outside the row read position 0; mask_batch zeroes what does
// not belong to the row.  Otherwise: guarded element loads.
template <int V, int RB, bool FAST>
__device__ __forceinline__ void load_batch(float4 (&a)[RB][V], const float *__restrict__ Ap, u32 n,
                                           u32 g, u32 G, u32 q0, u32 tid)
{
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        u32 i = row_of_slot(n, g, G, q0 + (u32)r);
#pragma unroll
        for (int v = 0; v < V; ++v) {
            u32 c0 = 4u * (tid + (u32)BT * v);
            if constexpr (FAST) {
                bool touch = i < n && c0 + 3u >= i && c0 < n;
                u32 pos = touch ? row_sym2<u32>(n, i) + c0 - i : 0u;   // c0 - i may wrap: sum is exact mod 2^32
                // byte offset in 32 bits (n <= 8192: the array is below 2^28 bytes): scalar base + vector offset
                f4u t = *reinterpret_cast<const f4u *>(reinterpret_cast<const char *>(Ap) + (pos << 2));
                a[r][v] = make_float4(t.x, t.y, t.z, t.w);
            } else {
                float e[4] = {0.f, 0.f, 0.f, 0.f};
                if (i < n) {
                    const float *rowp = Ap + row_sym2<u32>(n, i);
#pragma unroll
                    for (u32 q = 0; q < 4; ++q) {
                        u32 c = c0 + q;
                        if (c >= i && c < n) e[q] = rowp[c - i];
                    }
                }
                a[r][v] = make_float4(e[0], e[1], e[2], e[3]);
            }
        }
    }
}

template <int V, int RB>
__device__ __forceinline__ void mask_batch(float4 (&a)[RB][V], u32 n, u32 g, u32 G, u32 q0, u32 tid)
{
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        u32 i = row_of_slot(n, g, G, q0 + (u32)r);
#pragma unroll
        for (int v = 0; v < V; ++v) {
            u32 c0 = 4u * (tid + (u32)BT * v);
            // element q of the group is in the row iff q >= i - c0 (and the row / group exist)
            int d = (i < n && c0 < n) ? (int)i - (int)c0 : 4;
            a[r][v].x = (0 >= d) ? a[r][v].x : 0.f;
            a[r][v].y = (1 >= d) ? a[r][v].y : 0.f;
            a[r][v].z = (2 >= d) ? a[r][v].z : 0.f;
            a[r][v].w = (3 >= d) ? a[r][v].w : 0.f;
        }
    }
}

template <int V, int RB>
__device__ __forceinline__ void process_batch(const float4 (&a)[RB][V], const float4 (&xs)[V],
                                              float4 (&ya)[V], float (*red)[RB][BT / 64], int pb,
                                              u32 lane, u32 wave)
{
    constexpr int NW = BT / 64;
    static_assert(NW * RB <= 64 && (NW == 4 || NW == 8 || NW == 16), "cross-wave reduction layout");
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
    // Every wave adds the NW wave partials of each row in the same fixed tree:
    // lane l holds partial (row l / NW, wave l % NW); DPP adds inside aligned
    // groups of NW lanes; the row sums are then read as wave-uniform scalars.
    float c = (lane < (u32)(NW * RB)) ? (&red[pb][0][0])[lane] : 0.f;
    c += wave_dpp<0xB1>(c);
    c += wave_dpp<0x4E>(c);
    if constexpr (NW >= 8) c += wave_dpp<0x141>(c);
    if constexpr (NW >= 16) c += wave_dpp<0x140>(c);
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const float t = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, c), r * NW));
#pragma unroll
        for (int v = 0; v < V; ++v) {
            ya[v].x += t * a[r][v].x; ya[v].y += t * a[r][v].y;
            ya[v].z += t * a[r][v].z; ya[v].w += t * a[r][v].w;
        }
    }
}

template <int V, int RB, bool FAST>
__global__ __launch_bounds__(BT) void batax_onepass_kernel(const float *__restrict__ Ap,
                                                          const float *__restrict__ x,
                                                          float *__restrict__ part, u32 n, u32 npad,
                                                          u32 G)
{
    __shared__ float red[2][RB][BT / 64];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6, g = blockIdx.x;

    // batch b holds the slots RB*b .. RB*b + RB-1 of this workgroup (row_of_slot)
    const u32 mid = (n - 1u) / 2u;                 // last row dealt from the top
    const u32 nslots = (mid >= g) ? 2u * ((mid - g) / G + 1u) : 0u;
    const u32 nb = (nslots + RB - 1) / RB;
    float4 a0[RB][V], a1[RB][V];
    load_batch<V, RB, FAST>(a0, Ap, n, g, G, 0u, tid); // first rows go out before anything else

    // x for the owned columns: branch-free (index clamped, value selected), so these
    // loads overlap the first batch instead of serialising in front of it
    float4 xs[V], ya[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        u32 c0 = 4u * (tid + (u32)BT * v);
        float e[4];
#pragma unroll
        for (u32 q = 0; q < 4; ++q) {
            float t = x[min(c0 + q, n - 1u)];
            e[q] = (c0 + q < n) ? t : 0.f;
        }
        xs[v] = make_float4(e[0], e[1], e[2], e[3]);
        ya[v] = make_float4(0.f, 0.f, 0.f, 0.f);
    }

    for (u32 b = 0; b < nb; b += 2) {
        load_batch<V, RB, FAST>(a1, Ap, n, g, G, RB * (b + 1), tid);
        __builtin_amdgcn_sched_barrier(0);
        mask_batch<V, RB>(a0, n, g, G, RB * b, tid);
        process_batch<V, RB>(a0, xs, ya, red, 0, lane, wave);
        __builtin_amdgcn_sched_barrier(0);
        load_batch<V, RB, FAST>(a0, Ap, n, g, G, RB * (b + 2), tid);
        __builtin_amdgcn_sched_barrier(0);
        mask_batch<V, RB>(a1, n, g, G, RB * (b + 1), tid);
        process_batch<V, RB>(a1, xs, ya, red, 1, lane, wave);
        __builtin_amdgcn_sched_barrier(0);
    }

    float *dst = part + (size_t)g * npad;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        u32 c0 = 4u * (tid + (u32)BT * v);
        if (c0 < npad) *reinterpret_cast<float4 *>(dst + c0) = ya[v];
    }
}

// y[j] = beta * sum_g part[g][j]: a block owns 8 groups of four columns and cuts
// the G partials into 32 slices (g ascending inside a slice, slices ascending).
__global__ __launch_bounds__(256) void batax_reduce_kernel(const float *__restrict__ part,
                                                          float *__restrict__ y, u32 n, u32 npad, u32 G,
                                                          float beta)
{
    __shared__ float4 acc[32][8];
    const u32 cq = threadIdx.x & 7u, sl = threadIdx.x >> 3;
    const u32 c0 = (blockIdx.x * 8u + cq) * 4u;
    const u32 per = (G + 31u) / 32u;
    const u32 g0 = min(G, sl * per), g1 = min(G, g0 + per);
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c0 < npad) {
        const float *src = part + c0;
#pragma unroll 8
        for (u32 g = g0; g < g1; ++g) {
            float4 v = *reinterpret_cast<const float4 *>(src + (size_t)g * npad);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    }
    acc[sl][cq] = s;
    __syncthreads();
    if (sl == 0 && c0 < npad) {
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int q = 0; q < 32; ++q) {
            float4 v = acc[q][cq];
            t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
        }
        float e[4] = {beta * t.x, beta * t.y, beta * t.z, beta * t.w};
#pragma unroll
        for (u32 q = 0; q < 4; ++q)
            if (c0 + q < n) y[c0 + q] = e[q];
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

// y partial of one row slice: thread j adds A(i,j) t_i over the rows i <= j of slice blockIdx.y (rows
// ascending; the loads of a wave are contiguous in j)
constexpr u32 ATY_SLICES = 64;
__global__ __launch_bounds__(256) void batax_aty_kernel(const float *__restrict__ Ap,
                                                       const float *__restrict__ t, float *__restrict__ part,
                                                       u32 n, u32 npad)
{
    u32 j = blockIdx.x * 256u + threadIdx.x;
    if (j >= n) return;
    const u32 per = (n + ATY_SLICES - 1u) / ATY_SLICES, i0 = blockIdx.y * per, i1 = min(min(n, i0 + per), j + 1u);
    float s = 0.f;
#pragma unroll 4
    for (u32 i = i0; i < i1; ++i) s += Ap[row_sym2<u32>(n, i) + (j - i)] * t[i];
    part[(size_t)blockIdx.y * npad + j] = s;
}

__global__ __launch_bounds__(256) void batax_aty_reduce_kernel(const float *__restrict__ part, float *__restrict__ y,
                                                              u32 n, u32 npad, float beta)
{
    u32 j = blockIdx.x * 256u + threadIdx.x;
    if (j >= n) return;
    float s = 0.f;
#pragma unroll 8
    for (u32 q = 0; q < ATY_SLICES; ++q) s += part[(size_t)q * npad + j];
    y[j] = beta * s;
}

constexpr int NMAX_ONEPASS = 16384;         // rows of up to 64 KB stay in one workgroup's registers

static inline u32 onepass_grid(int n) { return (u32)(n < GMAX ? n : GMAX); }
static inline u32 pad4(int n) { return ((u32)n + 3u) & ~3u; }

size_t batax_workspace(int n)
{
    if (n <= NMAX_ONEPASS) return (size_t)onepass_grid(n) * pad4(n) * sizeof(float);
    return (size_t)(1u + ATY_SLICES) * pad4(n) * sizeof(float);       // t, then the slice partials of y
}

// V column groups per thread; a batch is RB_SHORT rows up to two groups, two rows at three, one row at four (the
// registers of a 1024-thread workgroup hold that much twice)
template <int V, int RB>
static void launch_onepass(bool fast, u32 G, hipStream_t s, const float *Ap, const float *x, float *wsf, u32 un,
                           u32 npad)
{
    if (fast)
        hipLaunchKernelGGL((batax_onepass_kernel<V, RB, true>), dim3(G), dim3(BT), 0, s, Ap, x, wsf, un, npad, G);
    else
        hipLaunchKernelGGL((batax_onepass_kernel<V, RB, false>), dim3(G), dim3(BT), 0, s, Ap, x, wsf, un, npad, G);
}

st_status launch_batax(const float *Ap, const float *x, float *y, int n, float beta, void *ws,
                       hipStream_t s)
{
    u32 un = (u32)n;
    float *wsf = static_cast<float *>(ws);
    if (n <= NMAX_ONEPASS) {
        u32 G = onepass_grid(n), npad = pad4(n);
        const bool fast = (n % 4 == 0) && n >= 4;
        int V = (n + 4 * BT - 1) / (4 * BT);
        if (V <= 1) launch_onepass<1, RB_SHORT>(fast, G, s, Ap, x, wsf, un, npad);
        else if (V == 2) launch_onepass<2, RB_SHORT>(fast, G, s, Ap, x, wsf, un, npad);
        else if (V == 3) launch_onepass<3, 2>(fast, G, s, Ap, x, wsf, un, npad);
        else launch_onepass<4, 1>(fast, G, s, Ap, x, wsf, un, npad);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(batax_reduce_kernel, dim3((npad / 4u + 7u) / 8u), dim3(256), 0, s, wsf, y, un, npad,
                           G, beta);
        return launch_status();
    }
    const u32 npad = pad4(n);
    hipLaunchKernelGGL(batax_ax_kernel, dim3((un + 3u) / 4u), dim3(256), 0, s, Ap, x, wsf, un);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    hipLaunchKernelGGL(batax_aty_kernel, dim3((un + 255u) / 256u, ATY_SLICES), dim3(256), 0, s, Ap, wsf, wsf + npad, un,
                       npad);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    hipLaunchKernelGGL(batax_aty_reduce_kernel, dim3((un + 255u) / 256u), dim3(256), 0, s, wsf + npad, y, un, npad, beta);
    return launch_status();
}

// ---- the same computation for callers that cannot allocate ------------------------------------------
// The per-workgroup partial results live in a file-scope device array instead of a caller workspace.  The
// array's name is only a host-side handle: its device address is looked up once per device (each GPU holds
// its own copy at its own address) and that address is what the kernels receive, exactly as they receive
// the caller's workspace in launch_batax.  Every call on a GPU uses the same array, so two calls that
// overlap in time on one GPU race; nothing in it has to start at zero (every word a call reads, it has
// written before).
constexpr int NMAX_STATIC = 8192;
constexpr size_t SCRATCH_BYTES = (size_t)GMAX * NMAX_STATIC * sizeof(float);        // 8 MiB
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

int batax_static_max_n() { return NMAX_STATIC; }

st_status launch_batax_static(const float *Ap, const float *x, float *y, int n, float beta, hipStream_t s)
{
    static std::mutex mu;
    static void *scratch_of_device[64] = {nullptr};
    if (n < 1 || n > NMAX_STATIC || batax_workspace(n) > SCRATCH_BYTES) return ST_ERR_UNSUPPORTED;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return ST_ERR_LAUNCH;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (scratch_of_device[dev] == nullptr) {
            void *p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return ST_ERR_LAUNCH;
            scratch_of_device[dev] = p;
        }
        ptr = scratch_of_device[dev];
    }
    return launch_batax(Ap, x, y, n, beta, ptr, s);
}

}  // namespace st
