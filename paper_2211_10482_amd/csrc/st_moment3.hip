// Third-moment accumulation over the unique set i<=j<=k,
//     Sc(rank3(i,j,k)) (+)= sum_s X(s,i) X(s,j) X(s,k).
//
// The sum over samples is a dense contraction  S(i,(j,k)) = sum_s X(s,i) P(s,(j,k))
// with P = x_j x_k formed on the fly, so it runs on the fp32 matrix cores
// (v_mfma_f32_16x16x4_f32: a 16 x 16 tile of outputs, four samples per
// instruction).  What keeps it in the unique space is the choice of tiles.
//
// MFMA path (n <= 64, indices padded to 64).  The 64 indices are split into
// four groups of 16, group g = {4m+g}; one 16-byte load per lane then delivers
// the A operand of all four groups at once (lane = (m, sample slot)).  An
// unordered index triple is classified by the groups it touches:
//   * three different groups: columns = (fixed element m of group b) x (16 elements
//     of group c), rows = a group outside {b, c}.  P = xa[c] * broadcast_m(xa[b]) is
//     ONE VALU multiply with a DPP row broadcast, and it serves BOTH row groups
//     outside {b, c}: the column pairs (0,1) carry the rows of groups 2 and 3, the
//     column pairs (2,3) those of groups 0 and 1.  2 * 16 products, 4 * 16 tiles, all
//     outputs unique.
//   * a pair inside one group g, third index anywhere (group r): columns = the
//     16 pairs (m, m-d mod 16) of g at cyclic distance d = 0..8, rows = group r.
//     P = xa[g] * rotate_d(xa[g]) is one VALU multiply with a DPP row rotate
//     and is shared by the four row groups.  When r = g all three indices lie in
//     one group of 16 and two of them have the same parity, i.e. an even
//     distance: the tiles (g, odd d, r = g) are not needed.  At distance 8 there
//     are only 8 pairs per group, so two groups share a tile (a lane select
//     between two products).  4 * (4 * 4 + 4 * 3) + 8 tiles.
// The tiles are dealt to the eight waves by PRODUCT: all tiles that multiply by the
// same pair product go to one wave, so every product is formed once per K-step in
// the whole workgroup (70 vector instructions for the 184 MFMAs; on this chip vector
// instructions and single-precision MFMAs do not overlap).
// 184 tiles cover every unordered triple (47,104 accumulators for the 45,760
// unique entries, against 64^3 = 262,144 dense ones).  A workgroup (8 waves,
// 23 tiles = 92 accumulator
// registers per wave) owns ALL accumulators and streams a contiguous slice of
// the samples through a double-buffered LDS chunk of 64 samples that the whole
// workgroup loads once (X is read from HBM exactly once; the loads of chunk c+2
// are in flight while chunk c is multiplied).  Workgroup partials go to the
// workspace in raw tile layout (coalesced) and a second kernel adds them in a
// fixed order, drops the padding / duplicate positions and scatters through
// rank3.  No float atomics.
//
// Other feature counts: a table-driven matrix-core kernel for 64 < n <= 256 with
// n >= 14 * ceil(n/16) (st_moment_mfma.hip), register tiles on the vector ALUs for
// n <= 40 and the rest up to 256, one thread per unique entry and sample slice beyond.
#include <type_traits>
#include <utility>

#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int... Is, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F &&f)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F &&>(f));
}

constexpr int M3_WAVES = 8;
constexpr int M3_TPW = 23;                         // tiles per wave
constexpr int M3_TILES = M3_WAVES * M3_TPW;        // 184
constexpr int M3_ACC = M3_TILES * 256;             // accumulators per workgroup
constexpr int M3_GMAX = 256;

// lane m of each 16-lane row reads lane (m - D) mod 16 of the same row
template <int D> __device__ __forceinline__ float row_ror(float v)
{
    if constexpr (D == 0) return v;
    else
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v),
                                                                     0x120 + D, 0xf, 0xf, false));
}
// every lane of a 16-lane row reads lane M of that row
template <int M> __device__ __forceinline__ float row_bcast(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v),
                                                                 0x150 + M, 0xf, 0xf, false));
}

// other * (lane M of bsrc's 16-lane row) in one VALU instruction.  Written out because
// the compiler materialises a broadcast that has two users as a separate move.  The
// instruction is opaque to the compiler's hazard checks, so the caller keeps VALU writes
// of `bsrc` at least two instructions away (here: bsrc only ever comes from LDS loads,
// and the block of these products starts with the required wait states).
template <int M> __device__ __forceinline__ float mul_bcast(float bsrc, float other)
{
#ifdef ST_NO_GPU_ASSEMBLY   // a build of this source for another target (the CPU bounds check of the tests)
    return row_bcast<M>(bsrc) * other;
#else
    float r;
    asm volatile("v_mul_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                 : "=v"(r)
                 : "v"(bsrc), "v"(other), "n"(M));
    return r;
#endif
}

// Tile descriptor shared by the accumulation kernel (compile time) and the
// reduction kernel (run time).  A unit is the set of tiles that use one product:
//   E(g, d even) : pairs of group g at distance d = 0, 2, 4, 6, row groups 0..3        (4 tiles, 1 multiply)
//   O(g, d odd)  : the same at d = 1, 3, 5, 7, row groups other than g                 (3 tiles, 1 multiply)
//   D(g, g+1)    : distance 8 of the groups (0,1) or (2,3), row groups 0..3            (4 tiles, 2 multiplies + select)
//   K(b, c; m)   : element m of group b times group c, (b,c) = (0,1) with row groups 2, 3
//                  or (2,3) with row groups 0, 1                                        (2 tiles, 1 multiply)
// 16 + 16 + 2 + 32 units.  Every wave holds 23 tiles: waves 0..3 two E, three O, three K (8 vector
// instructions per K-step); waves 4, 5 two E, one O, one D, four K (10); waves 6, 7 two E, one O, six K (9).
// Waves w and w+4 share a SIMD: 18, 18, 17, 17 vector instructions per SIMD and K-step.
struct TileDesc {
    int kind;   // 0: pair inside group gb at distance d; 1: (element m of gb) x (group gc);
                // 2: pairs at distance 8, columns 0..7 of group gb, columns 8..15 of group gc
    int r;      // row group
    int gb, gc; // column groups (gc unused for kind 0)
    int d;      // cyclic distance (kinds 0, 2) or fixed element m (kind 1)
};
__host__ __device__ constexpr TileDesc tile_desc(int w, int local)
{
    // pair-in-group units at an even distance (four tiles, r = 0..3): every wave takes two
    if (local < 8) {
        const int eu = 2 * w + local / 4;
        return TileDesc{0, local % 4, eu / 4, 0, 2 * (eu % 4)};
    }
    int l = local - 8;
    // at an odd distance (three tiles, r != g): waves 0..3 take three units, waves 4..7 one
    const int no = w < 4 ? 3 : 1, o0 = w < 4 ? 3 * w : 8 + w;
    if (l < 3 * no) {
        const int ou = o0 + l / 3, g = ou / 4, v = l % 3;
        return TileDesc{0, v + (v >= g ? 1 : 0), g, 0, 2 * (ou % 4) + 1};
    }
    l -= 3 * no;
    // distance 8 (four tiles, r = 0..3): waves 4 and 5
    if (w == 4 || w == 5) {
        if (l < 4) return TileDesc{2, l, 2 * (w - 4), 2 * (w - 4) + 1, 8};
        l -= 4;
    }
    // broadcast units (two tiles): three for waves 0..3, four for waves 4 and 5, six for waves 6 and 7
    const int k0 = w < 4 ? 3 * w : w == 4 ? 12 : w == 5 ? 16 : w == 6 ? 20 : 26;
    const int ku = k0 + l / 2;
    if (ku < 16) return TileDesc{1, 2 + l % 2, 0, 1, ku};
    return TileDesc{1, l % 2, 2, 3, ku - 16};
}
// first tile of the wave that multiplies by the same pair product
__host__ __device__ constexpr int m3_product_of(int w, int local)
{
    const TileDesc a = tile_desc(w, local);
    for (int u = 0; u < local; ++u) {
        const TileDesc b = tile_desc(w, u);
        if (a.kind == b.kind && a.gb == b.gb && a.gc == b.gc && a.d == b.d) return u;
    }
    return local;
}

// every pair product is formed by exactly one wave: 66 products (16 + 16 + 2 + 32 units) in 70 vector instructions
__host__ __device__ constexpr int m3_products_formed()
{
    int formed = 0;
    for (int w = 0; w < M3_WAVES; ++w)
        for (int t = 0; t < M3_TPW; ++t)
            if (m3_product_of(w, t) == t) ++formed;
    return formed;
}
__host__ __device__ constexpr bool m3_product_in_one_wave()
{
    for (int w = 0; w < M3_WAVES; ++w)
        for (int t = 0; t < M3_TPW; ++t) {
            const TileDesc a = tile_desc(w, t);
            for (int w2 = w + 1; w2 < M3_WAVES; ++w2)
                for (int u = 0; u < M3_TPW; ++u) {
                    const TileDesc b = tile_desc(w2, u);
                    if (a.kind == b.kind && a.gb == b.gb && a.gc == b.gc && a.d == b.d) return false;
                }
        }
    return true;
}
static_assert(m3_products_formed() == 66 && m3_product_in_one_wave(), "tiles are dealt to the waves by product");

#ifndef ST_M3_CH
#define ST_M3_CH 64
#endif
constexpr int M3_CH = ST_M3_CH;                    // samples per staged chunk (a multiple of 16)
constexpr int M3_THREADS = M3_WAVES * 64;
constexpr int M3_LPT = M3_CH * 16 / M3_THREADS;    // 16-byte pieces of a chunk per thread (2)

// A chunk of 64 samples is staged in LDS as [sample][64 columns] by the whole
// workgroup (each row of X is fetched from HBM exactly once), columns >= n and
// samples past the end of the slice as zeros.  load_chunk only issues the loads
// (row clamped into the slice, nothing touches the results) so that they stay in
// flight under the MFMAs of the previous chunks; store_chunk masks and writes.
template <bool FULL>
__device__ __forceinline__ void load_chunk(f32x4 (&r)[M3_LPT], const float *__restrict__ X, int64_t s0,
                                           int64_t s_end, u32 n, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M3_LPT; ++k) {
        const u32 j = tid + (u32)M3_THREADS * k, smp = j >> 4, c0 = 4u * (j & 15u);
        const int64_t s = s0 + smp, sc = s < s_end ? s : s_end - 1;
        if constexpr (FULL) {
            float4 t = *reinterpret_cast<const float4 *>(X + sc * 64 + c0);
            r[k] = (f32x4){t.x, t.y, t.z, t.w};
        } else {
            const float *row = X + sc * (int64_t)n;
#pragma unroll
            for (u32 g = 0; g < 4; ++g) r[k][g] = row[c0 + g < n ? c0 + g : n - 1];
        }
    }
}
template <bool FULL>
__device__ __forceinline__ void store_chunk(const f32x4 (&r)[M3_LPT], float *__restrict__ buf, int64_t s0,
                                            int64_t s_end, u32 n, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M3_LPT; ++k) {
        const u32 j = tid + (u32)M3_THREADS * k, smp = j >> 4, c0 = 4u * (j & 15u);
        const bool live = s0 + smp < s_end;
        f32x4 v;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) v[g] = (live && (FULL || c0 + g < n)) ? r[k][g] : 0.f;
        *reinterpret_cast<f32x4 *>(buf + smp * 64u + c0) = v;
    }
}

// The same two steps for a chunk that lies wholly inside the slice, 64 features: every address is a wave-uniform
// base plus an offset the lane keeps for the whole kernel, nothing is masked (the general forms above cost about
// fifty vector instructions per chunk and wave in 64-bit index arithmetic, compares and selects, and on this chip
// those are not hidden behind the MFMAs).
__device__ __forceinline__ void load_whole_chunk(f32x4 (&r)[M3_LPT], const float *__restrict__ chunk, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M3_LPT; ++k) {
        const float4 t = *reinterpret_cast<const float4 *>(chunk + 4u * (tid + (u32)M3_THREADS * k));
        r[k] = (f32x4){t.x, t.y, t.z, t.w};
    }
}
__device__ __forceinline__ void store_whole_chunk(const f32x4 (&r)[M3_LPT], float *__restrict__ buf, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M3_LPT; ++k) *reinterpret_cast<f32x4 *>(buf + 4u * (tid + (u32)M3_THREADS * k)) = r[k];
}

template <int W>
__device__ __forceinline__ void m3_step(f32x4 (&acc)[M3_TPW], const f32x4 &xa, bool upper)
{
    // All pair products of the step first, each in a register of its own, then the
    // MFMAs back to back: a product that is formed right in front of its MFMA in
    // a recycled register has to wait for the previous MFMA to release it.
    float p[M3_TPW];
    ST_WAIT_STATES(1);
    static_for<M3_TPW>([&](auto T) {
        constexpr TileDesc td = tile_desc(W, decltype(T)::value);
        if constexpr (td.kind == 1 && m3_product_of(W, decltype(T)::value) == decltype(T)::value)
            p[T] = mul_bcast<td.d>(xa[td.gb], xa[td.gc]);
    });
    static_for<M3_TPW>([&](auto T) {
        constexpr TileDesc td = tile_desc(W, decltype(T)::value);
        if constexpr (m3_product_of(W, decltype(T)::value) == decltype(T)::value) {
            if constexpr (td.kind == 0) p[T] = xa[td.gb] * row_ror<td.d>(xa[td.gb]);
            if constexpr (td.kind == 2) {
                // lanes m < 8: pair (m, m+8) of group gb; lanes m >= 8: pair (m-8, m) of group gc
                const float lo = xa[td.gb] * row_ror<8>(xa[td.gb]), hi = xa[td.gc] * row_ror<8>(xa[td.gc]);
                p[T] = upper ? hi : lo;
            }
        }
    });
    __builtin_amdgcn_sched_barrier(0);
    static_for<M3_TPW>([&](auto T) {
        constexpr TileDesc td = tile_desc(W, decltype(T)::value);
        constexpr int pi = m3_product_of(W, decltype(T)::value);
        acc[T] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[td.r], p[pi], acc[T], 0, 0, 0);
    });
    __builtin_amdgcn_sched_barrier(0);
}

template <int W, bool FULL>
__device__ __forceinline__ void m3_wave(const float *__restrict__ X, int64_t s_begin, int64_t s_end,
                                        u32 n, float *__restrict__ part, float (*xs)[M3_CH * 64], u32 tid)
{
    const u32 lane = tid & 63u;
    const bool upper = (lane & 8u) != 0u;
    f32x4 acc[M3_TPW];
#pragma unroll
    for (int t = 0; t < M3_TPW; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int64_t nchunks = (s_end - s_begin + M3_CH - 1) / M3_CH;
    f32x4 r[M3_LPT];
    load_chunk<FULL>(r, X, s_begin, s_end, n, tid);
    store_chunk<FULL>(r, xs[0], s_begin, s_end, n, tid);
    if (nchunks > 1) load_chunk<FULL>(r, X, s_begin + M3_CH, s_end, n, tid);
    __syncthreads();

    // lane (m, q) reads X(s + q, 4m .. 4m+3): component g is the A operand of group g
    const float *mine = &xs[0][0] + lane * 4u;
    // One chunk: the registers hold chunk c+1: park it in the other buffer (its readers finished before the
    // barrier that ended the previous iteration), put chunk c+2 in flight, then the MFMAs of chunk c.
    // WHOLE: chunks c+1 and c+2 exist and lie wholly inside the slice (all iterations but the last three): the
    // staging has no conditions, no masks and no 64-bit index arithmetic per lane.
    auto chunk = [&](int64_t c, auto whole) {
        constexpr bool WHOLE = FULL && decltype(whole)::value;
        const u32 cb = (u32)(c & 1);
        if constexpr (WHOLE) {
            store_whole_chunk(r, xs[cb ^ 1u], tid);
            load_whole_chunk(r, X + (s_begin + (c + 2) * M3_CH) * 64, tid);
        } else {
            if (c + 1 < nchunks) store_chunk<FULL>(r, xs[cb ^ 1u], s_begin + (c + 1) * M3_CH, s_end, n, tid);
            if (c + 2 < nchunks) load_chunk<FULL>(r, X, s_begin + (c + 2) * M3_CH, s_end, n, tid);
        }
        __builtin_amdgcn_sched_barrier(0);
        const float *src = mine + cb * (M3_CH * 64);
        f32x4 xa[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) xa[k] = *reinterpret_cast<const f32x4 *>(src + k * 256);
        // groups of four K-steps; kept as a real loop so that the eight per-wave
        // code streams stay small enough for the instruction cache
        constexpr int NG = M3_CH / 16;
#pragma unroll 1
        for (int g = 0; g < NG; ++g) {
            // (the last group re-reads itself, which is harmless)
            const float *nsrc = src + (g < NG - 1 ? g + 1 : NG - 1) * 1024;
            // each operand register is refilled with the next group's K-step right after
            // its last use, so three steps of MFMAs cover the LDS latency
            m3_step<W>(acc, xa[0], upper);
            xa[0] = *reinterpret_cast<const f32x4 *>(nsrc);
            m3_step<W>(acc, xa[1], upper);
            xa[1] = *reinterpret_cast<const f32x4 *>(nsrc + 256);
            m3_step<W>(acc, xa[2], upper);
            xa[2] = *reinterpret_cast<const f32x4 *>(nsrc + 512);
            m3_step<W>(acc, xa[3], upper);
            xa[3] = *reinterpret_cast<const f32x4 *>(nsrc + 768);
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    };
    int64_t c = 0;
    if constexpr (FULL)
        for (; c + 3 < nchunks; ++c) chunk(c, std::true_type{});
    for (; c < nchunks; ++c) chunk(c, std::false_type{});

    float *dst = part + (size_t)W * M3_TPW * 256 + lane;
#pragma unroll
    for (int t = 0; t < M3_TPW; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) dst[(t * 4 + v) * 64] = acc[t][v];
}

template <bool FULL>
__global__ __launch_bounds__(M3_THREADS) void moment3_mfma_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                                int64_t chunk, float *__restrict__ ws)
{
    __shared__ __attribute__((aligned(16))) float xs[2][M3_CH * 64];
    const u32 tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane((int)(tid >> 6));
    int64_t s_begin = (int64_t)blockIdx.x * chunk;
    int64_t s_end = s_begin + chunk < N ? s_begin + chunk : N;
    float *part = ws + (size_t)blockIdx.x * M3_ACC;
    // every wave runs the same chunk loop (same number of barriers) over its own tiles
    switch (wave) {
    case 0: m3_wave<0, FULL>(X, s_begin, s_end, n, part, xs, tid); break;
    case 1: m3_wave<1, FULL>(X, s_begin, s_end, n, part, xs, tid); break;
    case 2: m3_wave<2, FULL>(X, s_begin, s_end, n, part, xs, tid); break;
    case 3: m3_wave<3, FULL>(X, s_begin, s_end, n, part, xs, tid); break;
    case 4: m3_wave<4, FULL>(X, s_begin, s_end, n, part, xs, tid); break;
    case 5: m3_wave<5, FULL>(X, s_begin, s_end, n, part, xs, tid); break;
    case 6: m3_wave<6, FULL>(X, s_begin, s_end, n, part, xs, tid); break;
    default: m3_wave<7, FULL>(X, s_begin, s_end, n, part, xs, tid); break;
    }
}

__device__ __forceinline__ void sort3u(u32 &a, u32 &b, u32 &c)
{
    u32 lo = min(a, b), hi = max(a, b);
    u32 mn = min(lo, c), mx = max(hi, c), md = max(lo, min(hi, c));
    a = mn; b = md; c = mx;
}

// Adds the G workgroup partials and scatters the unique ones.  A block owns 64 raw
// accumulators and cuts the partials into 4 slices (g ascending inside a slice,
// slices ascending).
__global__ __launch_bounds__(256) void moment3_reduce_kernel(const float *__restrict__ ws, u32 G, u32 n,
                                                            float *__restrict__ Sc, int accumulate)
{
    __shared__ float accs[4][64];
    const u32 lane = threadIdx.x & 63u, sl = threadIdx.x >> 6;
    const u32 e = blockIdx.x * 64u + lane;        // raw accumulator id, < M3_ACC
    const u32 tile = e >> 8, v = (e >> 6) & 3u;
    TileDesc td = tile_desc((int)(tile / M3_TPW), (int)(tile % M3_TPW));
    // D layout of the 16x16 MFMA: lane holds column lane%16 of rows 4*(lane/16) + v
    u32 rowel = 4u * (lane >> 4) + v, col = lane & 15u;
    u32 i = 4u * rowel + (u32)td.r, j, k;
    bool keep;
    if (td.kind != 1) {
        const u32 other = (col - (u32)td.d) & 15u;
        const u32 g = (td.kind == 0 || col < 8u) ? (u32)td.gb : (u32)td.gc;
        j = 4u * col + g;
        k = 4u * other + g;
        keep = true;
        if ((u32)td.r == g) {
            // all three in one group: the triple has up to three (row, pair) positions, and only pairs at an
            // even distance have a tile with r = g (two of three indices have the same parity); the position
            // whose pair is closest (then: whose row is smallest) is kept.
            const u32 d1 = (rowel - other) & 15u, d2 = (rowel - col) & 15u;
            const u32 c1 = min(d1, 16u - d1), c2 = min(d2, 16u - d2);
            const u32 key = 16u * (u32)td.d + rowel;
            const u32 key1 = (c1 & 1u) ? 0xffffu : 16u * c1 + col, key2 = (c2 & 1u) ? 0xffffu : 16u * c2 + other;
            keep = key <= key1 && key <= key2;
        }
    } else {
        j = 4u * (u32)td.d + (u32)td.gb;
        k = 4u * col + (u32)td.gc;
        keep = true;
    }
    keep = keep && i < n && j < n && k < n;
    float s = 0.f;
    if (keep) {
        const u32 per = (G + 3u) / 4u, g0 = min(G, sl * per), g1 = min(G, g0 + per);
        const float *src = ws + e;
#pragma unroll 8
        for (u32 g = g0; g < g1; ++g) s += src[(size_t)g * M3_ACC];
    }
    accs[sl][lane] = s;
    __syncthreads();
    if (sl == 0 && keep) {
        s = (accs[0][lane] + accs[1][lane]) + (accs[2][lane] + accs[3][lane]);
        sort3u(i, j, k);
        u32 p = rank_sym3<u32>(n, i, j, k);
        Sc[p] = accumulate ? Sc[p] + s : s;
    }
}

// ---- general path -----------------------------------------------------------------
__global__ __launch_bounds__(256) void moment3_plain_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                           u32 count, int64_t slice,
                                                           float *__restrict__ part)
{
    u32 p = blockIdx.x * 256u + threadIdx.x;
    if (p >= count) return;
    u32 i, j, k;
    unrank_sym3<u32>(n, p, i, j, k);
    int64_t s0 = (int64_t)blockIdx.y * slice, s1 = s0 + slice < N ? s0 + slice : N;
    float s = 0.f;
    for (int64_t q = s0; q < s1; ++q) {
        const float *row = X + q * (int64_t)n;
        s += row[i] * row[j] * row[k];
    }
    part[(size_t)blockIdx.y * count + p] = s;
}

__global__ __launch_bounds__(256) void moment3_plain_reduce_kernel(const float *__restrict__ part, u32 SY,
                                                                  u32 count, float *__restrict__ Sc,
                                                                  int accumulate)
{
    u32 p = blockIdx.x * 256u + threadIdx.x;
    if (p >= count) return;
    float s = 0.f;
    for (u32 y = 0; y < SY; ++y) s += part[(size_t)y * count + p];
    Sc[p] = accumulate ? Sc[p] + s : s;
}

__global__ __launch_bounds__(256) void zero_kernel(float *__restrict__ p, u32 count)
{
    u32 t = blockIdx.x * 256u + threadIdx.x;
    if (t < count) p[t] = 0.f;
}

static inline int64_t m3_chunk(int64_t N)
{
    int64_t c = (N + M3_GMAX - 1) / M3_GMAX;
    c = (c + M3_CH - 1) / M3_CH * M3_CH;
    return c;
}
static inline u32 m3_groups(int64_t N) { return N == 0 ? 0u : (u32)((N + m3_chunk(N) - 1) / m3_chunk(N)); }
static inline u32 plain_slices(int64_t N)
{
    int64_t s = (N + 1023) / 1024;
    return (u32)(s < 1 ? 1 : s > 16 ? 16 : s);
}


// ---- tile path: any n <= 256, plain fp32 vector arithmetic ------------------------------------
// For feature counts other than the 64 the matrix-core kernel above is built around.  The indices are
// cut into blocks of four; a block triple I <= J <= K (unranked with the closed form of the entries
// themselves, on n/4 blocks) is owned by ONE lane with its 4 x 4 x 4 accumulators in registers: per
// sample the lane reads the three 16-byte groups x_I, x_J, x_K from the staged sample row and does
// 16 + 64 multiply(-add)s (a_ij = x_i x_j, acc_ijk += a_ij x_k).  Only the block diagonals are padded.
// Samples go through a double-buffered LDS chunk per workgroup (rows padded to 4*ceil(n/4) floats,
// loads of chunk c+2 in flight while chunk c is consumed); the sample range is cut into slices
// (grid.y) so that the grid fills the chip; with fewer than 64 block triples (n <= 24) a wave holds every
// triple several times and the copies share out the samples of a chunk.  Slice partials -> second kernel
// adds them in a fixed order, keeps i <= j <= k < n and scatters through rank3.  No atomics.
constexpr int M3T_LPT = 8;                         // 16-byte pieces of a chunk per thread
constexpr int M3T_WGTARGET = 1024;                 // workgroups to aim for

struct M3TPlan {
    u32 nb4, np, nbt, threads, gx, ch, S;
    u32 sub;                 // fewer than 64 block triples: a wave holds `sub` copies, copy q takes the samples = q mod sub
    int64_t slice;
};
static inline M3TPlan m3t_plan(int64_t N, int n)
{
    M3TPlan p;
    p.nb4 = ((u32)n + 3u) / 4u;
    p.np = 4u * p.nb4;
    p.nbt = (u32)count_sym3<int64_t>(p.nb4);
    p.threads = p.nbt >= 256u ? 256u : ((p.nbt + 63u) / 64u) * 64u;
    p.sub = p.nbt < 64u ? 64u / p.nbt : 1u;
    p.gx = (p.nbt + p.threads - 1u) / p.threads;
    u32 ch = (u32)M3T_LPT * p.threads * 4u / p.np;           // samples whose pieces fit the threads' registers
    ch = ch > 64u ? 64u : ch & ~7u;
    p.ch = ch;
    int64_t S = (M3T_WGTARGET + p.gx - 1) / p.gx;
    const int64_t smax = (N + p.ch - 1) / p.ch;
    if (S > smax) S = smax;
    if (S > 1024) S = 1024;
    if (S < 1) S = 1;
    p.slice = ((N + S - 1) / S + p.ch - 1) / p.ch * p.ch;    // whole chunks
    p.S = (u32)((N + p.slice - 1) / p.slice);
    return p;
}

__device__ __forceinline__ void m3t_load_chunk(f32x4 (&r)[M3T_LPT], const float *__restrict__ X, int64_t s0,
                                               int64_t s_end, u32 n, u32 np4, u32 pieces, u32 tid, u32 nthreads)
{
#pragma unroll
    for (int k = 0; k < M3T_LPT; ++k) {
        const u32 j = min(tid + nthreads * (u32)k, pieces - 1u), smp = j / np4, c0 = 4u * (j - smp * np4);
        const int64_t s = s0 + smp, sc = s < s_end ? s : s_end - 1;
        const float *row = X + sc * (int64_t)n;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) r[k][g] = row[c0 + g < n ? c0 + g : n - 1u];
    }
}

__device__ __forceinline__ void m3t_store_chunk(const f32x4 (&r)[M3T_LPT], float *__restrict__ buf, int64_t s0,
                                                int64_t s_end, u32 n, u32 np4, u32 pieces, u32 tid, u32 nthreads)
{
#pragma unroll
    for (int k = 0; k < M3T_LPT; ++k) {
        const u32 j = tid + nthreads * (u32)k, smp = j / np4, c0 = 4u * (j - smp * np4);
        if (j >= pieces) continue;
        const bool row_ok = s0 + smp < s_end;
        f32x4 v;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) v[g] = (row_ok && c0 + g < n) ? r[k][g] : 0.f;
        *reinterpret_cast<f32x4 *>(buf + (size_t)j * 4u) = v;       // [sample][np] = piece order
    }
}

// grid.x = block triples / blockDim.x, grid.y = sample slices; dynamic LDS: 2 chunks of ch x np floats.
// SUBBED (fewer than 64 block triples, one wave per workgroup): the wave holds every triple `sub` times,
// copy q takes the samples = q (mod sub) of a chunk, and the copies are added through LDS in a fixed
// order before the slice partial is written.
template <bool SUBBED>
__global__ __launch_bounds__(256) void moment3_tile_kernel(const float *__restrict__ X, int64_t N, u32 n, u32 nb4,
                                                          u32 nbt, u32 ch, u32 sub, int64_t slice,
                                                          float *__restrict__ ws)
{
    extern __shared__ float lds[];
    float *m3t_lds = lds;
    const u32 tid = threadIdx.x, nthreads = blockDim.x, np = 4u * nb4, np4 = nb4;
    const u32 pieces = ch * np4, chunk_f = ch * np;
    // SUBBED: lane = (copy, triple)
    const u32 copy = SUBBED ? tid / nbt : 0u;
    const u32 bt = SUBBED ? tid - copy * nbt : blockIdx.x * nthreads + tid;
    const bool active = SUBBED ? copy < sub : bt < nbt;
    u32 I, J, K;
    unrank_sym3<u32>(nb4, min(bt, nbt - 1u), I, J, K);
    const u32 oi = 4u * I, oj = 4u * J, ok = 4u * K;

    const int64_t s_begin = (int64_t)blockIdx.y * slice;
    const int64_t s_end = s_begin + slice < N ? s_begin + slice : N;
    const int64_t nchunks = s_end > s_begin ? (s_end - s_begin + ch - 1) / ch : 0;

    float acc[64];
#pragma unroll
    for (int e = 0; e < 64; ++e) acc[e] = 0.f;

    if (nchunks > 0) {
        f32x4 r[M3T_LPT];
        m3t_load_chunk(r, X, s_begin, s_end, n, np4, pieces, tid, nthreads);
        m3t_store_chunk(r, m3t_lds, s_begin, s_end, n, np4, pieces, tid, nthreads);
        if (nchunks > 1) m3t_load_chunk(r, X, s_begin + ch, s_end, n, np4, pieces, tid, nthreads);
        __syncthreads();
        for (int64_t c = 0; c < nchunks; ++c) {
            const u32 cb = (u32)(c & 1);
            // registers hold chunk c+1: park it in the other buffer (its readers finished before the
            // barrier that ended the previous iteration), then put chunk c+2 in flight
            if (c + 1 < nchunks)
                m3t_store_chunk(r, m3t_lds + (cb ^ 1u) * chunk_f, s_begin + (c + 1) * ch, s_end, n, np4, pieces, tid,
                                nthreads);
            if (c + 2 < nchunks) m3t_load_chunk(r, X, s_begin + (c + 2) * ch, s_end, n, np4, pieces, tid, nthreads);
            __builtin_amdgcn_sched_barrier(0);
            const float *row = m3t_lds + cb * chunk_f + (SUBBED && active ? copy : 0u) * np;
            const u32 sstep = SUBBED ? sub : 1u, rstep = sstep * np;
#pragma unroll 2
            for (u32 smp = SUBBED && active ? copy : 0u; smp < ch; smp += sstep, row += rstep) {
                const f32x4 xi = *reinterpret_cast<const f32x4 *>(row + oi);
                const f32x4 xj = *reinterpret_cast<const f32x4 *>(row + oj);
                const f32x4 xk = *reinterpret_cast<const f32x4 *>(row + ok);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float a = xi[i] * xj[j];
#pragma unroll
                        for (int k = 0; k < 4; ++k) acc[(i * 4 + j) * 4 + k] += a * xk[k];
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
        }
    }

    if constexpr (SUBBED) {
        // add the copies: lane -> LDS row (stride 65: conflict free), then thread e adds accumulator e of
        // every triple over the copies in ascending order (the loop above ended with a barrier)
        float *red = m3t_lds;
#pragma unroll
        for (int e = 0; e < 64; ++e) red[tid * 65u + e] = active ? acc[e] : 0.f;
        __syncthreads();
        for (u32 b = 0; b < nbt; ++b) {
            float v = 0.f;
            for (u32 c = 0; c < sub; ++c) v += red[(c * nbt + b) * 65u + tid];
            ws[((size_t)blockIdx.y * nbt + b) * 64u + tid] = v;
        }
    } else if (active) {
        f32x4 *dst = reinterpret_cast<f32x4 *>(ws + ((size_t)blockIdx.y * nbt + bt) * 64u);
#pragma unroll
        for (int e = 0; e < 16; ++e) dst[e] = (f32x4){acc[4 * e], acc[4 * e + 1], acc[4 * e + 2], acc[4 * e + 3]};
    }
}

// A block owns 16 raw accumulators (block triple, i, j, k) and cuts the S slice partials into 16 groups
// (slices g, g+16, ... ascending inside a group, groups ascending); stores the entries of the unique set.
__global__ __launch_bounds__(256) void moment3_tile_reduce_kernel(const float *__restrict__ ws, u32 S, u32 n,
                                                                 u32 nb4, u32 nbt, float *__restrict__ Sc,
                                                                 int accumulate)
{
    __shared__ float part[16][16];
    const u32 a = threadIdx.x & 15u, g = threadIdx.x >> 4;
    const u32 t = blockIdx.x * 16u + a;                  // < nbt * 64
    const size_t stride = (size_t)nbt * 64u;
    float s = 0.f;
    if (t < nbt * 64u) {
#pragma unroll 4
        for (u32 y = g; y < S; y += 16u) s += ws[(size_t)y * stride + t];
    }
    part[g][a] = s;
    __syncthreads();
    if (g != 0u || t >= nbt * 64u) return;
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) v += part[q][a];
    const u32 bt = t >> 6, e = t & 63u;
    u32 I, J, K;
    unrank_sym3<u32>(nb4, bt, I, J, K);
    const u32 i = 4u * I + (e >> 4), j = 4u * J + ((e >> 2) & 3u), k = 4u * K + (e & 3u);
    if (!(i <= j && j <= k && k < n)) return;
    const u32 p = rank_sym3<u32>(n, i, j, k);
    Sc[p] = accumulate ? Sc[p] + v : v;
}

constexpr int M3T_NMAX = 256;                      // rows of up to 1 KB in LDS
// the matrix-core kernel pads every n <= 64 to 64 features: the tile path wins below about 40
static inline bool m3_use_tiles(int n) { return n <= 40 || (n > 64 && n <= M3T_NMAX); }

size_t moment3_workspace(int64_t N, int n)
{
    if (N == 0) return 0;
    if (moment_mfma_wins(3, n)) return moment_mfma_workspace(3, N, n);
    if (m3_use_tiles(n)) {
        const M3TPlan p = m3t_plan(N, n);
        return (size_t)p.S * p.nbt * 64u * sizeof(float);
    }
    if (n <= 64) return (size_t)m3_groups(N) * M3_ACC * sizeof(float);
    return (size_t)plain_slices(N) * (size_t)count_sym3<int64_t>(n) * sizeof(float);
}

st_status launch_moment3(const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws,
                         hipStream_t s)
{
    u32 count = (u32)count_sym3<int64_t>(n);
    if (N == 0) {
        if (!accumulate) hipLaunchKernelGGL(zero_kernel, dim3((count + 255u) / 256u), dim3(256), 0, s, Sc, count);
        return launch_status();
    }
    if (moment_mfma_wins(3, n)) return launch_moment_mfma(3, X, N, n, Sc, accumulate, ws, s);
    float *wsf = static_cast<float *>(ws);
    if (m3_use_tiles(n)) {
        const M3TPlan p = m3t_plan(N, n);
        size_t lds_bytes = (size_t)2u * p.ch * p.np * sizeof(float);                // at most 64 KB
        const bool subbed = p.sub > 1u;
        if (subbed && lds_bytes < 64u * 65u * sizeof(float)) lds_bytes = 64u * 65u * sizeof(float);
        if (!allow_dynamic_lds(reinterpret_cast<const void *>(moment3_tile_kernel<false>), 64 * 1024) ||
            !allow_dynamic_lds(reinterpret_cast<const void *>(moment3_tile_kernel<true>), 64 * 1024))
            return ST_ERR_LAUNCH;
        if (subbed)
            hipLaunchKernelGGL(moment3_tile_kernel<true>, dim3(p.gx, p.S), dim3(p.threads), lds_bytes, s, X, N, (u32)n,
                               p.nb4, p.nbt, p.ch, p.sub, p.slice, wsf);
        else
            hipLaunchKernelGGL(moment3_tile_kernel<false>, dim3(p.gx, p.S), dim3(p.threads), lds_bytes, s, X, N, (u32)n,
                               p.nb4, p.nbt, p.ch, p.sub, p.slice, wsf);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment3_tile_reduce_kernel, dim3((p.nbt * 64u + 15u) / 16u), dim3(256), 0, s, wsf, p.S,
                           (u32)n, p.nb4, p.nbt, Sc, accumulate);
        return launch_status();
    }
    if (n <= 64) {
        int64_t chunk = m3_chunk(N);
        u32 G = m3_groups(N);
        if (n == 64)
            hipLaunchKernelGGL(moment3_mfma_kernel<true>, dim3(G), dim3(M3_WAVES * 64), 0, s, X, N, (u32)n,
                               chunk, wsf);
        else
            hipLaunchKernelGGL(moment3_mfma_kernel<false>, dim3(G), dim3(M3_WAVES * 64), 0, s, X, N, (u32)n,
                               chunk, wsf);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment3_reduce_kernel, dim3(M3_ACC / 64), dim3(256), 0, s, wsf, G, (u32)n, Sc,
                           accumulate);
        return launch_status();
    }
    u32 SY = plain_slices(N);
    int64_t slice = (N + SY - 1) / SY;
    hipLaunchKernelGGL(moment3_plain_kernel, dim3((count + 255u) / 256u, SY), dim3(256), 0, s, X, N, (u32)n,
                       count, slice, wsf);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    hipLaunchKernelGGL(moment3_plain_reduce_kernel, dim3((count + 255u) / 256u), dim3(256), 0, s, wsf, SY,
                       count, Sc, accumulate);
    return launch_status();
}

}  // namespace st
