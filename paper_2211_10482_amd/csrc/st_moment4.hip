// Fourth-moment accumulation over N samples, unique entries only:
//     Sc(rank4(i,j,k,l)) (+)= sum_s X(s,i) X(s,j) X(s,k) X(s,l)      for i <= j <= k <= l
// (the M3 = vec(f (x) f) (x) vec(f (x) f) term of the degree-2 polynomial-regression
// covariance, summed over the data; about 23 of every 24 dense entries are redundant).
//
// Three paths: matrix cores for 52 < n <= 64 (described at its kernels below), and fp32
// vector arithmetic for the other sizes, where padding every index range to 64 would cost
// more than the matrix cores gain.
//
// Tile path (n <= 52), plain fp32 vector arithmetic: on the vector ALUs any set of entries
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
//
// 64 < n <= 256: the same tiles with sample rows of 4*ceil(n/4) floats in dynamic LDS.
#include <mutex>
#include <vector>

#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int M4_THREADS = 256;                    // 64 block quadruples x 4 lanes
constexpr int M4_CH = 64;                          // samples per staged chunk
constexpr int M4_LPT = M4_CH * 16 / M4_THREADS;    // 16-byte pieces of a chunk per thread (4)
constexpr int M4_WGTARGET = 1024;                  // workgroups to aim for (four per CU)

// A chunk of M4_CH samples is staged as [sample][64 columns]; columns >= n and samples
// past the end of the slice become zeros.  load_chunk only issues the loads (row clamped
// into the slice), store_chunk masks and writes.
template <bool FULL>
__device__ __forceinline__ void m4_load_chunk(f32x4 (&r)[M4_LPT], const float *__restrict__ X, int64_t s0,
                                              int64_t s_end, u32 n, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M4_LPT; ++k) {
        const u32 j = tid + (u32)M4_THREADS * k, smp = j >> 4, c0 = 4u * (j & 15u);
        const int64_t s = s0 + smp, sc = s < s_end ? s : s_end - 1;
        if constexpr (FULL) {
            const float4 t = *reinterpret_cast<const float4 *>(X + sc * 64 + c0);
            r[k] = (f32x4){t.x, t.y, t.z, t.w};
        } else {
            const float *row = X + sc * (int64_t)n;
#pragma unroll
            for (u32 g = 0; g < 4; ++g) r[k][g] = row[c0 + g < n ? c0 + g : n - 1];
        }
    }
}

template <bool FULL>
__device__ __forceinline__ void m4_store_chunk(const f32x4 (&r)[M4_LPT], float *__restrict__ buf, int64_t s0,
                                               int64_t s_end, u32 n, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M4_LPT; ++k) {
        const u32 j = tid + (u32)M4_THREADS * k, smp = j >> 4, c0 = 4u * (j & 15u);
        const bool row_ok = s0 + smp < s_end;
        f32x4 v;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) v[g] = (row_ok && (FULL || c0 + g < n)) ? r[k][g] : 0.f;
        *reinterpret_cast<f32x4 *>(buf + smp * 64u + c0) = v;
    }
}

// grid.x = block quadruples / 64, grid.y = sample slices
template <bool FULL>
__global__ __launch_bounds__(M4_THREADS) void moment4_tile_kernel(const float *__restrict__ X, int64_t N, u32 n,
                                                                u32 nb4, u32 nbq, int64_t slice,
                                                                float *__restrict__ ws)
{
    __shared__ __attribute__((aligned(16))) float xs[2][M4_CH * 64];
    const u32 tid = threadIdx.x, ii = tid & 3u;
    const u32 bq = blockIdx.x * 64u + (tid >> 2);
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
        m4_load_chunk<FULL>(r, X, s_begin, s_end, n, tid);
        m4_store_chunk<FULL>(r, xs[0], s_begin, s_end, n, tid);
        if (nchunks > 1) m4_load_chunk<FULL>(r, X, s_begin + M4_CH, s_end, n, tid);
        __syncthreads();
        for (int64_t c = 0; c < nchunks; ++c) {
            const u32 cb = (u32)(c & 1);
            // registers hold chunk c+1: park it in the other buffer (its readers finished
            // before the barrier that ended the previous iteration), then put chunk c+2 in flight
            if (c + 1 < nchunks) m4_store_chunk<FULL>(r, xs[cb ^ 1u], s_begin + (c + 1) * M4_CH, s_end, n, tid);
            if (c + 2 < nchunks) m4_load_chunk<FULL>(r, X, s_begin + (c + 2) * M4_CH, s_end, n, tid);
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

    if (bq < nbq) {
        f32x4 *dst = reinterpret_cast<f32x4 *>(ws + (((size_t)blockIdx.y * nbq + bq) * 4u + ii) * 64u);
#pragma unroll
        for (int e = 0; e < 16; ++e) dst[e] = (f32x4){acc[4 * e], acc[4 * e + 1], acc[4 * e + 2], acc[4 * e + 3]};
    }
}

// ---- tile path for 64 < n <= 256: the same lanes and register tiles, sample rows of 4*ceil(n/4) floats ----
// (dynamic LDS: two chunks of `ch` samples; a chunk is as many samples as the workgroup's threads can
// hold in flight, four 16-byte pieces each)
__device__ __forceinline__ void m4g_load_chunk(f32x4 (&r)[M4_LPT], const float *__restrict__ X, int64_t s0,
                                               int64_t s_end, u32 n, u32 np4, u32 pieces, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M4_LPT; ++k) {
        const u32 j = min(tid + (u32)M4_THREADS * k, pieces - 1u), smp = j / np4, c0 = 4u * (j - smp * np4);
        const int64_t s = s0 + smp, sc = s < s_end ? s : s_end - 1;
        const float *row = X + sc * (int64_t)n;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) r[k][g] = row[c0 + g < n ? c0 + g : n - 1u];
    }
}

__device__ __forceinline__ void m4g_store_chunk(const f32x4 (&r)[M4_LPT], float *__restrict__ buf, int64_t s0,
                                                int64_t s_end, u32 n, u32 np4, u32 pieces, u32 tid)
{
#pragma unroll
    for (int k = 0; k < M4_LPT; ++k) {
        const u32 j = tid + (u32)M4_THREADS * k, smp = j / np4, c0 = 4u * (j - smp * np4);
        if (j >= pieces) continue;
        const bool row_ok = s0 + smp < s_end;
        f32x4 v;
#pragma unroll
        for (u32 g = 0; g < 4; ++g) v[g] = (row_ok && c0 + g < n) ? r[k][g] : 0.f;
        *reinterpret_cast<f32x4 *>(buf + (size_t)j * 4u) = v;
    }
}

__global__ __launch_bounds__(M4_THREADS) void moment4_tile_general_kernel(const float *__restrict__ X, int64_t N,
                                                                        u32 n, u32 nb4, u32 nbq, u32 ch,
                                                                        int64_t slice, float *__restrict__ ws)
{
    extern __shared__ float lds[];
    const u32 tid = threadIdx.x, ii = tid & 3u, np4 = nb4, np = 4u * nb4;
    const u32 pieces = ch * np4, chunk_f = ch * np;
    const u32 bq = blockIdx.x * 64u + (tid >> 2);
    u32 I, J, K, L;
    unrank_sym4<u32>(nb4, min(bq, nbq - 1u), I, J, K, L);
    const u32 oi = 4u * I + ii, oj = 4u * J, ok = 4u * K, ol = 4u * L;

    const int64_t s_begin = (int64_t)blockIdx.y * slice;
    const int64_t s_end = s_begin + slice < N ? s_begin + slice : N;
    const int64_t nchunks = s_end > s_begin ? (s_end - s_begin + ch - 1) / ch : 0;

    float acc[64];
#pragma unroll
    for (int e = 0; e < 64; ++e) acc[e] = 0.f;

    if (nchunks > 0) {
        f32x4 r[M4_LPT];
        m4g_load_chunk(r, X, s_begin, s_end, n, np4, pieces, tid);
        m4g_store_chunk(r, lds, s_begin, s_end, n, np4, pieces, tid);
        if (nchunks > 1) m4g_load_chunk(r, X, s_begin + ch, s_end, n, np4, pieces, tid);
        __syncthreads();
        for (int64_t c = 0; c < nchunks; ++c) {
            const u32 cb = (u32)(c & 1);
            if (c + 1 < nchunks) m4g_store_chunk(r, lds + (cb ^ 1u) * chunk_f, s_begin + (c + 1) * ch, s_end, n, np4, pieces, tid);
            if (c + 2 < nchunks) m4g_load_chunk(r, X, s_begin + (c + 2) * ch, s_end, n, np4, pieces, tid);
            __builtin_amdgcn_sched_barrier(0);
            const float *row = lds + cb * chunk_f;
#pragma unroll 2
            for (u32 smp = 0; smp < ch; ++smp, row += np) {
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

    if (bq < nbq) {
        f32x4 *dst = reinterpret_cast<f32x4 *>(ws + (((size_t)blockIdx.y * nbq + bq) * 4u + ii) * 64u);
#pragma unroll
        for (int e = 0; e < 16; ++e) dst[e] = (f32x4){acc[4 * e], acc[4 * e + 1], acc[4 * e + 2], acc[4 * e + 3]};
    }
}

// One thread per raw accumulator (block quadruple, lane, j, k, l): adds the S slice
// partials in ascending order and stores the entries of the unique set.
__global__ __launch_bounds__(256) void moment4_reduce_kernel(const float *__restrict__ ws, u32 S, u32 n, u32 nb4,
                                                            u32 nbq, float *__restrict__ Sc, int accumulate)
{
    const u32 t = blockIdx.x * 256u + threadIdx.x;       // < nbq * 256
    if (t >= nbq * 256u) return;
    const u32 bq = t >> 8, ii = (t >> 6) & 3u, e = t & 63u;
    u32 I, J, K, L;
    unrank_sym4<u32>(nb4, bq, I, J, K, L);
    const u32 i = 4u * I + ii, j = 4u * J + (e >> 4), k = 4u * K + ((e >> 2) & 3u), l = 4u * L + (e & 3u);
    if (!(i <= j && j <= k && k <= l && l < n)) return;
    float s = 0.f;
    const size_t stride = (size_t)nbq * 256u;
#pragma unroll 4
    for (u32 y = 0; y < S; ++y) s += ws[(size_t)y * stride + t];
    const u32 p = rank_sym4<u32>(n, i, j, k, l);
    Sc[p] = accumulate ? Sc[p] + s : s;
}

__global__ __launch_bounds__(256) void moment4_zero_kernel(float *__restrict__ p, u32 count)
{
    u32 t = blockIdx.x * 256u + threadIdx.x;
    if (t < count) p[t] = 0.f;
}

// ---- matrix-core path (indices padded to G = ceil(n/16) groups of 16) --------------------
// Sc(i,j,k,l) = sum_s (x_i x_j)(x_k x_l): a contraction over the samples of pair products with
// pair products, so a 16 x 16 MFMA tile is (16 row pairs) x (16 column pairs).  Index i is
// position m = i mod 16 of group g = i / 16; a PAIR SET (ga, gb, d) holds the 16 pairs
// (position m of group ga, position m-d mod 16 of group gb): in-group sets ga = gb, d = 0..8
// (d = 8 names every pair twice), cross sets ga < gb, d = 0..15.  Every 4-multiset of indices is
// covered exactly once by the following (row set) x (column set) tiles, by the groups of the
// four indices (a, b, c, d different groups):
//   {a,b,c,d}: cross(a,b,.) x cross(c,d,.) for a < b < c < d                 all unique
//   {a,a,b,c}: in(a,.) x cross(b,c,.)                                        all unique
//   {a,a,b,b}: in(a,.) x in(b,.), a < b                                      all unique
//   {a,a,a,b}: in(a, even d) x cross(a,b,.): two of the three positions in a have the same
//              parity; the position whose row pair is the closest even pair is kept
//   {a,a,a,a}: in(a, even d) x in(a,.); smallest (d_row, d_col, row pair) is kept
// (the reduce kernel applies the rules; a brute-force count over all multisets of 64 and of 80
// indices gives exactly one kept accumulator each).  Tiles are grouped into wave blocks of 3 row
// sets x 8 column sets = 24 MFMAs fed by 11 products per four samples (n = 64: 175 blocks, 4,200
// tiles for the 2,994 that the unique entries would fill; the ragged edges weigh less as G grows).
// A workgroup of 8 waves owns 8 blocks and streams a slice of the samples through a
// double-buffered LDS chunk stored as [group][step of 4 samples][sample slot][position], so that
// a wave reads either operand of a product, rotated or not, as 64 consecutive floats.  The sets
// are run-time data (a table built on the host per G, copied into the workspace): one code
// stream for all waves; per product two LDS reads and one multiply.
constexpr int M4M_ROWS = 3, M4M_COLS = 8, M4M_SPECS = M4M_ROWS + M4M_COLS, M4M_TPB = M4M_ROWS * M4M_COLS;
constexpr int M4M_WAVES = 8;
constexpr int M4M_ACC = M4M_TPB * 256;               // accumulators per wave block
constexpr int M4M_THREADS = M4M_WAVES * 64;
constexpr int M4M_UNITS = 4;                         // staging units (one group x 16 samples) per wave and chunk
constexpr int M4M_FLUSH_SAMPLES = 8192;              // samples per fp32 accumulation chain

// pair set: bit 12 = valid, bits 8..11 = ga, bits 4..7 = gb, bits 0..3 = d
static inline int m4m_set(int ga, int gb, int d) { return 0x1000 | (ga << 8) | (gb << 4) | d; }

struct M4MTable {
    std::vector<int> spec;     // [slots][M4M_SPECS], slots = 8 * kinds
    u32 blocks = 0, kinds = 0;
};
static void m4m_add(M4MTable &t, const std::vector<int> &rows, const std::vector<int> &cols)
{
    if (rows.empty() || cols.empty()) return;
    for (size_t r0 = 0; r0 < rows.size(); r0 += M4M_ROWS)
        for (size_t c0 = 0; c0 < cols.size(); c0 += M4M_COLS) {
            for (size_t i = 0; i < (size_t)M4M_ROWS; ++i) t.spec.push_back(r0 + i < rows.size() ? rows[r0 + i] : 0);
            for (size_t j = 0; j < (size_t)M4M_COLS; ++j) t.spec.push_back(c0 + j < cols.size() ? cols[c0 + j] : 0);
            ++t.blocks;
        }
}
static M4MTable m4m_build_table(int G)
{
    M4MTable t;
    std::vector<int> rows, cols;
    // four different groups: rows cross(a,b,.) for all a < b (b fixed), columns cross(c,d,.) for b < c < d
    for (int b = 1; b < G; ++b) {
        rows.clear(); cols.clear();
        for (int a = 0; a < b; ++a)
            for (int d = 0; d < 16; ++d) rows.push_back(m4m_set(a, b, d));
        for (int c = b + 1; c < G; ++c)
            for (int e = c + 1; e < G; ++e)
                for (int d = 0; d < 16; ++d) cols.push_back(m4m_set(c, e, d));
        m4m_add(t, rows, cols);
    }
    // a pair in group a with two other groups, or with a pair in a later group
    for (int a = 0; a < G; ++a) {
        rows.clear(); cols.clear();
        for (int d = 0; d < 9; ++d) rows.push_back(m4m_set(a, a, d));
        for (int b = 0; b < G; ++b)
            for (int c = b + 1; c < G; ++c)
                if (b != a && c != a)
                    for (int d = 0; d < 16; ++d) cols.push_back(m4m_set(b, c, d));
        for (int b = a + 1; b < G; ++b)
            for (int d = 0; d < 9; ++d) cols.push_back(m4m_set(b, b, d));
        m4m_add(t, rows, cols);
    }
    // three or four indices in group a
    for (int a = 0; a < G; ++a) {
        rows.clear(); cols.clear();
        for (int e = 0; e < 5; ++e) rows.push_back(m4m_set(a, a, 2 * e));
        for (int b = 0; b < G; ++b)
            if (b != a)
                for (int d = 0; d < 16; ++d) cols.push_back(m4m_set(a < b ? a : b, a < b ? b : a, d));
        for (int d = 0; d < 9; ++d) cols.push_back(m4m_set(a, a, d));
        m4m_add(t, rows, cols);
    }
    t.kinds = (t.blocks + M4M_WAVES - 1) / M4M_WAVES;
    t.spec.resize((size_t)t.kinds * M4M_WAVES * M4M_SPECS, 0);     // empty slots of the last workgroup kind
    return t;
}
// one table per G, built at first use and kept (the copies into workspaces read from it)
static const M4MTable &m4m_table(int G)
{
    static std::mutex mu;
    static M4MTable *cache[17] = {nullptr};
    std::lock_guard<std::mutex> lock(mu);
    if (!cache[G]) cache[G] = new M4MTable(m4m_build_table(G));
    return *cache[G];
}

// Staging: a unit is (group g, 16 consecutive samples): lane (sample, quarter) loads X(s, 16g + 4*quarter ..+3)
// of sample s = 16*sq + lane/4 and stores it at [g][step][slot][4*quarter ..] (16 floats per sample, so the
// wave writes 1 KB of consecutive LDS).  What does not change from chunk to chunk is computed once.
struct M4MStage {
    u32 go[M4M_UNITS];      // float offset of the lane's piece from the first sample of the chunk
    u32 lo[M4M_UNITS];      // float offset of the piece in a chunk buffer
    u32 units;              // units of this wave
};
// sample inside the chunk and first column of the lane's piece of unit k (only the guarded paths need them)
template <int STEPS>
__device__ __forceinline__ void m4m_piece(u32 k, u32 G, u32 wave, u32 lane, u32 &smp, u32 &c0, u32 &lo)
{
    const u32 unit = wave + (u32)M4M_WAVES * k, g = unit % G, sq = unit / G;
    smp = 16u * sq + (lane >> 2);
    c0 = 16u * g + 4u * (lane & 3u);
    lo = (g * (u32)STEPS + 4u * sq) * 64u + 4u * lane;
}
template <int STEPS>
__device__ __forceinline__ M4MStage m4m_stage(u32 n, u32 G, u32 wave, u32 lane)
{
    M4MStage st;
    st.units = 0;
#pragma unroll
    for (int k = 0; k < M4M_UNITS; ++k) {
        u32 smp, c0;
        m4m_piece<STEPS>((u32)k, G, wave, lane, smp, c0, st.lo[k]);
        if (wave + (u32)M4M_WAVES * k < G * (u32)(STEPS / 4)) st.units = (u32)k + 1u;
        st.go[k] = smp * n + (c0 + 4u <= n ? c0 : 0u);
    }
    return st;
}
// rows: samples of the chunk that exist (a whole chunk except at the end of the slice)
template <int STEPS, bool V4>
__device__ __forceinline__ void m4m_load_chunk(f32x4 (&r)[M4M_UNITS], const M4MStage &st, const float *__restrict__ Xc,
                                               u32 rows, u32 n, u32 G, u32 wave, u32 lane)
{
    if (V4 && rows == (u32)STEPS * 4u) {
#pragma unroll
        for (int k = 0; k < M4M_UNITS; ++k) {
            if ((u32)k >= st.units) continue;
            const float4 t = *reinterpret_cast<const float4 *>(Xc + st.go[k]);
            r[k] = (f32x4){t.x, t.y, t.z, t.w};
        }
    } else {
#pragma unroll
        for (int k = 0; k < M4M_UNITS; ++k) {
            if ((u32)k >= st.units) continue;
            u32 smp, c0, lo;
            m4m_piece<STEPS>((u32)k, G, wave, lane, smp, c0, lo);
            const float *row = Xc + (size_t)(smp < rows ? smp : rows - 1u) * n;
#pragma unroll
            for (u32 e = 0; e < 4; ++e) r[k][e] = row[c0 + e < n ? c0 + e : n - 1u];
        }
    }
}
// padded: some column of the 16*G staged ones is >= n
template <int STEPS>
__device__ __forceinline__ void m4m_store_chunk(const f32x4 (&r)[M4M_UNITS], const M4MStage &st, float *__restrict__ buf,
                                                u32 rows, u32 n, u32 G, u32 wave, u32 lane, bool padded)
{
    if (!padded && rows == (u32)STEPS * 4u) {
#pragma unroll
        for (int k = 0; k < M4M_UNITS; ++k) {
            if ((u32)k >= st.units) continue;
            *reinterpret_cast<f32x4 *>(buf + st.lo[k]) = r[k];
        }
    } else {
#pragma unroll
        for (int k = 0; k < M4M_UNITS; ++k) {
            if ((u32)k >= st.units) continue;
            u32 smp, c0, lo;
            m4m_piece<STEPS>((u32)k, G, wave, lane, smp, c0, lo);
            f32x4 v;
#pragma unroll
            for (u32 e = 0; e < 4; ++e) v[e] = (smp < rows && c0 + e < n) ? r[k][e] : 0.f;
            *reinterpret_cast<f32x4 *>(buf + lo) = v;
        }
    }
}

// partial (+)= accumulators, six tiles at a time (all 96 values in flight at once would not fit the registers)
__device__ __forceinline__ void m4m_flush(const f32x4 (&acc)[M4M_TPB], float *dst, bool add)
{
#ifndef ST_HOST_EMULATION
    // the 96 addresses are formed here, from immediates, and not ahead of the chunk loop (where they would be
    // kept in registers the loop needs)
    asm volatile("" : "+v"(dst));
#endif
#pragma unroll
    for (int t0 = 0; t0 < M4M_TPB; t0 += 6) {
        float old[6][4];
        if (add) {
#pragma unroll
            for (int t = 0; t < 6; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) old[t][v] = dst[((t0 + t) * 4 + v) * 64];
        }
#pragma unroll
        for (int t = 0; t < 6; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) dst[((t0 + t) * 4 + v) * 64] = add ? old[t][v] + acc[t0 + t][v] : acc[t0 + t][v];
        __builtin_amdgcn_sched_barrier(0);
    }
}

// STEPS K-steps (4 samples each) per staged chunk; V4: rows are read with 16-byte loads (n % 4 == 0)
template <int STEPS, bool V4>
__global__ __launch_bounds__(M4M_THREADS) void moment4_mfma_kernel(const float *__restrict__ X, int64_t N, u32 n, u32 G,
                                                                 u32 kinds, int64_t slice,
                                                                 const int *__restrict__ table, float *__restrict__ ws)
{
    extern __shared__ float lds[];                      // two chunks of G * STEPS * 64 floats
    constexpr int CH = STEPS * 4;
    constexpr int FLUSH = M4M_FLUSH_SAMPLES / CH;       // chunks per fp32 accumulation chain
    const u32 tid = threadIdx.x, lane = tid & 63u;
    const u32 wave = (u32)__builtin_amdgcn_readfirstlane((int)(tid >> 6));
    const u32 kind = blockIdx.x % kinds, sl = blockIdx.x / kinds;
    const u32 block = kind * (u32)M4M_WAVES + wave;     // the last slots of the last kind may be empty
    const u32 chunk_f = G * (u32)STEPS * 64u;
    const int64_t s_begin = (int64_t)sl * slice, s_end = s_begin + slice < N ? s_begin + slice : N;

    // per-lane float offsets of the two operands of every product inside a chunk buffer (step 0)
    u32 oa[M4M_SPECS], ob[M4M_SPECS];
#pragma unroll
    for (int u = 0; u < M4M_SPECS; ++u) {
        const u32 sp = (u32)table[(size_t)block * M4M_SPECS + u];
        const u32 ga = (sp >> 8) & 15u, gb = (sp >> 4) & 15u, d = sp & 15u;
        oa[u] = ga * (u32)STEPS * 64u + lane;
        ob[u] = gb * (u32)STEPS * 64u + (lane & 48u) + ((lane - d) & 15u);
    }
    f32x4 acc[M4M_TPB];
#pragma unroll
    for (int t = 0; t < M4M_TPB; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int64_t nchunks = (s_end - s_begin + CH - 1) / CH;
    const size_t slots = (size_t)kinds * M4M_WAVES;
    float *dst = ws + ((size_t)sl * slots + block) * M4M_ACC + lane;
    const M4MStage stg = m4m_stage<STEPS>(n, G, wave, lane);
    const bool padded = n != 16u * G;
    // samples of chunk c that exist
    auto rows_of = [&](int64_t c) -> u32 {
        const int64_t left = s_end - (s_begin + c * CH);
        return left < CH ? (u32)left : (u32)CH;
    };
    f32x4 r[M4M_UNITS];
    m4m_load_chunk<STEPS, V4>(r, stg, X + s_begin * (int64_t)n, rows_of(0), n, G, wave, lane);
    m4m_store_chunk<STEPS>(r, stg, lds, rows_of(0), n, G, wave, lane, padded);
    if (nchunks > 1) m4m_load_chunk<STEPS, V4>(r, stg, X + (s_begin + CH) * (int64_t)n, rows_of(1), n, G, wave, lane);
    __syncthreads();

    for (int64_t c = 0; c < nchunks; ++c) {
        const u32 cb = (u32)(c & 1);
        // registers hold chunk c+1: park it in the other buffer (its readers finished before the
        // barrier that ended the previous iteration), then put chunk c+2 in flight
        if (c + 1 < nchunks)
            m4m_store_chunk<STEPS>(r, stg, lds + (cb ^ 1u) * chunk_f, rows_of(c + 1), n, G, wave, lane, padded);
        if (c + 2 < nchunks)
            m4m_load_chunk<STEPS, V4>(r, stg, X + (s_begin + (c + 2) * CH) * (int64_t)n, rows_of(c + 2), n, G, wave, lane);
        __builtin_amdgcn_sched_barrier(0);
        const float *base = lds + cb * chunk_f;
        float a[2][M4M_SPECS], b[2][M4M_SPECS];
#pragma unroll
        for (int u = 0; u < M4M_SPECS; ++u) { a[0][u] = base[oa[u]]; b[0][u] = base[ob[u]]; }
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            const int cur = st & 1, nxt = cur ^ 1;
            if (st + 1 < STEPS) {          // operands of the next step are in flight under this step's MFMAs
#pragma unroll
                for (int u = 0; u < M4M_SPECS; ++u) {
                    a[nxt][u] = base[(st + 1) * 64 + oa[u]];
                    b[nxt][u] = base[(st + 1) * 64 + ob[u]];
                }
            }
            float p[M4M_SPECS];
#pragma unroll
            for (int u = 0; u < M4M_SPECS; ++u) p[u] = a[cur][u] * b[cur][u];
#pragma unroll
            for (int i = 0; i < M4M_ROWS; ++i)
#pragma unroll
                for (int j = 0; j < M4M_COLS; ++j)
                    acc[i * M4M_COLS + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(p[i], p[M4M_ROWS + j],
                                                                               acc[i * M4M_COLS + j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);      // keeps the operand reads of later steps out of this one
        }
        __syncthreads();
        // Long fp32 accumulation chains lose accuracy (1.2e-4 norm-wise after 180,000 samples): every FLUSH
        // chunks the accumulators are added to the wave's own partial in the workspace and cleared.
        if ((c + 1) % FLUSH == 0 && c + 1 < nchunks) {
            m4m_flush(acc, dst, c + 1 != FLUSH);
#pragma unroll
            for (int t = 0; t < M4M_TPB; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
    }
    m4m_flush(acc, dst, nchunks > FLUSH);
}

__device__ __forceinline__ u32 m4m_cyc(u32 x, u32 y)
{
    const u32 t = (x - y) & 15u;
    return min(t, 16u - t);
}

// One thread per raw accumulator: decides whether it is the kept position of its index multiset,
// adds the S slice partials in ascending order and scatters through rank4.
__global__ __launch_bounds__(256) void moment4_mfma_reduce_kernel(const float *__restrict__ ws,
                                                                 const int *__restrict__ table, u32 blocks, u32 slots,
                                                                 u32 S, u32 n, float *__restrict__ Sc, int accumulate)
{
    const size_t e = (size_t)blockIdx.x * 256u + threadIdx.x;      // < blocks * M4M_ACC
    if (e >= (size_t)blocks * M4M_ACC) return;
    const u32 block = (u32)(e / (u32)M4M_ACC), loc = (u32)(e - (size_t)block * M4M_ACC);
    const u32 t = loc >> 8, v = (loc >> 6) & 3u, lane = loc & 63u;
    // D layout of the 16x16 MFMA: lane holds column lane%16 of rows 4*(lane/16) + v
    const u32 m = 4u * (lane >> 4) + v, mp = lane & 15u;
    const u32 rs = (u32)table[(size_t)block * M4M_SPECS + t / (u32)M4M_COLS];
    const u32 cs = (u32)table[(size_t)block * M4M_SPECS + (u32)M4M_ROWS + t % (u32)M4M_COLS];
    if (!(rs & 0x1000u) || !(cs & 0x1000u)) return;
    const u32 g1 = (rs >> 8) & 15u, g2 = (rs >> 4) & 15u, dr = rs & 15u;
    const u32 g3 = (cs >> 8) & 15u, g4 = (cs >> 4) & 15u, dc = cs & 15u;
    const u32 x1 = m, x2 = (m - dr) & 15u, x3 = mp, x4 = (mp - dc) & 15u;
    // an in-group set at distance 8 names every pair twice
    if ((g1 == g2 && dr == 8u && m >= 8u) || (g3 == g4 && dc == 8u && mp >= 8u)) return;
    bool keep = true;
    if (g1 == g2) {
        const u32 a = g1;
        if (g3 != g4) {
            if (g3 == a || g4 == a) {
                // three positions in group a: the row pair must be the closest even pair (ties: smallest third)
                const u32 z = g3 == a ? x3 : x4;
                const u32 d1 = m4m_cyc(x1, z), d2 = m4m_cyc(x2, z);
                const u32 k0 = 16u * dr + z;
                const u32 k1 = (d1 & 1u) ? 0xffffu : 16u * d1 + x2, k2 = (d2 & 1u) ? 0xffffu : 16u * d2 + x1;
                keep = k0 <= k1 && k0 <= k2;
            }
        } else if (g3 == a) {
            // all four in group a: of the three pairings (either pair as the row pair, which needs an even
            // distance) the smallest (d_row, d_col, row pair) is kept
            auto key = [](u32 r0, u32 r1, u32 c0, u32 c1) -> u32 {
                const u32 d = m4m_cyc(r0, r1);
                if (d & 1u) return 0xffffffffu;
                return ((d * 9u + m4m_cyc(c0, c1)) * 16u + min(r0, r1)) * 16u + max(r0, r1);
            };
            const u32 k0 = key(x1, x2, x3, x4);
            keep = key(x3, x4, x1, x2) >= k0 && key(x1, x3, x2, x4) >= k0 && key(x2, x4, x1, x3) >= k0 &&
                   key(x1, x4, x2, x3) >= k0 && key(x2, x3, x1, x4) >= k0;
        }
    }
    u32 i = 16u * g1 + x1, j = 16u * g2 + x2, k = 16u * g3 + x3, l = 16u * g4 + x4;
    if (!keep || i >= n || j >= n || k >= n || l >= n) return;
    float s = 0.f;
    const size_t stride = (size_t)slots * M4M_ACC;
#pragma unroll 4
    for (u32 y = 0; y < S; ++y) s += ws[(size_t)y * stride + e];
    // sort the four indices
    u32 lo = min(i, j), hi = max(i, j); i = lo; j = hi;
    lo = min(k, l); hi = max(k, l); k = lo; l = hi;
    lo = min(i, k); hi = max(i, k); i = lo; k = hi;
    lo = min(j, l); hi = max(j, l); j = lo; l = hi;
    lo = min(j, k); hi = max(j, k); j = lo; k = hi;
    const u32 pos = rank_sym4<u32>(n, i, j, k, l);
    Sc[pos] = accumulate ? Sc[pos] + s : s;
}

// Plan of the matrix-core path.  Workspace: the table (padded to 256 bytes), then S * slots blocks of partials.
struct M4MPlan { u32 G, steps, kinds, blocks, S; int64_t slice; size_t table_bytes; };
static inline bool m4_use_mfma(int n)
{
    // worth it while padding every index range to 16*G costs less than the matrix cores gain
    const int G = (n + 15) / 16;
    return n >= 53 && n <= 256 && 8 * G <= n * 4 / 7;          // 16 G <= 8/7 n
}
static inline M4MPlan m4m_plan(int64_t N, int n)
{
    M4MPlan p;
    p.G = ((u32)n + 15u) / 16u;
    p.steps = p.G <= 8u ? 16u : 8u;                            // two chunks of G * steps * 64 floats: at most 64 KB
    const M4MTable &t = m4m_table((int)p.G);
    p.kinds = t.kinds;
    p.blocks = t.blocks;
    p.table_bytes = (t.spec.size() * sizeof(int) + 255u) / 256u * 256u;
    const int64_t ch = 4 * p.steps;
    // Sample slices: every workgroup does the same work, so the kinds * S workgroups run in whole rounds of one
    // per compute unit; the smallest S that fills at least 93 % of its rounds (else the best one), each slice at
    // least four chunks long and the partials of all slices below 2 GB.
    const int64_t cus = num_cus();
    int64_t smax = (N + 4 * ch - 1) / (4 * ch);
    const int64_t scap = (int64_t)(((size_t)2 << 30) / ((size_t)p.kinds * M4M_WAVES * M4M_ACC * sizeof(float)));
    if (smax > scap) smax = scap;
    if (smax > 64) smax = 64;
    if (smax < 1) smax = 1;
    int64_t S = 1;
    double best = 0.0;
    for (int64_t c = 1; c <= smax; ++c) {
        const int64_t wgs = (int64_t)p.kinds * c, rounds = (wgs + cus - 1) / cus;
        const double fill = (double)wgs / (double)(rounds * cus);
        if (fill > best + 1e-9) { best = fill; S = c; }
        if (fill >= 0.93) { S = c; break; }
    }
    p.slice = ((N + S - 1) / S + ch - 1) / ch * ch;
    p.S = (u32)((N + p.slice - 1) / p.slice);
    return p;
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
    // samples per chunk: 64 up to n = 64; beyond, what the threads' 4 pieces each can hold (16 at n = 256)
    p.ch = n <= 64 ? (u32)M4_CH : ((u32)(M4_LPT * M4_THREADS) / p.nb4) & ~3u;
    if (p.ch > (u32)M4_CH) p.ch = (u32)M4_CH;
    int64_t S = (M4_WGTARGET + p.gx - 1) / p.gx;           // enough slices to fill the chip ...
    int64_t smax = (N + p.ch - 1) / p.ch;                  // ... each of at least one chunk
    if (S > smax) S = smax;
    if (S > 64) S = 64;
    if (S < 1) S = 1;
    p.slice = ((N + S - 1) / S + p.ch - 1) / p.ch * p.ch;      // whole chunks
    p.S = (u32)((N + p.slice - 1) / p.slice);
    return p;
}

size_t moment4_workspace(int64_t N, int n)
{
    if (N == 0) return 0;
    if (m4_use_mfma(n)) {
        const M4MPlan p = m4m_plan(N, n);
        return p.table_bytes + (size_t)p.S * p.kinds * M4M_WAVES * M4M_ACC * sizeof(float);
    }
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
    if (m4_use_mfma(n)) {
        const M4MPlan p = m4m_plan(N, n);
        const M4MTable &tab = m4m_table((int)p.G);
        int *table = static_cast<int *>(ws);
        float *wsf = reinterpret_cast<float *>(static_cast<char *>(ws) + p.table_bytes);
        // the table lives for the life of the process, so the copy may complete after this call returns
        if (hipMemcpyAsync(table, tab.spec.data(), tab.spec.size() * sizeof(int), hipMemcpyHostToDevice, s) != hipSuccess)
            return ST_ERR_LAUNCH;
        const dim3 grid(p.kinds * p.S), block(M4M_THREADS);
        const size_t lds_bytes = (size_t)2u * p.G * p.steps * 64u * sizeof(float);
        const bool v4 = n % 4 == 0;
        if (p.steps == 16u) {
            if (v4) hipLaunchKernelGGL((moment4_mfma_kernel<16, true>), grid, block, lds_bytes, s, X, N, (u32)n, p.G, p.kinds, p.slice, table, wsf);
            else hipLaunchKernelGGL((moment4_mfma_kernel<16, false>), grid, block, lds_bytes, s, X, N, (u32)n, p.G, p.kinds, p.slice, table, wsf);
        } else {
            if (v4) hipLaunchKernelGGL((moment4_mfma_kernel<8, true>), grid, block, lds_bytes, s, X, N, (u32)n, p.G, p.kinds, p.slice, table, wsf);
            else hipLaunchKernelGGL((moment4_mfma_kernel<8, false>), grid, block, lds_bytes, s, X, N, (u32)n, p.G, p.kinds, p.slice, table, wsf);
        }
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        const size_t racc = (size_t)p.blocks * M4M_ACC;
        hipLaunchKernelGGL(moment4_mfma_reduce_kernel, dim3((u32)((racc + 255) / 256)), dim3(256), 0, s, wsf, table,
                           p.blocks, p.kinds * (u32)M4M_WAVES, p.S, (u32)n, Sc, accumulate);
        return launch_status();
    }
    if (n <= 64) {
        const M4Plan p = m4_plan(N, n);
        float *wsf = static_cast<float *>(ws);
        if (n == 64)
            hipLaunchKernelGGL(moment4_tile_kernel<true>, dim3(p.gx, p.S), dim3(M4_THREADS), 0, s, X, N, (u32)n,
                               p.nb4, p.nbq, p.slice, wsf);
        else
            hipLaunchKernelGGL(moment4_tile_kernel<false>, dim3(p.gx, p.S), dim3(M4_THREADS), 0, s, X, N, (u32)n,
                               p.nb4, p.nbq, p.slice, wsf);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment4_reduce_kernel, dim3(p.nbq), dim3(256), 0, s, wsf, p.S, (u32)n, p.nb4, p.nbq, Sc,
                           accumulate);
        return launch_status();
    }
    {
        const M4Plan p = m4_plan(N, n);
        float *wsf = static_cast<float *>(ws);
        const size_t lds_bytes = (size_t)2u * p.ch * 4u * p.nb4 * sizeof(float);      // at most 64 KB
        static bool attr = false;
        if (!attr) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(moment4_tile_general_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024) != hipSuccess)
                return ST_ERR_LAUNCH;
            attr = true;
        }
        hipLaunchKernelGGL(moment4_tile_general_kernel, dim3(p.gx, p.S), dim3(M4_THREADS), lds_bytes, s, X, N, (u32)n,
                           p.nb4, p.nbq, p.ch, p.slice, wsf);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        hipLaunchKernelGGL(moment4_reduce_kernel, dim3(p.nbq), dim3(256), 0, s, wsf, p.S, (u32)n, p.nb4, p.nbq, Sc,
                           accumulate);
        return launch_status();
    }
}

}  // namespace st
