// Moment accumulation on the matrix cores for any feature count up to 256: third and fourth
// moments over the unique sets i <= j <= k (<= l), as one table-driven kernel.
//
// Index i is position m = i mod 16 of group g = i / 16 (G = ceil(n/16) groups, the last one
// padded with zeros).  A SET holds 16 values per sample: a pair set (ga, gb, d) the products
// (position m of group ga) * (position m-d mod 16 of group gb) -- in-group sets ga = gb,
// d = 0..8 (d = 8 names every pair twice), cross sets ga < gb, d = 0..15 -- and a single set (g)
// the 16 values of group g themselves (in the table a product with a plane of ones; the third-moment
// instance of the kernel, whose row sets are all single, reads the values and skips the multiply).  A 16 x 16
// MFMA tile contracts a row set with a column set over the samples:
//     acc(m, m') += sum_s rowset(s, m) * colset(s, m').
// Fourth moment, Sc(i,j,k,l) = sum_s (x_i x_j)(x_k x_l): pair sets x pair sets.  Every 4-multiset
// of indices is covered exactly once by the following tiles, by the groups of its indices
// (a, b, c, d different groups):
//   {a,b,c,d}: cross(a,b,.) x cross(c,d,.) for a < b < c < d                 all unique
//   {a,a,b,c}: in(a,.) x cross(b,c,.)                                        all unique
//   {a,a,b,b}: in(a,.) x in(b,.), a < b                                      all unique
//   {a,a,a,b}: in(a, even d) x cross(a,b,.): two of the three positions in a have the same
//              parity; the position whose row pair is the closest even pair is kept
//   {a,a,a,a}: in(a, even d) x in(a,.); smallest (d_row, d_col, row pair) is kept
// Third moment, Sc(i,j,k) = sum_s x_i (x_j x_k): single sets x pair sets:
//   {a,b,c}  : single(z) x cross(x,y,.), every group triple given to ONE of its three pairs when
//              the table is built (in threes, so that the row blocks are full)
//   {a,a,b}  : single(b) x in(a,.)                                           all unique
//   {a,a,a}  : single(a) x in(a, even d), closest even pair kept
// (the reduce kernels apply the rules; brute-force counts over all multisets of 64 and of 80
// indices give exactly one kept accumulator each).  Tiles are grouped into wave blocks of 3 row
// sets x 8 column sets = 24 MFMAs fed by 11 products per four samples (fourth moment, n = 64: 175
// blocks, 4,200 tiles for the 2,994 that the unique entries would fill; the ragged edges weigh
// less as G grows; a block at the ragged end of a row list runs an instance of the kernel body that issues no
// MFMAs for the row sets it does not have).  A workgroup of 8 waves owns 8 blocks and streams a slice of the samples
// through a double-buffered LDS chunk stored as [group][step of 4 samples][sample slot]
// [position], so that a wave reads either operand of a product, rotated or not, as 64
// consecutive floats.  The sets are run-time data (a table built on the host per moment and G,
// copied into the workspace): one code stream for all waves; per product two LDS reads and one
// multiply (a single row set: one read).  Slice partials -> reduce kernel: keeps the positions above, adds the slices in
// ascending order, sorts the indices and scatters through the closed-form rank.  No atomics.
#include <algorithm>
#include <cstring>
#include <type_traits>
#include <mutex>
#include <vector>

#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int MM_ROWS = 3, MM_COLS = 8, MM_SPECS = MM_ROWS + MM_COLS, MM_TPB = MM_ROWS * MM_COLS;
constexpr int MM_WAVES = 8;
constexpr int MM_ACC = MM_TPB * 256;               // accumulators per wave block
constexpr int MM_THREADS = MM_WAVES * 64;
constexpr int MM_UNITS = 4;                         // staging units (one group x 16 samples) per wave and chunk
constexpr int MM_FLUSH_SAMPLES = 8192;              // samples per fp32 accumulation chain

// set: bit 14 = valid, bits 9..13 = ga, bits 4..8 = gb (G = the plane of ones: a single set), bits 0..3 = d
constexpr u32 MM_VALID = 0x4000u;
static inline int mm_set(int ga, int gb, int d) { return (int)MM_VALID | (ga << 9) | (gb << 4) | d; }
__host__ __device__ __forceinline__ u32 mm_ga(u32 sp) { return (sp >> 9) & 31u; }
__host__ __device__ __forceinline__ u32 mm_gb(u32 sp) { return (sp >> 4) & 31u; }
__host__ __device__ __forceinline__ u32 mm_d(u32 sp) { return sp & 15u; }

struct MMTable {
    std::vector<int> spec;     // [slots][MM_SPECS], slots = 8 * kinds
    u32 blocks = 0, kinds = 0;
    int *pinned = nullptr;     // the same table in pinned, device-visible host memory (what a call's copy kernel reads)
};
static void mm_add(MMTable &t, const std::vector<int> &rows, const std::vector<int> &cols)
{
    if (rows.empty() || cols.empty()) return;
    for (size_t r0 = 0; r0 < rows.size(); r0 += MM_ROWS)
        for (size_t c0 = 0; c0 < cols.size(); c0 += MM_COLS) {
            for (size_t i = 0; i < (size_t)MM_ROWS; ++i) t.spec.push_back(r0 + i < rows.size() ? rows[r0 + i] : 0);
            for (size_t j = 0; j < (size_t)MM_COLS; ++j) t.spec.push_back(c0 + j < cols.size() ? cols[c0 + j] : 0);
            ++t.blocks;
        }
}
// The blocks in the order the kernel wants them: a block costs as many MFMAs as it has row sets in use, the eight
// blocks of a workgroup run side by side until the slowest is done, and waves w and w+4 share a SIMD.  So the
// blocks are sorted by their row sets in use, which makes the workgroups uniform (a workgroup of ragged blocks is
// short instead of waiting for one full block), and inside a workgroup the k-th largest shares its SIMD with the
// k-th smallest.  The reduce kernels read a tile's sets from the table and do not care about the order.
static void mm_arrange(MMTable &t)
{
    auto used = [&](size_t b) {
        int nr = 0;
        for (int u = 0; u < MM_ROWS; ++u) nr += (t.spec[b * MM_SPECS + u] & (int)MM_VALID) ? 1 : 0;
        return nr;
    };
    const size_t nb = t.blocks;
    std::vector<size_t> order(nb);
    for (size_t b = 0; b < nb; ++b) order[b] = b;
    std::stable_sort(order.begin(), order.end(), [&](size_t x, size_t y) { return used(x) > used(y); });
    std::vector<int> out(t.spec.size(), 0);
    for (size_t w0 = 0; w0 < nb; w0 += MM_WAVES) {
        const size_t cnt = nb - w0 < (size_t)MM_WAVES ? nb - w0 : (size_t)MM_WAVES;
        for (size_t k = 0; k < cnt; ++k) {
            // sorted position k of this workgroup -> wave: 0, 1, 2, 3 take the four largest, 7, 6, 5, 4 the rest
            // (a last workgroup that is not full keeps its blocks in front: the reduce kernels walk `blocks` slots)
            const size_t wave = cnt < (size_t)MM_WAVES || k < 4 ? k : (size_t)MM_WAVES + 3u - k;
            const size_t src = order[w0 + k];
            for (int u = 0; u < MM_SPECS; ++u) out[(w0 + wave) * MM_SPECS + u] = t.spec[src * MM_SPECS + u];
        }
    }
    t.spec.swap(out);
}
static MMTable mm_build_table4(int G)
{
    MMTable t;
    std::vector<int> rows, cols;
    // four different groups: rows cross(a,b,.) for all a < b (b fixed), columns cross(c,d,.) for b < c < d
    for (int b = 1; b < G; ++b) {
        rows.clear(); cols.clear();
        for (int a = 0; a < b; ++a)
            for (int d = 0; d < 16; ++d) rows.push_back(mm_set(a, b, d));
        for (int c = b + 1; c < G; ++c)
            for (int e = c + 1; e < G; ++e)
                for (int d = 0; d < 16; ++d) cols.push_back(mm_set(c, e, d));
        mm_add(t, rows, cols);
    }
    // a pair in group a with two other groups, or with a pair in a later group
    for (int a = 0; a < G; ++a) {
        rows.clear(); cols.clear();
        for (int d = 0; d < 9; ++d) rows.push_back(mm_set(a, a, d));
        for (int b = 0; b < G; ++b)
            for (int c = b + 1; c < G; ++c)
                if (b != a && c != a)
                    for (int d = 0; d < 16; ++d) cols.push_back(mm_set(b, c, d));
        for (int b = a + 1; b < G; ++b)
            for (int d = 0; d < 9; ++d) cols.push_back(mm_set(b, b, d));
        mm_add(t, rows, cols);
    }
    // three or four indices in group a
    for (int a = 0; a < G; ++a) {
        rows.clear(); cols.clear();
        for (int e = 0; e < 5; ++e) rows.push_back(mm_set(a, a, 2 * e));
        for (int b = 0; b < G; ++b)
            if (b != a)
                for (int d = 0; d < 16; ++d) cols.push_back(mm_set(a < b ? a : b, a < b ? b : a, d));
        for (int d = 0; d < 9; ++d) cols.push_back(mm_set(a, a, d));
        mm_add(t, rows, cols);
    }
    t.kinds = (t.blocks + MM_WAVES - 1) / MM_WAVES;
    t.spec.resize((size_t)t.kinds * MM_WAVES * MM_SPECS, 0);     // empty slots of the last workgroup kind
    mm_arrange(t);
    return t;
}
static MMTable mm_build_table3(int G)
{
    MMTable t;
    std::vector<int> rows, cols;
    // a pair inside one group, third index anywhere: all single sets against all in-group sets (when the single
    // is of the same group only the even distances are kept)
    for (int g = 0; g < G; ++g) rows.push_back(mm_set(g, G, 0));
    for (int a = 0; a < G; ++a)
        for (int d = 0; d < 9; ++d) cols.push_back(mm_set(a, a, d));
    mm_add(t, rows, cols);
    // three different groups: each group triple is given to one of its three pairs (x, y) as the column sets
    // cross(x,y,.), its third group z as a single row set; first in threes (full row blocks), then what is left
    std::vector<char> done((size_t)G * G * G, 0);
    auto id = [&](int p, int q, int r) {
        int lo = p < q ? (p < r ? p : r) : (q < r ? q : r), hi = p > q ? (p > r ? p : r) : (q > r ? q : r);
        int mid = p + q + r - lo - hi;
        return ((size_t)lo * G + mid) * G + hi;
    };
    for (int pass = 0; pass < 2; ++pass)
        for (int x = 0; x < G; ++x)
            for (int y = x + 1; y < G; ++y) {
                std::vector<int> zs;
                for (int z = 0; z < G; ++z)
                    if (z != x && z != y && !done[id(x, y, z)]) zs.push_back(z);
                const size_t take = pass == 0 ? zs.size() / 3 * 3 : zs.size();
                if (take == 0) continue;
                rows.clear(); cols.clear();
                for (size_t q = 0; q < take; ++q) { rows.push_back(mm_set(zs[q], G, 0)); done[id(x, y, zs[q])] = 1; }
                for (int d = 0; d < 16; ++d) cols.push_back(mm_set(x, y, d));
                mm_add(t, rows, cols);
            }
    t.kinds = (t.blocks + MM_WAVES - 1) / MM_WAVES;
    t.spec.resize((size_t)t.kinds * MM_WAVES * MM_SPECS, 0);
    mm_arrange(t);
    return t;
}
// One table per moment and G, built at first use and kept for the life of the process, with a copy in pinned
// host memory that every GPU can read: a call brings the table into its workspace with a small KERNEL that
// reads that copy, so the call enqueues kernels only (nothing blocks the host, and a caller may capture it).
static const MMTable &mm_table(int order, int G)
{
    static std::mutex mu;
    static MMTable *cache[2][17] = {{nullptr}};
    std::lock_guard<std::mutex> lock(mu);
    MMTable *&slot = cache[order - 3][G];
    if (!slot) {
        slot = new MMTable(order == 3 ? mm_build_table3(G) : mm_build_table4(G));
        void *host = nullptr;
        const size_t bytes = slot->spec.size() * sizeof(int);
        if (hipHostMalloc(&host, bytes ? bytes : sizeof(int), hipHostMallocPortable) == hipSuccess && host) {
            memcpy(host, slot->spec.data(), bytes);
            slot->pinned = static_cast<int *>(host);
        }
    }
    return *slot;
}

__global__ __launch_bounds__(256) void mm_table_copy_kernel(const int *__restrict__ src, int *__restrict__ dst, u32 count)
{
    for (u32 e = blockIdx.x * 256u + threadIdx.x; e < count; e += gridDim.x * 256u) dst[e] = src[e];
}

// Staging: a unit is (group g, 16 consecutive samples): lane (sample, quarter) loads X(s, 16g + 4*quarter ..+3)
// of sample s = 16*sq + lane/4 and stores it at [g][step][slot][4*quarter ..] (16 floats per sample, so the
// wave writes 1 KB of consecutive LDS).  What does not change from chunk to chunk is computed once.
struct MMStage {
    u32 go[MM_UNITS];      // float offset of the lane's piece from the first sample of the chunk
    u32 lo[MM_UNITS];      // float offset of the piece in a chunk buffer
    u32 units;              // units of this wave
};
// sample inside the chunk and first column of the lane's piece of unit k (only the guarded paths need them)
template <int STEPS>
__device__ __forceinline__ void mm_piece(u32 k, u32 G, u32 wave, u32 lane, u32 &smp, u32 &c0, u32 &lo)
{
    const u32 unit = wave + (u32)MM_WAVES * k, g = unit % G, sq = unit / G;
    smp = 16u * sq + (lane >> 2);
    c0 = 16u * g + 4u * (lane & 3u);
    lo = (g * (u32)STEPS + 4u * sq) * 64u + 4u * lane;
}
template <int STEPS>
__device__ __forceinline__ MMStage mm_stage(u32 n, u32 G, u32 wave, u32 lane)
{
    MMStage st;
    st.units = 0;
#pragma unroll
    for (int k = 0; k < MM_UNITS; ++k) {
        u32 smp, c0;
        mm_piece<STEPS>((u32)k, G, wave, lane, smp, c0, st.lo[k]);
        if (wave + (u32)MM_WAVES * k < G * (u32)(STEPS / 4)) st.units = (u32)k + 1u;
        st.go[k] = smp * n + (c0 + 4u <= n ? c0 : 0u);
    }
    return st;
}
// rows: samples of the chunk that exist (a whole chunk except at the end of the slice)
template <int STEPS, bool V4>
__device__ __forceinline__ void mm_load_chunk(f32x4 (&r)[MM_UNITS], const MMStage &st, const float *__restrict__ Xc,
                                               u32 rows, u32 n, u32 G, u32 wave, u32 lane)
{
    if (V4 && rows == (u32)STEPS * 4u) {
#pragma unroll
        for (int k = 0; k < MM_UNITS; ++k) {
            if ((u32)k >= st.units) continue;
            const float4 t = *reinterpret_cast<const float4 *>(Xc + st.go[k]);
            r[k] = (f32x4){t.x, t.y, t.z, t.w};
        }
    } else {
#pragma unroll
        for (int k = 0; k < MM_UNITS; ++k) {
            if ((u32)k >= st.units) continue;
            u32 smp, c0, lo;
            mm_piece<STEPS>((u32)k, G, wave, lane, smp, c0, lo);
            const float *row = Xc + (size_t)(smp < rows ? smp : rows - 1u) * n;
#pragma unroll
            for (u32 e = 0; e < 4; ++e) r[k][e] = row[c0 + e < n ? c0 + e : n - 1u];
        }
    }
}
// padded: some column of the 16*G staged ones is >= n
template <int STEPS>
__device__ __forceinline__ void mm_store_chunk(const f32x4 (&r)[MM_UNITS], const MMStage &st, float *__restrict__ buf,
                                                u32 rows, u32 n, u32 G, u32 wave, u32 lane, bool padded)
{
    if (!padded && rows == (u32)STEPS * 4u) {
#pragma unroll
        for (int k = 0; k < MM_UNITS; ++k) {
            if ((u32)k >= st.units) continue;
            *reinterpret_cast<f32x4 *>(buf + st.lo[k]) = r[k];
        }
    } else {
#pragma unroll
        for (int k = 0; k < MM_UNITS; ++k) {
            if ((u32)k >= st.units) continue;
            u32 smp, c0, lo;
            mm_piece<STEPS>((u32)k, G, wave, lane, smp, c0, lo);
            f32x4 v;
#pragma unroll
            for (u32 e = 0; e < 4; ++e) v[e] = (smp < rows && c0 + e < n) ? r[k][e] : 0.f;
            *reinterpret_cast<f32x4 *>(buf + lo) = v;
        }
    }
}

// partial (+)= accumulators, six (or four) tiles at a time (all 96 values in flight at once would not fit the registers)
template <int NT>                                   // NT: tiles in use (the first NT accumulators)
__device__ __forceinline__ void mm_flush(const f32x4 (&acc)[MM_TPB], float *dst, bool add)
{
    constexpr int STEP = NT % 6 == 0 ? 6 : 4;
    // the 96 addresses are formed here, from immediates, and not ahead of the chunk loop (where they would be
    // kept in registers the loop needs)
    ST_PIN_VGPR(dst);
#pragma unroll
    for (int t0 = 0; t0 < NT; t0 += STEP) {
        float old[STEP][4];
        if (add) {
#pragma unroll
            for (int t = 0; t < STEP; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) old[t][v] = dst[((t0 + t) * 4 + v) * 64];
        }
#pragma unroll
        for (int t = 0; t < STEP; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) dst[((t0 + t) * 4 + v) * 64] = add ? old[t][v] + acc[t0 + t][v] : acc[t0 + t][v];
        __builtin_amdgcn_sched_barrier(0);
    }
}

// STEPS K-steps (4 samples each) per staged chunk; V4: rows are read with 16-byte loads (n % 4 == 0); SINGLE: the
// row sets are single sets (third moment): no product, one read; NR: row sets this wave's block uses (the first NR
// of its three: a block at the ragged end of a row list issues no MFMAs for the sets it does not have; every
// instance runs the same chunk loop with the same barriers, so waves of one workgroup may run different ones).
template <int STEPS, bool V4, bool SINGLE, int NR>
__device__ __forceinline__ void mm_body(float *lds, const float *__restrict__ X, int64_t N, u32 n, u32 G, u32 kinds,
                                        int64_t slice, const int *__restrict__ table, float *__restrict__ ws,
                                        u32 tid, u32 wave, u32 block, u32 sl)
{
    constexpr int CH = STEPS * 4;
    constexpr int FLUSH = MM_FLUSH_SAMPLES / CH;       // chunks per fp32 accumulation chain
    const u32 lane = tid & 63u;
    auto used = [](int u) { return u >= MM_ROWS || u < NR; };      // spec u of the block is used by this instance
    const u32 chunk_f = (G + 1u) * (u32)STEPS * 64u;
    const int64_t s_begin = (int64_t)sl * slice, s_end = s_begin + slice < N ? s_begin + slice : N;

    // per-lane float offsets of the two operands of every product inside a chunk buffer (step 0)
    u32 oa[MM_SPECS], ob[MM_SPECS];
#pragma unroll
    for (int u = 0; u < MM_SPECS; ++u) {
        const u32 sp = (u32)table[(size_t)block * MM_SPECS + u];
        const u32 ga = mm_ga(sp), gb = mm_gb(sp), d = mm_d(sp);
        oa[u] = ga * (u32)STEPS * 64u + lane;
        ob[u] = gb * (u32)STEPS * 64u + (lane & 48u) + ((lane - d) & 15u);
    }
    f32x4 acc[MM_TPB];
#pragma unroll
    for (int t = 0; t < MM_TPB; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int64_t nchunks = (s_end - s_begin + CH - 1) / CH;
    const size_t slots = (size_t)kinds * MM_WAVES;
    float *dst = ws + ((size_t)sl * slots + block) * MM_ACC + lane;
    const MMStage stg = mm_stage<STEPS>(n, G, wave, lane);
    const bool padded = n != 16u * G;
    // samples of chunk c that exist
    auto rows_of = [&](int64_t c) -> u32 {
        const int64_t left = s_end - (s_begin + c * CH);
        return left < CH ? (u32)left : (u32)CH;
    };
    for (u32 q = tid; q < (u32)STEPS * 64u; q += (u32)MM_THREADS) {     // the plane of ones of both buffers
        lds[G * (u32)STEPS * 64u + q] = 1.f;
        lds[chunk_f + G * (u32)STEPS * 64u + q] = 1.f;
    }
    f32x4 r[MM_UNITS];
    mm_load_chunk<STEPS, V4>(r, stg, X + s_begin * (int64_t)n, rows_of(0), n, G, wave, lane);
    mm_store_chunk<STEPS>(r, stg, lds, rows_of(0), n, G, wave, lane, padded);
    if (nchunks > 1) mm_load_chunk<STEPS, V4>(r, stg, X + (s_begin + CH) * (int64_t)n, rows_of(1), n, G, wave, lane);
    __syncthreads();

    // One chunk.  WHOLE: chunks c+1 and c+2 exist and are whole (every iteration but the last three of a slice):
    // their staging is compiled for a full row count and without the tests on c, which leaves no conditional
    // definitions of the staging registers (they cost a register copy each per chunk) and, for n a multiple of 16,
    // no per-lane index arithmetic; on this chip none of that would be hidden behind the MFMAs.
    auto chunk = [&](int64_t c, auto whole) {
        constexpr bool WHOLE = decltype(whole)::value;
        const u32 cb = (u32)(c & 1);
        // registers hold chunk c+1: park it in the other buffer (its readers finished before the
        // barrier that ended the previous iteration), then put chunk c+2 in flight
        if constexpr (WHOLE) {
            mm_store_chunk<STEPS>(r, stg, lds + (cb ^ 1u) * chunk_f, (u32)CH, n, G, wave, lane, padded);
            mm_load_chunk<STEPS, V4>(r, stg, X + (s_begin + (c + 2) * CH) * (int64_t)n, (u32)CH, n, G, wave, lane);
        } else {
            if (c + 1 < nchunks)
                mm_store_chunk<STEPS>(r, stg, lds + (cb ^ 1u) * chunk_f, rows_of(c + 1), n, G, wave, lane, padded);
            if (c + 2 < nchunks)
                mm_load_chunk<STEPS, V4>(r, stg, X + (s_begin + (c + 2) * CH) * (int64_t)n, rows_of(c + 2), n, G, wave, lane);
        }
        __builtin_amdgcn_sched_barrier(0);
        const float *base = lds + cb * chunk_f;
        float a[2][MM_SPECS], b[2][MM_SPECS];
#pragma unroll
        for (int u = 0; u < MM_SPECS; ++u) {
            if (!used(u)) continue;
            a[0][u] = base[oa[u]];
            if (!(SINGLE && u < MM_ROWS)) b[0][u] = base[ob[u]];
        }
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            // The 22 operands of the next step are read under this step's MFMAs in three batches (8, 7, 7), one
            // before each third of the MFMAs: the counter of outstanding LDS operations holds 15, and with more
            // in flight the waits in front of the products drain everything.
            const int cur = st & 1, nxt = cur ^ 1;
            const bool more = st + 1 < STEPS;
            auto fetch = [&](int q0, int q1) {          // operands q of the next step: q < 11 first, else second
#pragma unroll
                for (int q = q0; q < q1; ++q) {
                    if (!used(q < MM_SPECS ? q : q - MM_SPECS)) continue;
                    if (q < MM_SPECS) a[nxt][q] = base[(st + 1) * 64 + oa[q]];
                    else if (!(SINGLE && q - MM_SPECS < MM_ROWS)) b[nxt][q - MM_SPECS] = base[(st + 1) * 64 + ob[q - MM_SPECS]];
                }
            };
            if (more) fetch(0, 8);
            __builtin_amdgcn_sched_barrier(0);
            float p[MM_SPECS];
#pragma unroll
            for (int u = 0; u < MM_SPECS; ++u)
                if (used(u)) p[u] = (SINGLE && u < MM_ROWS) ? a[cur][u] : a[cur][u] * b[cur][u];
#pragma unroll
            for (int t = 0; t < 8; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(p[t / MM_COLS], p[MM_ROWS + t % MM_COLS], acc[t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (more) fetch(8, 15);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (NR > 1) {
#pragma unroll
                for (int t = 8; t < 16; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(p[t / MM_COLS], p[MM_ROWS + t % MM_COLS], acc[t], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (more) fetch(15, 22);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (NR > 2) {
#pragma unroll
                for (int t = 16; t < MM_TPB; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(p[t / MM_COLS], p[MM_ROWS + t % MM_COLS], acc[t], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        // Long fp32 accumulation chains lose accuracy (1.2e-4 norm-wise after 180,000 samples): every FLUSH
        // chunks the accumulators are added to the wave's own partial in the workspace and cleared.
        if ((c + 1) % FLUSH == 0 && c + 1 < nchunks) {
            mm_flush<NR * MM_COLS>(acc, dst, c + 1 != FLUSH);
#pragma unroll
            for (int t = 0; t < MM_TPB; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
    };
    int64_t c = 0;
    for (; c + 3 < nchunks; ++c) chunk(c, std::true_type{});
    for (; c < nchunks; ++c) chunk(c, std::false_type{});
    mm_flush<NR * MM_COLS>(acc, dst, nchunks > FLUSH);
}

template <int STEPS, bool V4, bool SINGLE>
__global__ __launch_bounds__(MM_THREADS) void moment_mfma_kernel(const float *__restrict__ X, int64_t N, u32 n, u32 G,
                                                                 u32 kinds, int64_t slice,
                                                                 const int *__restrict__ table, float *__restrict__ ws)
{
    extern __shared__ float lds[];                      // two chunks of (G + 1) * STEPS * 64 floats (last plane: ones)
    const u32 tid = threadIdx.x;
    const u32 wave = (u32)__builtin_amdgcn_readfirstlane((int)(tid >> 6));
    const u32 kind = blockIdx.x % kinds, sl = blockIdx.x / kinds;
    const u32 block = kind * (u32)MM_WAVES + wave;     // the last slots of the last kind may be empty
    // row sets in use (the valid ones come first); an empty slot runs the one-row instance on sets that the reduce
    // kernel passes over
    u32 nr = 0;
#pragma unroll
    for (int u = 0; u < MM_ROWS; ++u) nr += ((u32)table[(size_t)block * MM_SPECS + u] & MM_VALID) ? 1u : 0u;
    nr = (u32)__builtin_amdgcn_readfirstlane((int)nr);
    if (nr >= 3u) mm_body<STEPS, V4, SINGLE, 3>(lds, X, N, n, G, kinds, slice, table, ws, tid, wave, block, sl);
    else if (nr == 2u) mm_body<STEPS, V4, SINGLE, 2>(lds, X, N, n, G, kinds, slice, table, ws, tid, wave, block, sl);
    else mm_body<STEPS, V4, SINGLE, 1>(lds, X, N, n, G, kinds, slice, table, ws, tid, wave, block, sl);
}

__device__ __forceinline__ u32 mm_cyc(u32 x, u32 y)
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
    const size_t e = (size_t)blockIdx.x * 256u + threadIdx.x;      // < blocks * MM_ACC
    if (e >= (size_t)blocks * MM_ACC) return;
    const u32 block = (u32)(e / (u32)MM_ACC), loc = (u32)(e - (size_t)block * MM_ACC);
    const u32 t = loc >> 8, v = (loc >> 6) & 3u, lane = loc & 63u;
    // D layout of the 16x16 MFMA: lane holds column lane%16 of rows 4*(lane/16) + v
    const u32 m = 4u * (lane >> 4) + v, mp = lane & 15u;
    const u32 rs = (u32)table[(size_t)block * MM_SPECS + t / (u32)MM_COLS];
    const u32 cs = (u32)table[(size_t)block * MM_SPECS + (u32)MM_ROWS + t % (u32)MM_COLS];
    if (!(rs & MM_VALID) || !(cs & MM_VALID)) return;
    const u32 g1 = mm_ga(rs), g2 = mm_gb(rs), dr = mm_d(rs);
    const u32 g3 = mm_ga(cs), g4 = mm_gb(cs), dc = mm_d(cs);
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
                const u32 d1 = mm_cyc(x1, z), d2 = mm_cyc(x2, z);
                const u32 k0 = 16u * dr + z;
                const u32 k1 = (d1 & 1u) ? 0xffffu : 16u * d1 + x2, k2 = (d2 & 1u) ? 0xffffu : 16u * d2 + x1;
                keep = k0 <= k1 && k0 <= k2;
            }
        } else if (g3 == a) {
            // all four in group a: of the three pairings (either pair as the row pair, which needs an even
            // distance) the smallest (d_row, d_col, row pair) is kept
            auto key = [](u32 r0, u32 r1, u32 c0, u32 c1) -> u32 {
                const u32 d = mm_cyc(r0, r1);
                if (d & 1u) return 0xffffffffu;
                return ((d * 9u + mm_cyc(c0, c1)) * 16u + min(r0, r1)) * 16u + max(r0, r1);
            };
            const u32 k0 = key(x1, x2, x3, x4);
            keep = key(x3, x4, x1, x2) >= k0 && key(x1, x3, x2, x4) >= k0 && key(x2, x4, x1, x3) >= k0 &&
                   key(x1, x4, x2, x3) >= k0 && key(x2, x3, x1, x4) >= k0;
        }
    }
    u32 i = 16u * g1 + x1, j = 16u * g2 + x2, k = 16u * g3 + x3, l = 16u * g4 + x4;
    if (!keep || i >= n || j >= n || k >= n || l >= n) return;
    float s = 0.f;
    const size_t stride = (size_t)slots * MM_ACC;
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

// One thread per raw accumulator of the third moment: row = a single set, column = a pair set.
__global__ __launch_bounds__(256) void moment3_mfma_reduce_kernel(const float *__restrict__ ws,
                                                                 const int *__restrict__ table, u32 blocks, u32 slots,
                                                                 u32 S, u32 n, float *__restrict__ Sc, int accumulate)
{
    const size_t e = (size_t)blockIdx.x * 256u + threadIdx.x;      // < blocks * MM_ACC
    if (e >= (size_t)blocks * MM_ACC) return;
    const u32 block = (u32)(e / (u32)MM_ACC), loc = (u32)(e - (size_t)block * MM_ACC);
    const u32 t = loc >> 8, v = (loc >> 6) & 3u, lane = loc & 63u;
    const u32 m = 4u * (lane >> 4) + v, mp = lane & 15u;
    const u32 rs = (u32)table[(size_t)block * MM_SPECS + t / (u32)MM_COLS];
    const u32 cs = (u32)table[(size_t)block * MM_SPECS + (u32)MM_ROWS + t % (u32)MM_COLS];
    if (!(rs & MM_VALID) || !(cs & MM_VALID)) return;
    const u32 g1 = mm_ga(rs), g3 = mm_ga(cs), g4 = mm_gb(cs), dc = mm_d(cs);
    const u32 other = (mp - dc) & 15u;
    if (g3 == g4 && dc == 8u && mp >= 8u) return;         // an in-group set at distance 8 names every pair twice
    if (g3 == g4 && g1 == g3) {
        // all three in one group: only pairs at an even distance count (two of three positions have the same
        // parity); the position whose pair is closest (then: whose row is smallest) is kept
        if (dc & 1u) return;
        const u32 d1 = mm_cyc(m, other), d2 = mm_cyc(m, mp);
        const u32 key = 16u * dc + m;
        const u32 key1 = (d1 & 1u) ? 0xffffu : 16u * d1 + mp, key2 = (d2 & 1u) ? 0xffffu : 16u * d2 + other;
        if (!(key <= key1 && key <= key2)) return;
    }
    u32 i = 16u * g1 + m, j = 16u * g3 + mp, k = 16u * g4 + other;
    if (i >= n || j >= n || k >= n) return;
    float s = 0.f;
    const size_t stride = (size_t)slots * MM_ACC;
#pragma unroll 4
    for (u32 y = 0; y < S; ++y) s += ws[(size_t)y * stride + e];
    const u32 lo = min(i, j), hi = max(i, j);
    const u32 a = min(lo, k), c = max(hi, k), b = max(lo, min(hi, k));
    const u32 pos = rank_sym3<u32>(n, a, b, c);
    Sc[pos] = accumulate ? Sc[pos] + s : s;
}

// Plan.  Workspace: the table (padded to 256 bytes), then S * slots blocks of partials.
struct MMPlan { u32 G, steps, kinds, blocks, S; int64_t slice; size_t table_bytes; };
static inline MMPlan mm_plan(int order, int64_t N, int n)
{
    MMPlan p;
    p.G = ((u32)n + 15u) / 16u;
    p.steps = p.G <= 8u ? 16u : 8u;                            // at most four staging units per wave
    const MMTable &t = mm_table(order, (int)p.G);
    p.kinds = t.kinds;
    p.blocks = t.blocks;
    p.table_bytes = (t.spec.size() * sizeof(int) + 255u) / 256u * 256u;
    const int64_t ch = 4 * p.steps;
    // Sample slices: every workgroup does the same work, so the kinds * S workgroups run in whole rounds of one
    // per compute unit; S is chosen for the best filled rounds, less what the partials of a slice cost (written
    // and read once, priced at 4 TB/s against the MFMA time of the whole job), each slice at least four chunks
    // long and the partials of all slices below 2 GB.
    const int64_t cus = num_cus();
    int64_t smax = (N + 4 * ch - 1) / (4 * ch);
    const int64_t scap = (int64_t)(((size_t)2 << 30) / ((size_t)p.kinds * MM_WAVES * MM_ACC * sizeof(float)));
    if (smax > scap) smax = scap;
    if (smax > 256) smax = 256;
    if (smax < 1) smax = 1;
    const double slice_bytes = (double)p.kinds * MM_WAVES * MM_ACC * sizeof(float);
    const double mfma_seconds = (double)p.blocks * MM_TPB * ((double)N / 4.0) * 32.0 / (4.0 * (double)cus * 2.3e9);
    const double per_slice = 0.001 + (2.0 * slice_bytes / 4e12) / mfma_seconds;
    int64_t S = 1;
    double best = -1.0;
    for (int64_t c = 1; c <= smax; ++c) {
        const int64_t wgs = (int64_t)p.kinds * c, rounds = (wgs + cus - 1) / cus;
        const double score = (double)wgs / (double)(rounds * cus) - per_slice * (double)c;
        if (score > best + 1e-9) { best = score; S = c; }
    }
    p.slice = ((N + S - 1) / S + ch - 1) / ch * ch;
    p.S = (u32)((N + p.slice - 1) / p.slice);
    return p;
}

// Used where it was measured faster than the vector-ALU tiles (which pad to blocks of 4, not of 16): the fourth
// moment in the upper part of every group count (29..32, 41..48, 53..64 features) and beyond 64, the third
// moment beyond the 64-feature kernel while 16 G <= 8/7 n.
bool moment_mfma_wins(int order, int n)
{
    const int G = (n + 15) / 16;
    if (order == 4) return n <= 256 && (n > 64 || n >= (G == 2 ? 29 : G == 3 ? 41 : G == 4 ? 53 : 999));
    return n > 64 && n <= 256 && 14 * G <= n;
}

size_t moment_mfma_workspace(int order, int64_t N, int n)
{
    if (N <= 0) return 0;
    const MMPlan p = mm_plan(order, N, n);
    return p.table_bytes + (size_t)p.S * p.kinds * MM_WAVES * MM_ACC * sizeof(float);
}

st_status launch_moment_mfma(int order, const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws,
                             hipStream_t s)
{
    const MMPlan p = mm_plan(order, N, n);
    const MMTable &tab = mm_table(order, (int)p.G);
    int *table = static_cast<int *>(ws);
    float *wsf = reinterpret_cast<float *>(static_cast<char *>(ws) + p.table_bytes);
    // the table: pinned host memory -> workspace, by a kernel on the caller's stream
    if (tab.pinned == nullptr) return ST_ERR_LAUNCH;
    {
        const u32 count = (u32)tab.spec.size();
        u32 cb = (count + 255u) / 256u;
        if (cb > 64u) cb = 64u;
        if (cb > 0u) hipLaunchKernelGGL(mm_table_copy_kernel, dim3(cb), dim3(256), 0, s, tab.pinned, table, count);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    }
    const dim3 grid(p.kinds * p.S), block(MM_THREADS);
    const size_t lds_bytes = (size_t)2u * (p.G + 1u) * p.steps * 64u * sizeof(float);
    const bool v4 = n % 4 == 0;
    bool ok;
#define ST_MM_LAUNCH(STEPS, V4, SINGLE)                                                                                 \
    do {                                                                                                                \
        ok = allow_dynamic_lds(reinterpret_cast<const void *>(moment_mfma_kernel<STEPS, V4, SINGLE>), 96 * 1024); /* up to 74 KB */ \
        if (ok) hipLaunchKernelGGL((moment_mfma_kernel<STEPS, V4, SINGLE>), grid, block, lds_bytes, s, X, N, (u32)n, p.G,  \
                                   p.kinds, p.slice, table, wsf);                                                       \
    } while (0)
    const bool single = order == 3;
    if (p.steps == 16u) {
        if (v4) { if (single) ST_MM_LAUNCH(16, true, true); else ST_MM_LAUNCH(16, true, false); }
        else { if (single) ST_MM_LAUNCH(16, false, true); else ST_MM_LAUNCH(16, false, false); }
    } else {
        if (v4) { if (single) ST_MM_LAUNCH(8, true, true); else ST_MM_LAUNCH(8, true, false); }
        else { if (single) ST_MM_LAUNCH(8, false, true); else ST_MM_LAUNCH(8, false, false); }
    }
#undef ST_MM_LAUNCH
    if (!ok || hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    const size_t racc = (size_t)p.blocks * MM_ACC;
    const dim3 rgrid((u32)((racc + 255) / 256));
    if (order == 3)
        hipLaunchKernelGGL(moment3_mfma_reduce_kernel, rgrid, dim3(256), 0, s, wsf, table, p.blocks,
                           p.kinds * (u32)MM_WAVES, p.S, (u32)n, Sc, accumulate);
    else
        hipLaunchKernelGGL(moment4_mfma_reduce_kernel, rgrid, dim3(256), 0, s, wsf, table, p.blocks,
                           p.kinds * (u32)MM_WAVES, p.S, (u32)n, Sc, accumulate);
    return launch_status();
}

}  // namespace st
