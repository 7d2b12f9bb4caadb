// The three covariance terms of degree-2 polynomial regression in ONE pass over the samples,
// for at most sixteen features (the paper's two end-to-end data sets have six and thirteen):
//     S1(i,j) (+)= sum_s x_i x_j,   S2(i,j,k) (+)= sum_s x_i x_j x_k,   S3(i,j,k,l) (+)= sum_s x_i x_j x_k x_l
// over the unique sets i <= j (<= k (<= l)).  A lane takes whole samples and walks the nest
// for i, for j = i, for k = j, for l = k  with the running products x_i x_j and x_i x_j x_k shared
// by the inner loops, every accumulator a register.
//   * up to six features all 21 + 56 + 126 unique entries fit ONE lane: every lane of the grid has
//     its own samples (a wave reads 64 consecutive rows, every byte of them used); the lanes of a
//     wave (through LDS), then the four waves of a workgroup, are added in a fixed order at the end;
//   * seven to sixteen features: the waves of a workgroup take the same 64 samples and different
//     parts of the nest (second half of this file).
// Workgroup partials -> reduce kernel (fixed order, no atomics).  Bound by the HBM stream (six
// features) or the fp32 vector rate (thirteen and more).
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
    constexpr int CS_PH = NP <= 4 ? 33 : 52;          // accumulators per pass of the lane sum through LDS (at most 64)
    __shared__ float tr[4][CS_PH * 65];
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
    // The 64 lanes of a wave are added through LDS, CS_PH accumulators at a time: every lane writes its values
    // as column `lane` of a [CS_PH][64] block (rows padded to 65 floats: no bank conflicts either way), lane a
    // then adds row a in lane order.  A DPP tree per accumulator would be seven vector instructions for each of
    // the 203, a quarter of everything this kernel issues at two million samples.  Then the four waves.
    constexpr int PHASES = (C::ALL + CS_PH - 1) / CS_PH;
#pragma unroll
    for (int ph = 0; ph < PHASES; ++ph) {
#pragma unroll
        for (int a = 0; a < CS_PH; ++a)
            if (ph * CS_PH + a < C::ALL) tr[wave][a * 65 + (int)lane] = acc[ph * CS_PH + a];
        __syncthreads();
        if (lane < (u32)CS_PH && ph * CS_PH + (int)lane < C::ALL) {
            float v = 0.f;
#pragma unroll 16
            for (int q = 0; q < 64; ++q) v += tr[wave][lane * 65u + (u32)q];
            red[wave][ph * CS_PH + (int)lane] = v;
        }
        __syncthreads();
    }
    for (u32 a = tid; a < (u32)C::ALL; a += 256u)
        ws[(size_t)blockIdx.x * C::ALL + a] = (red[0][a] + red[1][a]) + (red[2][a] + red[3][a]);
}

// 4 accumulators x 64 slices of the workgroup partials per block (at most 8 partials per thread for the 512
// workgroups of the one-lane kernel, all loads in flight together; slices added in ascending order, y ascending
// inside a slice); keeps the entries with every index < n (S1 or S2 may be null: that term is not wanted)
__global__ __launch_bounds__(256) void covar_small_reduce_kernel(const float *__restrict__ ws, u32 G, u32 n, u32 np,
                                                                float *__restrict__ S1, float *__restrict__ S2,
                                                                float *__restrict__ S3, int accumulate)
{
    __shared__ float part[64][4];
    const u32 a = threadIdx.x & 3u, g = threadIdx.x >> 2;
    const u32 a2 = count_sym2<u32>(np), a3 = count_sym3<u32>(np), a4 = count_sym4<u32>(np), all = a2 + a3 + a4;
    const u32 t = blockIdx.x * 4u + a;
    float s = 0.f;
    if (t < all) {
        const u32 per = (G + 63u) / 64u, y0 = min(G, g * per), y1 = min(G, y0 + per);
#pragma unroll 8
        for (u32 y = y0; y < y1; ++y) s += ws[(size_t)y * all + t];
    }
    part[g][a] = s;
    __syncthreads();
    if (g != 0u || t >= all) return;
    s = 0.f;
#pragma unroll
    for (int q = 0; q < 64; ++q) s += part[q][a];
    u32 i, j, k, l;
    if (t < a2) {
        unrank_sym2<u32>(np, t, i, j);
        if (j >= n || !S1) return;
        const u32 p = rank_sym2<u32>(n, i, j);
        S1[p] = accumulate ? S1[p] + s : s;
    } else if (t < a2 + a3) {
        unrank_sym3<u32>(np, t - a2, i, j, k);
        if (k >= n || !S2) return;
        const u32 p = rank_sym3<u32>(n, i, j, k);
        S2[p] = accumulate ? S2[p] + s : s;
    } else {
        unrank_sym4<u32>(np, t - a2 - a3, i, j, k, l);
        if (l >= n) return;
        const u32 p = rank_sym4<u32>(n, i, j, k, l);
        S3[p] = accumulate ? S3[p] + s : s;
    }
}

// ---- seven to sixteen features: the same lanes, the accumulators split over the waves -------------
// A lane still takes whole samples, but the unique entries no longer fit one lane's registers (13 features:
// 91 + 455 + 1,820), so the waves of a workgroup take the SAME 64 samples and different parts of the loop nest:
// the nest is cut by its (i, j) prefix -- S1(i,j), S2(i,j,k >= j) and S3(i,j,k,l >= k) belong together and
// share the running products -- and the prefixes are dealt to 4, 8, 16 or 24 waves of at most CSP_BUDGET
// accumulators each, 4 or 8 waves to a workgroup (one, two or three kinds of workgroup).  The 64 rows are
// staged once per workgroup in LDS (coalesced; read back one column of 64 rows at a time).  No accumulator
// has two owners in a workgroup, so a wave writes its sums straight into the workgroup's partial; X is read
// once per kind of workgroup.
constexpr int CSP_BUDGET = 210;                   // accumulators per wave at most (about 240 registers per lane in all)
constexpr int CSP_NMAX = 16;
template <int NP> constexpr int csp_prefix_count(int j) { return 1 + (NP - j) + (NP - j) * (NP - j + 1) / 2; }
template <int NP> struct CspPlan {
    int pi[NP * (NP + 1) / 2], pj[NP * (NP + 1) / 2];   // the prefixes (i, j), j >= i, in nest order
    int first[65];            // wave w (over all kinds) owns the prefixes first[w] .. first[w+1]-1
    int accs[64];             // accumulators of each wave
    int waves;
};
// Prefixes are dealt to the waves largest first, each to the wave with the fewest accumulators so far; the
// number of waves is the smallest of 4, 8, 16, 24, 32 that keeps a wave within CSP_BUDGET (whole SIMDs' worth
// of equally loaded waves: a workgroup is 4 or 8 of them).
template <int NP> constexpr CspPlan<NP> csp_make_plan()
{
    constexpr int NPAIR = NP * (NP + 1) / 2;
    CspPlan<NP> p{};
    int total = 0;
    for (int i = 0; i < NP; ++i)
        for (int j = i; j < NP; ++j) total += csp_prefix_count<NP>(j);
    const int choices[5] = {4, 8, 16, 24, 32};
    int K = 32;
    for (int c = 4; c >= 0; --c)
        if ((total + choices[c] - 1) / choices[c] <= CSP_BUDGET - 8) K = choices[c];
    int load[32] = {}, owner[NPAIR] = {}, oi[NPAIR] = {}, oj[NPAIR] = {};
    // prefixes by decreasing count: the count depends on j only and falls with j
    int q = 0;
    for (int j = 0; j < NP; ++j)
        for (int i = 0; i <= j; ++i) {
            int best = 0;
            for (int w = 1; w < K; ++w)
                if (load[w] < load[best]) best = w;
            load[best] += csp_prefix_count<NP>(j);
            owner[q] = best;
            oi[q] = i;
            oj[q] = j;
            ++q;
        }
    q = 0;
    for (int w = 0; w < K; ++w) {
        p.first[w] = q;
        p.accs[w] = load[w];
        for (int t = 0; t < NPAIR; ++t)
            if (owner[t] == w) { p.pi[q] = oi[t]; p.pj[q] = oj[t]; ++q; }
    }
    p.first[K] = q;
    p.waves = K;
    return p;
}
template <int NP> struct CspStatic { static constexpr CspPlan<NP> plan = csp_make_plan<NP>(); };
template <int NP> constexpr int csp_kinds() { return (CspStatic<NP>::plan.waves + 7) / 8; }
template <int NP> constexpr int csp_wpk() { return CspStatic<NP>::plan.waves < 8 ? CspStatic<NP>::plan.waves : 8; }

// Staging of a group of 64 consecutive samples: the workgroup's threads read the 64 n floats (contiguous in X) in
// order and park them as rows of LS = NP | 1 floats (odd: lanes that read one column of 64 rows hit 64 banks).
constexpr int CSP_STAGE = 3;                      // elements per thread: 64 * 16 floats over at least 448 threads
template <int NP> struct CspLds { static constexpr int LS = NP | 1, FLOATS = 64 * LS; };
__device__ __forceinline__ void csp_stage_load(float (&r)[CSP_STAGE], const float *__restrict__ X, int64_t N, u32 n,
                                               int64_t group, u32 tid, u32 nthreads)
{
    const int64_t base = group * 64 * (int64_t)n, end = N * (int64_t)n;
#pragma unroll
    for (int k = 0; k < CSP_STAGE; ++k) {
        const u32 e = tid + nthreads * (u32)k;
        r[k] = (e < 64u * n && base + e < end) ? X[base + e] : 0.f;
    }
}
template <int NP>
__device__ __forceinline__ void csp_stage_store(const float (&r)[CSP_STAGE], float *__restrict__ buf, u32 n, u32 tid,
                                                u32 nthreads)
{
#pragma unroll
    for (int k = 0; k < CSP_STAGE; ++k) {
        const u32 e = tid + nthreads * (u32)k;
        if (e < 64u * n) {
            const u32 smp = e / n, c = e - smp * n;
            buf[smp * (u32)CspLds<NP>::LS + c] = r[k];
        }
    }
}

// Wave W of the plan (W >= the number of waves: a wave that only helps with the staging).  Every wave of the
// workgroup runs the same loop over the sample groups g, g + G, .. with one barrier per group.
template <int NP, int W>
__device__ __forceinline__ void csp_body(const float *__restrict__ X, int64_t N, u32 n, int64_t g, int64_t G,
                                         float *__restrict__ part, float *__restrict__ lds, u32 tid, u32 nthreads)
{
    typedef CsCounts<NP> C;
    constexpr bool REAL = W < CspStatic<NP>::plan.waves;
    constexpr int NA = REAL ? CspStatic<NP>::plan.accs[REAL ? W : 0] : 1;
    constexpr int Q0 = REAL ? CspStatic<NP>::plan.first[REAL ? W : 0] : 0;
    constexpr int Q1 = REAL ? CspStatic<NP>::plan.first[REAL ? W + 1 : 0] : 0;
    constexpr int LS = CspLds<NP>::LS;
    const u32 lane = tid & 63u;
    float acc[NA];
#pragma unroll
    for (int a = 0; a < NA; ++a) acc[a] = 0.f;
    const int64_t ngroups = (N + 63) / 64;
    // columns >= n of a staged row are never written: zero both buffers once
    for (u32 e = tid; e < 2u * (u32)CspLds<NP>::FLOATS; e += nthreads) lds[e] = 0.f;
    __syncthreads();
    float r[CSP_STAGE];
    csp_stage_load(r, X, N, n, g, tid, nthreads);
    csp_stage_store<NP>(r, lds, n, tid, nthreads);
    __syncthreads();
    u32 cur = 0;
    for (int64_t grp = g; grp < ngroups; grp += G, cur ^= 1u) {
        const bool more = grp + G < ngroups;
        if (more) csp_stage_load(r, X, N, n, grp + G, tid, nthreads);       // in flight under the products
        if constexpr (REAL) {
            const float *row = lds + cur * (u32)CspLds<NP>::FLOATS + lane * (u32)LS;
            float x[NP];
#pragma unroll
            for (int c = 0; c < NP; ++c) x[c] = row[c];
            int a = 0;
#pragma unroll
            for (int q = Q0; q < Q1; ++q) {
                const int i = CspStatic<NP>::plan.pi[q], j = CspStatic<NP>::plan.pj[q];
                const float pij = x[i] * x[j];
                acc[a++] += pij;
#pragma unroll
                for (int k = j; k < NP; ++k) {
                    const float pijk = pij * x[k];
                    acc[a++] += pijk;
#pragma unroll
                    for (int l = k; l < NP; ++l) acc[a++] += pijk * x[l];
                }
            }
        }
        // the other buffer was read in the previous iteration, which ended with a barrier
        if (more) csp_stage_store<NP>(r, lds + (cur ^ 1u) * (u32)CspLds<NP>::FLOATS, n, tid, nthreads);
        __syncthreads();
    }
    if constexpr (REAL) {
        int a = 0;
#pragma unroll
        for (int q = Q0; q < Q1; ++q) {
            const int i = CspStatic<NP>::plan.pi[q], j = CspStatic<NP>::plan.pj[q];
            float v = wave_sum(acc[a++]);
            if (lane == 0u) part[rank_sym2<u32>(NP, i, j)] = v;
#pragma unroll
            for (int k = j; k < NP; ++k) {
                v = wave_sum(acc[a++]);
                if (lane == 0u) part[C::A2 + rank_sym3<u32>(NP, i, j, k)] = v;
#pragma unroll
                for (int l = k; l < NP; ++l) {
                    v = wave_sum(acc[a++]);
                    if (lane == 0u) part[C::A2 + C::A3 + rank_sym4<u32>(NP, i, j, k, l)] = v;
                }
            }
        }
    }
}
// gw in 0 .. kinds * waves-per-kind - 1; the slots past the plan's last wave run the helper body
template <int NP, int W>
__device__ __forceinline__ void csp_dispatch(int gw, const float *__restrict__ X, int64_t N, u32 n, int64_t g,
                                             int64_t G, float *__restrict__ part, float *__restrict__ lds, u32 tid,
                                             u32 nthreads)
{
    if constexpr (W + 1 < csp_kinds<NP>() * csp_wpk<NP>()) {
        if (gw == W) csp_body<NP, W>(X, N, n, g, G, part, lds, tid, nthreads);
        else csp_dispatch<NP, W + 1>(gw, X, N, n, g, G, part, lds, tid, nthreads);
    } else {
        csp_body<NP, W>(X, N, n, g, G, part, lds, tid, nthreads);
    }
}
// grid.x = kinds * G: workgroup (kind, g) takes the sample groups g, g + G, .. of 64 samples
template <int NP>
__global__ __launch_bounds__(512) void covar_split_kernel(const float *__restrict__ X, int64_t N, u32 n, u32 G,
                                                         float *__restrict__ ws)
{
    typedef CsCounts<NP> C;
    __shared__ float lds[2 * CspLds<NP>::FLOATS];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const u32 kind = blockIdx.x % (u32)csp_kinds<NP>(), g = blockIdx.x / (u32)csp_kinds<NP>();
    const int gw = (int)kind * csp_wpk<NP>() + wave;
    csp_dispatch<NP, 0>(gw, X, N, n, (int64_t)g, (int64_t)G, ws + (size_t)g * C::ALL, lds, threadIdx.x,
                        64u * (u32)csp_wpk<NP>());
}
static inline u32 csp_np(int n) { return n <= 8 ? 8u : n <= 10 ? 10u : n <= 13 ? 13u : 16u; }
template <int NP> static st_status csp_launch(const float *X, int64_t N, int n, u32 G, float *wsf, hipStream_t s)
{
    hipLaunchKernelGGL(covar_split_kernel<NP>, dim3(G * (u32)csp_kinds<NP>()), dim3(64u * (u32)csp_wpk<NP>()), 0, s, X, N,
                       (u32)n, G, wsf);
    return hipGetLastError() == hipSuccess ? ST_OK : ST_ERR_LAUNCH;
}
static inline u32 csp_groups(int64_t N, u32 np)
{
    const u32 kinds = np == 8u ? (u32)csp_kinds<8>() : np == 10u ? (u32)csp_kinds<10>()
                                                   : np == 13u ? (u32)csp_kinds<13>() : (u32)csp_kinds<16>();
    int64_t g = 2 * (int64_t)num_cus() / kinds;            // about two workgroups per compute unit in all
    const int64_t gmax = (N + 63) / 64;
    if (g > gmax) g = gmax;
    return (u32)(g < 1 ? 1 : g);
}

static inline u32 cs_groups(int64_t N)
{
    const int64_t g = (N + 255) / 256;
    return (u32)(g < 1 ? 1 : g > CS_WGS ? CS_WGS : g);
}
static inline u32 cs_np(int n) { return n <= 4 ? 4u : n <= CS_NMAX ? 6u : csp_np(n); }
static inline u32 cs_all(u32 np) { return count_sym2<u32>(np) + count_sym3<u32>(np) + count_sym4<u32>(np); }

bool covar_small_applies(int n) { return n >= 1 && n <= CSP_NMAX; }

size_t covar_small_workspace(int64_t N, int n)
{
    if (N <= 0) return 0;
    const u32 np = cs_np(n);
    const u32 G = n <= CS_NMAX ? cs_groups(N) : csp_groups(N, np);
    return (size_t)G * cs_all(np) * sizeof(float);
}

// N >= 1; S1 and S2 may be null (the fourth moment alone)
st_status launch_covar_small(const float *X, int64_t N, int n, float *S1, float *S2, float *S3, int accumulate,
                             void *ws, hipStream_t s)
{
    const u32 np = cs_np(n);
    float *wsf = static_cast<float *>(ws);
    u32 G;
    if (n <= CS_NMAX) {
        G = cs_groups(N);
        if (np == 4u) hipLaunchKernelGGL(covar_small_kernel<4>, dim3(G), dim3(256), 0, s, X, N, (u32)n, wsf);
        else hipLaunchKernelGGL(covar_small_kernel<6>, dim3(G), dim3(256), 0, s, X, N, (u32)n, wsf);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    } else {
        G = csp_groups(N, np);
        st_status rc;
        if (np == 8u) rc = csp_launch<8>(X, N, n, G, wsf, s);
        else if (np == 10u) rc = csp_launch<10>(X, N, n, G, wsf, s);
        else if (np == 13u) rc = csp_launch<13>(X, N, n, G, wsf, s);
        else rc = csp_launch<16>(X, N, n, G, wsf, s);
        if (rc != ST_OK) return rc;
    }
    const u32 all = cs_all(np);
    hipLaunchKernelGGL(covar_small_reduce_kernel, dim3((all + 3u) / 4u), dim3(256), 0, s, wsf, G, (u32)n, np, S1, S2,
                       S3, accumulate);
    return launch_status();
}

}  // namespace st
