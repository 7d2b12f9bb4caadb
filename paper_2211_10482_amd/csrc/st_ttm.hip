// Tensor-times-matrix along mode 3 of a band tensor,
//     Y(i,j,r) = sum_l T(i,j,l) U(l,r)   for the in-band pairs (i,j) only.
//
// In packed band storage the in-band fibres T(i,j,:) are the rows of a plain
// row-major matrix [band_pairs][nl], and the output keeps the same unique set,
// so the kernel is a dense contraction [rows x nl] . [nl x R] and runs on the
// fp32 matrix cores (v_mfma_f32_16x16x4_f32).  The band itself only decides
// which rows exist (rank/unrank of the row id is the caller's business).
//
// Split-K path (nl in {64,128,256,512}, R in {16,32,48,64}): workgroups of 16
// waves, one per CU.  A wave owns a 16-row tile and one quarter of the l range
// for all R columns: it issues every 16-byte load of its quarter rows at once,
// before U is staged, so the HBM latency is paid once and overlaps the staging.
// U is staged into LDS already permuted into MFMA B-operand order; per 16 values
// of l a wave issues one ds_read_b128 of U per 16 columns and four MFMAs per
// read (lane = (row, l-quad); the four components of a load feed four MFMAs whose
// K slots are permuted consistently on the U side).  The four quarter sums of a
// tile are added through LDS in a fixed order ((q0+q2)+(q1+q3)).
//
// General MFMA path (nl % 16 == 0, R % 16 == 0, R <= 256): persistent workgroups,
// a work unit is a 16-row x 16-column output tile over the whole l range, U is
// staged in chunks of l.  Any other shape: one thread per output value.
//
// Algorithmic traffic per output row: 4*nl bytes read + 4*R written (+ U once).
#include "st_common.h"

namespace st {

typedef uint32_t u32;
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int TW = 16;        // waves per workgroup
constexpr int MAXR = 4;       // row tiles a wave keeps accumulators for at once

// Stage rows [k0, k0+kc) of U (nl x R, row-major) into LDS in B-operand order:
// value U(k0 + 16 s + 4 q + t, 16 ct + c) goes to ((s*CT + ct)*64 + 16 q + c)*4 + t.
// A thread gathers the four rows t = 0..3 of one column (each of its loads is
// coalesced along the column index across the wave) and writes them with one
// conflict-free 16-byte LDS store.
__device__ __forceinline__ void stage_u(float *lds, const float *__restrict__ U, u32 k0, u32 kc, u32 R,
                                        u32 CT, u32 tid, u32 nthreads)
{
    const u32 kq = kc / 4u;
    for (u32 e = tid; e < kq * R; e += nthreads) {
        u32 k4 = e / R, col = e - k4 * R;
        const float *src = U + (size_t)(k0 + 4u * k4) * R + col;
        float4 v = make_float4(src[0], src[R], src[2 * (size_t)R], src[3 * (size_t)R]);
        u32 s = k4 >> 2, q = k4 & 3u, ct = col >> 4, c = col & 15u;
        *reinterpret_cast<float4 *>(lds + ((size_t)((s * CT + ct) * 64u + 16u * q + c)) * 4u) = v;
    }
}

__global__ __launch_bounds__(TW * 64) void ttm_mfma_kernel(const float *__restrict__ Tc,
                                                         const float *__restrict__ U, float *__restrict__ Yc,
                                                         u32 rows, u32 nl, u32 R, u32 KC)
{
    extern __shared__ float lds[];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 CT = R / 16u;
    const u32 SLOTS = TW / CT;                 // row tiles in flight per workgroup
    const u32 slot = wave / CT, ct = wave - slot * CT;
    const bool active = slot < SLOTS;
    const u32 rtiles = (rows + 15u) / 16u;
    const u32 per_super = gridDim.x * SLOTS * MAXR;
    const u32 nsuper = (rtiles + per_super - 1u) / per_super;
    const u32 nchunks = (nl + KC - 1u) / KC;
    const u32 lrow = lane & 15u, lq = lane >> 4;

    for (u32 sr = 0; sr < nsuper; ++sr) {
        f32x4 acc[MAXR];
#pragma unroll
        for (int r = 0; r < MAXR; ++r) acc[r] = (f32x4){0.f, 0.f, 0.f, 0.f};

        for (u32 ch = 0; ch < nchunks; ++ch) {
            const u32 k0 = ch * KC, kc = min(KC, nl - k0);
            if (!(nchunks == 1u && sr > 0u)) {
                __syncthreads();
                stage_u(lds, U, k0, kc, R, CT, tid, TW * 64u);
                __syncthreads();
            }
            if (!active) continue;
            const u32 steps = kc / 16u;
#pragma unroll
            for (int r = 0; r < MAXR; ++r) {
                u32 rt = blockIdx.x + gridDim.x * (slot + SLOTS * ((u32)r + MAXR * sr));
                if (rt >= rtiles) continue;
                u32 row = min(rt * 16u + lrow, rows - 1u);          // clamp: tail rows are discarded
                const float4 *ap = reinterpret_cast<const float4 *>(Tc + (size_t)row * nl + k0) + lq;
                const f32x4 *bp = reinterpret_cast<const f32x4 *>(lds) + (size_t)ct * 64u + lane;
                f32x4 c = acc[r];
                u32 s = 0;
                for (; s + 4u <= steps; s += 4u) {
                    float4 a0 = ap[(s + 0u) * 4u], a1 = ap[(s + 1u) * 4u];
                    float4 a2 = ap[(s + 2u) * 4u], a3 = ap[(s + 3u) * 4u];
                    f32x4 b0 = bp[(size_t)(s + 0u) * CT * 64u], b1 = bp[(size_t)(s + 1u) * CT * 64u];
                    f32x4 b2 = bp[(size_t)(s + 2u) * CT * 64u], b3 = bp[(size_t)(s + 3u) * CT * 64u];
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.x, b0[0], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.y, b0[1], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.z, b0[2], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.w, b0[3], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a1.x, b1[0], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a1.y, b1[1], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a1.z, b1[2], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a1.w, b1[3], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a2.x, b2[0], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a2.y, b2[1], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a2.z, b2[2], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a2.w, b2[3], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a3.x, b3[0], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a3.y, b3[1], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a3.z, b3[2], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a3.w, b3[3], c, 0, 0, 0);
                }
                for (; s < steps; ++s) {
                    float4 a0 = ap[s * 4u];
                    f32x4 b0 = bp[(size_t)s * CT * 64u];
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.x, b0[0], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.y, b0[1], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.z, b0[2], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.w, b0[3], c, 0, 0, 0);
                }
                acc[r] = c;
            }
        }

        if (active) {
#pragma unroll
            for (int r = 0; r < MAXR; ++r) {
                u32 rt = blockIdx.x + gridDim.x * (slot + SLOTS * ((u32)r + MAXR * sr));
                if (rt >= rtiles) continue;
                // D layout: lane holds column lane%16 of rows 4*(lane/16) + v
#pragma unroll
                for (u32 v = 0; v < 4; ++v) {
                    u32 row = rt * 16u + 4u * lq + v;
                    if (row < rows) Yc[(size_t)row * R + ct * 16u + lrow] = acc[r][v];
                }
            }
        }
    }
}

// Same staging with the shape known at compile time: every thread issues all of
// its loads before the first LDS store, so the staging pays one memory latency.
template <u32 NL, u32 RR, u32 NTHREADS>
__device__ __forceinline__ void stage_u_static(float *lds, const float *__restrict__ U, u32 tid)
{
    constexpr u32 CT = RR / 16u, ITEMS = (NL / 4u) * RR, PER = (ITEMS + NTHREADS - 1u) / NTHREADS;
    float4 v[PER];
#pragma unroll
    for (u32 it = 0; it < PER; ++it) {
        const u32 e = min(tid + NTHREADS * it, ITEMS - 1u);
        const u32 k4 = e / RR, col = e % RR;
        const float *src = U + (size_t)(4u * k4) * RR + col;
        v[it] = make_float4(src[0], src[RR], src[2u * RR], src[3u * RR]);
    }
#pragma unroll
    for (u32 it = 0; it < PER; ++it) {
        const u32 e = tid + NTHREADS * it;
        const u32 k4 = e / RR, col = e % RR;
        const u32 s = k4 >> 2, q = k4 & 3u, ct = col >> 4, c = col & 15u;
        if (e < ITEMS) *reinterpret_cast<float4 *>(lds + ((size_t)((s * CT + ct) * 64u + 16u * q + c)) * 4u) = v[it];
    }
}

// ---- split-K kernel ---------------------------------------------------------------
// NS = 16-value steps of l per wave (nl = 64*NS), CT = R/16.
template <int NS, int CT>
__global__ __launch_bounds__(TW * 64) void ttm_splitk_kernel(const float *__restrict__ Tc,
                                                           const float *__restrict__ U, float *__restrict__ Yc,
                                                           u32 rows)
{
    extern __shared__ float lds[];
    constexpr u32 nl = 64u * NS, R = 16u * CT;
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 slot = wave >> 2, kq = wave & 3u;            // row-tile slot, quarter of the l range
    const u32 rtiles = (rows + 15u) / 16u;
    const u32 nrounds = (rtiles + gridDim.x * 4u - 1u) / (gridDim.x * 4u);
    const u32 lrow = lane & 15u, lq = lane >> 4;
    f32x4 *xch = reinterpret_cast<f32x4 *>(lds);           // exchange area, aliases the staged U

    for (u32 round = 0; round < nrounds; ++round) {
        const u32 rt = blockIdx.x + gridDim.x * (slot + 4u * round);
        const bool live = rt < rtiles;
        // all loads of this wave's quarter rows go out first
        float4 a[NS];
        {
            const u32 row = min((live ? rt : 0u) * 16u + lrow, rows - 1u);   // clamp: tail rows are discarded
            const float4 *ap = reinterpret_cast<const float4 *>(Tc + (size_t)row * nl + kq * (16u * NS)) + lq;
#pragma unroll
            for (int s = 0; s < NS; ++s) a[s] = ap[s * 4];
        }
        if (round > 0) __syncthreads();                    // exchange area of the previous round is free
        stage_u_static<nl, R, TW * 64u>(lds, U, tid);
        __syncthreads();

        f32x4 acc[CT];
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
        const f32x4 *bp = reinterpret_cast<const f32x4 *>(lds) + (size_t)(kq * NS) * CT * 64u + lane;
        if (live) {   // wave-uniform: idle slots leave the matrix cores to the live ones
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            f32x4 b[CT];
#pragma unroll
            for (int c = 0; c < CT; ++c) b[c] = bp[(s * CT + c) * 64];
            const float av[4] = {a[s].x, a[s].y, a[s].z, a[s].w};
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int c = 0; c < CT; ++c)
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[t], b[c][t], acc[c], 0, 0, 0);
        }
        }
        __syncthreads();                                   // every wave is done reading U

        // quarters 2,3 -> quarters 0,1 ; then quarter 1 -> quarter 0
        f32x4 *mine = xch + (size_t)(slot * 2u) * CT * 64u + lane;
        if (kq >= 2u) {
#pragma unroll
            for (int c = 0; c < CT; ++c) mine[((kq - 2u) * CT + c) * 64u] = acc[c];
        }
        __syncthreads();
        if (kq < 2u) {
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                const f32x4 o = mine[(kq * CT + c) * 64u];
                acc[c] += o;
            }
        }
        __syncthreads();
        if (kq == 1u) {
#pragma unroll
            for (int c = 0; c < CT; ++c) mine[c * 64u] = acc[c];
        }
        __syncthreads();
        if (kq == 0u && live) {
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                const f32x4 o = mine[c * 64u];
                // D layout: lane holds column lane%16 of rows 4*(lane/16) + v
#pragma unroll
                for (u32 v = 0; v < 4; ++v) {
                    const u32 row = rt * 16u + 4u * lq + v;
                    if (row < rows) Yc[(size_t)row * R + c * 16u + lrow] = acc[c][v] + o[v];
                }
            }
        }
    }
}

template <int NS>
static bool launch_splitk_ct(int CT, u32 grid, size_t lds_bytes, hipStream_t s, const float *Tc, const float *U,
                             float *Yc, u32 rows)
{
#define ST_TTM_CASE(C)                                                                                   \
    case C: {                                                                                            \
        static bool attr = false;                                                                        \
        if (!attr) {                                                                                     \
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(ttm_splitk_kernel<NS, C>),            \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess) \
                return false;                                                                            \
            attr = true;                                                                                 \
        }                                                                                                \
        hipLaunchKernelGGL((ttm_splitk_kernel<NS, C>), dim3(grid), dim3(TW * 64), lds_bytes, s, Tc, U, Yc, rows); \
        return true;                                                                                     \
    }
    switch (CT) {
        ST_TTM_CASE(1)
        ST_TTM_CASE(2)
        ST_TTM_CASE(3)
        ST_TTM_CASE(4)
    }
#undef ST_TTM_CASE
    return false;
}

// Any shape: one thread per output value.
__global__ __launch_bounds__(256) void ttm_plain_kernel(const float *__restrict__ Tc,
                                                       const float *__restrict__ U, float *__restrict__ Yc,
                                                       uint64_t rows, u32 nl, u32 R)
{
    uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (t >= rows * R) return;
    uint64_t row = t / R;
    u32 r = (u32)(t - row * R);
    const float *a = Tc + row * nl;
    float s = 0.f;
    for (u32 l = 0; l < nl; ++l) s += a[l] * U[(size_t)l * R + r];
    Yc[t] = s;
}

size_t ttm_workspace(int, int, int, int) { return 0; }

st_status launch_ttm(const float *Tc, const float *U, float *Yc, int64_t rows, int nl, int R, void *,
                     hipStream_t s)
{
    if (rows == 0) return ST_OK;
    const bool splitk = (nl == 64 || nl == 128 || nl == 256 || nl == 512) && (R % 16 == 0) && R <= 64 &&
                        rows < ((int64_t)1 << 31);
    if (splitk) {
        const u32 rtiles = (u32)((rows + 15) / 16);
        u32 grid = (u32)num_cus();
        if (grid > rtiles) grid = rtiles;
        size_t lds_bytes = (size_t)nl * R * 4u;
        if (lds_bytes < 32u * 1024u) lds_bytes = 32u * 1024u;     // room for the exchange area
        bool ok = false;
        switch (nl / 64) {
        case 1: ok = launch_splitk_ct<1>(R / 16, grid, lds_bytes, s, Tc, U, Yc, (u32)rows); break;
        case 2: ok = launch_splitk_ct<2>(R / 16, grid, lds_bytes, s, Tc, U, Yc, (u32)rows); break;
        case 4: ok = launch_splitk_ct<4>(R / 16, grid, lds_bytes, s, Tc, U, Yc, (u32)rows); break;
        case 8: ok = launch_splitk_ct<8>(R / 16, grid, lds_bytes, s, Tc, U, Yc, (u32)rows); break;
        }
        return ok ? launch_status() : ST_ERR_LAUNCH;
    }
    bool mfma = (nl % 16 == 0) && (R % 16 == 0) && R <= 256 && rows < ((int64_t)1 << 31);
    if (mfma) {
        const u32 lds_budget = 128u * 1024u;
        u32 KC = (lds_budget / ((u32)R * 4u)) & ~15u;      // rows of U per LDS chunk, multiple of 16
        if (KC > (u32)nl) KC = (u32)nl;
        size_t lds_bytes = (size_t)KC * R * 4u;
        static bool attr_set = false;
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(ttm_mfma_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_budget) != hipSuccess)
                return ST_ERR_LAUNCH;
            attr_set = true;
        }
        u32 rtiles = (u32)((rows + 15) / 16);
        u32 grid = (u32)num_cus();
        if (grid > rtiles) grid = rtiles;
        hipLaunchKernelGGL(ttm_mfma_kernel, dim3(grid), dim3(TW * 64), lds_bytes, s, Tc, U, Yc, (u32)rows,
                           (u32)nl, (u32)R, KC);
        return launch_status();
    }
    uint64_t total = (uint64_t)rows * R;
    if ((total + 255) / 256 > 0x7fffffffull) return ST_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(ttm_plain_kernel, dim3((u32)((total + 255) / 256)), dim3(256), 0, s, Tc, U, Yc,
                       (uint64_t)rows, (u32)nl, (u32)R);
    return launch_status();
}

}  // namespace st
