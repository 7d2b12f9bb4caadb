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
// waves, one per CU, persistent over rounds of four 16-row tiles.  A wave owns
// one tile and one quarter of the l range for all R columns; the rows of a
// round are requested while the MFMAs of the round before run (those of the
// first round right after U is staged).  U is staged once, in its natural
// row-major order (the column tiles of a row tile are interleaved, see below),
// per 16 values of l a wave issues four LDS reads of R/16 floats and 4*R/16
// MFMAs (lane = (row, l-quad); the four components of a 16-byte load of T feed
// four MFMAs whose K slots are permuted consistently on the U side).  The four
// quarter sums of a tile are added through LDS in a fixed order
// ((q0+q2)+(q1+q3)).
//
// General MFMA path (R <= 256): persistent workgroups, a work unit is a 16-row x
// 16-column output tile over the whole l range, U is staged in chunks of l; sizes
// that are not multiples of 16 are tiled over the next multiple with zeros staged
// for what lies outside U and element loads of T.  R > 256: one thread per output
// value.
//
// Algorithmic traffic per output row: 4*nl bytes read + 4*R written (+ U once).
#include <mutex>

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
// RAGGED: nl and R are the true sizes, the tiling runs over their multiples of 16 (kc, CT) and what lies
// outside U is staged as zeros.
template <bool RAGGED>
__device__ __forceinline__ void stage_u(float *lds, const float *__restrict__ U, u32 k0, u32 kc, u32 nl, u32 R,
                                        u32 CT, u32 tid, u32 nthreads)
{
    const u32 kq = kc / 4u, Rp = CT * 16u;
    for (u32 e = tid; e < kq * Rp; e += nthreads) {
        u32 k4 = e / Rp, col = e - k4 * Rp;
        const u32 l = k0 + 4u * k4;
        float4 v;
        if constexpr (RAGGED) {
            const u32 cc = min(col, R - 1u);
            float t[4];
#pragma unroll
            for (u32 q = 0; q < 4; ++q) {
                const float x = U[(size_t)min(l + q, nl - 1u) * R + cc];
                t[q] = (l + q < nl && col < R) ? x : 0.f;
            }
            v = make_float4(t[0], t[1], t[2], t[3]);
        } else {
            const float *src = U + (size_t)l * R + col;
            v = make_float4(src[0], src[R], src[2 * (size_t)R], src[3 * (size_t)R]);
        }
        u32 s = k4 >> 2, q = k4 & 3u, ct = col >> 4, c = col & 15u;
        *reinterpret_cast<float4 *>(lds + ((size_t)((s * CT + ct) * 64u + 16u * q + c)) * 4u) = v;
    }
}

// four values T(row, l .. l+3) of the A operand; RAGGED: element loads, zeros past the end of the row
template <bool RAGGED>
__device__ __forceinline__ float4 ttm_load_a(const float *__restrict__ rowp, u32 l, u32 nl)
{
    if constexpr (RAGGED) {
        float t[4];
#pragma unroll
        for (u32 q = 0; q < 4; ++q) {
            const float x = rowp[min(l + q, nl - 1u)];
            t[q] = l + q < nl ? x : 0.f;
        }
        return make_float4(t[0], t[1], t[2], t[3]);
    } else {
        return *reinterpret_cast<const float4 *>(rowp + l);
    }
}

template <bool RAGGED>
__global__ __launch_bounds__(TW * 64) void ttm_mfma_kernel(const float *__restrict__ Tc,
                                                         const float *__restrict__ U, float *__restrict__ Yc,
                                                         u32 rows, u32 nl, u32 R, u32 KC)
{
    extern __shared__ float lds[];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 CT = (R + 15u) / 16u, nlp = (nl + 15u) & ~15u;   // the tiling runs over multiples of 16
    const u32 SLOTS = TW / CT;                 // row tiles in flight per workgroup
    const u32 slot = wave / CT, ct = wave - slot * CT;
    const bool active = slot < SLOTS;
    const u32 rtiles = (rows + 15u) / 16u;
    const u32 per_super = gridDim.x * SLOTS * MAXR;
    const u32 nsuper = (rtiles + per_super - 1u) / per_super;
    const u32 nchunks = (nlp + KC - 1u) / KC;
    const u32 lrow = lane & 15u, lq = lane >> 4;

    for (u32 sr = 0; sr < nsuper; ++sr) {
        f32x4 acc[MAXR];
#pragma unroll
        for (int r = 0; r < MAXR; ++r) acc[r] = (f32x4){0.f, 0.f, 0.f, 0.f};

        for (u32 ch = 0; ch < nchunks; ++ch) {
            const u32 k0 = ch * KC, kc = min(KC, nlp - k0);
            if (!(nchunks == 1u && sr > 0u)) {
                __syncthreads();
                stage_u<RAGGED>(lds, U, k0, kc, nl, R, CT, tid, TW * 64u);
                __syncthreads();
            }
            if (!active) continue;
            const u32 steps = kc / 16u;
#pragma unroll
            for (int r = 0; r < MAXR; ++r) {
                u32 rt = blockIdx.x + gridDim.x * (slot + SLOTS * ((u32)r + MAXR * sr));
                if (rt >= rtiles) continue;
                u32 row = min(rt * 16u + lrow, rows - 1u);          // clamp: tail rows are discarded
                const float *rowp = Tc + (size_t)row * nl;
                const u32 l0 = k0 + 4u * lq;
                const f32x4 *bp = reinterpret_cast<const f32x4 *>(lds) + (size_t)ct * 64u + lane;
                f32x4 c = acc[r];
                u32 s = 0;
                for (; s + 4u <= steps; s += 4u) {
                    float4 a0 = ttm_load_a<RAGGED>(rowp, l0 + 16u * (s + 0u), nl), a1 = ttm_load_a<RAGGED>(rowp, l0 + 16u * (s + 1u), nl);
                    float4 a2 = ttm_load_a<RAGGED>(rowp, l0 + 16u * (s + 2u), nl), a3 = ttm_load_a<RAGGED>(rowp, l0 + 16u * (s + 3u), nl);
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
                    float4 a0 = ttm_load_a<RAGGED>(rowp, l0 + 16u * s, nl);
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
                    if (row < rows && ct * 16u + lrow < R) Yc[(size_t)row * R + ct * 16u + lrow] = acc[r][v];
                }
            }
        }
    }
}

// ---- split-K kernel --------------------------------------------------------------------
// NS = 16-value steps of l per wave (nl = 64*NS), CT = R/16.
//
// Column mapping.  A lane of an MFMA B operand / D result stands for one column n = lane % 16 of a
// 16-column tile.  Here the CT tiles of a row tile are interleaved: tile j holds the columns CT*n + j,
// so the CT values a lane needs from one row of U, and the CT results it holds for one output row, are
// CONSECUTIVE in memory.  U therefore stays in its natural row-major order in LDS (staged with plain
// 16-byte copies), one LDS read of CT floats feeds CT MFMAs, and a lane stores CT consecutive columns
// of Y at once.
template <int CT> struct cols { float v[CT]; };

template <int CT> __device__ __forceinline__ cols<CT> load_cols(const float *p)
{
    cols<CT> r;
    if constexpr (CT == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
    } else if constexpr (CT == 2) {
        const float2 t = *reinterpret_cast<const float2 *>(p);
        r.v[0] = t.x; r.v[1] = t.y;
    } else {
#pragma unroll
        for (int j = 0; j < CT; ++j) r.v[j] = p[j];
    }
    return r;
}

template <int CT> __device__ __forceinline__ void store_cols(float *p, const cols<CT> &r)
{
    if constexpr (CT == 4) *reinterpret_cast<float4 *>(p) = make_float4(r.v[0], r.v[1], r.v[2], r.v[3]);
    else if constexpr (CT == 2) *reinterpret_cast<float2 *>(p) = make_float2(r.v[0], r.v[1]);
    else {
#pragma unroll
        for (int j = 0; j < CT; ++j) p[j] = r.v[j];
    }
}

// U (nl x R, row-major) into LDS, same order: every thread issues all its 16-byte loads before its
// first LDS store, so the staging pays one memory latency.
template <u32 NL, u32 RR, u32 NTHREADS>
__device__ __forceinline__ void stage_u_rowmajor(float *lds, const float *__restrict__ U, u32 tid)
{
    constexpr u32 ITEMS = NL * RR / 4u, PER = (ITEMS + NTHREADS - 1u) / NTHREADS;
    float4 v[PER];
#pragma unroll
    for (u32 it = 0; it < PER; ++it)
        v[it] = reinterpret_cast<const float4 *>(U)[min(tid + NTHREADS * it, ITEMS - 1u)];
#pragma unroll
    for (u32 it = 0; it < PER; ++it) {
        const u32 e = tid + NTHREADS * it;
        if (e < ITEMS) reinterpret_cast<float4 *>(lds)[e] = v[it];
    }
}

// The 16-byte loads of a wave's quarter rows of row tile rt (A-operand layout: lane = (row, l-quad)).
template <int NS>
__device__ __forceinline__ const float4 *ttm_row_ptr(const float *__restrict__ Tc, u32 rt, u32 rtiles, u32 rows,
                                                     u32 lrow, u32 lq, u32 kq)
{
    const u32 row = min((rt < rtiles ? rt : 0u) * 16u + lrow, rows - 1u);    // clamp: tail rows are discarded
    return reinterpret_cast<const float4 *>(Tc + (size_t)row * (64u * NS) + kq * (16u * NS)) + lq;
}

// One round of a wave: the MFMAs of its quarter of a row tile, the addition of the four quarter sums
// through LDS in the order (q0+q2)+(q1+q3), and the store of one output row in four (row 4*(lane/16) + kq:
// every wave of the slot stores, so all waves issue the same memory operations per round).
//   FULL: every tile of the round is a full tile and a next round exists: nothing is conditional, and
//         the rows of the next round are requested one load per MFMA step (a wave whose request waits
//         for room in the memory pipeline then holds up only its own MFMAs).  The wait counters the
//         compiler derives for the prefetched rows are exact here; a conditional store between the
//         request of a row and its use would make the wave wait for the store as well.
//   else: guarded tail rounds; `prefetch` (workgroup-uniform) says whether another round follows.
template <int NS, int CT, bool FULL>
__device__ __forceinline__ void ttm_round(const float4 (&a)[NS], float4 (&an)[NS], const float4 *apn, bool prefetch,
                                          const float *__restrict__ ub, f32x4 *mine, float *__restrict__ Yc, u32 rt,
                                          u32 rtiles, u32 rows, u32 kq, u32 lrow, u32 lq)
{
    constexpr u32 R = 16u * CT;
    const bool live = FULL ? true : rt < rtiles;
    if (!FULL && prefetch) {
#pragma unroll
        for (int s = 0; s < NS; ++s) an[s] = apn[s * 4];
    }
    f32x4 acc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
    if (live) {   // wave-uniform
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (FULL) {
                an[s] = apn[s * 4];
                __builtin_amdgcn_sched_barrier(0);
            }
            const float av[4] = {a[s].x, a[s].y, a[s].z, a[s].w};
            cols<CT> b[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) b[t] = load_cols<CT>(ub + (size_t)(16 * s + t) * R);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int c = 0; c < CT; ++c)
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[t], b[t].v[c], acc[c], 0, 0, 0);
        }
    }
    if (kq >= 2u) {
#pragma unroll
        for (int c = 0; c < CT; ++c) mine[((kq - 2u) * CT + c) * 64u] = acc[c];
    }
    __syncthreads();
    if (kq < 2u) {       // q0 += q2, q1 += q3; each wave overwrites only what it has just read
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            acc[c] += mine[(kq * CT + c) * 64u];
            mine[(kq * CT + c) * 64u] = acc[c];
        }
    }
    __syncthreads();
    {
        // D layout: a lane holds, for column tile c, the rows 4*(lane/16) + v of column CT*(lane%16) + c
        const float *sums = reinterpret_cast<const float *>(mine);
        const u32 row = rt * 16u + 4u * lq + kq;
        cols<CT> y;
#pragma unroll
        for (int c = 0; c < CT; ++c) y.v[c] = sums[c * 256 + kq] + sums[(CT + c) * 256 + kq];
        if (FULL || (live && row < rows)) store_cols<CT>(Yc + (size_t)row * R + CT * lrow, y);
    }
    __syncthreads();     // the exchange area is free for the next round
}

// Workgroups of 16 waves, one per CU, persistent over rounds of four row tiles.  U is staged once and
// stays in LDS (nl*R*4 bytes) with the exchange area (4 slots * 2 * CT KB) behind it: 160 KB at
// nl = 512, R = 64.
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
    const u32 stride = gridDim.x * 4u;
    const u32 nrounds = (rtiles + stride - 1u) / stride;
    // leading rounds in which the tiles of all four slots of this workgroup are full tiles
    const u32 last_slot0 = blockIdx.x + gridDim.x * 3u, full_tiles = rows / 16u;
    u32 nfull = full_tiles > last_slot0 ? (full_tiles - last_slot0 + stride - 1u) / stride : 0u;
    if (nfull == nrounds && nfull > 0u) --nfull;           // the last round has nothing to prefetch
    const u32 lrow = lane & 15u, lq = lane >> 4;
    f32x4 *mine = reinterpret_cast<f32x4 *>(lds + nl * R) + (size_t)(slot * 2u) * CT * 64u + lane;
    // B operand of MFMA t of step s: lane (k = lane/16, n = lane%16) takes U(l, CT*n + c), l = 16 s + 4 k + t
    const float *ub = lds + (size_t)(kq * (16u * NS) + 4u * lq) * R + CT * lrow;
    const u32 rt0 = blockIdx.x + gridDim.x * slot;

    // U first, then the rows of the first round: a wave cannot pass the request of its rows before the
    // memory pipeline has room for them (with cold rows that takes microseconds for the last waves), so
    // nothing that all waves have to finish is put behind those requests.  The waves whose rows arrive
    // first start their MFMAs while the others still wait.
    stage_u_rowmajor<nl, R, TW * 64u>(lds, U, tid);
    __syncthreads();
    float4 a0[NS], a1[NS];
    {
        const float4 *ap = ttm_row_ptr<NS>(Tc, rt0, rtiles, rows, lrow, lq, kq);
#pragma unroll
        for (int s = 0; s < NS; ++s) a0[s] = ap[s * 4];
    }
    u32 round = 0;
    for (; round + 2u <= nfull; round += 2u) {
        const u32 rt = rt0 + stride * round;
        ttm_round<NS, CT, true>(a0, a1, ttm_row_ptr<NS>(Tc, rt + stride, rtiles, rows, lrow, lq, kq), true, ub, mine,
                                Yc, rt, rtiles, rows, kq, lrow, lq);
        __builtin_amdgcn_sched_barrier(0);
        ttm_round<NS, CT, true>(a1, a0, ttm_row_ptr<NS>(Tc, rt + 2u * stride, rtiles, rows, lrow, lq, kq), true, ub,
                                mine, Yc, rt + stride, rtiles, rows, kq, lrow, lq);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (; round < nrounds; round += 2u) {
        const u32 rt = rt0 + stride * round;
        ttm_round<NS, CT, false>(a0, a1, ttm_row_ptr<NS>(Tc, rt + stride, rtiles, rows, lrow, lq, kq),
                                 round + 1u < nrounds, ub, mine, Yc, rt, rtiles, rows, kq, lrow, lq);
        __builtin_amdgcn_sched_barrier(0);
        if (round + 1u < nrounds) {                        // workgroup-uniform
            ttm_round<NS, CT, false>(a1, a0, ttm_row_ptr<NS>(Tc, rt + 2u * stride, rtiles, rows, lrow, lq, kq),
                                     round + 2u < nrounds, ub, mine, Yc, rt + stride, rtiles, rows, kq, lrow, lq);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// ---- one-shot kernel: a few row tiles per workgroup -------------------------------------------------------
// With so few rows (the band workload: 540 row tiles on 256 CUs) a call is a few microseconds of memory
// latency around a few microseconds of MFMA work: everything is requested at once, no wave waits for
// another before its last MFMA, and the MFMA work is dealt evenly.
//   * Work: a workgroup owns FULL row tiles b, b+G, .. and, when the tile count is not a multiple of G,
//     single COLUMN tiles of the left-over row tiles (unit q = b + G e is column tile q % CT of row tile
//     full*G + q / CT): the left-over tiles are dealt in quarters, so no CU carries a whole tile more than
//     another (540 tiles on 256 CUs: 2.25 tiles at most instead of 3).
//   * Split of the l range over the W waves of the workgroup (W = 16, or nl/16 when that is less): wave w
//     owns l in [LW w, LW (w+1)), LW = nl / W, for ALL columns.  Its slice of U is LW x R floats, which it
//     keeps in REGISTERS as MFMA B operands, loaded straight from L2 with CT-float loads (the interleaved
//     column mapping of the persistent kernel: column tile j holds the columns CT n + j); its slice of the
//     rows of a tile is LW consecutive floats per row, 16-byte loads straight into A-operand registers.
//     Nothing is staged, there is no barrier in front of the MFMAs, every byte is requested once.
//   * The W partial results of a tile meet in LDS at the end and are added in wave order (fixed), one
//     output value per thread.
template <int NS, int CT, int FULL, bool EX>
__global__ __launch_bounds__((NS >= 4 ? 16 : 4 * NS) * 64) void ttm_oneshot_kernel(const float *__restrict__ Tc,
                                                             const float *__restrict__ U, float *__restrict__ Yc,
                                                             u32 rows)
{
    extern __shared__ float lds[];
    constexpr u32 nl = 64u * NS, R = 16u * CT, W = NS >= 4 ? 16u : 4u * NS, LW = nl / W, SPW = LW / 16u;
    constexpr u32 SLOTF = W * CT * 256u;                 // floats of one exchange buffer: [W][CT][64 lanes][4]
    constexpr int TT = FULL + (EX ? 1 : 0);              // tile slots: FULL whole row tiles, then one column-tile unit
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 lrow = lane & 15u, lq = lane >> 4;
    const u32 rtiles = (rows + 15u) / 16u, G = gridDim.x;
    // the column-tile unit of this workgroup: column tile xc of row tile xrt (xrt >= rtiles: none)
    const u32 xrt = FULL * G + blockIdx.x / CT, xc = blockIdx.x % CT;

    // B operands: MFMA t of step s, lane (k = lane/16, n = lane%16), column tile c: U(l, CT n + c), l = LW w + 16 s + 4 k + t
    // A operands: lane (row = lane%16, k = lane/16) takes T(row, LW w + 16 s + 4 k .. +3)
    // Request order: the rows of the first slot (cold, the longest latency of the launch), then the slice of U (the
    // same for every workgroup, so it comes from L2), then the rows of the other slots.
    float4 a[TT][SPW];
    cols<CT> u[SPW][4];
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        const u32 rt = t < FULL ? blockIdx.x + G * (u32)t : xrt;
        const u32 grow = min(rt * 16u + lrow, rows - 1u);            // clamp: rows past the end are never stored
        const float4 *ap = reinterpret_cast<const float4 *>(Tc + (size_t)grow * nl + wave * LW) + lq;
#pragma unroll
        for (u32 s = 0; s < SPW; ++s) a[t][s] = ap[4u * s];
        if (t == 0) {
            __builtin_amdgcn_sched_barrier(0);
            const float *up = U + (size_t)(wave * LW + 4u * lq) * R + CT * lrow;
#pragma unroll
            for (u32 s = 0; s < SPW; ++s)
#pragma unroll
                for (u32 q = 0; q < 4; ++q) u[s][q] = load_cols<CT>(up + (size_t)(16u * s + q) * R);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // every request of the wave is issued before its first MFMA (left to itself the compiler moves the requests
    // of the later tiles down between the MFMAs of the earlier ones, and their latency then adds to the MFMA time
    // instead of running under it)
    __builtin_amdgcn_sched_barrier(0);
    // all MFMAs first, slot after slot as the rows arrive (each slot has an exchange buffer of its own), then ONE
    // barrier, then the additions: no wave waits for another before its last MFMA
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        float *buf = lds + (size_t)t * SLOTF;
        if (t < FULL) {
            f32x4 acc[CT];
#pragma unroll
            for (int c = 0; c < CT; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (u32 s = 0; s < SPW; ++s) {
                const float av[4] = {a[t][s].x, a[t][s].y, a[t][s].z, a[t][s].w};
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int c = 0; c < CT; ++c)
                        acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[k], u[s][k].v[c], acc[c], 0, 0, 0);
            }
#pragma unroll
            for (int c = 0; c < CT; ++c)
                *reinterpret_cast<f32x4 *>(buf + ((size_t)(wave * CT + (u32)c) * 64u + lane) * 4u) = acc[c];
        } else {                                         // one column tile, chosen by selects (a workgroup without a
                                                         // unit multiplies clamped rows; its result is never read)
            f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (u32 s = 0; s < SPW; ++s) {
                const float av[4] = {a[t][s].x, a[t][s].y, a[t][s].z, a[t][s].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float b = u[s][k].v[0];
#pragma unroll
                    for (int c = 1; c < CT; ++c) b = xc == (u32)c ? u[s][k].v[c] : b;
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[k], b, acc, 0, 0, 0);
                }
            }
            *reinterpret_cast<f32x4 *>(buf + ((size_t)wave * 64u + lane) * 4u) = acc;     // [W][64 lanes][4]
        }
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        const float *buf = lds + (size_t)t * SLOTF;
        const bool whole = t < FULL;
        const u32 rt = whole ? blockIdx.x + G * (u32)t : xrt;
        if (rt >= rtiles) continue;
        // one output value per thread and pass, the W partial results added in wave order; value j of a
        // column tile c is element v = j % 4 of lane j / 4: row 4 (lane/16) + v, column CT (lane%16) + c
#pragma unroll 1
        for (u32 j = tid; j < (whole ? CT : 1u) * 256u; j += W * 64u) {
            const u32 c = whole ? j >> 8 : xc, jl = j & 255u, ln = jl >> 2, v = jl & 3u;
            const u32 wstride = whole ? CT * 256u : 256u, off = whole ? c * 256u + jl : jl;
            float y = 0.f;
#pragma unroll
            for (u32 w = 0; w < W; ++w) y += buf[(size_t)w * wstride + off];
            const u32 row = rt * 16u + 4u * (ln >> 4) + v;
            if (row < rows) Yc[(size_t)row * R + CT * (ln & 15u) + c] = y;
        }
    }
}

constexpr u32 ONESHOT_FULL = 2;    // whole row tiles per workgroup the one-shot kernel is built for (+ one column-tile unit)

// whole row tiles per workgroup, and whether the left-over tiles, dealt as single column tiles, fit one unit per
// workgroup; ok = false when the shape needs more than the kernel is built for
static inline void oneshot_split(u32 rtiles, u32 grid, u32 CT, u32 &full, bool &extra, bool &ok)
{
    full = rtiles / grid;
    const u32 rem = rtiles - full * grid;
    extra = rem > 0;
    ok = full <= ONESHOT_FULL && rem * CT <= grid && full + (extra ? 1u : 0u) >= 1u;
}

template <int NS, int CT>
static bool launch_oneshot_tt(u32 full, bool extra, u32 grid, hipStream_t s, const float *Tc, const float *U, float *Yc,
                              u32 rows)
{
    constexpr u32 W = NS >= 4 ? 16u : 4u * NS;
#define ST_TTM_ONESHOT(F, X)                                                                               \
    {                                                                                                      \
        const size_t lds_bytes = (size_t)F * W * CT * 1024u + (X ? W * 1024u : 0u);   /* one exchange buffer per slot */ \
        if (!allow_dynamic_lds(reinterpret_cast<const void *>(ttm_oneshot_kernel<NS, CT, F, X>), 160 * 1024)) return false; \
        hipLaunchKernelGGL((ttm_oneshot_kernel<NS, CT, F, X>), dim3(grid), dim3(W * 64u), lds_bytes, s, Tc, U, Yc, rows); \
        return true;                                                                                       \
    }
    if (full == 0 && extra) ST_TTM_ONESHOT(0, true)
    if (full == 1 && !extra) ST_TTM_ONESHOT(1, false)
    if (full == 1 && extra) ST_TTM_ONESHOT(1, true)
    if (full == 2 && !extra) ST_TTM_ONESHOT(2, false)
    if (full == 2 && extra) ST_TTM_ONESHOT(2, true)
#undef ST_TTM_ONESHOT
    return false;
}

template <int NS>
static bool launch_oneshot_ct(int CT, u32 full, bool extra, u32 grid, hipStream_t s, const float *Tc, const float *U,
                              float *Yc, u32 rows)
{
    switch (CT) {
    case 1: return launch_oneshot_tt<NS, 1>(full, extra, grid, s, Tc, U, Yc, rows);
    case 2: return launch_oneshot_tt<NS, 2>(full, extra, grid, s, Tc, U, Yc, rows);
    case 3: return launch_oneshot_tt<NS, 3>(full, extra, grid, s, Tc, U, Yc, rows);
    case 4: return launch_oneshot_tt<NS, 4>(full, extra, grid, s, Tc, U, Yc, rows);
    }
    return false;
}

template <int NS>
static bool launch_splitk_ct(int CT, u32 grid, size_t lds_bytes, hipStream_t s, const float *Tc, const float *U,
                             float *Yc, u32 rows)
{
#define ST_TTM_CASE(C)                                                                                   \
    case C: {                                                                                            \
        if (!allow_dynamic_lds(reinterpret_cast<const void *>(ttm_splitk_kernel<NS, C>), 160 * 1024)) return false; \
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

// whether a workgroup of the current device may hold 160 KB of LDS (asked once per device)
static bool lds_budget_160k()
{
    static std::mutex mu;
    static int cached[64] = {0};                       // 0 unknown, 1 yes, 2 no
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return false;
        cached[dev] = v >= 160 * 1024 ? 1 : 2;
    }
    return cached[dev] == 1;
}

st_status launch_ttm(const float *Tc, const float *U, float *Yc, int64_t rows, int nl, int R, void *,
                     hipStream_t s)
{
    if (rows == 0) return ST_OK;
    const bool splitk = (nl == 64 || nl == 128 || nl == 256 || nl == 512) && (R % 16 == 0) && R <= 64 &&
                        rows < ((int64_t)1 << 31) && lds_budget_160k();
    if (splitk) {
        const u32 rtiles = (u32)((rows + 15) / 16);
        u32 grid = (u32)num_cus();
        if (grid > rtiles) grid = rtiles;
        bool ok = false;
        u32 full = 0;
        bool extra = false, fits = false;
        oneshot_split(rtiles, grid, (u32)R / 16u, full, extra, fits);
        if (fits) {                                      // a few row tiles per CU: everything in one round
            switch (nl / 64) {
            case 1: ok = launch_oneshot_ct<1>(R / 16, full, extra, grid, s, Tc, U, Yc, (u32)rows); break;
            case 2: ok = launch_oneshot_ct<2>(R / 16, full, extra, grid, s, Tc, U, Yc, (u32)rows); break;
            case 4: ok = launch_oneshot_ct<4>(R / 16, full, extra, grid, s, Tc, U, Yc, (u32)rows); break;
            case 8: ok = launch_oneshot_ct<8>(R / 16, full, extra, grid, s, Tc, U, Yc, (u32)rows); break;
            }
            return ok ? launch_status() : ST_ERR_LAUNCH;
        }
        const size_t lds_bytes = (size_t)nl * R * 4u + (size_t)8u * (R / 16u) * 1024u;   // U + exchange area
        switch (nl / 64) {
        case 1: ok = launch_splitk_ct<1>(R / 16, grid, lds_bytes, s, Tc, U, Yc, (u32)rows); break;
        case 2: ok = launch_splitk_ct<2>(R / 16, grid, lds_bytes, s, Tc, U, Yc, (u32)rows); break;
        case 4: ok = launch_splitk_ct<4>(R / 16, grid, lds_bytes, s, Tc, U, Yc, (u32)rows); break;
        case 8: ok = launch_splitk_ct<8>(R / 16, grid, lds_bytes, s, Tc, U, Yc, (u32)rows); break;
        }
        return ok ? launch_status() : ST_ERR_LAUNCH;
    }
    bool mfma = R <= 256 && rows < ((int64_t)1 << 31) && (int64_t)nl < ((int64_t)1 << 30);
    if (mfma) {
        const bool ragged = (nl % 16 != 0) || (R % 16 != 0);
        const u32 Rp = ((u32)R + 15u) & ~15u, nlp = ((u32)nl + 15u) & ~15u;
        const u32 lds_budget = 128u * 1024u;
        u32 KC = (lds_budget / (Rp * 4u)) & ~15u;          // rows of U per LDS chunk, multiple of 16
        if (KC > nlp) KC = nlp;
        size_t lds_bytes = (size_t)KC * Rp * 4u;
        if (!allow_dynamic_lds(reinterpret_cast<const void *>(ttm_mfma_kernel<false>), (int)lds_budget) ||
            !allow_dynamic_lds(reinterpret_cast<const void *>(ttm_mfma_kernel<true>), (int)lds_budget))
            return ST_ERR_LAUNCH;
        u32 rtiles = (u32)((rows + 15) / 16);
        u32 grid = (u32)num_cus();
        if (grid > rtiles) grid = rtiles;
        if (ragged)
            hipLaunchKernelGGL(ttm_mfma_kernel<true>, dim3(grid), dim3(TW * 64), lds_bytes, s, Tc, U, Yc, (u32)rows,
                               (u32)nl, (u32)R, KC);
        else
            hipLaunchKernelGGL(ttm_mfma_kernel<false>, dim3(grid), dim3(TW * 64), lds_bytes, s, Tc, U, Yc, (u32)rows,
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
