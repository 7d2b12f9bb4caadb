// MTTKRP with a fully symmetric order-3 tensor and equal factors,
//     M(i,r) = sum_{j,k} T(i,j,k) B(j,r) B(k,r),
// reading only the packed unique entries i<=j<=k.
//
// The index range is cut into blocks of 16.  For a block X of output rows and
// an unordered pair of blocks P <= Q the 16^3 sub-tensor D[x][p][q] =
// T(sort(x,p,q)) contributes  M(x,r) += w * sum_{p,q} D[x][p][q] B(p,r) B(q,r)
// with w = 2 for P < Q (the mirrored pair Q,P) and 1 for P = Q.  That is a
// dense contraction [16 x 256] . [256 x R] against Khatri-Rao rows formed on
// the fly, and runs on the fp32 matrix cores (v_mfma_f32_16x16x4_f32).
//
// "Owner computes": a workgroup owns the output rows of one block X and a
// contiguous range of block pairs, so no two workgroups ever add into the same
// output and the result is deterministic; a packed entry is visited by the (up
// to three) owners of its indices.  Per visit the sub-tensor is staged in LDS.
// The visits of X come in two classes, each with its own closed-form
// enumeration and its own branch-free, software-pipelined loop:
//   * "run" visits, P < Q both different from X (and n a multiple of 16): the
//     sub-tensor is made of contiguous runs of packed storage -- along q when Q
//     is the largest block (16-byte loads, 16-byte LDS writes), along x when X is
//     (16-byte loads transposed into the tile by the LDS writes);
//   * "gather" visits, two of the three blocks equal (2*NB-1 pairs per X), or
//     every visit when n is ragged: per element sort + closed-form rank3.
// The 16 x 64 blocks of B for P (pre-scaled by w) and Q are staged beside the
// tile.  While visit v is multiplied, visit v+1 sits in the second LDS buffer
// and the loads of visit v+2 are in flight in registers; one barrier per visit.
// Each of the 4 waves owns 16 columns r: per p one ds_read_b128 of D (lane =
// (x, q-quad); the four components feed four MFMAs with consistently permuted K
// slots and separate accumulators), four VALU multiplies for the Khatri-Rao
// operand, four MFMAs.  Workgroup partials go to the workspace; a second kernel
// adds them in a fixed order.
//
// Algorithmic traffic: 4 bytes per stored entry (each read by three owners,
// two of them out of cache) + B + M.
#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr u32 XS = 260;            // LDS stride between x-planes of the tile (16*16 + 4 pad)
constexpr u32 TILE_F = 16 * XS;    // floats per staged tile
constexpr u32 BS = 68;             // LDS row stride of a staged 16 x 64 block of B (bank spread)
constexpr u32 BBLK_F = 16 * BS;
#ifndef ST_MTTKRP_NT
#define ST_MTTKRP_NT 512
#endif
constexpr u32 NT = ST_MTTKRP_NT;   // threads per workgroup: 4 column waves x PSPLIT halves of the p range
constexpr u32 PSPLIT = NT / 256;
constexpr u32 TPT = 4096 / NT;     // tile values staged per thread
constexpr u32 BPT = 512 / NT;      // float4 pieces of the two B blocks staged per thread
static_assert(NT == 256 || NT == 512, "workgroup size");

struct __attribute__((packed, aligned(4))) f4u { float x, y, z, w; };

__device__ __forceinline__ void sort3u(u32 &a, u32 &b, u32 &c)
{
    u32 lo = min(a, b), hi = max(a, b);
    u32 mn = min(lo, c), mx = max(hi, c), md = max(lo, min(hi, c));
    a = mn; b = md; c = mx;
}

// One visit = (row block X, block pair P <= Q).
struct Visit {
    u32 p0, q0;   // first index of blocks P and Q
    bool qruns;   // run visits: runs along q (Q above X) or along x
    float wgt;    // 2 for P < Q, 1 for P = Q
};

// Cursor over the visits of one class for row block X.  Only the first position
// is unranked; after that the cursor steps (all of it wave-uniform scalar work).
//   run visits   : u-th strict pair a < b+1 of the NB-1 blocks other than X,
//                  kept as (a, b) with a <= b < NB-2 in sym2 order
//   gather visits: ragged n -> every pair P <= Q in sym2 order (a, b);
//                  otherwise the 2*NB-1 pairs with two equal blocks: (g,g) for
//                  g < NB, then (g',X) for g' < X, then (X,g'+1)   (a = g)
template <bool GATHER> struct Cursor {
    u32 NB, X, a, b;
    bool all_pairs;

    __device__ __forceinline__ Cursor(u32 NB_, u32 X_, bool all_pairs_, u32 u) : NB(NB_), X(X_), all_pairs(all_pairs_)
    {
        if (!GATHER) unrank_sym2<u32>(NB - 2u, u, a, b);
        else if (all_pairs) unrank_sym2<u32>(NB, u, a, b);
        else { a = u; b = 0; }
    }
    __device__ __forceinline__ void step()
    {
        if (!GATHER || all_pairs) {
            const u32 last = (GATHER ? NB : NB - 2u) - 1u;
            if (b < last) ++b; else { ++a; b = a; }
        } else {
            ++a;
        }
    }
    __device__ __forceinline__ Visit get() const
    {
        u32 P, Q;
        if (!GATHER) {
            P = a + (a >= X ? 1u : 0u);
            Q = b + 1u + (b + 1u >= X ? 1u : 0u);
        } else if (all_pairs) {
            P = a; Q = b;
        } else if (a < NB) {
            P = Q = a;
        } else {
            const u32 h = a - NB;
            P = h < X ? h : X;
            Q = h < X ? X : h + 1u;
        }
        Visit v;
        v.p0 = P * 16u; v.q0 = Q * 16u; v.qruns = !GATHER && Q > X; v.wgt = (P < Q) ? 2.f : 1.f;
        return v;
    }
};

// Global -> registers for one visit: 16 tile values and one float4 of each staged
// B block per thread.  Every load is unconditional (addresses clamped) and the
// results are not touched here, so they stay in flight while the previous visit
// is multiplied; store_visit zeroes what lies outside the tensor.
template <bool GATHER, bool R4>
__device__ __forceinline__ void load_visit(const Visit &v, const float *__restrict__ Tc,
                                           const float *__restrict__ B, u32 n, u32 R, u32 x0, u32 rbase,
                                           u32 tid, float (&pf)[TPT], float (&bb)[BPT][4])
{
    if constexpr (!GATHER) {
#pragma unroll
        for (u32 it = 0; it < TPT / 4; ++it) {
            const u32 e = tid + NT * it, row = e >> 2, qr = e & 3u;
            const u32 hi = row >> 4, lo = row & 15u;
            // runs along q: row = (x, p), D[x][p][q] = Tc[run(min, max) + (q0 + q - max)]
            // runs along x: row = (p, q), D[x][p][q] = Tc[run(p, q) + (x0 + x - q)]
            const u32 i1 = v.qruns ? x0 + hi : v.p0 + hi;
            const u32 i2 = v.qruns ? v.p0 + lo : v.q0 + lo;
            const u32 a = min(i1, i2), b = max(i1, i2);
            const u32 first = v.qruns ? v.q0 : x0;
            f4u t = *reinterpret_cast<const f4u *>(Tc + run_sym3<u32>(n, a, b) + (first - b) + 4u * qr);
            pf[4 * it] = t.x; pf[4 * it + 1] = t.y; pf[4 * it + 2] = t.z; pf[4 * it + 3] = t.w;
        }
    } else {
#pragma unroll
        for (u32 it = 0; it < TPT; ++it) {
            const u32 e = tid + NT * it;
            u32 a = x0 + (e >> 8), b = v.p0 + ((e >> 4) & 15u), c = v.q0 + (e & 15u);
            sort3u(a, b, c);
            pf[it] = Tc[c < n ? rank_sym3<u32>(n, a, b, c) : 0u];
        }
    }
    // piece j = tid + NT*k of the two 16 x 64 blocks of B: block j/256 (P, then Q),
    // row (j%256)/16, columns rbase + 4*(j%16) .. +3
#pragma unroll
    for (u32 k = 0; k < BPT; ++k) {
        const u32 j = tid + NT * k, h = j >> 8, row = (j & 255u) >> 4, col = rbase + 4u * (j & 15u);
        const u32 gr = (h == 0 ? v.p0 : v.q0) + row;
        float(&dst)[4] = bb[k];
        if constexpr (R4) {   // R % 4 == 0: rows of B are 16-byte aligned
            const bool ok = gr < n && col < R;
            float4 t = *reinterpret_cast<const float4 *>(B + (ok ? (size_t)gr * R + col : 0));
            dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w;
        } else {
#pragma unroll
            for (u32 q = 0; q < 4; ++q) dst[q] = B[(gr < n && col + q < R) ? (size_t)gr * R + col + q : 0];
        }
    }
}

// Registers -> LDS: dense tile D[x][p][q] (x-stride XS) and the two B blocks, the
// P block scaled by the pair weight; positions outside the tensor become zero.
template <bool GATHER>
__device__ __forceinline__ void store_visit(const Visit &v, u32 n, u32 R, u32 x0, u32 rbase,
                                            float *__restrict__ tile, float *__restrict__ bp,
                                            float *__restrict__ bq, u32 tid, const float (&pf)[TPT],
                                            const float (&bb)[BPT][4])
{
    if constexpr (!GATHER) {
        if (v.qruns) {
#pragma unroll
            for (u32 it = 0; it < TPT / 4; ++it) {
                const u32 e = tid + NT * it, row = e >> 2, qr = e & 3u;
                *reinterpret_cast<float4 *>(&tile[(row >> 4) * XS + (row & 15u) * 16u + 4u * qr]) =
                    make_float4(pf[4 * it], pf[4 * it + 1], pf[4 * it + 2], pf[4 * it + 3]);
            }
        } else {
#pragma unroll
            for (u32 it = 0; it < TPT / 4; ++it) {
                const u32 e = tid + NT * it, row = e >> 2, xr = e & 3u;
                float *d = &tile[(4u * xr) * XS + (row >> 4) * 16u + (row & 15u)];
                d[0] = pf[4 * it]; d[XS] = pf[4 * it + 1]; d[2 * XS] = pf[4 * it + 2]; d[3 * XS] = pf[4 * it + 3];
            }
        }
    } else {
#pragma unroll
        for (u32 it = 0; it < TPT; ++it) {
            const u32 e = tid + NT * it;
            const u32 x = e >> 8, p = (e >> 4) & 15u, q = e & 15u;
            const bool ok = max(x0 + x, max(v.p0 + p, v.q0 + q)) < n;
            tile[x * XS + p * 16u + q] = ok ? pf[it] : 0.f;
        }
    }
#pragma unroll
    for (u32 k = 0; k < BPT; ++k) {
        const u32 j = tid + NT * k, h = j >> 8, row = (j & 255u) >> 4, col = rbase + 4u * (j & 15u);
        const bool rok = (h == 0 ? v.p0 : v.q0) + row < n;
        const float w = (h == 0) ? v.wgt : 1.f;
        float *dst = (h == 0 ? bp : bq) + row * BS + 4u * (j & 15u);
        *reinterpret_cast<float4 *>(dst) =
            make_float4((rok && col + 0u < R) ? w * bb[k][0] : 0.f, (rok && col + 1u < R) ? w * bb[k][1] : 0.f,
                        (rok && col + 2u < R) ? w * bb[k][2] : 0.f, (rok && col + 3u < R) ? w * bb[k][3] : 0.f);
    }
}

struct MttkrpLds {
    float tile[2][TILE_F];
    float bp[2][BBLK_F];
    float bq[2][BBLK_F];
};

// Visits [v0, v1) of one class for row block X, accumulated into acc.
template <bool GATHER, bool R4>
__device__ __forceinline__ void visit_loop(MttkrpLds &L, const float *__restrict__ Tc,
                                           const float *__restrict__ B, u32 n, u32 R, u32 NB, u32 X,
                                           bool all_pairs, u32 v0, u32 v1, u32 rbase, bool has_rt,
                                           f32x4 (&acc)[4])
{
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 x0 = X * 16u, lrow = lane & 15u, lq = lane >> 4;
    if (v0 >= v1) return;
    const u32 nv = v1 - v0;
    Cursor<GATHER> cur(NB, X, all_pairs, v0);

    float pf[TPT], bb[BPT][4];
    Visit nxt = cur.get();
    load_visit<GATHER, R4>(nxt, Tc, B, n, R, x0, rbase, tid, pf, bb);
    store_visit<GATHER>(nxt, n, R, x0, rbase, L.tile[0], L.bp[0], L.bq[0], tid, pf, bb);
    if (nv > 1) {
        cur.step();
        nxt = cur.get();
        load_visit<GATHER, R4>(nxt, Tc, B, n, R, x0, rbase, tid, pf, bb);
    }
    __syncthreads();

    for (u32 v = 0; v < nv; ++v) {
        const u32 cb = v & 1u;
        // registers hold visit v+1: park it in the other buffer (its last readers
        // finished before the barrier that ended iteration v-1) ...
        if (v + 1 < nv)
            store_visit<GATHER>(nxt, n, R, x0, rbase, L.tile[cb ^ 1u], L.bp[cb ^ 1u], L.bq[cb ^ 1u], tid, pf, bb);
        // ... and put visit v+2 in flight
        if (v + 2 < nv) {
            cur.step();
            nxt = cur.get();
            load_visit<GATHER, R4>(nxt, Tc, B, n, R, x0, rbase, tid, pf, bb);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (has_rt) {
            const u32 cw = wave & 3u, pbeg = (wave >> 2) * (16u / PSPLIT);   // column block, first p
            const float *bqp = &L.bq[cb][(4u * lq) * BS + cw * 16u + lrow];
            const float bq0 = bqp[0], bq1 = bqp[BS], bq2 = bqp[2 * BS], bq3 = bqp[3 * BS];
            const float *bpp = &L.bp[cb][pbeg * BS + cw * 16u + lrow];
            const float *arow = &L.tile[cb][lrow * XS + pbeg * 16u + 4u * lq];
#pragma unroll
            for (u32 p = 0; p < 16u / PSPLIT; ++p) {
                const float bpv = bpp[p * BS];
                const f32x4 a = *reinterpret_cast<const f32x4 *>(arow + p * 16u);
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], bpv * bq0, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], bpv * bq1, acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], bpv * bq2, acc[2], 0, 0, 0);
                acc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], bpv * bq3, acc[3], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    }
}

struct MttkrpPlan {
    u32 NB, RT, Rpad;
    u32 all_pairs;        // ragged n: every visit takes the gather loop
    u32 nrun, ngat;       // visits per row block in each class
    u32 PPR, PPG;         // visits per workgroup in each class
    u32 NCHR, NCHG, NCH;  // workgroups (chunks) per row block
};

template <bool R4>
__global__ __launch_bounds__(NT) void mttkrp_mfma_kernel(const float *__restrict__ Tc,
                                                        const float *__restrict__ B,
                                                        float *__restrict__ part, u32 n, u32 R, MttkrpPlan pl)
{
    __shared__ __attribute__((aligned(16))) MttkrpLds L;
    const u32 lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const u32 X = blockIdx.y, ch = blockIdx.x;
    const u32 rbase = blockIdx.z * 64u;               // this workgroup's 64 columns of R
    const u32 rt = blockIdx.z * 4u + (wave & 3u);     // this wave's block of 16 columns
    const bool has_rt = rt * 16u < R;

    f32x4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};

    if (ch < pl.NCHR) {
        const u32 v0 = ch * pl.PPR;
        visit_loop<false, R4>(L, Tc, B, n, R, pl.NB, X, false, v0, min(pl.nrun, v0 + pl.PPR), rbase, has_rt, acc);
    } else {
        const u32 v0 = (ch - pl.NCHR) * pl.PPG;
        visit_loop<true, R4>(L, Tc, B, n, R, pl.NB, X, pl.all_pairs != 0u, v0, min(pl.ngat, v0 + pl.PPG), rbase,
                         has_rt, acc);
    }

    f32x4 sum;
#pragma unroll
    for (u32 v = 0; v < 4; ++v) sum[v] = (acc[0][v] + acc[1][v]) + (acc[2][v] + acc[3][v]);
    if constexpr (PSPLIT == 2) {
        // the waves of the upper half of the p range hand their sums to the lower half
        // (the visit loops end with a barrier, so the tile buffer is free)
        f32x4 *xch = reinterpret_cast<f32x4 *>(&L.tile[0][0]);
        if (wave >= 4u) xch[(wave - 4u) * 64u + lane] = sum;
        __syncthreads();
        if (wave < 4u) {
            const f32x4 o = xch[wave * 64u + lane];
#pragma unroll
            for (u32 v = 0; v < 4; ++v) sum[v] += o[v];
        }
    }
    if (has_rt && wave < 4u) {
        // D layout: lane holds column lane%16 of rows 4*(lane/16) + v
        const u32 lrow = lane & 15u, lq = lane >> 4;
        float *dst = part + ((size_t)(X * pl.NCH + ch) * 16u) * pl.Rpad + rt * 16u + lrow;
#pragma unroll
        for (u32 v = 0; v < 4; ++v) dst[(size_t)(4u * lq + v) * pl.Rpad] = sum[v];
    }
}

// M(16X + x, r) = sum_ch part[X][ch][x][r]: a thread owns one output value and
// one of 8 slices of the chunks (ch ascending inside a slice, slices ascending).
__global__ __launch_bounds__(256) void mttkrp_reduce_kernel(const float *__restrict__ part,
                                                          float *__restrict__ M, u32 n, u32 R, u32 NCH,
                                                          u32 Rpad)
{
    __shared__ float acc[8][32];
    const u32 o = threadIdx.x & 31u, sl = threadIdx.x >> 5;
    const u32 t = blockIdx.x * 32u + o;
    float s = 0.f;
    if (t < n * R) {
        const u32 i = t / R, r = t - i * R;
        const u32 per = (NCH + 7u) / 8u, c0 = min(NCH, sl * per), c1 = min(NCH, c0 + per);
        const float *src = part + ((size_t)((i >> 4) * NCH) * 16u + (i & 15u)) * Rpad + r;
#pragma unroll 4
        for (u32 c = c0; c < c1; ++c) s += src[(size_t)c * 16u * Rpad];
    }
    acc[sl][o] = s;
    __syncthreads();
    if (sl == 0 && t < n * R) {
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) v += acc[q][o];
        M[t] = v;
    }
}

static inline MttkrpPlan plan(int n, int R)
{
    MttkrpPlan p;
    p.NB = ((u32)n + 15u) / 16u;
    p.RT = ((u32)R + 15u) / 16u;
    p.Rpad = p.RT * 16u;
    p.all_pairs = (n % 16 != 0) ? 1u : 0u;
    const u32 npairs = p.NB * (p.NB + 1u) / 2u;
    if (p.all_pairs) {
        p.nrun = 0;
        p.ngat = npairs;
    } else {
        p.nrun = p.NB >= 3u ? (p.NB - 1u) * (p.NB - 2u) / 2u : 0u;
        p.ngat = 2u * p.NB - 1u;
    }
    // about 1500 workgroups in all (two rounds of three per CU); a gather visit costs
    // roughly two run visits
    uint64_t work = (uint64_t)p.NB * ((uint64_t)p.nrun + 2u * (uint64_t)p.ngat);
    u32 unit = (u32)((work + 1499u) / 1500u);
    if (unit < 2u) unit = 2u;
    p.PPR = unit;
    p.PPG = unit / 2u;
    p.NCHR = (p.nrun + p.PPR - 1u) / p.PPR;
    p.NCHG = (p.ngat + p.PPG - 1u) / p.PPG;
    p.NCH = p.NCHR + p.NCHG;
    return p;
}

size_t mttkrp_workspace(int n, int R)
{
    MttkrpPlan p = plan(n, R);
    return (size_t)p.NB * p.NCH * 16u * p.Rpad * sizeof(float);
}

st_status launch_mttkrp(const float *Tc, const float *B, float *M, int n, int R, void *ws, hipStream_t s)
{
    MttkrpPlan p = plan(n, R);
    u32 gz = (p.RT + 3u) / 4u;
    if (p.NB > 65535u || gz > 65535u) return ST_ERR_UNSUPPORTED;
    float *part = static_cast<float *>(ws);
    if (R % 4 == 0)
        hipLaunchKernelGGL(mttkrp_mfma_kernel<true>, dim3(p.NCH, p.NB, gz), dim3(NT), 0, s, Tc, B, part, (u32)n,
                           (u32)R, p);
    else
        hipLaunchKernelGGL(mttkrp_mfma_kernel<false>, dim3(p.NCH, p.NB, gz), dim3(NT), 0, s, Tc, B, part, (u32)n,
                           (u32)R, p);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    u32 total = (u32)n * (u32)R;
    hipLaunchKernelGGL(mttkrp_reduce_kernel, dim3((total + 31u) / 32u), dim3(256), 0, s, part, M, (u32)n,
                       (u32)R, p.NCH, p.Rpad);
    return launch_status();
}

}  // namespace st
