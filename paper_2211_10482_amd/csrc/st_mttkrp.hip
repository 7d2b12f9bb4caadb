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
// to three) owners of its indices.  Per visit the sub-tensor is staged in LDS:
//   * Q above both other blocks : the runs T(a,b,q0..q0+15) are contiguous in
//     packed storage -> 16-byte loads, 16-byte LDS writes;
//   * X above both other blocks : the runs T(p,q,x0..x0+15) are contiguous ->
//     16-byte loads, transposed into the tile by the LDS writes;
//   * any two blocks equal (or a ragged last block): per element sort + closed
//     form rank3 gather.
// The 16 x 64 blocks of B for P (pre-scaled by w) and Q are staged beside it.
// Staging is software pipelined: while visit v is multiplied, visit v+1 sits in
// the second LDS buffer and the loads of visit v+2 are in flight in registers;
// one barrier per visit.  Each of the 4 waves owns 16 columns r: per p one
// ds_read_b128 of D (lane = (x, q-quad); the four components feed four MFMAs
// with consistently permuted K slots and separate accumulators), four VALU
// multiplies for the Khatri-Rao operand, four MFMAs.  Workgroup partials go to
// the workspace; a second kernel adds them in a fixed order.
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

struct __attribute__((packed, aligned(4))) f4u { float x, y, z, w; };

__device__ __forceinline__ void sort3u(u32 &a, u32 &b, u32 &c)
{
    u32 lo = min(a, b), hi = max(a, b);
    u32 mn = min(lo, c), mx = max(hi, c), md = max(lo, min(hi, c));
    a = mn; b = md; c = mx;
}

// One visit = (row block X, block pair P <= Q).  kind: 0 runs along q, 1 runs
// along x (transposed into the tile), 2 per-element gather.
struct Visit {
    u32 p0, q0;
    int kind;
    float wgt;
};

__device__ __forceinline__ Visit decode_visit(u32 NB, u32 pi, u32 X, u32 n)
{
    u32 P, Q;
    unrank_sym2<u32>(NB, pi, P, Q);
    Visit v;
    v.p0 = P * 16u;
    v.q0 = Q * 16u;
    const bool full = max(X, Q) * 16u + 16u <= n;
    v.kind = (full && Q > X && Q > P && X != P) ? 0 : (full && X > Q && Q > P) ? 1 : 2;
    v.wgt = (P < Q) ? 2.f : 1.f;
    return v;
}

// Global -> registers for one visit: 16 tile values and one float4 of each staged
// B block per thread.  All loads are unconditional (addresses clamped) and their
// results are not touched here, so that they stay in flight while the previous
// visit is being multiplied; `mask` records which of them are real (bits 0..15
// tile values, 16..19 P-block, 20..23 Q-block) for store_visit to apply.
__device__ __forceinline__ void load_visit(const Visit &v, const float *__restrict__ Tc,
                                           const float *__restrict__ B, u32 n, u32 R, u32 x0, u32 rbase,
                                           u32 tid, float (&pf)[16], float4 &pb, float4 &qb, u32 &mask)
{
    mask = 0xffffu;
    if (v.kind == 0) {
        // D[x][p][q] = Tc[run(min, max) + (q0 + q - max)], 16 consecutive q per (x, p)
#pragma unroll
        for (u32 it = 0; it < 4; ++it) {
            u32 e = tid + 256u * it, row = e >> 2, qr = e & 3u;
            u32 a = min(x0 + (row >> 4), v.p0 + (row & 15u)), b = max(x0 + (row >> 4), v.p0 + (row & 15u));
            f4u t = *reinterpret_cast<const f4u *>(Tc + run_sym3<u32>(n, a, b) + (v.q0 - b) + 4u * qr);
            pf[4 * it] = t.x; pf[4 * it + 1] = t.y; pf[4 * it + 2] = t.z; pf[4 * it + 3] = t.w;
        }
    } else if (v.kind == 1) {
        // D[x][p][q] = Tc[run(p, q) + (x0 + x - q)], 16 consecutive x per (p, q)
#pragma unroll
        for (u32 it = 0; it < 4; ++it) {
            u32 e = tid + 256u * it, row = e >> 2, xr = e & 3u;
            u32 pp = v.p0 + (row >> 4), qq = v.q0 + (row & 15u);
            f4u t = *reinterpret_cast<const f4u *>(Tc + run_sym3<u32>(n, pp, qq) + (x0 - qq) + 4u * xr);
            pf[4 * it] = t.x; pf[4 * it + 1] = t.y; pf[4 * it + 2] = t.z; pf[4 * it + 3] = t.w;
        }
    } else {
        mask = 0;
#pragma unroll
        for (u32 it = 0; it < 16; ++it) {
            u32 e = tid + 256u * it;
            u32 a = x0 + (e >> 8), b = v.p0 + ((e >> 4) & 15u), c = v.q0 + (e & 15u);
            sort3u(a, b, c);
            const bool ok = c < n;
            pf[it] = Tc[ok ? rank_sym3<u32>(n, a, b, c) : 0u];
            mask |= ok ? (1u << it) : 0u;
        }
    }
    // rows p0 + tid/16 and q0 + tid/16 of B, columns rbase + 4*(tid%16) .. +3
    const u32 row = tid >> 4, col = rbase + 4u * (tid & 15u);
    float e[2][4];
#pragma unroll
    for (u32 h = 0; h < 2; ++h) {
        const u32 gr = (h == 0 ? v.p0 : v.q0) + row;
        if ((R & 3u) == 0) {
            const bool ok = gr < n && col < R;
            float4 t = *reinterpret_cast<const float4 *>(B + (ok ? (size_t)gr * R + col : 0));
            e[h][0] = t.x; e[h][1] = t.y; e[h][2] = t.z; e[h][3] = t.w;
            mask |= ok ? (0xfu << (16u + 4u * h)) : 0u;
        } else {
#pragma unroll
            for (u32 q = 0; q < 4; ++q) {
                const bool ok = gr < n && col + q < R;
                e[h][q] = B[ok ? (size_t)gr * R + col + q : 0];
                mask |= ok ? (1u << (16u + 4u * h + q)) : 0u;
            }
        }
    }
    pb = make_float4(e[0][0], e[0][1], e[0][2], e[0][3]);
    qb = make_float4(e[1][0], e[1][1], e[1][2], e[1][3]);
}

// Registers -> LDS (dense tile D[x][p][q] with x-stride XS, and the two B blocks;
// the P block is pre-scaled by the pair weight).
__device__ __forceinline__ void store_visit(int kind, float wgt, float *__restrict__ tile,
                                            float *__restrict__ bp, float *__restrict__ bq, u32 tid,
                                            const float (&pf)[16], const float4 &pb, const float4 &qb, u32 mask)
{
    if (kind == 0) {
#pragma unroll
        for (u32 it = 0; it < 4; ++it) {
            u32 e = tid + 256u * it, row = e >> 2, qr = e & 3u;
            *reinterpret_cast<float4 *>(&tile[(row >> 4) * XS + (row & 15u) * 16u + 4u * qr]) =
                make_float4(pf[4 * it], pf[4 * it + 1], pf[4 * it + 2], pf[4 * it + 3]);
        }
    } else if (kind == 1) {
#pragma unroll
        for (u32 it = 0; it < 4; ++it) {
            u32 e = tid + 256u * it, row = e >> 2, xr = e & 3u;
            float *d = &tile[(4u * xr) * XS + (row >> 4) * 16u + (row & 15u)];
            d[0] = pf[4 * it]; d[XS] = pf[4 * it + 1]; d[2 * XS] = pf[4 * it + 2]; d[3 * XS] = pf[4 * it + 3];
        }
    } else {
#pragma unroll
        for (u32 it = 0; it < 16; ++it) {
            u32 e = tid + 256u * it;
            tile[(e >> 8) * XS + ((e >> 4) & 15u) * 16u + (e & 15u)] = ((mask >> it) & 1u) ? pf[it] : 0.f;
        }
    }
    const u32 o = (tid >> 4) * BS + 4u * (tid & 15u);
    *reinterpret_cast<float4 *>(&bp[o]) =
        make_float4(((mask >> 16) & 1u) ? wgt * pb.x : 0.f, ((mask >> 17) & 1u) ? wgt * pb.y : 0.f,
                    ((mask >> 18) & 1u) ? wgt * pb.z : 0.f, ((mask >> 19) & 1u) ? wgt * pb.w : 0.f);
    *reinterpret_cast<float4 *>(&bq[o]) =
        make_float4(((mask >> 20) & 1u) ? qb.x : 0.f, ((mask >> 21) & 1u) ? qb.y : 0.f,
                    ((mask >> 22) & 1u) ? qb.z : 0.f, ((mask >> 23) & 1u) ? qb.w : 0.f);
}

__global__ __launch_bounds__(256) void mttkrp_mfma_kernel(const float *__restrict__ Tc,
                                                        const float *__restrict__ B,
                                                        float *__restrict__ part, u32 n, u32 R, u32 NB,
                                                        u32 npairs, u32 PPC, u32 NCH, u32 Rpad)
{
    __shared__ __attribute__((aligned(16))) float tile[2][TILE_F];
    __shared__ __attribute__((aligned(16))) float bpb[2][BBLK_F];
    __shared__ __attribute__((aligned(16))) float bqb[2][BBLK_F];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 X = blockIdx.y, ch = blockIdx.x;
    const u32 rbase = blockIdx.z * 64u;               // this workgroup's 64 columns of R
    const u32 rt = blockIdx.z * 4u + wave;            // this wave's block of 16 columns
    const bool has_rt = rt * 16u < R;
    const u32 x0 = X * 16u;
    const u32 lrow = lane & 15u, lq = lane >> 4;

    f32x4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const u32 pi0 = ch * PPC, pi1 = min(npairs, pi0 + PPC);
    const u32 nv = pi1 - pi0;

    float pf[16];
    float4 pb, qb;
    u32 mask;
    Visit cur = decode_visit(NB, pi0, X, n);
    load_visit(cur, Tc, B, n, R, x0, rbase, tid, pf, pb, qb, mask);
    store_visit(cur.kind, cur.wgt, tile[0], bpb[0], bqb[0], tid, pf, pb, qb, mask);
    Visit nxt = cur;
    if (nv > 1) {
        nxt = decode_visit(NB, pi0 + 1, X, n);
        load_visit(nxt, Tc, B, n, R, x0, rbase, tid, pf, pb, qb, mask);
    }
    __syncthreads();

    for (u32 v = 0; v < nv; ++v) {
        const u32 cb = v & 1u;
        // registers hold visit v+1: park it in the other buffer (its last readers
        // finished before the barrier that ended iteration v-1) ...
        if (v + 1 < nv)
            store_visit(nxt.kind, nxt.wgt, tile[cb ^ 1u], bpb[cb ^ 1u], bqb[cb ^ 1u], tid, pf, pb, qb, mask);
        // ... and put visit v+2 in flight
        if (v + 2 < nv) {
            nxt = decode_visit(NB, pi0 + v + 2, X, n);
            load_visit(nxt, Tc, B, n, R, x0, rbase, tid, pf, pb, qb, mask);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (has_rt) {
            const float *bqp = &bqb[cb][(4u * lq) * BS + wave * 16u + lrow];
            const float bq0 = bqp[0], bq1 = bqp[BS], bq2 = bqp[2 * BS], bq3 = bqp[3 * BS];
            const float *bpp = &bpb[cb][wave * 16u + lrow];
            const float *arow = &tile[cb][lrow * XS + 4u * lq];
#pragma unroll
            for (u32 p = 0; p < 16; ++p) {
                const float bp = bpp[p * BS];
                const f32x4 a = *reinterpret_cast<const f32x4 *>(arow + p * 16u);
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], bp * bq0, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], bp * bq1, acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], bp * bq2, acc[2], 0, 0, 0);
                acc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], bp * bq3, acc[3], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    }

    if (has_rt) {
        // D layout: lane holds column lane%16 of rows 4*(lane/16) + v
        float *dst = part + ((size_t)(X * NCH + ch) * 16u) * Rpad + rt * 16u + lrow;
#pragma unroll
        for (u32 v = 0; v < 4; ++v)
            dst[(size_t)(4u * lq + v) * Rpad] = (acc[0][v] + acc[1][v]) + (acc[2][v] + acc[3][v]);
    }
}

// M(16X + x, r) = sum_ch part[X][ch][x][r], ch ascending.
__global__ __launch_bounds__(256) void mttkrp_reduce_kernel(const float *__restrict__ part,
                                                          float *__restrict__ M, u32 n, u32 R, u32 NCH,
                                                          u32 Rpad)
{
    u32 t = blockIdx.x * 256u + threadIdx.x;
    if (t >= n * R) return;
    u32 i = t / R, r = t - i * R;
    u32 X = i >> 4, x = i & 15u;
    const float *src = part + ((size_t)(X * NCH) * 16u + x) * Rpad + r;
    float s = 0.f;
    for (u32 c = 0; c < NCH; ++c) s += src[(size_t)c * 16u * Rpad];
    M[t] = s;
}

struct MttkrpPlan { u32 NB, npairs, PPC, NCH, RT, Rpad; };

static inline MttkrpPlan plan(int n, int R)
{
    MttkrpPlan p;
    p.NB = ((u32)n + 15u) / 16u;
    p.npairs = p.NB * (p.NB + 1u) / 2u;
    uint64_t visits = (uint64_t)p.NB * p.npairs;
    p.PPC = (u32)((visits + 1535u) / 1536u);   // about 1536 workgroups: two rounds of three per CU
    if (p.PPC < 1u) p.PPC = 1u;
    p.NCH = (p.npairs + p.PPC - 1u) / p.PPC;
    p.RT = ((u32)R + 15u) / 16u;
    p.Rpad = p.RT * 16u;
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
    hipLaunchKernelGGL(mttkrp_mfma_kernel, dim3(p.NCH, p.NB, gz), dim3(256), 0, s, Tc, B, part, (u32)n, (u32)R,
                       p.NB, p.npairs, p.PPC, p.NCH, p.Rpad);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    u32 total = (u32)n * (u32)R;
    hipLaunchKernelGGL(mttkrp_reduce_kernel, dim3((total + 255u) / 256u), dim3(256), 0, s, part, M, (u32)n,
                       (u32)R, p.NCH, p.Rpad);
    return launch_status();
}

}  // namespace st
