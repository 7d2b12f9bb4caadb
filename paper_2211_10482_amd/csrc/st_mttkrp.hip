// MTTKRP with a fully symmetric order-3 tensor and equal factors,
//     M(i,r) = sum_{j,k} T(i,j,k) B(j,r) B(k,r),
// reading only the packed unique entries i<=j<=k.
//
// The index range is cut into blocks of 16, so the packed tensor is a set of
// 16^3 sub-tensors, one per block triple A <= B <= C.  Every contraction below is
// dense and runs on the fp32 matrix cores (v_mfma_f32_16x16x4_f32).  Three kinds
// of work item, each a workgroup of 8 waves with its own branch-free,
// software-pipelined loop over "visits" (one staged sub-tensor each):
//
//   * row items (row block X, a range of block pairs X < P < Q):
//         M(x,r) += 2 * sum_{p,q} T(x,p,q) B(p,r) B(q,r)
//     a [16 x 256] . [256 x R] contraction against Khatri-Rao rows formed on the
//     fly (one VALU multiply per MFMA); the sub-tensor is made of contiguous runs
//     along q -> 16-byte loads, 16-byte LDS writes.
//   * pair items (block pair P < Q, a range of row blocks X < P):
//         U(p,q;r) = sum_X sum_x T(x,p,q) B(x,r)        (accumulated over the visits)
//         M(p,r) += 2 * sum_q B(q,r) U(p,q;r),   M(q,r) += 2 * sum_p B(p,r) U(p,q;r)
//     a [256 x 16] . [16 x R] contraction per visit with plain rows of B as the
//     second operand (no products at all); the two outputs come from ONE
//     accumulator, so a sub-tensor with three different blocks is multiplied
//     twice, not three times, for its three output blocks.
//   * gather items (row block X, the 2*NB-1 block pairs that repeat a block, or
//     every pair when n is not a multiple of 16): owner-computes with a per-element
//     sort + closed-form rank3 gather,
//         M(x,r) += w * sum_{p,q} T(sort(x,p,q)) B(p,r) B(q,r),  w = 2 for P < Q.
//
// No two workgroups add into the same output: each item writes its own partial
// block(s) and a second kernel adds them in a fixed order (deterministic, no
// float atomics).  Staging is double buffered in LDS with the loads of visit v+2
// in flight in registers while visit v is multiplied; one barrier per visit.  In
// the row/gather loops lane = (x, q-quad): one ds_read_b128 of the sub-tensor
// feeds four MFMAs whose K slots are permuted consistently on the B side; in the
// pair loop lane = (q, x-quad) on a transposed staging layout.
//
// Algorithmic traffic: 4 bytes per stored entry (read by two or three items) + B + M.
#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr u32 NT = 512;            // threads per workgroup: 4 column waves x 2 halves
constexpr u32 XS = 260;            // row/gather tile D[x][p][q]: stride between x-planes (16*16 + 4 pad)
constexpr u32 TILE_F = 16 * XS;
constexpr u32 QS = 20;             // pair tile D[p][q][x]: stride between q rows (16 + 4 pad)
constexpr u32 PS = 16 * QS;        //                       stride between p planes
constexpr u32 TILEB_F = 16 * PS;
constexpr u32 BS = 68;             // LDS row stride of a staged 16 x 64 block of B (bank spread)
constexpr u32 BBLK_F = 16 * BS;

struct __attribute__((packed, aligned(4))) f4u { float x, y, z, w; };

__device__ __forceinline__ void sort3u(u32 &a, u32 &b, u32 &c)
{
    u32 lo = min(a, b), hi = max(a, b);
    u32 mn = min(lo, c), mx = max(hi, c), md = max(lo, min(hi, c));
    a = mn; b = md; c = mx;
}

struct MttkrpPlan {
    u32 NB, RT, Rpad;
    u32 all_pairs;          // ragged n: every visit is a gather visit, no row/pair items
    u32 ngat;               // gather visits per row block
    u32 PPR, PPG, PPB;      // visits per row / gather / pair item
    u32 NCHR, NCHG, NCHA;   // row chunks (of row block 0, the longest), gather chunks, NCHA = NCHR + NCHG
    u32 CHB;                // chunk slots per block pair
    u32 nitemsA;            // NB * NCHA row+gather items (unused row slots exit at once)
    u32 npairs_strict;      // block pairs P < Q
};

__host__ __device__ inline u32 strict_pairs(u32 m) { return m >= 2u ? m * (m - 1u) / 2u : 0u; }
__host__ __device__ inline u32 row_chunks(const MttkrpPlan &pl, u32 X)       // row items of row block X
{
    return pl.all_pairs ? 0u : (strict_pairs(pl.NB - 1u - X) + pl.PPR - 1u) / pl.PPR;
}
__host__ __device__ inline u32 pair_chunks(const MttkrpPlan &pl, u32 P)      // pair items of a pair (P, .)
{
    return pl.all_pairs ? 0u : (P + pl.PPB - 1u) / pl.PPB;
}
__host__ __device__ inline u32 pair_index(u32 NB, u32 P, u32 Q)              // P < Q  ->  0 .. C(NB,2)-1
{
    return P * (NB - 1u) - (P * (P - 1u)) / 2u + (Q - 1u - P);
}

// ---- row and gather items ----------------------------------------------------------
struct Visit {
    u32 p0, q0;   // first index of blocks P and Q
    float wgt;    // 2 for P < Q, 1 for P = Q
};

// Cursor over the visits of a row or gather item.  Only the first position is
// unranked; after that the cursor steps (wave-uniform scalar work).
//   row    : u-th strict pair P < Q of the m = NB-1-X blocks above X, kept as (a, b)
//            with a <= b < m-1 in sym2 order: P = X+1+a, Q = X+2+b
//   gather : ragged n -> every pair P <= Q in sym2 order (a, b); otherwise the 2*NB-1
//            pairs with two equal blocks: (g,g) for g < NB, then (g',X) for g' < X,
//            then (X,g'+1)   (a = g)
template <bool GATHER> struct Cursor {
    u32 NB, X, a, b;
    bool all_pairs;

    __device__ __forceinline__ Cursor(u32 NB_, u32 X_, bool all_pairs_, u32 u) : NB(NB_), X(X_), all_pairs(all_pairs_)
    {
        if (!GATHER) unrank_sym2<u32>(NB - 2u - X, u, a, b);
        else if (all_pairs) unrank_sym2<u32>(NB, u, a, b);
        else { a = u; b = 0; }
    }
    __device__ __forceinline__ void step()
    {
        if (!GATHER || all_pairs) {
            const u32 last = (GATHER ? NB : NB - 2u - X) - 1u;
            if (b < last) ++b; else { ++a; b = a; }
        } else {
            ++a;
        }
    }
    __device__ __forceinline__ Visit get() const
    {
        u32 P, Q;
        if (!GATHER) {
            P = X + 1u + a;
            Q = X + 2u + b;
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
        v.p0 = P * 16u; v.q0 = Q * 16u; v.wgt = (P < Q) ? 2.f : 1.f;
        return v;
    }
};

// Global -> registers for one visit: 8 sub-tensor values and one 16-byte piece of
// the two staged blocks of B per thread.  Every load is unconditional (addresses
// clamped) and the results are not touched here, so they stay in flight while
// the previous visit is multiplied; store_visit zeroes what lies outside.
template <bool GATHER, bool R4>
__device__ __forceinline__ void load_visit(const Visit &v, const float *__restrict__ Tc,
                                           const float *__restrict__ B, u32 n, u32 R, u32 x0, u32 rbase,
                                           u32 tid, float (&pf)[8], float (&bb)[4])
{
    if constexpr (!GATHER) {
        // X < P < Q: D[x][p][q] = Tc[run(x, p) + (q0 + q - p)], 16 consecutive q per (x, p)
#pragma unroll
        for (u32 it = 0; it < 2; ++it) {
            const u32 e = tid + NT * it, row = e >> 2, qr = e & 3u;
            const u32 xi = x0 + (row >> 4), pi = v.p0 + (row & 15u);
            f4u t = *reinterpret_cast<const f4u *>(Tc + run_sym3<u32>(n, xi, pi) + (v.q0 - pi) + 4u * qr);
            pf[4 * it] = t.x; pf[4 * it + 1] = t.y; pf[4 * it + 2] = t.z; pf[4 * it + 3] = t.w;
        }
    } else {
#pragma unroll
        for (u32 it = 0; it < 8; ++it) {
            const u32 e = tid + NT * it;
            u32 a = x0 + (e >> 8), b = v.p0 + ((e >> 4) & 15u), c = v.q0 + (e & 15u);
            sort3u(a, b, c);
            pf[it] = Tc[c < n ? rank_sym3<u32>(n, a, b, c) : 0u];
        }
    }
    // piece tid of the two 16 x 64 blocks of B: block tid/256 (P, then Q), row
    // (tid%256)/16, columns rbase + 4*(tid%16) .. +3
    const u32 h = tid >> 8, row = (tid & 255u) >> 4, col = rbase + 4u * (tid & 15u);
    const u32 gr = (h == 0 ? v.p0 : v.q0) + row;
    if constexpr (R4) {   // R % 4 == 0: rows of B are 16-byte aligned
        const bool ok = gr < n && col < R;
        float4 t = *reinterpret_cast<const float4 *>(B + (ok ? (size_t)gr * R + col : 0));
        bb[0] = t.x; bb[1] = t.y; bb[2] = t.z; bb[3] = t.w;
    } else {
#pragma unroll
        for (u32 q = 0; q < 4; ++q) bb[q] = B[(gr < n && col + q < R) ? (size_t)gr * R + col + q : 0];
    }
}

// Registers -> LDS: dense tile D[x][p][q] (x-stride XS) and the two B blocks, the
// P block scaled by the pair weight; positions outside the tensor become zero.
template <bool GATHER>
__device__ __forceinline__ void store_visit(const Visit &v, u32 n, u32 R, u32 x0, u32 rbase,
                                            float *__restrict__ tile, float *__restrict__ bp,
                                            float *__restrict__ bq, u32 tid, const float (&pf)[8],
                                            const float (&bb)[4])
{
    if constexpr (!GATHER) {
#pragma unroll
        for (u32 it = 0; it < 2; ++it) {
            const u32 e = tid + NT * it, row = e >> 2, qr = e & 3u;
            *reinterpret_cast<float4 *>(&tile[(row >> 4) * XS + (row & 15u) * 16u + 4u * qr]) =
                make_float4(pf[4 * it], pf[4 * it + 1], pf[4 * it + 2], pf[4 * it + 3]);
        }
    } else {
#pragma unroll
        for (u32 it = 0; it < 8; ++it) {
            const u32 e = tid + NT * it;
            const u32 x = e >> 8, p = (e >> 4) & 15u, q = e & 15u;
            const bool ok = max(x0 + x, max(v.p0 + p, v.q0 + q)) < n;
            tile[x * XS + p * 16u + q] = ok ? pf[it] : 0.f;
        }
    }
    const u32 h = tid >> 8, row = (tid & 255u) >> 4, col = rbase + 4u * (tid & 15u);
    const bool rok = (h == 0 ? v.p0 : v.q0) + row < n;
    const float w = (h == 0) ? v.wgt : 1.f;
    float *dst = (h == 0 ? bp : bq) + row * BS + 4u * (tid & 15u);
    *reinterpret_cast<float4 *>(dst) =
        make_float4((rok && col + 0u < R) ? w * bb[0] : 0.f, (rok && col + 1u < R) ? w * bb[1] : 0.f,
                    (rok && col + 2u < R) ? w * bb[2] : 0.f, (rok && col + 3u < R) ? w * bb[3] : 0.f);
}

struct LdsRow {
    float tile[2][TILE_F];
    float bp[2][BBLK_F];
    float bq[2][BBLK_F];
};
struct LdsPair {
    float tile[2][TILEB_F];
    float bx[2][BBLK_F];
};
constexpr size_t LDS_BYTES = sizeof(LdsRow) > sizeof(LdsPair) ? sizeof(LdsRow) : sizeof(LdsPair);

// Visits [v0, v1) of a row (GATHER = false) or gather item of row block X.
// Wave (cw, half) accumulates columns 16*cw.. of its half of the p range.
template <bool GATHER, bool R4>
__device__ __forceinline__ void visit_loop(LdsRow &L, const float *__restrict__ Tc,
                                           const float *__restrict__ B, u32 n, u32 R, u32 NB, u32 X,
                                           bool all_pairs, u32 v0, u32 v1, u32 rbase, bool has_rt,
                                           f32x4 (&acc)[4])
{
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 x0 = X * 16u, lrow = lane & 15u, lq = lane >> 4;
    if (v0 >= v1) return;
    const u32 nv = v1 - v0;
    Cursor<GATHER> cur(NB, X, all_pairs, v0);

    float pf[8], bb[4];
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
            const u32 cw = wave & 3u, pbeg = (wave >> 2) * 8u;   // column block, first p
            const float *bqp = &L.bq[cb][(4u * lq) * BS + cw * 16u + lrow];
            const float bq0 = bqp[0], bq1 = bqp[BS], bq2 = bqp[2 * BS], bq3 = bqp[3 * BS];
            const float *bpp = &L.bp[cb][pbeg * BS + cw * 16u + lrow];
            const float *arow = &L.tile[cb][lrow * XS + pbeg * 16u + 4u * lq];
#pragma unroll
            for (u32 p = 0; p < 8; ++p) {
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

// ---- pair items -----------------------------------------------------------------------
// Global -> registers for the visit (X, P, Q), X < P < Q: thread (qr, x, p) takes
// T(x, p, q0 + 4qr .. +3); threads below 256 also take one 16-byte piece of the 16 x 64
// block of B for the rows of X.
template <bool R4>
__device__ __forceinline__ void load_pair_visit(u32 x0, u32 p0, u32 q0, const float *__restrict__ Tc,
                                                const float *__restrict__ B, u32 n, u32 R, u32 rbase, u32 tid,
                                                float (&pf)[8], float (&bb)[4])
{
#pragma unroll
    for (u32 it = 0; it < 2; ++it) {
        const u32 e = tid + NT * it, qr = e & 3u, xi = x0 + ((e >> 2) & 15u), pi = p0 + (e >> 6);
        f4u t = *reinterpret_cast<const f4u *>(Tc + run_sym3<u32>(n, xi, pi) + (q0 - pi) + 4u * qr);
        pf[4 * it] = t.x; pf[4 * it + 1] = t.y; pf[4 * it + 2] = t.z; pf[4 * it + 3] = t.w;
    }
    const u32 row = (tid & 255u) >> 4, col = rbase + 4u * (tid & 15u);
    if constexpr (R4) {
        const bool ok = col < R;
        float4 t = *reinterpret_cast<const float4 *>(B + (ok ? (size_t)(x0 + row) * R + col : 0));
        bb[0] = t.x; bb[1] = t.y; bb[2] = t.z; bb[3] = t.w;
    } else {
#pragma unroll
        for (u32 q = 0; q < 4; ++q) bb[q] = B[(col + q < R) ? (size_t)(x0 + row) * R + col + q : 0];
    }
}

// Registers -> LDS, transposed: D[p][q][x] with x fastest (q-stride QS, p-stride PS).
__device__ __forceinline__ void store_pair_visit(u32 R, u32 rbase, float *__restrict__ tile,
                                                 float *__restrict__ bx, u32 tid, const float (&pf)[8],
                                                 const float (&bb)[4])
{
#pragma unroll
    for (u32 it = 0; it < 2; ++it) {
        const u32 e = tid + NT * it, qr = e & 3u, x = (e >> 2) & 15u, p = e >> 6;
        float *d = &tile[p * PS + (4u * qr) * QS + x];
        d[0] = pf[4 * it]; d[QS] = pf[4 * it + 1]; d[2 * QS] = pf[4 * it + 2]; d[3 * QS] = pf[4 * it + 3];
    }
    if (tid < 256u) {
        const u32 row = tid >> 4, col = rbase + 4u * (tid & 15u);
        *reinterpret_cast<float4 *>(&bx[row * BS + 4u * (tid & 15u)]) =
            make_float4(col + 0u < R ? bb[0] : 0.f, col + 1u < R ? bb[1] : 0.f, col + 2u < R ? bb[2] : 0.f,
                        col + 3u < R ? bb[3] : 0.f);
    }
}

// Pair item (P, Q), row blocks X in [xa, xb): accumulates U(p,q;r) over the visits,
// then writes the two output blocks (rows of P, rows of Q) to out[2][16][Rpad].
template <bool R4>
__device__ __forceinline__ void pair_loop(LdsPair &L, const float *__restrict__ Tc, const float *__restrict__ B,
                                          u32 n, u32 R, u32 P, u32 Q, u32 xa, u32 xb, u32 rbase, u32 rt,
                                          bool has_rt, float *__restrict__ out, u32 Rpad)
{
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 cw = wave & 3u, half = wave >> 2, lrow = lane & 15u, lq = lane >> 4;
    const u32 p0 = P * 16u, q0 = Q * 16u;
    const u32 nv = xb - xa;

    f32x4 acc[8];                                         // U(p = 8*half + j, q = 4*(lane/16) + v; r)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    float pf[8], bb[4];
    load_pair_visit<R4>(xa * 16u, p0, q0, Tc, B, n, R, rbase, tid, pf, bb);
    store_pair_visit(R, rbase, L.tile[0], L.bx[0], tid, pf, bb);
    if (nv > 1) load_pair_visit<R4>((xa + 1u) * 16u, p0, q0, Tc, B, n, R, rbase, tid, pf, bb);
    __syncthreads();

    for (u32 v = 0; v < nv; ++v) {
        const u32 cb = v & 1u;
        if (v + 1 < nv) store_pair_visit(R, rbase, L.tile[cb ^ 1u], L.bx[cb ^ 1u], tid, pf, bb);
        if (v + 2 < nv) load_pair_visit<R4>((xa + v + 2u) * 16u, p0, q0, Tc, B, n, R, rbase, tid, pf, bb);
        __builtin_amdgcn_sched_barrier(0);
        if (has_rt) {
            // lane = (q, x-quad): component t of the 16-byte read is x = 4*(lane/16) + t
            const float *bxp = &L.bx[cb][(4u * lq) * BS + cw * 16u + lrow];
            const float bx0 = bxp[0], bx1 = bxp[BS], bx2 = bxp[2 * BS], bx3 = bxp[3 * BS];
            const float *ap = &L.tile[cb][(half * 8u) * PS + lrow * QS + 4u * lq];
            // two groups of four p: 16 independent MFMAs per group keep the matrix pipe
            // busy with half the operand registers
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                f32x4 a[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) a[j] = *reinterpret_cast<const f32x4 *>(ap + (4 * g + j) * PS);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * g + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][0], bx0, acc[4 * g + j], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * g + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][1], bx1, acc[4 * g + j], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * g + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][2], bx2, acc[4 * g + j], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * g + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][3], bx3, acc[4 * g + j], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    }

    // outputs: rows of P from sums over q, rows of Q from sums over p
    const u32 r = rt * 16u + lrow;
    const bool r_ok = has_rt && r < R;
    float mk[4] = {0.f, 0.f, 0.f, 0.f};
    float mj[8];
    float bqv[4];
#pragma unroll
    for (u32 v = 0; v < 4; ++v) bqv[v] = r_ok ? B[(size_t)(q0 + 4u * lq + v) * R + r] : 0.f;
#pragma unroll
    for (u32 j = 0; j < 8; ++j) {
        const float bpv = r_ok ? B[(size_t)(p0 + half * 8u + j) * R + r] : 0.f;
        float s = 0.f;
#pragma unroll
        for (u32 v = 0; v < 4; ++v) {
            mk[v] += bpv * acc[j][v];
            s += bqv[v] * acc[j][v];
        }
        // add the four q-quads (lanes l, l^16, l^32, l^48); every lane ends with the same sum
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        mj[j] = s;
    }
    // the two halves of the p range meet in LDS for the rows of Q (the loop ended
    // with a barrier, so the tile buffer is free)
    f32x4 *xch = reinterpret_cast<f32x4 *>(&L.tile[0][0]);
    if (half == 1u) xch[cw * 64u + lane] = (f32x4){mk[0], mk[1], mk[2], mk[3]};
    __syncthreads();
    if (has_rt) {
        if (lq == 0u) {
#pragma unroll
            for (u32 j = 0; j < 8; ++j) out[(size_t)(half * 8u + j) * Rpad + rt * 16u + lrow] = 2.f * mj[j];
        }
        if (half == 0u) {
            const f32x4 o = xch[cw * 64u + lane];
            // D layout: lane holds column lane%16 of rows 4*(lane/16) + v
#pragma unroll
            for (u32 v = 0; v < 4; ++v)
                out[(size_t)(16u + 4u * lq + v) * Rpad + rt * 16u + lrow] = 2.f * (mk[v] + o[v]);
        }
    }
}

// ---- the kernel ----------------------------------------------------------------------------
// items [0, nitemsA): row block X = item / NCHA, chunk ch = item % NCHA (ch < NCHR: row
// item, else gather item);  items [nitemsA, ..): block pair (P, Q) and chunk c.
template <bool R4>
__global__ __launch_bounds__(NT) void mttkrp_mfma_kernel(const float *__restrict__ Tc,
                                                       const float *__restrict__ B,
                                                       float *__restrict__ partA, float *__restrict__ partB,
                                                       u32 n, u32 R, MttkrpPlan pl)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds_raw[LDS_BYTES];
    const u32 lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const u32 rbase = blockIdx.y * 64u;                  // this workgroup's 64 columns of R
    const u32 rt = blockIdx.y * 4u + (wave & 3u);        // this wave's block of 16 columns
    const bool has_rt = rt * 16u < R;
    const u32 item = blockIdx.x;

    if (item >= pl.nitemsA) {
        const u32 it = item - pl.nitemsA, pidx = it / pl.CHB, c = it - pidx * pl.CHB;
        u32 P, Qm;
        unrank_sym2<u32>(pl.NB - 1u, pidx, P, Qm);      // inverse of pair_index: (P, Q-1)
        if (c >= pair_chunks(pl, P)) return;
        const u32 xa = c * pl.PPB, xb = min(P, xa + pl.PPB);
        pair_loop<R4>(*reinterpret_cast<LdsPair *>(lds_raw), Tc, B, n, R, P, Qm + 1u, xa, xb, rbase, rt, has_rt,
                      partB + (size_t)it * 32u * pl.Rpad, pl.Rpad);
        return;
    }

    const u32 X = item / pl.NCHA, ch = item - X * pl.NCHA;
    if (ch < pl.NCHR && ch >= row_chunks(pl, X)) return;

    f32x4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    LdsRow &L = *reinterpret_cast<LdsRow *>(lds_raw);
    if (ch < pl.NCHR) {
        const u32 v0 = ch * pl.PPR;
        visit_loop<false, R4>(L, Tc, B, n, R, pl.NB, X, false, v0, min(strict_pairs(pl.NB - 1u - X), v0 + pl.PPR),
                              rbase, has_rt, acc);
    } else {
        const u32 v0 = (ch - pl.NCHR) * pl.PPG;
        visit_loop<true, R4>(L, Tc, B, n, R, pl.NB, X, pl.all_pairs != 0u, v0, min(pl.ngat, v0 + pl.PPG), rbase,
                             has_rt, acc);
    }

    f32x4 sum;
#pragma unroll
    for (u32 v = 0; v < 4; ++v) sum[v] = (acc[0][v] + acc[1][v]) + (acc[2][v] + acc[3][v]);
    // the waves of the upper half of the p range hand their sums to the lower half
    // (the visit loops end with a barrier, so the tile buffer is free)
    f32x4 *xch = reinterpret_cast<f32x4 *>(&L.tile[0][0]);
    if (wave >= 4u) xch[(wave - 4u) * 64u + lane] = sum;
    __syncthreads();
    if (has_rt && wave < 4u) {
        const f32x4 o = xch[wave * 64u + lane];
        // D layout: lane holds column lane%16 of rows 4*(lane/16) + v
        const u32 lrow = lane & 15u, lq = lane >> 4;
        float *dst = partA + ((size_t)item * 16u) * pl.Rpad + rt * 16u + lrow;
#pragma unroll
        for (u32 v = 0; v < 4; ++v) dst[(size_t)(4u * lq + v) * pl.Rpad] = sum[v] + o[v];
    }
}

// M(16X + x, r) = sum of the partial blocks that target row block X, in a fixed
// order: 16 slices per output value -- slices 0..7 the row/gather chunks (ch mod 8),
// slices 8..11 the pair items (X, Q) by Q mod 4, slices 12..15 the pair items
// (P, X) by P mod 4; inside a slice ascending, then slices ascending.
__global__ __launch_bounds__(512) void mttkrp_reduce_kernel(const float *__restrict__ partA,
                                                          const float *__restrict__ partB,
                                                          float *__restrict__ M, u32 n, u32 R, MttkrpPlan pl)
{
    __shared__ float accs[16][32];
    const u32 o = threadIdx.x & 31u, sl = threadIdx.x >> 5;
    const u32 t = blockIdx.x * 32u + o;
    float s = 0.f;
    if (t < n * R) {
        const u32 i = t / R, r = t - i * R, X = i >> 4, x = i & 15u;
        const size_t blk = (size_t)16u * pl.Rpad, off = (size_t)x * pl.Rpad + r;
        if (sl < 8u) {
            const u32 nr = row_chunks(pl, X);
            const float *src = partA + (size_t)X * pl.NCHA * blk + off;
#pragma unroll 4
            for (u32 c = sl; c < nr; c += 8u) s += src[(size_t)c * blk];
#pragma unroll 2
            for (u32 c = sl; c < pl.NCHG; c += 8u) s += src[(size_t)(pl.NCHR + c) * blk];
        } else if (sl < 12u) {
            const u32 nc = pair_chunks(pl, X);
            if (nc > 0u) {
                // pair_index(X, Q) is consecutive in Q
                const float *src = partB + (size_t)pair_index(pl.NB, X, X + 1u) * pl.CHB * 2u * blk + off;
#pragma unroll 2
                for (u32 dq = sl - 8u; X + 1u + dq < pl.NB; dq += 4u)
                    for (u32 c = 0; c < nc; ++c) s += src[((size_t)dq * pl.CHB + c) * 2u * blk];
            }
        } else if (!pl.all_pairs) {
#pragma unroll 2
            for (u32 P = 1u + (sl - 12u); P < X; P += 4u) {
                const u32 nc = pair_chunks(pl, P);
                const float *src = partB + (size_t)pair_index(pl.NB, P, X) * pl.CHB * 2u * blk + blk + off;
                for (u32 c = 0; c < nc; ++c) s += src[(size_t)c * 2u * blk];
            }
        }
    }
    accs[sl][o] = s;
    __syncthreads();
    if (sl == 0 && t < n * R) {
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q) v += accs[q][o];
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
    p.ngat = p.all_pairs ? npairs : 2u * p.NB - 1u;
    p.npairs_strict = p.all_pairs ? 0u : strict_pairs(p.NB);
    // work in visits: row and pair visits of the C(NB,3) sub-tensors with three different
    // blocks, and gather visits (weighted 2: per-element address arithmetic)
    uint64_t triples = p.all_pairs ? 0u : (uint64_t)p.NB * (p.NB - 1u) * (p.NB >= 2u ? p.NB - 2u : 0u) / 6u;
    uint64_t work = 2u * triples + 2u * (uint64_t)p.NB * p.ngat;
    u32 unit = (u32)((work + 1499u) / 1500u);          // about 1500 items in all
    if (unit < 2u) unit = 2u;
    p.PPR = unit;
    p.PPB = unit;
    p.PPG = unit / 2u;
    p.NCHR = p.all_pairs ? 0u : (strict_pairs(p.NB - 1u) + p.PPR - 1u) / p.PPR;
    p.NCHG = (p.ngat + p.PPG - 1u) / p.PPG;
    p.NCHA = p.NCHR + p.NCHG;
    p.CHB = (p.all_pairs || p.NB < 3u) ? 1u : (p.NB - 2u + p.PPB - 1u) / p.PPB;
    p.nitemsA = p.NB * p.NCHA;
    return p;
}

static inline size_t partA_floats(const MttkrpPlan &p) { return (size_t)p.nitemsA * 16u * p.Rpad; }
static inline size_t partB_floats(const MttkrpPlan &p) { return (size_t)p.npairs_strict * p.CHB * 32u * p.Rpad; }

size_t mttkrp_workspace(int n, int R)
{
    MttkrpPlan p = plan(n, R);
    return (partA_floats(p) + partB_floats(p)) * sizeof(float);
}

st_status launch_mttkrp(const float *Tc, const float *B, float *M, int n, int R, void *ws, hipStream_t s)
{
    MttkrpPlan p = plan(n, R);
    u32 gy = (p.RT + 3u) / 4u;
    uint64_t items = (uint64_t)p.nitemsA + (uint64_t)p.npairs_strict * p.CHB;
    if (items > 0x7fffffffull || gy > 65535u) return ST_ERR_UNSUPPORTED;
    float *partA = static_cast<float *>(ws), *partB = partA + partA_floats(p);
    if (R % 4 == 0)
        hipLaunchKernelGGL(mttkrp_mfma_kernel<true>, dim3((u32)items, gy), dim3(NT), 0, s, Tc, B, partA, partB,
                           (u32)n, (u32)R, p);
    else
        hipLaunchKernelGGL(mttkrp_mfma_kernel<false>, dim3((u32)items, gy), dim3(NT), 0, s, Tc, B, partA, partB,
                           (u32)n, (u32)R, p);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    u32 total = (u32)n * (u32)R;
    hipLaunchKernelGGL(mttkrp_reduce_kernel, dim3((total + 31u) / 32u), dim3(512), 0, s, partA, partB, M, (u32)n,
                       (u32)R, p);
    return launch_status();
}

}  // namespace st
