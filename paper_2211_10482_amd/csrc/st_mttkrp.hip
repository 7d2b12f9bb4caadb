// MTTKRP with a fully symmetric order-3 tensor and equal factors,
//     M(i,r) = sum_{j,k} T(i,j,k) B(j,r) B(k,r),
// reading only the packed unique entries i<=j<=k.
//
// The index range is cut into blocks of 16, so the packed tensor is a set of
// 16^3 sub-tensors, one per block triple A <= B <= C.  Every contraction below is
// dense and runs on the fp32 matrix cores (v_mfma_f32_16x16x4_f32).  All work is done
// by two kinds of pair item, each a workgroup of
// 8 waves with a branch-free, software-pipelined loop over "visits" (one staged
// 16^3 tile each) that uses plain rows of B as the second MFMA operand (no
// Khatri-Rao products are ever formed):
//
//   * (P,Q) items (block pair P <= Q, a range of row blocks X <= P):
//         U(p,q;r) = sum_X w_X sum_x T(x,p,q) B(x,r)     (accumulated over the visits)
//         M(p,r) += 2 * sum_q B(q,r) U(p,q;r),   M(q,r) += 2 * sum_p B(p,r) U(p,q;r)
//     two output blocks from ONE accumulator (P = Q: one, the two are the same);
//   * (X,P) items (block pair X <= P, a range of blocks Q >= P):
//         V(x,p;r) = sum_Q w_Q sum_q T(x,p,q) B(q,r),    M(x,r) += 2 * sum_p B(p,r) V(x,p;r)
//     consecutive visits read consecutive 64-byte runs.
//
// A block triple X < P < Q is visited once by each kind (weight 1), which gives its
// three output blocks from two contractions.  Triples that repeat a block use the
// symmetry of the tile instead of a gather: the staged tile is completed from the
// stored half (canonical min/max addressing, or a mirrored LDS write when the
// stored runs are ragged), and the visits X = P, Q = P and all visits of an (X,X)
// item carry weight 1/2, so that every ordered pair (j,k) of
// M(i,r) = sum_{j,k} T(i,j,k) B(j,r) B(k,r) is counted exactly once:
//     {A,A,C}: M[A] from item (P=A,Q=C) visit X=A (1/2) and item (X=A,P=A) visit Q=C (1/2),
//              M[C] from item (P=A,Q=C) visit X=A (1/2);
//     {A,C,C}: M[C] from item (P=C,Q=C) visit X=A,  M[A] from item (X=A,P=C) visit Q=C (1/2);
//     {A,A,A}: item (X=A,P=A) visit Q=A (1/2), the only tile that needs a per-element sort.
//
// When n is not a multiple of 16 the packed tensor is first copied into the packed layout of the
// next multiple, zeros for every entry with an index >= n (mttkrp_repack_kernel), and the pair items
// run on the copy.
//
// Both pair kinds run the same [256 x 16] . [16 x R] MFMA loop on a staged tile
// D[i1][i2][k] (k fastest): (P,Q) items stage it transposed (i1 = p, i2 = q, k = x),
// (X,P) items as it lies in memory (i1 = x, i2 = p, k = q; 16-byte LDS writes).
//
// No two workgroups add into the same output: each item writes its own partial
// block(s) and a second kernel adds them in a fixed order (deterministic, no
// float atomics).  Staging is double buffered in LDS with the loads of visit v+2
// in flight in registers while visit v is multiplied; one barrier per visit.  One
// ds_read_b128 of the tile feeds four MFMAs whose K slots are permuted
// consistently on the B side.
//
// Small tensors (n <= 96, R <= 32) skip all of this: one launch, one workgroup per
// output row, on the vector ALUs (mttkrp_rows_kernel, near the end of this file).
//
// Algorithmic traffic: 4 bytes per stored entry (read by two or three items) + B + M.
#include "st_common.h"
#include "st_index.h"

namespace st {

typedef uint32_t u32;
typedef float f32x4 __attribute__((ext_vector_type(4)));

#ifndef ST_MTTKRP_WPE
#define ST_MTTKRP_WPE 4
#endif
#ifndef ST_MTTKRP_ITEMS
#define ST_MTTKRP_ITEMS 350u
#endif
constexpr u32 NT = 512;            // threads per workgroup: 4 column waves x 2 halves
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
    u32 PPB;                // visits per pair item
    u32 CHB;                // chunk slots per block pair (either pair kind)
    u32 npairs;             // block pairs P <= Q
};

// visits of a (P,Q) item: row blocks X <= P (P = Q: X < P, the tile of three equal
// blocks belongs to the (X,P) kind); of an (X,P) item: blocks Q >= P
__host__ __device__ inline u32 visits_pq(u32 P, u32 Q) { return P < Q ? P + 1u : P; }
__host__ __device__ inline u32 visits_xp(u32 NB, u32 P) { return NB - P; }
__host__ __device__ inline u32 chunks_of(const MttkrpPlan &pl, u32 visits) { return (visits + pl.PPB - 1u) / pl.PPB; }

struct LdsPair {
    float tile[2][TILEB_F];
    float bk[2][BBLK_F];
};

// ---- pair items -----------------------------------------------------------------------
// The staged tile is D[i1][i2][k] with k fastest (i2-stride QS, i1-stride PS); block b1
// supplies i1, block b2 supplies i2 and the visit supplies the block of k:
//   KIND 0: item (P, Q), visits X <= P:  i1 = p, i2 = q, k = x
//   KIND 1: item (X, P), visits Q >= P:  i1 = x, i2 = p, k = q
// Global -> registers for one visit: thread (qr, ., .) takes the four values
// T(min(x,p), max(x,p), q0 + 4qr .. +3) of one stored run (x and p only meet in the same
// block when X = P, where the tile is symmetric in them); threads below 256 also take
// one 16-byte piece of the 16 x 64 block of B for the rows of the k block.  Where the q
// block equals the p block the values with q < p are not part of the run (they are
// whatever precedes it in memory, p >= 16 there) and store_pair_visit<MIRROR> drops them.
template <int KIND, bool R4>
__device__ __forceinline__ void load_pair_visit(u32 b1_0, u32 b2_0, u32 k0, const float *__restrict__ Tc,
                                                const float *__restrict__ B, u32 n, u32 R, u32 rbase, u32 tid,
                                                float (&pf)[8], float (&bb)[4])
{
#pragma unroll
    for (u32 it = 0; it < 2; ++it) {
        const u32 e = tid + NT * it, qr = e & 3u, mid = (e >> 2) & 15u, hi = e >> 6;
        const u32 x = (KIND == 0) ? k0 + mid : b1_0 + hi;
        const u32 pp = (KIND == 0) ? b1_0 + hi : b2_0 + mid;
        const u32 q0 = (KIND == 0) ? b2_0 : k0;
        const u32 lo = min(x, pp), up = max(x, pp);
        // one 32-bit sum: q0 - up is negative (wraps) where the q block is the p block
        const u32 pos = run_sym3<u32>(n, lo, up) + (q0 - up) + 4u * qr;
        f4u t = *reinterpret_cast<const f4u *>(Tc + pos);
        pf[4 * it] = t.x; pf[4 * it + 1] = t.y; pf[4 * it + 2] = t.z; pf[4 * it + 3] = t.w;
    }
    const u32 row = (tid & 255u) >> 4, col = rbase + 4u * (tid & 15u);
    if constexpr (R4) {
        const bool ok = col < R;
        float4 t = *reinterpret_cast<const float4 *>(B + (ok ? (size_t)(k0 + row) * R + col : 0));
        bb[0] = t.x; bb[1] = t.y; bb[2] = t.z; bb[3] = t.w;
    } else {
#pragma unroll
        for (u32 q = 0; q < 4; ++q) bb[q] = B[(col + q < R) ? (size_t)(k0 + row) * R + col + q : 0];
    }
}

// The tile of three equal blocks (item (X,X), visit Q = X): one sorted gather per value.
template <bool R4>
__device__ __forceinline__ void load_diag_visit(u32 b0, const float *__restrict__ Tc, const float *__restrict__ B,
                                                u32 n, u32 R, u32 rbase, u32 tid, float (&pf)[8], float (&bb)[4])
{
#pragma unroll
    for (u32 it = 0; it < 2; ++it) {
        const u32 e = tid + NT * it, qr = e & 3u, mid = (e >> 2) & 15u, hi = e >> 6;
#pragma unroll
        for (u32 t = 0; t < 4; ++t) {
            u32 a = b0 + hi, b = b0 + mid, c = b0 + 4u * qr + t;
            sort3u(a, b, c);
            pf[4 * it + t] = Tc[rank_sym3<u32>(n, a, b, c)];
        }
    }
    const u32 row = (tid & 255u) >> 4, col = rbase + 4u * (tid & 15u);
    if constexpr (R4) {
        const bool ok = col < R;
        float4 t = *reinterpret_cast<const float4 *>(B + (ok ? (size_t)(b0 + row) * R + col : 0));
        bb[0] = t.x; bb[1] = t.y; bb[2] = t.z; bb[3] = t.w;
    } else {
#pragma unroll
        for (u32 q = 0; q < 4; ++q) bb[q] = B[(col + q < R) ? (size_t)(b0 + row) * R + col + q : 0];
    }
}

// Registers -> LDS, the block of B scaled by the weight w of the visit.  KIND 0
// transposes (the loaded run lies along i2), KIND 1 keeps the run as one 16-byte write
// along k.  MIRROR (the q block is the p block): the loaded values with q >= p are
// written to (p, q) and to (q, p), the others dropped.
template <int KIND, bool MIRROR>
__device__ __forceinline__ void store_pair_visit(u32 R, u32 rbase, float w, float *__restrict__ tile,
                                                 float *__restrict__ bk, u32 tid, const float (&pf)[8],
                                                 const float (&bb)[4])
{
#pragma unroll
    for (u32 it = 0; it < 2; ++it) {
        const u32 e = tid + NT * it, qr = e & 3u, mid = (e >> 2) & 15u, hi = e >> 6;
        if constexpr (!MIRROR) {
            if constexpr (KIND == 0) {
                float *d = &tile[hi * PS + (4u * qr) * QS + mid];
                d[0] = pf[4 * it]; d[QS] = pf[4 * it + 1]; d[2 * QS] = pf[4 * it + 2]; d[3 * QS] = pf[4 * it + 3];
            } else {
                *reinterpret_cast<float4 *>(&tile[hi * PS + mid * QS + 4u * qr]) =
                    make_float4(pf[4 * it], pf[4 * it + 1], pf[4 * it + 2], pf[4 * it + 3]);
            }
        } else {
            // KIND 0: (p, q, x) = (hi, 4qr+t, mid) at [p][q][x];  KIND 1: (x, p, q) = (hi, mid, 4qr+t) at [x][p][q]
            const u32 pl = (KIND == 0) ? hi : mid;
#pragma unroll
            for (u32 t = 0; t < 4; ++t) {
                const u32 ql = 4u * qr + t;
                const float v = pf[4 * it + t];
                if constexpr (KIND == 0) {
                    if (ql >= pl) tile[pl * PS + ql * QS + mid] = v;
                    if (ql > pl) tile[ql * PS + pl * QS + mid] = v;
                } else {
                    if (ql >= pl) tile[hi * PS + pl * QS + ql] = v;
                    if (ql > pl) tile[hi * PS + ql * QS + pl] = v;
                }
            }
        }
    }
    if (tid < 256u) {
        const u32 row = tid >> 4, col = rbase + 4u * (tid & 15u);
        *reinterpret_cast<float4 *>(&bk[row * BS + 4u * (tid & 15u)]) =
            make_float4(col + 0u < R ? w * bb[0] : 0.f, col + 1u < R ? w * bb[1] : 0.f,
                        col + 2u < R ? w * bb[2] : 0.f, col + 3u < R ? w * bb[3] : 0.f);
    }
}

// Weight of the visit with k block kb (see the table at the top of the file).
template <int KIND> __device__ __forceinline__ float visit_weight(u32 b1, u32 b2, u32 kb)
{
    if (KIND == 0) return (kb == b1 && b1 != b2) ? 0.5f : 1.f;
    return (b1 == b2 || kb == b2) ? 0.5f : 1.f;
}

// Pair item of blocks (b1, b2), k blocks [va, vb): accumulates U(i1,i2;r) over the
// visits, then writes the rows of b1 (sums over i2) to out[0][16][Rpad] and, for
// KIND 0 with b1 < b2, the rows of b2 (sums over i1) to out[1][16][Rpad].
// SYM: a (P,P) item, every tile is completed by mirroring.
template <int KIND, bool SYM, bool R4>
__device__ __forceinline__ void pair_loop(LdsPair &L, const float *__restrict__ Tc, const float *__restrict__ B,
                                          u32 n, u32 R, u32 b1, u32 b2, u32 va, u32 vb, u32 rbase, u32 rt,
                                          bool has_rt, float *__restrict__ out, u32 Rpad)
{
    static_assert(!(SYM && KIND == 1), "only (P,P) items mirror every visit");
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 cw = wave & 3u, half = wave >> 2, lrow = lane & 15u, lq = lane >> 4;
    const u32 b1_0 = b1 * 16u, b2_0 = b2 * 16u;
    const u32 nv = vb - va;

    f32x4 acc[8];                                         // U(i1 = 8*half + j, i2 = 4*(lane/16) + v; r)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    float pf[8], bb[4];
    // first visit: for an (X,P) item that starts at Q = P the q block is the p block
    if (KIND == 1 && va == b2) {
        if (b1 == b2) {
            load_diag_visit<R4>(b1_0, Tc, B, n, R, rbase, tid, pf, bb);
            store_pair_visit<KIND, false>(R, rbase, 0.5f, L.tile[0], L.bk[0], tid, pf, bb);
        } else {
            load_pair_visit<KIND, R4>(b1_0, b2_0, va * 16u, Tc, B, n, R, rbase, tid, pf, bb);
            store_pair_visit<KIND, true>(R, rbase, 0.5f, L.tile[0], L.bk[0], tid, pf, bb);
        }
    } else {
        load_pair_visit<KIND, R4>(b1_0, b2_0, va * 16u, Tc, B, n, R, rbase, tid, pf, bb);
        store_pair_visit<KIND, SYM>(R, rbase, visit_weight<KIND>(b1, b2, va), L.tile[0], L.bk[0], tid, pf, bb);
    }
    if (nv > 1) load_pair_visit<KIND, R4>(b1_0, b2_0, (va + 1u) * 16u, Tc, B, n, R, rbase, tid, pf, bb);
    __syncthreads();

    for (u32 v = 0; v < nv; ++v) {
        const u32 cb = v & 1u;
        // The MFMAs of visit v are issued first: they run on the matrix pipe while this
        // wave waits for the loads of visit v+1, parks them in the other buffer (its last
        // readers finished before the barrier that ended iteration v-1) and puts visit
        // v+2 in flight.
        if (has_rt) {
            // lane = (i2, k-quad): component t of the 16-byte read is k = 4*(lane/16) + t
            const float *bkp = &L.bk[cb][(4u * lq) * BS + cw * 16u + lrow];
            const float bk0 = bkp[0], bk1 = bkp[BS], bk2 = bkp[2 * BS], bk3 = bkp[3 * BS];
            const float *ap = &L.tile[cb][(half * 8u) * PS + lrow * QS + 4u * lq];
            // two groups of four i1: 16 independent MFMAs per group keep the matrix pipe
            // busy with half the operand registers
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                f32x4 a[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) a[j] = *reinterpret_cast<const f32x4 *>(ap + (4 * g + j) * PS);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * g + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][0], bk0, acc[4 * g + j], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * g + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][1], bk1, acc[4 * g + j], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * g + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][2], bk2, acc[4 * g + j], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * g + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][3], bk3, acc[4 * g + j], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (v + 1 < nv)
            store_pair_visit<KIND, SYM>(R, rbase, visit_weight<KIND>(b1, b2, va + v + 1u), L.tile[cb ^ 1u],
                                        L.bk[cb ^ 1u], tid, pf, bb);
        if (v + 2 < nv) load_pair_visit<KIND, R4>(b1_0, b2_0, (va + v + 2u) * 16u, Tc, B, n, R, rbase, tid, pf, bb);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    }

    // outputs: rows of b1 from sums over i2, rows of b2 from sums over i1
    constexpr bool TWO = (KIND == 0) && !SYM;
    const u32 r = rt * 16u + lrow;
    const bool r_ok = has_rt && r < R;
    float mk[4] = {0.f, 0.f, 0.f, 0.f};
    float mj[8];
    float b2v[4];
#pragma unroll
    for (u32 v = 0; v < 4; ++v) b2v[v] = r_ok ? B[(size_t)(b2_0 + 4u * lq + v) * R + r] : 0.f;
#pragma unroll
    for (u32 j = 0; j < 8; ++j) {
        float s = 0.f;
        if constexpr (TWO) {
            const float b1v = r_ok ? B[(size_t)(b1_0 + half * 8u + j) * R + r] : 0.f;
#pragma unroll
            for (u32 v = 0; v < 4; ++v) mk[v] += b1v * acc[j][v];
        }
#pragma unroll
        for (u32 v = 0; v < 4; ++v) s += b2v[v] * acc[j][v];
        // add the four i2-quads (lanes l, l^16, l^32, l^48); every lane ends with the same sum
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        mj[j] = s;
    }
    if (has_rt && lq == 0u) {
#pragma unroll
        for (u32 j = 0; j < 8; ++j) out[(size_t)(half * 8u + j) * Rpad + rt * 16u + lrow] = 2.f * mj[j];
    }
    if constexpr (TWO) {
        // the two halves of the i1 range meet in LDS for the rows of b2 (the loop ended
        // with a barrier, so the tile buffer is free)
        f32x4 *xch = reinterpret_cast<f32x4 *>(&L.tile[0][0]);
        if (half == 1u) xch[cw * 64u + lane] = (f32x4){mk[0], mk[1], mk[2], mk[3]};
        __syncthreads();
        if (has_rt && half == 0u) {
            const f32x4 o = xch[cw * 64u + lane];
            // D layout: lane holds column lane%16 of rows 4*(lane/16) + v
#pragma unroll
            for (u32 v = 0; v < 4; ++v)
                out[(size_t)(16u + 4u * lq + v) * Rpad + rt * 16u + lrow] = 2.f * (mk[v] + o[v]);
        }
    }
}

// ---- the kernels --------------------------------------------------------------------------
// n a multiple of 16: 2*npairs*CHB pair items (block pair and chunk slot; slots beyond
// the pair's own number of chunks exit at once).
template <bool R4>
__global__ __launch_bounds__(NT, ST_MTTKRP_WPE) void mttkrp_pair_kernel(const float *__restrict__ Tc,
                                                       const float *__restrict__ B,
                                                       float *__restrict__ partPQ, float *__restrict__ partXP,
                                                       u32 n, u32 R, MttkrpPlan pl)
{
    __shared__ __attribute__((aligned(16))) LdsPair L;
    const u32 wave = threadIdx.x >> 6;
    const u32 rbase = blockIdx.y * 64u;                  // this workgroup's 64 columns of R
    const u32 rt = blockIdx.y * 4u + (wave & 3u);        // this wave's block of 16 columns
    const bool has_rt = rt * 16u < R;

    // Launch order: pair after pair, longest pairs first ((P,Q) items have about P visits
    // per pair, (X,P) items NB-P), the 2*CHB slots of a pair (kind, chunk) next to each
    // other, so that the long items start early.  Workgroups go to the XCDs round-robin
    // by index: the slots of a pair are rotated by a hash of the pair, or the empty
    // slots of the short pairs would all land on the same XCDs.
    const u32 g = 2u * pl.CHB;
    const u32 kp = blockIdx.x / g, pos = blockIdx.x - kp * g;
    const u32 slot = (pos + ((kp * 0x9E3779B1u) >> 16)) % g;
    const bool xp = (slot & 1u) != 0u;
    const u32 c = slot >> 1;
    // (P,Q) and (P,Q-1) read the two halves of the same 128-byte lines: with one slot
    // pair per block pair they are placed 8 workgroups apart, i.e. on the same XCD (same
    // L2) at about the same time.
    u32 kq = kp;
    if (!xp && g == 2u && (kp | 7u) < pl.npairs) kq = (kp & ~7u) + 2u * (kp & 3u) + ((kp >> 2) & 1u);
    u32 a, b;
    unrank_sym2<u32>(pl.NB, pl.npairs - 1u - kq, a, b);          // a <= b, a descending
    if (!xp) {
        const u32 P = a, Q = b, nvis = visits_pq(P, Q);
        const u32 nc = chunks_of(pl, nvis);
        if (c >= nc) return;
        const u32 va = c * nvis / nc, vb = (c + 1u) * nvis / nc;                  // row blocks X, even chunks
        float *out = partPQ + ((size_t)rank_sym2<u32>(pl.NB, P, Q) * pl.CHB + c) * 32u * pl.Rpad;
        if (P < Q) pair_loop<0, false, R4>(L, Tc, B, n, R, P, Q, va, vb, rbase, rt, has_rt, out, pl.Rpad);
        else pair_loop<0, true, R4>(L, Tc, B, n, R, P, Q, va, vb, rbase, rt, has_rt, out, pl.Rpad);
    } else {
        const u32 X = pl.NB - 1u - b, P = pl.NB - 1u - a;         // mirrored: X <= P, P ascending
        const u32 nvis = visits_xp(pl.NB, P), nc = chunks_of(pl, nvis);
        if (c >= nc) return;
        const u32 va = P + c * nvis / nc, vb = P + (c + 1u) * nvis / nc;          // blocks Q, even chunks
        float *out = partXP + ((size_t)rank_sym2<u32>(pl.NB, X, P) * pl.CHB + c) * 16u * pl.Rpad;
        pair_loop<1, false, R4>(L, Tc, B, n, R, X, P, va, vb, rbase, rt, has_rt, out, pl.Rpad);
    }
}

// M(16X + x, r) = sum of the partial blocks that target row block X, in a fixed
// order: 16 slices per output value: slices 0..5 the (X,P) items by P mod 6, slices 6..10 the (X,Q) items of
// kind (P,Q) by Q mod 5 (first output block), slices 11..15 the (P,X) items by
// P mod 5 (second output block); inside a slice ascending, then slices ascending.
__global__ __launch_bounds__(512) void mttkrp_reduce_kernel(const float *__restrict__ partPQ,
                                                          const float *__restrict__ partXP,
                                                          float *__restrict__ M, u32 n, u32 R, MttkrpPlan pl)
{
    __shared__ float accs[16][32];
    const u32 o = threadIdx.x & 31u, sl = threadIdx.x >> 5;
    const u32 t = blockIdx.x * 32u + o;
    float s = 0.f;
    if (t < n * R) {
        const u32 i = t / R, r = t - i * R, X = i >> 4, x = i & 15u;
        const size_t blk = (size_t)16u * pl.Rpad, off = (size_t)x * pl.Rpad + r;
        if (sl < 6u) {
            // rank_sym2(X, P) is consecutive in P
            const float *src = partXP + (size_t)rank_sym2<u32>(pl.NB, X, X) * pl.CHB * blk + off;
#pragma unroll 2
            for (u32 dp = sl; X + dp < pl.NB; dp += 6u) {
                const u32 nc = chunks_of(pl, visits_xp(pl.NB, X + dp));
                for (u32 c = 0; c < nc; ++c) s += src[((size_t)dp * pl.CHB + c) * blk];
            }
        } else if (sl < 11u) {
            const float *src = partPQ + (size_t)rank_sym2<u32>(pl.NB, X, X) * pl.CHB * 2u * blk + off;
#pragma unroll 2
            for (u32 dq = sl - 6u; X + dq < pl.NB; dq += 5u) {
                const u32 nc = chunks_of(pl, visits_pq(X, X + dq));
                for (u32 c = 0; c < nc; ++c) s += src[((size_t)dq * pl.CHB + c) * 2u * blk];
            }
        } else {
#pragma unroll 2
            for (u32 P = sl - 11u; P < X; P += 5u) {
                const u32 nc = chunks_of(pl, visits_pq(P, X));
                const float *src = partPQ + (size_t)rank_sym2<u32>(pl.NB, P, X) * pl.CHB * 2u * blk + blk + off;
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
    p.npairs = p.NB * (p.NB + 1u) / 2u;
    // work in visits: every block triple X <= P <= Q is visited twice (once by each pair kind; the
    // triples that repeat a block split differently but add up to the same)
    const uint64_t work = (uint64_t)p.NB * (p.NB + 1u) * (p.NB + 2u) / 3u;
    u32 unit = (u32)((work + (ST_MTTKRP_ITEMS - 1u)) / ST_MTTKRP_ITEMS);   // about that many items in all
    if (unit < 2u) unit = 2u;
    p.PPB = unit;
    p.CHB = (p.NB + p.PPB - 1u) / p.PPB;                  // the longest item has NB visits
    return p;
}

static inline size_t partPQ_floats(const MttkrpPlan &p) { return (size_t)p.npairs * p.CHB * 32u * p.Rpad; }
static inline size_t partXP_floats(const MttkrpPlan &p) { return (size_t)p.npairs * p.CHB * 16u * p.Rpad; }


// ---- small tensors: one workgroup per output row, one launch ------------------------------------
// When the whole packed tensor is a few hundred KB (n <= 96) the two-kernel item scheme above is all
// launch and pipeline start-up.  Here (R <= 32) a workgroup owns output row i and evaluates
//     M(i,r) = sum_{j<=k} w(j,k) T(sort(i,j,k)) B(j,r) B(k,r),   w = 1 for j = k, 2 otherwise,
// on the vector ALUs.  A wave takes the rows j = wave, wave+16, ... and its lanes the columns k = j + lane:
// every lane first gathers its (at most 12) weighted entries through rank3 of the sorted triple, all loads
// in flight together, while B is copied to LDS (rows padded to RC+4 floats: conflict-free 16-byte reads of
// different rows); it keeps RC accumulators, which are added over the sixteen waves through LDS and over
// the lanes with one DPP tree per output value, in a fixed order.  Each entry is read by the (up to three)
// rows it belongs to; at this size those re-reads come from the cache.
constexpr u32 ROWS_NMAX = 96;      // largest n of the row kernel
constexpr u32 ROWS_NT = 1024;      // threads per workgroup of the row kernel
constexpr u32 ROWS_NW = ROWS_NT / 64;
constexpr u32 ROWS_SLOTS = ((ROWS_NMAX + ROWS_NW - 1) / ROWS_NW) * ((ROWS_NMAX + 63) / 64);   // (j, k chunk) per wave: 12
template <int RC>                  // accumulators per lane: R rounded up to 16 or 32
__global__ __launch_bounds__(ROWS_NT) void mttkrp_rows_kernel(const float *__restrict__ Tc, const float *__restrict__ B,
                                                         float *__restrict__ M, u32 n, u32 R)
{
    constexpr u32 LS = RC + 4;                      // LDS row stride of B
    __shared__ __attribute__((aligned(16))) float Bs[ROWS_NMAX * LS];
    __shared__ float red[ROWS_NW][16][64];          // [wave][accumulator][lane]
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6, i = blockIdx.x;
    // A wave takes the rows j = wave, wave+16, ... and its lanes the columns k = j + lane (+64): slot q of
    // a lane is one weighted entry w T(sort(i,j,k)), gathered through rank3 of the sorted triple.  All
    // loads of a lane are issued before anything else (addresses clamped, results masked).
    const u32 kchunks = (n + 63u) / 64u;
    float tv[ROWS_SLOTS];
    u32 kk[ROWS_SLOTS];
#pragma unroll
    for (u32 q = 0; q < ROWS_SLOTS; ++q) {
        const u32 jq = wave + ROWS_NW * (q / 2u), k = jq + 64u * (q & 1u) + lane;
        const bool in = (q & 1u) < kchunks && jq < n && k < n;
        u32 a = i, b = in ? jq : i, c = in ? k : i;
        sort3u(a, b, c);
        const float t = Tc[rank_sym3<u32>(n, a, b, c)];
        tv[q] = in ? (k == jq ? t : 2.f * t) : 0.f;
        kk[q] = in ? k : 0u;
    }
    for (u32 e = tid; e < n * RC; e += ROWS_NT) {
        const u32 row = e / RC, r = e - row * RC;
        Bs[row * LS + r] = r < R ? B[(size_t)row * R + r] : 0.f;
    }
    __syncthreads();
    float acc[RC];
#pragma unroll
    for (int r = 0; r < RC; ++r) acc[r] = 0.f;
#pragma unroll
    for (u32 q = 0; q < ROWS_SLOTS; ++q) {
        const u32 jq = wave + ROWS_NW * (q / 2u);
        if (jq >= n || (q & 1u) >= kchunks) continue;           // wave-uniform
        const float *bj = &Bs[jq * LS];                         // wave-uniform: broadcast reads
        const float *bk = &Bs[kk[q] * LS];
        const float t = tv[q];
#pragma unroll
        for (int c = 0; c < RC / 4; ++c) {
            const float4 v = *reinterpret_cast<const float4 *>(bk + 4 * c);
            const float4 u = *reinterpret_cast<const float4 *>(bj + 4 * c);
            acc[4 * c] += t * u.x * v.x;
            acc[4 * c + 1] += t * u.y * v.y;
            acc[4 * c + 2] += t * u.z * v.z;
            acc[4 * c + 3] += t * u.w * v.w;
        }
    }
    // M(i,r) = sum over waves and lanes, 16 accumulators at a time: every lane parks its values in LDS, then
    // wave r adds accumulator r of all waves lane by lane (waves ascending) and over its 64 lanes (DPP tree)
#pragma unroll
    for (int h = 0; h < RC / 16; ++h) {
        if (h > 0) __syncthreads();
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave][r][lane] = acc[16 * h + r];
        __syncthreads();
        float v = 0.f;
#pragma unroll
        for (u32 w = 0; w < ROWS_NW; ++w) v += red[w][wave][lane];
        v = wave_sum(v);
        const u32 r = 16u * (u32)h + wave;
        if (lane == 0 && r < R) M[(size_t)i * R + r] = v;
    }
}

// ---- n not a multiple of 16: repack into the next multiple -------------------------------------
// The pair items need whole 16^3 tiles.  For other n the packed tensor is copied once into the packed
// layout of np = 16*ceil(n/16) with zeros for every entry that has an index >= n (one wave per run
// (i,j): both layouts store the run k = j.. contiguously), B gets zero rows, and the pair items run on
// the copy; rows >= n of the result are never written.  One extra read and write of the tensor (about
// 0.5x the time of the contraction itself) instead of per-element gathers in the inner loop.
__global__ __launch_bounds__(256) void mttkrp_repack_kernel(const float *__restrict__ Tc, const float *__restrict__ B,
                                                           float *__restrict__ Tp, float *__restrict__ Bp, u32 n,
                                                           u32 np, u32 R, u32 nruns)
{
    const u32 run = blockIdx.x * 4u + (threadIdx.x >> 6), lane = threadIdx.x & 63u;
    if (run < nruns) {
        u32 i, j;
        unrank_sym2<u32>(np, run, i, j);
        float *dst = Tp + rank_sym3<u32>(np, i, j, j);
        const bool live = j < n;                                  // i <= j
        const float *src = Tc + (live ? rank_sym3<u32>(n, i, j, j) : 0u);
        for (u32 q = lane; q < np - j; q += 64u) dst[q] = (live && j + q < n) ? src[q] : 0.f;
    }
    // the first blocks also copy B (n x R) into np x R
    const u32 e = blockIdx.x * 256u + threadIdx.x;
    if (e < np * R) Bp[e] = e < n * R ? B[e] : 0.f;
}

static inline bool use_rows(int n, int R) { return (u32)n <= ROWS_NMAX && R <= 32; }
static inline u32 pad16(int n) { return ((u32)n + 15u) & ~15u; }

size_t mttkrp_workspace(int n, int R)
{
    if (use_rows(n, R)) return 0;
    const u32 np = pad16(n);
    MttkrpPlan p = plan((int)np, R);
    size_t floats = partPQ_floats(p) + partXP_floats(p);
    if (np != (u32)n) floats += (size_t)count_sym3<int64_t>(np) + (size_t)np * R;   // repacked tensor and factor
    return floats * sizeof(float);
}

st_status launch_mttkrp(const float *Tc, const float *B, float *M, int n, int R, void *ws, hipStream_t s)
{
    if (use_rows(n, R)) {
        if (R <= 16) hipLaunchKernelGGL(mttkrp_rows_kernel<16>, dim3((u32)n), dim3(ROWS_NT), 0, s, Tc, B, M, (u32)n, (u32)R);
        else hipLaunchKernelGGL(mttkrp_rows_kernel<32>, dim3((u32)n), dim3(ROWS_NT), 0, s, Tc, B, M, (u32)n, (u32)R);
        return launch_status();
    }
    const u32 np = pad16(n);
    MttkrpPlan p = plan((int)np, R);
    u32 gy = (p.RT + 3u) / 4u;
    uint64_t items = 2u * (uint64_t)p.npairs * p.CHB;
    if (items > 0x7fffffffull || gy > 65535u) return ST_ERR_UNSUPPORTED;
    float *partPQ = static_cast<float *>(ws), *partXP = partPQ + partPQ_floats(p);
    if (np != (u32)n) {
        float *Tp = partXP + partXP_floats(p), *Bp = Tp + (size_t)count_sym3<int64_t>(np);
        const u32 nruns = count_sym2<u32>(np);
        u32 blocks = (nruns + 3u) / 4u, bblocks = (np * (u32)R + 255u) / 256u;
        if (blocks < bblocks) blocks = bblocks;
        hipLaunchKernelGGL(mttkrp_repack_kernel, dim3(blocks), dim3(256), 0, s, Tc, B, Tp, Bp, (u32)n, np, (u32)R, nruns);
        if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
        Tc = Tp;
        B = Bp;
    }
    const dim3 grid((u32)items, gy), block(NT);
    if (R % 4 == 0) hipLaunchKernelGGL(mttkrp_pair_kernel<true>, grid, block, 0, s, Tc, B, partPQ, partXP, np, (u32)R, p);
    else hipLaunchKernelGGL(mttkrp_pair_kernel<false>, grid, block, 0, s, Tc, B, partPQ, partXP, np, (u32)R, p);
    if (hipGetLastError() != hipSuccess) return ST_ERR_LAUNCH;
    u32 total = (u32)n * (u32)R;
    hipLaunchKernelGGL(mttkrp_reduce_kernel, dim3((total + 31u) / 32u), dim3(512), 0, s, partPQ, partXP, M,
                       (u32)n, (u32)R, p);
    return launch_status();
}

}  // namespace st
