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
// Each of the 4 waves then owns 16 columns r: per p one ds_read_b128 of D (lane =
// (x, q-quad); the four components feed four MFMAs with consistently permuted K
// slots), four VALU multiplies for the Khatri-Rao operand, four MFMAs.
// Workgroup partials go to the workspace; a second kernel adds them in order.
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

struct __attribute__((packed, aligned(4))) f4u { float x, y, z, w; };

__device__ __forceinline__ void sort3u(u32 &a, u32 &b, u32 &c)
{
    u32 lo = min(a, b), hi = max(a, b);
    u32 mn = min(lo, c), mx = max(hi, c), md = max(lo, min(hi, c));
    a = mn; b = md; c = mx;
}

__global__ __launch_bounds__(256) void mttkrp_mfma_kernel(const float *__restrict__ Tc,
                                                        const float *__restrict__ B,
                                                        float *__restrict__ part, u32 n, u32 R, u32 NB,
                                                        u32 npairs, u32 PPC, u32 NCH, u32 Rpad)
{
    __shared__ __attribute__((aligned(16))) float tile[TILE_F];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 X = blockIdx.y, ch = blockIdx.x;
    const u32 rt = blockIdx.z * 4u + wave;           // this wave's block of 16 columns of R
    const bool has_rt = rt * 16u < R;
    const u32 x0 = X * 16u;
    const u32 lrow = lane & 15u, lq = lane >> 4;
    const u32 r = rt * 16u + lrow;                    // column of B / M handled as MFMA column
    const bool r_ok = has_rt && r < R;

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const u32 pi0 = ch * PPC, pi1 = min(npairs, pi0 + PPC);
    for (u32 pi = pi0; pi < pi1; ++pi) {
        u32 P, Q;
        unrank_sym2<u32>(NB, pi, P, Q);
        const u32 p0 = P * 16u, q0 = Q * 16u;
        const bool full = (max(x0, q0) + 16u <= n);

        __syncthreads();                              // previous visit's readers are done
        if (full && Q > X && Q > P && X != P) {
            // runs along q: D[x][p][q] = Tc[run(min, max) + (q0 + q - max)]
#pragma unroll
            for (u32 it = 0; it < 4; ++it) {
                u32 e = tid + 256u * it, row = e >> 2, qr = e & 3u;
                u32 x = row >> 4, p = row & 15u;
                u32 a = min(x0 + x, p0 + p), b = max(x0 + x, p0 + p);
                const float *src = Tc + run_sym3<u32>(n, a, b) + (q0 - b) + 4u * qr;
                f4u v = *reinterpret_cast<const f4u *>(src);
                *reinterpret_cast<float4 *>(&tile[x * XS + p * 16u + 4u * qr]) = make_float4(v.x, v.y, v.z, v.w);
            }
        } else if (full && X > Q && Q > P) {
            // runs along x: D[x][p][q] = Tc[run(p, q) + (x0 + x - q)]
#pragma unroll
            for (u32 it = 0; it < 4; ++it) {
                u32 e = tid + 256u * it, row = e >> 2, xr = e & 3u;
                u32 p = row >> 4, q = row & 15u;
                const float *src = Tc + run_sym3<u32>(n, p0 + p, q0 + q) + (x0 - (q0 + q)) + 4u * xr;
                f4u v = *reinterpret_cast<const f4u *>(src);
                float *d = &tile[(4u * xr) * XS + p * 16u + q];
                d[0] = v.x; d[XS] = v.y; d[2 * XS] = v.z; d[3 * XS] = v.w;
            }
        } else {
#pragma unroll 4
            for (u32 it = 0; it < 16; ++it) {
                u32 e = tid + 256u * it;
                u32 x = e >> 8, p = (e >> 4) & 15u, q = e & 15u;
                u32 a = x0 + x, b = p0 + p, c = q0 + q;
                sort3u(a, b, c);
                float v = 0.f;
                if (c < n) v = Tc[rank_sym3<u32>(n, a, b, c)];
                tile[x * XS + p * 16u + q] = v;
            }
        }
        __syncthreads();

        if (has_rt) {
            const float wgt = (P < Q) ? 2.f : 1.f;
            float bq[4];
#pragma unroll
            for (u32 t = 0; t < 4; ++t) {
                u32 q = q0 + 4u * lq + t;
                bq[t] = (r_ok && q < n) ? B[(size_t)q * R + r] : 0.f;
            }
            const float *arow = &tile[lrow * XS + 4u * lq];
#pragma unroll 4
            for (u32 p = 0; p < 16; ++p) {
                u32 pg = p0 + p;
                float bp = (r_ok && pg < n) ? wgt * B[(size_t)pg * R + r] : 0.f;
                f32x4 a = *reinterpret_cast<const f32x4 *>(arow + p * 16u);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], bp * bq[0], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], bp * bq[1], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], bp * bq[2], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], bp * bq[3], acc, 0, 0, 0);
            }
        }
    }

    if (has_rt) {
        // D layout: lane holds column lane%16 of rows 4*(lane/16) + v
        float *dst = part + ((size_t)(X * NCH + ch) * 16u) * Rpad + rt * 16u + lrow;
#pragma unroll
        for (u32 v = 0; v < 4; ++v) dst[(size_t)(4u * lq + v) * Rpad] = acc[v];
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
    p.PPC = (u32)((visits + 2047u) / 2048u);
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
