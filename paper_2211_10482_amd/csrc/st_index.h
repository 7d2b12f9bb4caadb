// Closed-form index maps of the three packed unique sets (host and device).
//
//   sym2 : 0<=i<=j<n        (upper-triangular / symmetric unique set)
//   sym3 : 0<=i<=j<=k<n     (generalised symmetric order-3 unique set)
//   sym4 : 0<=i<=j<=k<=l<n  (order-4 analogue)
//   band : |i-j|<=w         (square pair, row-major)
//
// Packed order is lexicographic with the last index fastest, i.e. the order in
// which the paper's generated loop nests (for i; for j=i; for k=j) visit the
// unique set.  rank() turns indices into a packed position without tables or
// masks, unrank() inverts it.  I is the integer type (int64_t at the ABI;
// kernels instantiate uint32_t when every intermediate fits).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define ST_HD __host__ __device__ __forceinline__

namespace st {

template <typename I> ST_HD I tri(I m) { return m * (m + 1) / 2; }            // 1+2+..+m
template <typename I> ST_HD I tet(I m)                                       // tri(1)+..+tri(m)
{
    // tri(m) is exact and tri(m)*(m+2) = 3*tet(m): one division by a constant, no
    // branches.  The intermediate is 3*tet(m), so 32-bit use is valid to m = 2047.
    return tri<I>(m) * (m + 2) / 3;
}

template <typename I> ST_HD I pent(I m)                                      // tet(1)+..+tet(m)
{
    // tet(m)*(m+3) = 4*pent(m), exact; 32-bit use is valid to m = 320
    return tet<I>(m) * (m + 3) / 4;
}

template <typename I> ST_HD I count_sym2(I n) { return tri<I>(n); }
template <typename I> ST_HD I count_sym3(I n) { return tet<I>(n); }
template <typename I> ST_HD I count_sym4(I n) { return pent<I>(n); }
template <typename I> ST_HD I clamp_w(I n, I w) { return w > n - 1 ? n - 1 : w; }
template <typename I> ST_HD I count_band(I n, I w)
{
    w = clamp_w<I>(n, w);
    return n * (2 * w + 1) - w * (w + 1);
}

// position of (i,i) : rows 0..i-1 hold n, n-1, .., n-i+1 entries
template <typename I> ST_HD I row_sym2(I n, I i) { return i * n - (i * (i - 1)) / 2; }
template <typename I> ST_HD I rank_sym2(I n, I i, I j) { return row_sym2<I>(n, i) + (j - i); }

// position of (i,i,i) : slabs 0..i-1 hold tri(n), tri(n-1), .. entries
template <typename I> ST_HD I slab_sym3(I n, I i) { return tet<I>(n) - tet<I>(n - i); }
// position of (i,j,j)
template <typename I> ST_HD I run_sym3(I n, I i, I j)
{
    return slab_sym3<I>(n, i) + tri<I>(n - i) - tri<I>(n - j);
}
template <typename I> ST_HD I rank_sym3(I n, I i, I j, I k) { return run_sym3<I>(n, i, j) + (k - j); }

// position of (i,i,i,i) : the quadruples with first index i' < i are sym3 sets of sizes n, n-1, ..
template <typename I> ST_HD I hslab_sym4(I n, I i) { return pent<I>(n) - pent<I>(n - i); }
// the quadruples with first index i are the sym3 set of (j-i, k-i, l-i) over n-i values
template <typename I> ST_HD I rank_sym4(I n, I i, I j, I k, I l)
{
    return hslab_sym4<I>(n, i) + rank_sym3<I>(n - i, j - i, k - i, l - i);
}

// first packed position of band row i
template <typename I> ST_HD I row_band(I n, I w, I i)
{
    w = clamp_w<I>(n, w);
    I left = (i <= w) ? (i * w - (i * (i - 1)) / 2) : (w * (w + 1)) / 2;  // columns cut off at j<0
    I c = (i > n - w) ? (i - (n - w)) : 0;                               // rows already cut at j>=n
    return i * (2 * w + 1) - left - (c * (c + 1)) / 2;
}
template <typename I> ST_HD I rank_band(I n, I w, I i, I j)
{
    w = clamp_w<I>(n, w);
    I lo = (i > w) ? (i - w) : 0;
    return row_band<I>(n, w, i) + (j - lo);
}

// largest m with tri(m) <= q
template <typename I> ST_HD I tri_root(I q)
{
    I m = (I)((sqrt(8.0 * (double)q + 1.0) - 1.0) * 0.5);
    while (tri<I>(m + 1) <= q) ++m;
    while (m > 0 && tri<I>(m) > q) --m;
    return m;
}
// largest m with tet(m) <= q
template <typename I> ST_HD I tet_root(I q)
{
    I m = (I)cbrt(6.0 * (double)q);
    if (m > 0) --m;
    while (tet<I>(m + 1) <= q) ++m;
    while (m > 0 && tet<I>(m) > q) --m;
    return m;
}

// largest m with pent(m) <= q
template <typename I> ST_HD I pent_root(I q)
{
    I m = (I)sqrt(sqrt(24.0 * (double)q));
    m = m > 2 ? m - 2 : 0;
    while (pent<I>(m + 1) <= q) ++m;
    while (m > 0 && pent<I>(m) > q) --m;
    return m;
}

template <typename I> ST_HD void unrank_sym2(I n, I p, I &i, I &j)
{
    I q = tri<I>(n) - 1 - p;          // position counted from the end
    I m = tri_root<I>(q);             // rows n-m .. n-1 hold tri(m) <= q entries
    i = n - 1 - m;
    j = i + (p - row_sym2<I>(n, i));
}

template <typename I> ST_HD void unrank_sym3(I n, I p, I &i, I &j, I &k)
{
    I q = tet<I>(n) - 1 - p;
    I m = tet_root<I>(q);             // slabs n-m .. n-1 hold tet(m) <= q entries
    i = n - 1 - m;
    I jj, kk;
    unrank_sym2<I>(n - i, p - slab_sym3<I>(n, i), jj, kk);
    j = i + jj;
    k = i + kk;
}

template <typename I> ST_HD void unrank_sym4(I n, I p, I &i, I &j, I &k, I &l)
{
    I q = pent<I>(n) - 1 - p;
    I m = pent_root<I>(q);            // first indices n-m .. n-1 hold pent(m) <= q entries
    i = n - 1 - m;
    I jj, kk, ll;
    unrank_sym3<I>(n - i, p - hslab_sym4<I>(n, i), jj, kk, ll);
    j = i + jj;
    k = i + kk;
    l = i + ll;
}

template <typename I> ST_HD void unrank_band(I n, I w, I p, I &i, I &j)
{
    w = clamp_w<I>(n, w);
    I lo = 0, hi = n - 1;             // largest row whose first position is <= p
    while (lo < hi) {
        I mid = (lo + hi + 1) / 2;
        if (row_band<I>(n, w, mid) <= p) lo = mid; else hi = mid - 1;
    }
    i = lo;
    I c0 = (i > w) ? (i - w) : 0;
    j = c0 + (p - row_band<I>(n, w, i));
}

}  // namespace st
