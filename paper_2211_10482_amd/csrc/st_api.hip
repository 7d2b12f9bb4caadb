// C ABI of libstructtensor_hip.so: argument validation, host index utilities
// and dispatch to the kernel launchers.  Every error is detected here, on the
// host, before anything is enqueued.
#include <mutex>
#include <vector>

#include "st_common.h"
#include "st_index.h"

namespace st {

int num_cus()
{
    static std::mutex mu;
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
            v = 256;
        cached[dev] = v;
    }
    return cached[dev];
}

bool allow_dynamic_lds(const void *kernel, int bytes)
{
    struct Done { int dev; const void *kernel; int bytes; };
    static std::mutex mu;
    static std::vector<Done> done;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    std::lock_guard<std::mutex> lock(mu);
    for (const Done &d : done)
        if (d.dev == dev && d.kernel == kernel && d.bytes >= bytes) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
    done.push_back(Done{dev, kernel, bytes});
    return true;
}

}  // namespace st

using namespace st;
typedef int64_t i64;

extern "C" {

const char *st_status_string(st_status s)
{
    switch (s) {
    case ST_OK: return "ok";
    case ST_ERR_NULL: return "a required pointer is NULL";
    case ST_ERR_SHAPE: return "a size is out of range or buffers overlap";
    case ST_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    case ST_ERR_WORKSPACE: return "workspace missing or too small";
    case ST_ERR_LAUNCH: return "the HIP runtime reported a launch error";
    case ST_ERR_UNSUPPORTED: return "arguments outside the implemented range";
    default: return "unknown status";
    }
}

/* ---- counts / rank / unrank on the host -------------------------------- */
int64_t st_count_sym2(int64_t n) { return n < 0 ? -1 : count_sym2<i64>(n); }
int64_t st_count_sym3(int64_t n) { return n < 0 ? -1 : count_sym3<i64>(n); }
int64_t st_count_sym4(int64_t n) { return n < 0 ? -1 : count_sym4<i64>(n); }
int64_t st_count_band(int64_t n, int64_t w)
{
    if (n < 0 || w < 0) return -1;
    if (n == 0) return 0;
    return count_band<i64>(n, w);
}

int64_t st_rank_sym2(int64_t n, int64_t i, int64_t j)
{
    if (n < 1 || i < 0 || i > j || j >= n) return -1;
    return rank_sym2<i64>(n, i, j);
}
int64_t st_rank_sym3(int64_t n, int64_t i, int64_t j, int64_t k)
{
    if (n < 1 || i < 0 || i > j || j > k || k >= n) return -1;
    return rank_sym3<i64>(n, i, j, k);
}
int64_t st_rank_sym4(int64_t n, int64_t i, int64_t j, int64_t k, int64_t l)
{
    if (n < 1 || i < 0 || i > j || j > k || k > l || l >= n) return -1;
    return rank_sym4<i64>(n, i, j, k, l);
}
int64_t st_rank_band(int64_t n, int64_t w, int64_t i, int64_t j)
{
    if (n < 1 || w < 0 || i < 0 || j < 0 || i >= n || j >= n) return -1;
    i64 d = i > j ? i - j : j - i;
    if (d > w) return -1;
    return rank_band<i64>(n, w, i, j);
}

st_status st_unrank_sym2(int64_t n, int64_t p, int64_t *i, int64_t *j)
{
    if (!i || !j) return ST_ERR_NULL;
    if (n < 1 || p < 0 || p >= count_sym2<i64>(n)) return ST_ERR_SHAPE;
    unrank_sym2<i64>(n, p, *i, *j);
    return ST_OK;
}
st_status st_unrank_sym3(int64_t n, int64_t p, int64_t *i, int64_t *j, int64_t *k)
{
    if (!i || !j || !k) return ST_ERR_NULL;
    if (n < 1 || p < 0 || p >= count_sym3<i64>(n)) return ST_ERR_SHAPE;
    unrank_sym3<i64>(n, p, *i, *j, *k);
    return ST_OK;
}
st_status st_unrank_sym4(int64_t n, int64_t p, int64_t *i, int64_t *j, int64_t *k, int64_t *l)
{
    if (!i || !j || !k || !l) return ST_ERR_NULL;
    if (n < 1 || n > 50000 || p < 0 || p >= count_sym4<i64>(n)) return ST_ERR_SHAPE;   /* counts fit 64 bits */
    unrank_sym4<i64>(n, p, *i, *j, *k, *l);
    return ST_OK;
}
st_status st_unrank_band(int64_t n, int64_t w, int64_t p, int64_t *i, int64_t *j)
{
    if (!i || !j) return ST_ERR_NULL;
    if (n < 1 || w < 0 || p < 0 || p >= count_band<i64>(n, w)) return ST_ERR_SHAPE;
    unrank_band<i64>(n, w, p, *i, *j);
    return ST_OK;
}

st_status st_unrank_sym2_batch(int64_t n, int64_t p0, int64_t count, int32_t *out)
{
    if (count < 0) return ST_ERR_SHAPE;
    if (count == 0) return ST_OK;
    if (!out) return ST_ERR_NULL;
    if (n < 1 || n > INT32_MAX || p0 < 0 || p0 + count > count_sym2<i64>(n)) return ST_ERR_SHAPE;
    for (i64 q = 0; q < count; ++q) {
        i64 i, j;
        unrank_sym2<i64>(n, p0 + q, i, j);
        out[2 * q] = (int32_t)i; out[2 * q + 1] = (int32_t)j;
    }
    return ST_OK;
}
st_status st_unrank_sym3_batch(int64_t n, int64_t p0, int64_t count, int32_t *out)
{
    if (count < 0) return ST_ERR_SHAPE;
    if (count == 0) return ST_OK;
    if (!out) return ST_ERR_NULL;
    if (n < 1 || n > 2000000 || p0 < 0 || p0 + count > count_sym3<i64>(n)) return ST_ERR_SHAPE;
    for (i64 q = 0; q < count; ++q) {
        i64 i, j, k;
        unrank_sym3<i64>(n, p0 + q, i, j, k);
        out[3 * q] = (int32_t)i; out[3 * q + 1] = (int32_t)j; out[3 * q + 2] = (int32_t)k;
    }
    return ST_OK;
}
st_status st_unrank_sym4_batch(int64_t n, int64_t p0, int64_t count, int32_t *out)
{
    if (count < 0) return ST_ERR_SHAPE;
    if (count == 0) return ST_OK;
    if (!out) return ST_ERR_NULL;
    if (n < 1 || n > 50000 || p0 < 0 || p0 + count > count_sym4<i64>(n)) return ST_ERR_SHAPE;
    for (i64 q = 0; q < count; ++q) {
        i64 i, j, k, l;
        unrank_sym4<i64>(n, p0 + q, i, j, k, l);
        out[4 * q] = (int32_t)i; out[4 * q + 1] = (int32_t)j; out[4 * q + 2] = (int32_t)k; out[4 * q + 3] = (int32_t)l;
    }
    return ST_OK;
}
st_status st_unrank_band_batch(int64_t n, int64_t w, int64_t p0, int64_t count, int32_t *out)
{
    if (count < 0) return ST_ERR_SHAPE;
    if (count == 0) return ST_OK;
    if (!out) return ST_ERR_NULL;
    if (n < 1 || n > INT32_MAX || w < 0 || p0 < 0 || p0 + count > count_band<i64>(n, w))
        return ST_ERR_SHAPE;
    for (i64 q = 0; q < count; ++q) {
        i64 i, j;
        unrank_band<i64>(n, w, p0 + q, i, j);
        out[2 * q] = (int32_t)i; out[2 * q + 1] = (int32_t)j;
    }
    return ST_OK;
}

st_status st_unrank_device(int kind, int64_t n, int64_t w, int64_t p0, int64_t count,
                           int32_t *out, void *stream)
{
    if (count < 0) return ST_ERR_SHAPE;
    if (kind != 2 && kind != 3 && kind != 4 && kind != 5) return ST_ERR_SHAPE;
    if (n < 1 || p0 < 0 || (kind == 4 && w < 0)) return ST_ERR_SHAPE;
    if (n > (kind == 5 ? 50000 : 2000000)) return ST_ERR_UNSUPPORTED;
    i64 total = kind == 2 ? count_sym2<i64>(n) : kind == 3 ? count_sym3<i64>(n) : kind == 5 ? count_sym4<i64>(n)
                                                                                           : count_band<i64>(n, w);
    if (p0 + count > total) return ST_ERR_SHAPE;
    if (count == 0) return ST_OK;
    if (!out) return ST_ERR_NULL;
    return launch_unrank(kind, n, w, p0, count, out, (hipStream_t)stream);
}

/* ---- workspace queries ---------------------------------------------------- */
size_t st_mttkrp_sym3_workspace(int n, int R) { return (n < 1 || R < 1) ? 0 : mttkrp_workspace(n, R); }
size_t st_batax_utri_workspace(int n) { return n < 1 ? 0 : batax_workspace(n); }
size_t st_ttm_band_workspace(int n, int w, int nl, int R)
{
    return (n < 1 || w < 0 || nl < 1 || R < 1) ? 0 : ttm_workspace(n, w, nl, R);
}
size_t st_moment3_sym_workspace(int64_t N, int n) { return (N < 0 || n < 1) ? 0 : moment3_workspace(N, n); }
size_t st_moment4_sym_workspace(int64_t N, int n) { return (N < 0 || n < 1 || n > 256) ? 0 : moment4_workspace(N, n); }
size_t st_moment2_sym_workspace(int64_t N, int n) { return (N < 0 || n < 1 || n > 65000) ? 0 : moment2_workspace(N, n); }

static i64 struct_pairs(int structure, i64 ni, i64 nj)
{
    if (ni < 0 || nj < 0) return -1;
    switch (structure) {
    case ST_STRUCT_DIAG: return ni < nj ? ni : nj;
    case ST_STRUCT_FIXED_I: return nj;
    case ST_STRUCT_FIXED_J: return ni;
    case ST_STRUCT_UPPER: return ni == nj ? count_sym2<i64>(ni) : -1;
    default: return -1;
    }
}
int64_t st_count_struct(int structure, int64_t ni, int64_t nj) { return struct_pairs(structure, ni, nj); }
size_t st_ttm_struct_workspace(int, int, int, int, int) { return 0; }
size_t st_mttkrp_fixed_workspace(int kind, int ni, int nk, int nl, int R)
{
    if (kind < 0 || kind > 2 || ni < 1 || nk < 1 || nl < 1 || R < 1) return 0;
    return mttkrp_fixed_workspace(kind, ni, nk, nl, R);
}

/* ---- kernels ---------------------------------------------------------------- */
#define ST_REQUIRE_WS(need)                                                     \
    do {                                                                        \
        if ((need) > 0 && (!ws || ws_bytes < (need))) return ST_ERR_WORKSPACE;  \
        if ((need) > 0 && !aligned16(ws)) return ST_ERR_ALIGN;                  \
    } while (0)

st_status st_mttkrp_sym3(const float *Tc, const float *B, float *M, int n, int R, void *ws,
                         size_t ws_bytes, void *stream)
{
    if (!Tc || !B || !M) return ST_ERR_NULL;
    if (n < 1 || R < 1) return ST_ERR_SHAPE;
    if (n > 2000) return ST_ERR_UNSUPPORTED;   /* packed positions are 32-bit on the device */
    if (!aligned16(Tc) || !aligned16(B) || !aligned16(M)) return ST_ERR_ALIGN;
    size_t tb = (size_t)count_sym3<i64>(n) * 4, bb = (size_t)n * R * 4;
    if (overlap(M, bb, Tc, tb) || overlap(M, bb, B, bb)) return ST_ERR_SHAPE;
    size_t need = mttkrp_workspace(n, R);
    ST_REQUIRE_WS(need);
    if (need > 0 && (overlap(ws, need, Tc, tb) || overlap(ws, need, B, bb) || overlap(ws, need, M, bb)))
        return ST_ERR_SHAPE;
    return launch_mttkrp(Tc, B, M, n, R, ws, (hipStream_t)stream);
}

st_status st_batax_utri(const float *Ap, const float *x, float *y, int n, float beta, void *ws,
                        size_t ws_bytes, void *stream)
{
    if (!Ap || !x || !y) return ST_ERR_NULL;
    if (n < 1) return ST_ERR_SHAPE;
    if (n > 65000) return ST_ERR_UNSUPPORTED;  /* packed positions are 32-bit on the device */
    if (!aligned16(Ap) || !aligned16(x) || !aligned16(y)) return ST_ERR_ALIGN;
    size_t ab = (size_t)count_sym2<i64>(n) * 4, vb = (size_t)n * 4;
    if (overlap(y, vb, Ap, ab) || overlap(y, vb, x, vb)) return ST_ERR_SHAPE;
    size_t need = batax_workspace(n);
    ST_REQUIRE_WS(need);
    if (need > 0 && (overlap(ws, need, Ap, ab) || overlap(ws, need, x, vb) || overlap(ws, need, y, vb)))
        return ST_ERR_SHAPE;
    return launch_batax(Ap, x, y, n, beta, ws, (hipStream_t)stream);
}

int st_batax_utri_noalloc_max_n(void) { return batax_static_max_n(); }

st_status st_batax_utri_noalloc(const float *Ap, const float *x, float *y, int n, float beta, void *stream)
{
    if (!Ap || !x || !y) return ST_ERR_NULL;
    if (n < 1) return ST_ERR_SHAPE;
    if (n > batax_static_max_n()) return ST_ERR_UNSUPPORTED;   /* the library's static scratch array ends there */
    if (!aligned16(Ap) || !aligned16(x) || !aligned16(y)) return ST_ERR_ALIGN;
    size_t ab = (size_t)count_sym2<i64>(n) * 4, vb = (size_t)n * 4;
    if (overlap(y, vb, Ap, ab) || overlap(y, vb, x, vb)) return ST_ERR_SHAPE;
    return launch_batax_static(Ap, x, y, n, beta, (hipStream_t)stream);
}

st_status st_ttm_band(const float *Tc, const float *U, float *Yc, int n, int w, int nl, int R,
                      void *ws, size_t ws_bytes, void *stream)
{
    if (!Tc || !U || !Yc) return ST_ERR_NULL;
    if (n < 1 || w < 0 || nl < 1 || R < 1) return ST_ERR_SHAPE;
    if (!aligned16(Tc) || !aligned16(U) || !aligned16(Yc)) return ST_ERR_ALIGN;
    i64 rows = count_band<i64>(n, w);
    if (rows * (i64)nl > ((i64)1 << 40) || (i64)nl * R > ((i64)1 << 31)) return ST_ERR_UNSUPPORTED;
    size_t tb = (size_t)rows * nl * 4, ub = (size_t)nl * R * 4, yb = (size_t)rows * R * 4;
    if (overlap(Yc, yb, Tc, tb) || overlap(Yc, yb, U, ub)) return ST_ERR_SHAPE;
    size_t need = ttm_workspace(n, w, nl, R);
    ST_REQUIRE_WS(need);
    return launch_ttm(Tc, U, Yc, rows, nl, R, ws, (hipStream_t)stream);
}

st_status st_moment3_sym(const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws,
                         size_t ws_bytes, void *stream)
{
    if (!Sc || (N > 0 && !X)) return ST_ERR_NULL;
    if (N < 0 || n < 1 || (accumulate != 0 && accumulate != 1)) return ST_ERR_SHAPE;
    if (n > 2000) return ST_ERR_UNSUPPORTED;   /* packed positions are 32-bit on the device */
    if (!aligned16(Sc) || (X && !aligned16(X))) return ST_ERR_ALIGN;
    size_t sb = (size_t)count_sym3<i64>(n) * 4, xb = (size_t)N * n * 4;
    if (N > 0 && overlap(Sc, sb, X, xb)) return ST_ERR_SHAPE;
    size_t need = moment3_workspace(N, n);
    ST_REQUIRE_WS(need);
    if (need > 0 && (overlap(ws, need, Sc, sb) || (N > 0 && overlap(ws, need, X, xb)))) return ST_ERR_SHAPE;
    return launch_moment3(X, N, n, Sc, accumulate, ws, (hipStream_t)stream);
}

st_status st_moment2_sym(const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws,
                         size_t ws_bytes, void *stream)
{
    if (!Sc || (N > 0 && !X)) return ST_ERR_NULL;
    if (N < 0 || n < 1 || (accumulate != 0 && accumulate != 1)) return ST_ERR_SHAPE;
    if (n > 65000) return ST_ERR_UNSUPPORTED;  /* packed positions are 32-bit on the device */
    if (!aligned16(Sc) || (X && !aligned16(X))) return ST_ERR_ALIGN;
    size_t sb = (size_t)count_sym2<i64>(n) * 4, xb = (size_t)N * n * 4;
    if (N > 0 && overlap(Sc, sb, X, xb)) return ST_ERR_SHAPE;
    size_t need = moment2_workspace(N, n);
    ST_REQUIRE_WS(need);
    if (need > 0 && (overlap(ws, need, Sc, sb) || (N > 0 && overlap(ws, need, X, xb)))) return ST_ERR_SHAPE;
    return launch_moment2(X, N, n, Sc, accumulate, ws, (hipStream_t)stream);
}

st_status st_moment4_sym(const float *X, int64_t N, int n, float *Sc, int accumulate, void *ws,
                         size_t ws_bytes, void *stream)
{
    if (!Sc || (N > 0 && !X)) return ST_ERR_NULL;
    if (N < 0 || n < 1 || (accumulate != 0 && accumulate != 1)) return ST_ERR_SHAPE;
    if (n > 256) return ST_ERR_UNSUPPORTED;    /* packed positions are 32-bit on the device */
    if (!aligned16(Sc) || (X && !aligned16(X))) return ST_ERR_ALIGN;
    size_t sb = (size_t)count_sym4<i64>(n) * 4, xb = (size_t)N * n * 4;
    if (N > 0 && overlap(Sc, sb, X, xb)) return ST_ERR_SHAPE;
    size_t need = moment4_workspace(N, n);
    ST_REQUIRE_WS(need);
    if (need > 0 && (overlap(ws, need, Sc, sb) || (N > 0 && overlap(ws, need, X, xb)))) return ST_ERR_SHAPE;
    return launch_moment4(X, N, n, Sc, accumulate, ws, (hipStream_t)stream);
}

size_t st_covar_pr2_workspace(int64_t N, int n)
{
    if (N < 0 || n < 1 || n > 256) return 0;
    if (covar_small_applies(n)) return covar_small_workspace(N, n);
    size_t a = moment2_workspace(N, n), b = moment3_workspace(N, n), c = moment4_workspace(N, n);
    return a > b ? (a > c ? a : c) : (b > c ? b : c);
}

st_status st_covar_pr2(const float *X, int64_t N, int n, float *S1, float *S2, float *S3, int accumulate, void *ws,
                       size_t ws_bytes, void *stream)
{
    if (!S1 || !S2 || !S3 || (N > 0 && !X)) return ST_ERR_NULL;
    if (N < 0 || n < 1 || (accumulate != 0 && accumulate != 1)) return ST_ERR_SHAPE;
    if (n > 256) return ST_ERR_UNSUPPORTED;
    if (!aligned16(S1) || !aligned16(S2) || !aligned16(S3) || (X && !aligned16(X))) return ST_ERR_ALIGN;
    const size_t b1 = (size_t)count_sym2<i64>(n) * 4, b2 = (size_t)count_sym3<i64>(n) * 4,
                 b3 = (size_t)count_sym4<i64>(n) * 4, xb = (size_t)N * n * 4;
    if (overlap(S1, b1, S2, b2) || overlap(S1, b1, S3, b3) || overlap(S2, b2, S3, b3)) return ST_ERR_SHAPE;
    if (N > 0 && (overlap(S1, b1, X, xb) || overlap(S2, b2, X, xb) || overlap(S3, b3, X, xb))) return ST_ERR_SHAPE;
    size_t need = st_covar_pr2_workspace(N, n);
    ST_REQUIRE_WS(need);
    if (need > 0 && (overlap(ws, need, S1, b1) || overlap(ws, need, S2, b2) || overlap(ws, need, S3, b3) ||
                     (N > 0 && overlap(ws, need, X, xb))))
        return ST_ERR_SHAPE;
    if (N > 0 && covar_small_applies(n))         // one pass over the samples for all three terms
        return launch_covar_small(X, N, n, S1, S2, S3, accumulate, ws, (hipStream_t)stream);
    // the three kernels run one after the other on the stream, so they can share the workspace
    st_status rc = launch_moment2(X, N, n, S1, accumulate, ws, (hipStream_t)stream);
    if (rc != ST_OK) return rc;
    rc = launch_moment3(X, N, n, S2, accumulate, ws, (hipStream_t)stream);
    if (rc != ST_OK) return rc;
    return launch_moment4(X, N, n, S3, accumulate, ws, (hipStream_t)stream);
}

st_status st_expand_sym(const float *Sc, float *S, int n, int order, void *stream)
{
    if (!Sc || !S) return ST_ERR_NULL;
    if (n < 1 || (order != 2 && order != 3 && order != 4)) return ST_ERR_SHAPE;
    if (n > (order == 2 ? 65000 : order == 3 ? 2000 : 256)) return ST_ERR_UNSUPPORTED;
    if (!aligned16(Sc) || !aligned16(S)) return ST_ERR_ALIGN;
    size_t cb = (size_t)(order == 2 ? count_sym2<i64>(n) : order == 3 ? count_sym3<i64>(n) : count_sym4<i64>(n)) * 4;
    size_t db = (size_t)n * n * (order >= 3 ? n : 1) * (order == 4 ? n : 1) * 4;
    if (overlap(S, db, Sc, cb)) return ST_ERR_SHAPE;
    return launch_expand(Sc, S, n, order, (hipStream_t)stream);
}

st_status st_ttm_struct(int structure, const float *Bc, const float *U, float *Ac, int ni, int nj, int nl, int R,
                        void *, size_t, void *stream)
{
    if (!Bc || !U || !Ac) return ST_ERR_NULL;
    if (ni < 1 || nj < 1 || nl < 1 || R < 1) return ST_ERR_SHAPE;
    i64 rows = struct_pairs(structure, ni, nj);
    if (rows < 0) return ST_ERR_SHAPE;
    if (!aligned16(Bc) || !aligned16(U) || !aligned16(Ac)) return ST_ERR_ALIGN;
    if (rows * (i64)nl > ((i64)1 << 40) || (i64)nl * R > ((i64)1 << 31)) return ST_ERR_UNSUPPORTED;
    size_t tb = (size_t)rows * nl * 4, ub = (size_t)nl * R * 4, yb = (size_t)rows * R * 4;
    if (overlap(Ac, yb, Bc, tb) || overlap(Ac, yb, U, ub)) return ST_ERR_SHAPE;
    return launch_ttm(Bc, U, Ac, rows, nl, R, nullptr, (hipStream_t)stream);
}

st_status st_thp_struct(int structure, const float *Bc, const float *C, float *Ac, int ni, int nj, int nl, int fixed,
                        void *stream)
{
    if (!Bc || !C || !Ac) return ST_ERR_NULL;
    if (ni < 1 || nj < 1 || nl < 1) return ST_ERR_SHAPE;
    i64 rows = struct_pairs(structure, ni, nj);
    if (rows < 0) return ST_ERR_SHAPE;
    if (structure == ST_STRUCT_FIXED_I && (fixed < 0 || fixed >= ni)) return ST_ERR_SHAPE;
    if (structure == ST_STRUCT_FIXED_J && (fixed < 0 || fixed >= nj)) return ST_ERR_SHAPE;
    if (!aligned16(Bc) || !aligned16(C) || !aligned16(Ac)) return ST_ERR_ALIGN;
    if (ni > 65000 || nj > 65000 || (i64)ni * nj * nl > ((i64)1 << 40)) return ST_ERR_UNSUPPORTED;
    size_t pb = (size_t)rows * nl * 4, cb = (size_t)ni * nj * nl * 4;
    if (overlap(Ac, pb, Bc, pb) || overlap(Ac, pb, C, cb)) return ST_ERR_SHAPE;
    return launch_thp(structure, Bc, C, Ac, rows, nj, nl, fixed, (hipStream_t)stream);
}

st_status st_mttkrp_fixed(int kind, const float *Bc, const float *C, const float *D, float *A, int ni, int nk,
                          int nl, int R, int fixed_k, void *ws, size_t ws_bytes, void *stream)
{
    if (!Bc || !C || !D || !A) return ST_ERR_NULL;
    if (kind != ST_MTTKRP_FIXED_IK && kind != ST_MTTKRP_FIXED_I && kind != ST_MTTKRP_FIXED_K) return ST_ERR_SHAPE;
    if (ni < 1 || nk < 1 || nl < 1 || R < 1) return ST_ERR_SHAPE;
    if (kind != ST_MTTKRP_FIXED_I && (fixed_k < 0 || fixed_k >= nk)) return ST_ERR_SHAPE;
    if (!aligned16(Bc) || !aligned16(C) || !aligned16(D) || !aligned16(A)) return ST_ERR_ALIGN;
    if ((i64)nl * R > ((i64)1 << 31) || (i64)nk * R > ((i64)1 << 31) || (i64)ni * nl > ((i64)1 << 40) ||
        (i64)nk * nl > ((i64)1 << 40))
        return ST_ERR_UNSUPPORTED;
    const i64 brows = kind == ST_MTTKRP_FIXED_IK ? 1 : kind == ST_MTTKRP_FIXED_I ? nk : ni;
    const i64 arows = kind == ST_MTTKRP_FIXED_K ? ni : 1;
    size_t bb = (size_t)brows * nl * 4, cb = (size_t)nk * R * 4, db = (size_t)nl * R * 4, ab = (size_t)arows * R * 4;
    if (overlap(A, ab, Bc, bb) || overlap(A, ab, C, cb) || overlap(A, ab, D, db)) return ST_ERR_SHAPE;
    size_t need = mttkrp_fixed_workspace(kind, ni, nk, nl, R);
    ST_REQUIRE_WS(need);
    if (need > 0 && (overlap(ws, need, Bc, bb) || overlap(ws, need, C, cb) || overlap(ws, need, D, db) ||
                     overlap(ws, need, A, ab)))
        return ST_ERR_SHAPE;
    return launch_mttkrp_fixed(kind, Bc, C, D, A, ni, nk, nl, R, fixed_k, ws, (hipStream_t)stream);
}

st_status st_expand_band(const float *Tc, float *T, int n, int w, int nl, void *stream)
{
    if (!Tc || !T) return ST_ERR_NULL;
    if (n < 1 || w < 0 || nl < 1) return ST_ERR_SHAPE;
    if (n > 40000) return ST_ERR_UNSUPPORTED;   /* n*n and band positions are 32-bit on the device */
    if (!aligned16(Tc) || !aligned16(T)) return ST_ERR_ALIGN;
    size_t cb = (size_t)count_band<i64>(n, w) * nl * 4, db = (size_t)n * n * nl * 4;
    if (overlap(T, db, Tc, cb)) return ST_ERR_SHAPE;
    return launch_expand_band(Tc, T, n, w, nl, (hipStream_t)stream);
}

}  // extern "C"
