/*
 * st_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, fp64 CPU statement of what the structured-tensor kernels
 * compute.  Every function evaluates the *dense definition* of its
 * operation (the compression of the paper is lossless: reduction problem
 * R_T o P_T (T) = T, soundness section, and Property 5
 * T(x) = T_C(x) + T_R(x,x') * T_C(x')), never the unique-space algorithm.
 *
 * It shares no code with the GPU library.  In particular it owns its index
 * enumeration: positions in packed storage are found by *counting* inside
 * literal loop nests of the same shape as the paper's generated nests for
 * M1 / M2 (overview section: for i; for j=i; for k=j), never by a closed form.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * this file.  Nothing here is tuned.
 *
 * Conventions: 0-based indices, row-major dense arrays, last index fastest
 * in packed storage (the visiting order of the paper's loop nests, code
 * generation section).  Inputs are fp32 (as the GPU sees them) and are
 * widened exactly to fp64; all sums are fp64.
 *
 * Pins: every function below is checked in tests/test_oracle_pins.py against
 * something other than itself (closed-form counts, the 65-distinct-elements
 * example, numpy einsum / matmul on independently built dense tensors,
 * rank-one and all-ones special cases, permutation invariance).  Nothing is
 * "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define SO_API __attribute__((visibility("default")))

/* Threads the parallel loops below will use (for reporting timings). */
SO_API int so_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sets the number of threads of the parallel loops (timing on one thread, the paper's protocol, beside all
 * cores); no effect on any result: every output value is summed by one thread in a fixed order. */
SO_API void so_set_num_threads(int threads)
{
#ifdef _OPENMP
    if (threads >= 1) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
}

/* ------------------------------------------------------------------ */
/* enumeration by counting                                             */
/* ------------------------------------------------------------------ */

/* Unique set of a symmetric / upper-triangular matrix, T_U(i,j) = (0<=i<=j<n)
 * (structure catalogue, class S; upper-triangular compressed tensor example).
 * tab[i*n+j] = position in packed storage, -1 outside the unique set.
 * tab may be NULL (count only).  Returns the number of unique entries. */
SO_API int64_t so_enum_sym2(int64_t n, int64_t *tab)
{
    int64_t c = 0;
    if (tab) for (int64_t q = 0; q < n * n; ++q) tab[q] = -1;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = i; j < n; ++j) {
            if (tab) tab[i * n + j] = c;
            ++c;
        }
    return c;
}

/* Unique set of a fully symmetric order-3 tensor, 0<=i<=j<=k<n ("Tensor
 * Structures" paragraph; M2 nest).  tab[(i*n+j)*n+k] or NULL. */
SO_API int64_t so_enum_sym3(int64_t n, int64_t *tab)
{
    int64_t c = 0;
    if (tab) for (int64_t q = 0; q < n * n * n; ++q) tab[q] = -1;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = i; j < n; ++j)
            for (int64_t k = j; k < n; ++k) {
                if (tab) tab[(i * n + j) * n + k] = c;
                ++c;
            }
    return c;
}

/* Order-4 analogue 0<=i<=j<=k<=l<n (M3 nest); count only. */
SO_API int64_t so_count_sym4(int64_t n)
{
    int64_t c = 0;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = i; j < n; ++j)
            for (int64_t k = j; k < n; ++k)
                for (int64_t l = k; l < n; ++l) ++c;
    return c;
}

/* Band unique set |i-j|<=w of a square index pair, row-major, j fastest.
 * tab[i*n+j] or NULL. */
SO_API int64_t so_enum_band(int64_t n, int64_t w, int64_t *tab)
{
    int64_t c = 0;
    if (tab) for (int64_t q = 0; q < n * n; ++q) tab[q] = -1;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j) {
            int64_t d = i - j;
            if (d < 0) d = -d;
            if (d <= w) {
                if (tab) tab[i * n + j] = c;
                ++c;
            }
        }
    return c;
}

/* Listings of the unique sets in packed order (one index tuple per entry).
 * The caller sizes the output with the count returned by so_enum_*. */
SO_API int64_t so_list_sym2(int64_t n, int32_t *ij)
{
    int64_t c = 0;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = i; j < n; ++j) {
            ij[2 * c] = (int32_t)i; ij[2 * c + 1] = (int32_t)j; ++c;
        }
    return c;
}

SO_API int64_t so_list_sym3(int64_t n, int16_t *ijk)
{
    int64_t c = 0;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = i; j < n; ++j)
            for (int64_t k = j; k < n; ++k) {
                ijk[3 * c] = (int16_t)i; ijk[3 * c + 1] = (int16_t)j;
                ijk[3 * c + 2] = (int16_t)k; ++c;
            }
    return c;
}

/* Order-4 unique set in packed order (M3 nest: for i; for j=i; for k=j; for l=k). */
SO_API int64_t so_list_sym4(int64_t n, int16_t *ijkl)
{
    int64_t c = 0;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = i; j < n; ++j)
            for (int64_t k = j; k < n; ++k)
                for (int64_t l = k; l < n; ++l) {
                    ijkl[4 * c] = (int16_t)i; ijkl[4 * c + 1] = (int16_t)j;
                    ijkl[4 * c + 2] = (int16_t)k; ijkl[4 * c + 3] = (int16_t)l; ++c;
                }
    return c;
}

SO_API int64_t so_list_band(int64_t n, int64_t w, int32_t *ij)
{
    int64_t c = 0;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j) {
            int64_t d = i - j;
            if (d < 0) d = -d;
            if (d <= w) { ij[2 * c] = (int32_t)i; ij[2 * c + 1] = (int32_t)j; ++c; }
        }
    return c;
}

/* Start of each run (i,j,j..n-1) of the order-3 packed storage, found by
 * running the same nest and noting the counter on entry to the k loop.
 * run[i*n+j] for i<=j, -1 otherwise.  Used instead of the full n^3 table
 * when n is large. */
static int64_t *runs_sym3(int64_t n)
{
    int64_t *run = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n));
    int64_t c = 0;
    for (int64_t q = 0; q < n * n; ++q) run[q] = -1;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = i; j < n; ++j) {
            run[i * n + j] = c;
            for (int64_t k = j; k < n; ++k) ++c;
        }
    return run;
}

/* Start of each row of the order-2 packed storage, by counting. */
static int64_t *rows_sym2(int64_t n)
{
    int64_t *row = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    int64_t c = 0;
    for (int64_t i = 0; i < n; ++i) {
        row[i] = c;
        for (int64_t j = i; j < n; ++j) ++c;
    }
    return row;
}

static void sort3(int64_t *a, int64_t *b, int64_t *c)
{
    int64_t t;
    if (*a > *b) { t = *a; *a = *b; *b = t; }
    if (*b > *c) { t = *b; *b = *c; *c = t; }
    if (*a > *b) { t = *a; *a = *b; *b = t; }
}

/* Value of the full symmetric tensor at an arbitrary index: the redundancy
 * map sends (i,j,k) to its ascending sort (order-3 analogue of the class-S
 * map i'=j, j'=i for j<i; Property 5). */
static double sym3_at(const float *Tc, const int64_t *run, int64_t n,
                      int64_t i, int64_t j, int64_t k)
{
    sort3(&i, &j, &k);
    return (double)Tc[run[i * n + j] + (k - j)];
}

/* ------------------------------------------------------------------ */
/* dense materialisation (small n; used by the pins and tiny-n tests)  */
/* ------------------------------------------------------------------ */

SO_API void so_dense_sym3(const float *Tc, int64_t n, double *T)
{
    int64_t *tab = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n * n));
    so_enum_sym3(n, tab);
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j)
            for (int64_t k = 0; k < n; ++k) {
                int64_t a = i, b = j, c = k;
                sort3(&a, &b, &c);
                T[(i * n + j) * n + k] = (double)Tc[tab[(a * n + b) * n + c]];
            }
    free(tab);
}

SO_API void so_dense_utri(const float *Ap, int64_t n, double *A)
{
    int64_t *tab = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n));
    so_enum_sym2(n, tab);
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j)
            A[i * n + j] = (i <= j) ? (double)Ap[tab[i * n + j]] : 0.0;
    free(tab);
}

SO_API void so_dense_band(const float *Tc, int64_t n, int64_t w, int64_t nl, double *T)
{
    int64_t *tab = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n));
    so_enum_band(n, w, tab);
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j)
            for (int64_t l = 0; l < nl; ++l) {
                int64_t p = tab[i * n + j];
                T[(i * n + j) * nl + l] = (p >= 0) ? (double)Tc[p * nl + l] : 0.0;
            }
    free(tab);
}

/* ------------------------------------------------------------------ */
/* MTTKRP with a fully symmetric tensor and equal factors               */
/*   M(i,r) = sum_{j=0}^{n-1} sum_{k=0}^{n-1} T(i,j,k) B(j,r) B(k,r)    */
/* (kernel table: A(i,j) := B(i,k,l) * C(k,j) * D(l,j) with C = D)      */
/* rows[0..nrows) selects the output rows to evaluate (NULL = all n).   */
/* ------------------------------------------------------------------ */
SO_API void so_mttkrp_sym3(const float *Tc, const float *B, int64_t n, int64_t R,
                           const int64_t *rows, int64_t nrows, double *M)
{
    int64_t *run = runs_sym3(n);
    if (!rows) nrows = n;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nrows; ++q) {
        int64_t i = rows ? rows[q] : q;
        double *Mi = M + q * R;
        for (int64_t r = 0; r < R; ++r) Mi[r] = 0.0;
        for (int64_t j = 0; j < n; ++j)
            for (int64_t k = 0; k < n; ++k) {
                double t = sym3_at(Tc, run, n, i, j, k);
                const float *Bj = B + j * R, *Bk = B + k * R;
                for (int64_t r = 0; r < R; ++r)
                    Mi[r] += t * (double)Bj[r] * (double)Bk[r];
            }
    }
    free(run);
}

/* ------------------------------------------------------------------ */
/* y = beta * A^T (A x), A upper triangular, dense n^2 loops            */
/* ------------------------------------------------------------------ */
SO_API void so_batax_utri(const float *Ap, const float *x, int64_t n, double beta,
                          double *y)
{
    int64_t *row = rows_sym2(n);
    double *t = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            double a = (i <= j) ? (double)Ap[row[i] + (j - i)] : 0.0;
            s += a * (double)x[j];
        }
        t[i] = s;
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        double s = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double a = (i <= j) ? (double)Ap[row[i] + (j - i)] : 0.0;
            s += a * t[i];
        }
        y[j] = beta * s;
    }
    free(t);
    free(row);
}

/* ------------------------------------------------------------------ */
/* TTM along mode 3:  Y(i,j,r) = sum_l T(i,j,l) U(l,r)                  */
/* (kernel table: A(i,j,k) := B(i,j,l) * C(k,l), U(l,r) = C(r,l))       */
/* so_ttm_dense evaluates ALL n^2 (i,j), zeros included, into n*n*R.    */
/* so_ttm_band evaluates the in-band (i,j) only, in packed order.       */
/* ------------------------------------------------------------------ */
SO_API void so_ttm_dense(const float *Tc, const float *U, int64_t n, int64_t w,
                         int64_t nl, int64_t R, double *Y)
{
    int64_t *tab = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n));
    so_enum_band(n, w, tab);
#pragma omp parallel for schedule(static)
    for (int64_t ij = 0; ij < n * n; ++ij) {
        int64_t p = tab[ij];
        double *Yr = Y + ij * R;
        for (int64_t r = 0; r < R; ++r) Yr[r] = 0.0;
        for (int64_t l = 0; l < nl; ++l) {
            double t = (p >= 0) ? (double)Tc[p * nl + l] : 0.0;
            for (int64_t r = 0; r < R; ++r) Yr[r] += t * (double)U[l * R + r];
        }
    }
    free(tab);
}

SO_API void so_ttm_band(const float *Tc, const float *U, int64_t n, int64_t w,
                        int64_t nl, int64_t R, double *Yc)
{
    int64_t *tab = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n));
    so_enum_band(n, w, tab);
#pragma omp parallel for schedule(static)
    for (int64_t ij = 0; ij < n * n; ++ij) {
        int64_t p = tab[ij];
        if (p < 0) continue;
        double *Yr = Yc + p * R;
        for (int64_t r = 0; r < R; ++r) Yr[r] = 0.0;
        for (int64_t l = 0; l < nl; ++l) {
            double t = (double)Tc[p * nl + l];
            for (int64_t r = 0; r < R; ++r) Yr[r] += t * (double)U[l * R + r];
        }
    }
    free(tab);
}

/* ------------------------------------------------------------------ */
/* the three kernels of the kernel table on plain DENSE operands (the    */
/* sparsity structures of the table only decide which entries of B are   */
/* non-zero; the tests scatter a packed operand into a zero-filled dense  */
/* one and read the result back through the same support):               */
/*   TTM     A(i,j,k) = sum_l B(i,j,l) C(k,l)        (here U(l,k) = C(k,l)) */
/*   THP     A(i,j,k) = B(i,j,k) C(i,j,k)                                */
/*   MTTKRP  A(i,j)   = sum_{k,l} B(i,k,l) C(k,j) D(l,j)                 */
/* ------------------------------------------------------------------ */
SO_API void so_ttm_full(const float *B, const float *U, int64_t ni, int64_t nj, int64_t nl,
                        int64_t R, double *A)
{
#pragma omp parallel for schedule(static)
    for (int64_t ij = 0; ij < ni * nj; ++ij) {
        double *Ar = A + ij * R;
        for (int64_t r = 0; r < R; ++r) Ar[r] = 0.0;
        for (int64_t l = 0; l < nl; ++l) {
            double t = (double)B[ij * nl + l];
            for (int64_t r = 0; r < R; ++r) Ar[r] += t * (double)U[l * R + r];
        }
    }
}

SO_API void so_thp_full(const float *B, const float *C, int64_t count, double *A)
{
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < count; ++q) A[q] = (double)B[q] * (double)C[q];
}

SO_API void so_mttkrp_full(const float *B, const float *C, const float *D, int64_t ni, int64_t nk,
                           int64_t nl, int64_t R, double *A)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < ni; ++i)
        for (int64_t j = 0; j < R; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k < nk; ++k)
                for (int64_t l = 0; l < nl; ++l)
                    s += (double)B[(i * nk + k) * nl + l] * (double)C[k * R + j] * (double)D[l * R + j];
            A[i * R + j] = s;
        }
}

/* ------------------------------------------------------------------ */
/* third moment  S(i,j,k) = sum_s x_s(i) x_s(j) x_s(k)                  */
/* (degree-3 interaction term M2 = f (x) vec(f (x) f), summed over the  */
/* samples: "creation and addition of covariance matrices").  Raw sum,  */
/* no 1/N, no centring.                                                 */
/* so_moment3_dense: all n^3 positions.  so_moment3_entries: a list.    */
/* ------------------------------------------------------------------ */
SO_API void so_moment3_dense(const float *X, int64_t N, int64_t n, double *S)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j)
            for (int64_t k = 0; k < n; ++k) {
                double s = 0.0;
                for (int64_t q = 0; q < N; ++q) {
                    const float *xs = X + q * n;
                    s += (double)xs[i] * (double)xs[j] * (double)xs[k];
                }
                S[(i * n + j) * n + k] = s;
            }
}

SO_API void so_moment3_entries(const float *X, int64_t N, int64_t n,
                               const int32_t *ijk, int64_t count, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < count; ++e) {
        int64_t i = ijk[3 * e], j = ijk[3 * e + 1], k = ijk[3 * e + 2];
        double s = 0.0;
        for (int64_t q = 0; q < N; ++q) {
            const float *xs = X + q * n;
            s += (double)xs[i] * (double)xs[j] * (double)xs[k];
        }
        out[e] = s;
    }
}

/* ------------------------------------------------------------------ */
/* second and fourth moments: the other two terms of the degree-2       */
/* polynomial-regression covariance, summed over the samples,           */
/*   M1 = f (x) f              ->  S2(i,j)     = sum_s x_s(i) x_s(j)     */
/*   M3 = vec(f(x)f) (x) vec(f(x)f) -> S4(i,j,k,l) = sum_s x_i x_j x_k x_l */
/* Raw sums, all positions (dense) or a list of positions.              */
/* ------------------------------------------------------------------ */
SO_API void so_moment2_dense(const float *X, int64_t N, int64_t n, double *S)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double s = 0.0;
            for (int64_t q = 0; q < N; ++q) {
                const float *xs = X + q * n;
                s += (double)xs[i] * (double)xs[j];
            }
            S[i * n + j] = s;
        }
}

SO_API void so_moment4_dense(const float *X, int64_t N, int64_t n, double *S)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j)
            for (int64_t k = 0; k < n; ++k)
                for (int64_t l = 0; l < n; ++l) {
                    double s = 0.0;
                    for (int64_t q = 0; q < N; ++q) {
                        const float *xs = X + q * n;
                        s += (double)xs[i] * (double)xs[j] * (double)xs[k] * (double)xs[l];
                    }
                    S[((i * n + j) * n + k) * n + l] = s;
                }
}

SO_API void so_moment4_entries(const float *X, int64_t N, int64_t n,
                               const int32_t *ijkl, int64_t count, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < count; ++e) {
        int64_t i = ijkl[4 * e], j = ijkl[4 * e + 1], k = ijkl[4 * e + 2], l = ijkl[4 * e + 3];
        double s = 0.0;
        for (int64_t q = 0; q < N; ++q) {
            const float *xs = X + q * n;
            s += (double)xs[i] * (double)xs[j] * (double)xs[k] * (double)xs[l];
        }
        out[e] = s;
    }
}

/* Start of each run (i,j,k,k..n-1) of the order-4 packed storage, found by running
 * the M3 nest and noting the counter on entry to the l loop.  run[(i*n+j)*n+k] for
 * i<=j<=k, -1 otherwise. */
static int64_t *runs_sym4(int64_t n)
{
    int64_t *run = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n * n));
    for (int64_t q = 0; q < n * n * n; ++q) run[q] = -1;
    int64_t c = 0;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = i; j < n; ++j)
            for (int64_t k = j; k < n; ++k) {
                run[(i * n + j) * n + k] = c;
                for (int64_t l = k; l < n; ++l) ++c;
            }
    return run;
}

static void sort4(int64_t *a, int64_t *b, int64_t *c, int64_t *d)
{
    int64_t v[4] = {*a, *b, *c, *d};
    for (int x = 1; x < 4; ++x) {           /* insertion sort, ascending */
        int64_t t = v[x];
        int y = x - 1;
        while (y >= 0 && v[y] > t) { v[y + 1] = v[y]; --y; }
        v[y + 1] = t;
    }
    *a = v[0]; *b = v[1]; *c = v[2]; *d = v[3];
}

/* ------------------------------------------------------------------ */
/* reconstruction  T(x) = T_C(x) + T_R(x,x') * T_C(x')   (Property 5)   */
/* order 2: S(i,j) = Sc[pos(min,max)]  (class-S redundancy map)         */
/* order 3: S(i,j,k) = Sc[pos(sorted triple)]; order 4 likewise          */
/* fp32 in, fp32 out, a pure copy.                                      */
/* ------------------------------------------------------------------ */
SO_API int so_expand_sym(const float *Sc, int64_t n, int order, float *S)
{
    if (order == 2) {
        int64_t *tab = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n));
        so_enum_sym2(n, tab);
        for (int64_t i = 0; i < n; ++i)
            for (int64_t j = 0; j < n; ++j) {
                int64_t a = i < j ? i : j, b = i < j ? j : i;
                S[i * n + j] = Sc[tab[a * n + b]];
            }
        free(tab);
        return 0;
    }
    if (order == 3) {
        int64_t *run = runs_sym3(n);
        for (int64_t i = 0; i < n; ++i)
            for (int64_t j = 0; j < n; ++j)
                for (int64_t k = 0; k < n; ++k) {
                    int64_t a = i, b = j, c = k;
                    sort3(&a, &b, &c);
                    S[(i * n + j) * n + k] = Sc[run[a * n + b] + (c - b)];
                }
        free(run);
        return 0;
    }
    if (order == 4) {   /* S(i,j,k,l) = Sc[pos(sorted quadruple)] */
        int64_t *run = runs_sym4(n);
        for (int64_t i = 0; i < n; ++i)
            for (int64_t j = 0; j < n; ++j)
                for (int64_t k = 0; k < n; ++k)
                    for (int64_t l = 0; l < n; ++l) {
                        int64_t a = i, b = j, c = k, d = l;
                        sort4(&a, &b, &c, &d);
                        S[((i * n + j) * n + k) * n + l] = Sc[run[(a * n + b) * n + c] + (d - c)];
                    }
        free(run);
        return 0;
    }
    return 1;
}
