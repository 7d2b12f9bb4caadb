/* Driver of tests/test_oracle_sanitized.py: the oracle's C source compiled into this program with
 * AddressSanitizer and UndefinedBehaviorSanitizer, every function run once on small operands of exactly
 * the documented sizes (several sizes, the degenerate ones included).  Values are not checked here (the
 * pins do that); an out-of-bounds access, an overflow or a leak ends the program with a report. */
#include "../../oracle/st_oracle.c"
#include <stdio.h>

static float *fbuf(int64_t count)
{
    float *p = (float *)malloc(sizeof(float) * (size_t)(count > 0 ? count : 1));
    for (int64_t i = 0; i < count; ++i) p[i] = (float)((i * 37 % 101) - 50) / 64.f;
    return p;
}
static double *dbuf(int64_t count) { return (double *)malloc(sizeof(double) * (size_t)(count > 0 ? count : 1)); }

int main(void)
{
    const int64_t sizes[] = {1, 2, 5, 9};
    for (unsigned q = 0; q < sizeof(sizes) / sizeof(sizes[0]); ++q) {
        const int64_t n = sizes[q], R = 3, nl = 4, N = 6;
        const int64_t c2 = so_enum_sym2(n, NULL), c3 = so_enum_sym3(n, NULL), c4 = so_count_sym4(n);
        int64_t *tab2 = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n));
        int64_t *tab3 = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n * n));
        so_enum_sym2(n, tab2);
        so_enum_sym3(n, tab3);
        int32_t *l2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(2 * c2));
        int16_t *l3 = (int16_t *)malloc(sizeof(int16_t) * (size_t)(3 * c3));
        int16_t *l4 = (int16_t *)malloc(sizeof(int16_t) * (size_t)(4 * c4));
        so_list_sym2(n, l2);
        so_list_sym3(n, l3);
        so_list_sym4(n, l4);
        for (int64_t w = 0; w <= n; w += (n > 2 ? n / 2 : 1)) {
            const int64_t cb = so_enum_band(n, w, NULL);
            int64_t *tabb = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n * n));
            int32_t *lb = (int32_t *)malloc(sizeof(int32_t) * (size_t)(2 * cb));
            so_enum_band(n, w, tabb);
            so_list_band(n, w, lb);
            float *Tb = fbuf(cb * nl), *U = fbuf(nl * R);
            double *Td = dbuf(n * n * nl), *Y = dbuf(n * n * R), *Yc = dbuf(cb * R);
            so_dense_band(Tb, n, w, nl, Td);
            so_ttm_dense(Tb, U, n, w, nl, R, Y);
            so_ttm_band(Tb, U, n, w, nl, R, Yc);
            free(tabb); free(lb); free(Tb); free(U); free(Td); free(Y); free(Yc);
        }
        float *Tc = fbuf(c3), *B = fbuf(n * R), *Ap = fbuf(c2), *x = fbuf(n), *X = fbuf(N * n);
        double *T = dbuf(n * n * n), *A = dbuf(n * n), *M = dbuf((n > 2 ? n : 2) * R), *y = dbuf(n);
        so_dense_sym3(Tc, n, T);
        so_dense_utri(Ap, n, A);
        so_mttkrp_sym3(Tc, B, n, R, NULL, n, M);
        int64_t rows[2] = {n - 1, 0};
        so_mttkrp_sym3(Tc, B, n, R, rows, 2, M);
        so_batax_utri(Ap, x, n, 0.5, y);
        float *Bd = fbuf(n * n * nl), *Cd = fbuf(n * n * nl), *Cm = fbuf(n * R), *Dm = fbuf(nl * R), *U2 = fbuf(nl * R);
        double *Af = dbuf(n * n * R), *Ah = dbuf(n * n * nl), *Am = dbuf(n * R);
        so_ttm_full(Bd, U2, n, n, nl, R, Af);
        so_thp_full(Bd, Cd, n * n * nl, Ah);
        so_mttkrp_full(Bd, Cm, Dm, n, n, nl, R, Am);
        double *S2 = dbuf(n * n), *S3 = dbuf(n * n * n), *S4 = dbuf(n * n * n * n), *e3 = dbuf(c3), *e4 = dbuf(c4);
        int32_t *i3 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(3 * c3 + 1));
        int32_t *i4 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(4 * c4 + 1));
        for (int64_t p = 0; p < 3 * c3; ++p) i3[p] = l3[p];
        for (int64_t p = 0; p < 4 * c4; ++p) i4[p] = l4[p];
        so_moment2_dense(X, N, n, S2);
        so_moment3_dense(X, N, n, S3);
        so_moment4_dense(X, N, n, S4);
        so_moment3_entries(X, N, n, i3, c3, e3);
        so_moment4_entries(X, N, n, i4, c4, e4);
        so_moment3_dense(X, 0, n, S3);                       /* no samples */
        float *Sc2 = fbuf(c2), *Sc3 = fbuf(c3), *Sc4 = fbuf(c4);
        float *E2 = (float *)malloc(sizeof(float) * (size_t)(n * n)), *E3 = (float *)malloc(sizeof(float) * (size_t)(n * n * n)),
              *E4 = (float *)malloc(sizeof(float) * (size_t)(n * n * n * n));
        if (so_expand_sym(Sc2, n, 2, E2) || so_expand_sym(Sc3, n, 3, E3) || so_expand_sym(Sc4, n, 4, E4)) return 2;
        free(tab2); free(tab3); free(l2); free(l3); free(l4); free(Tc); free(B); free(Ap); free(x); free(X);
        free(T); free(A); free(M); free(y); free(Bd); free(Cd); free(Cm); free(Dm); free(U2); free(Af); free(Ah);
        free(Am); free(S2); free(S3); free(S4); free(e3); free(e4); free(i3); free(i4); free(Sc2); free(Sc3);
        free(Sc4); free(E2); free(E3); free(E4);
    }
    so_set_num_threads(1);
    printf("threads=%d ok\n", so_num_threads());
    return 0;
}
