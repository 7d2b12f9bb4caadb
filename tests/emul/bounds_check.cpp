// Driver of tests/test_kernel_bounds.py: one kernel family per build (-DCHECK_<NAME>),
// compiled against the host stand-in of the HIP runtime with AddressSanitizer.  Buffers
// have exactly the sizes the C-ABI documents, so any access outside them aborts.
#if defined(CHECK_MTTKRP)
#include "../../paper_2211_10482_amd/csrc/st_mttkrp.hip"
#elif defined(CHECK_BATAX)
#include "../../paper_2211_10482_amd/csrc/st_batax.hip"
#elif defined(CHECK_TTM)
#include "../../paper_2211_10482_amd/csrc/st_ttm.hip"
#elif defined(CHECK_MOMENT3)
#include "../../paper_2211_10482_amd/csrc/st_moment3.hip"
#include "../../paper_2211_10482_amd/csrc/st_moment_mfma.hip"
#elif defined(CHECK_MOMENT2)
#include "../../paper_2211_10482_amd/csrc/st_moment2.hip"
#elif defined(CHECK_MOMENT4)
#include "../../paper_2211_10482_amd/csrc/st_moment4.hip"
#include "../../paper_2211_10482_amd/csrc/st_moment_mfma.hip"
#define ST_STUB_COVAR_SMALL 1   // up to 16 features the fourth moment runs the kernels of the COVARSMALL family
#elif defined(CHECK_COVARSMALL)
#include "../../paper_2211_10482_amd/csrc/st_covar_small.hip"
#elif defined(CHECK_MCOVER)
#include "../../paper_2211_10482_amd/csrc/st_moment_mfma.hip"
#elif defined(CHECK_M2COVER)
#include "../../paper_2211_10482_amd/csrc/st_moment2.hip"
#elif defined(CHECK_EXPAND)
#include "../../paper_2211_10482_amd/csrc/st_expand.hip"
#elif defined(CHECK_TABLE)
#include "../../paper_2211_10482_amd/csrc/st_ttm.hip"
#include "../../paper_2211_10482_amd/csrc/st_table.hip"
#else
#error "define CHECK_<KERNEL>"
#endif
#include <cstdio>
#include <cstdlib>

namespace st {
float lds[160 * 1024 / 4];
int num_cus() { return 256; }
bool allow_dynamic_lds(const void *, int) { return true; }
#ifdef ST_STUB_COVAR_SMALL
bool covar_small_applies(int) { return false; }
size_t covar_small_workspace(int64_t, int) { return 0; }
st_status launch_covar_small(const float *, int64_t, int, float *, float *, float *, int, void *, hipStream_t) { return ST_OK; }
#endif
}  // namespace st

static float *fbuf(size_t count)
{
    float *p = static_cast<float *>(malloc(count ? count * sizeof(float) : 1));
    for (size_t i = 0; i < count; ++i) p[i] = 1.f;
    return p;
}

int main(int argc, char **argv)
{
    long a[6] = {0, 0, 0, 0, 0, 0};
    for (int i = 1; i < argc && i <= 6; ++i) a[i - 1] = atol(argv[i]);
    int rc = -1;
#if defined(CHECK_MTTKRP)
    const int n = (int)a[0], R = (int)a[1];
    const size_t cnt = (size_t)st::count_sym3<int64_t>(n), wsb = st::mttkrp_workspace(n, R);
    float *Tc = fbuf(cnt), *B = fbuf((size_t)n * R), *M = fbuf((size_t)n * R);
    void *ws = malloc(wsb ? wsb : 1);
    rc = st::launch_mttkrp(Tc, B, M, n, R, ws, nullptr);
    free(Tc); free(B); free(M); free(ws);
#elif defined(CHECK_BATAX)
    const int n = (int)a[0];
    const size_t cnt = (size_t)st::count_sym2<int64_t>(n), wsb = st::batax_workspace(n);
    float *Ap = fbuf(cnt), *x = fbuf(n), *y = fbuf(n);
    void *ws = malloc(wsb ? wsb : 1);
    rc = st::launch_batax(Ap, x, y, n, 0.5f, ws, nullptr);
    if (rc == 0 && n <= st::batax_static_max_n())      // the same kernels on the library's static scratch array
        rc = st::launch_batax_static(Ap, x, y, n, 0.5f, nullptr);
    free(Ap); free(x); free(y); free(ws);
#elif defined(CHECK_TTM)
    const long rows = a[0];
    const int nl = (int)a[1], R = (int)a[2];
    float *Tc = fbuf((size_t)rows * nl), *U = fbuf((size_t)nl * R), *Y = fbuf((size_t)rows * R);
    rc = st::launch_ttm(Tc, U, Y, rows, nl, R, nullptr, nullptr);
    free(Tc); free(U); free(Y);
#elif defined(CHECK_MOMENT3)
    const long N = a[0];
    const int n = (int)a[1], accumulate = (int)a[2];
    const size_t cnt = (size_t)st::count_sym3<int64_t>(n), wsb = st::moment3_workspace(N, n);
    float *X = fbuf((size_t)N * n), *Sc = fbuf(cnt);
    void *ws = malloc(wsb ? wsb : 1);
    rc = st::launch_moment3(X, N, n, Sc, accumulate, ws, nullptr);
    free(X); free(Sc); free(ws);
#elif defined(CHECK_COVARSMALL)
    const long N = a[0];
    const int n = (int)a[1], accumulate = (int)a[2];
    const size_t wsb = st::covar_small_workspace(N, n);
    float *X = fbuf((size_t)N * n), *S1 = fbuf((size_t)st::count_sym2<int64_t>(n)),
          *S2 = fbuf((size_t)st::count_sym3<int64_t>(n)), *S3 = fbuf((size_t)st::count_sym4<int64_t>(n));
    void *ws = malloc(wsb ? wsb : 1);
    rc = st::launch_covar_small(X, N, n, S1, S2, S3, accumulate, ws, nullptr);
    free(X); free(S1); free(S2); free(S3); free(ws);
#elif defined(CHECK_MCOVER)
    // The tile table and the kept-position rules of the matrix-core moment kernels: with every raw accumulator
    // set to 1 and Sc to 0, the reduce kernel in accumulate mode must leave exactly 1 in every unique entry
    // (each index multiset is kept at one position, no position falls outside the unique set).   args: order n
    const int order = (int)a[0], n = (int)a[1];
    const long N = 4;                                        // one slice
    const size_t cnt = (size_t)(order == 3 ? st::count_sym3<int64_t>(n) : st::count_sym4<int64_t>(n));
    const st::MMPlan p = st::mm_plan(order, N, n);
    const st::MMTable &tab = st::mm_table(order, (int)p.G);
    const size_t slots = (size_t)p.kinds * st::MM_WAVES, racc = (size_t)p.blocks * st::MM_ACC;
    float *part = fbuf(slots * st::MM_ACC), *Sc = fbuf(cnt);
    for (size_t q = 0; q < cnt; ++q) Sc[q] = 0.f;
    if (p.S != 1) return 3;
    if (order == 3)
        hipLaunchKernelGGL(st::moment3_mfma_reduce_kernel, dim3((unsigned)((racc + 255) / 256)), dim3(256), 0, nullptr,
                           part, tab.spec.data(), p.blocks, (unsigned)slots, 1u, (unsigned)n, Sc, 1);
    else
        hipLaunchKernelGGL(st::moment4_mfma_reduce_kernel, dim3((unsigned)((racc + 255) / 256)), dim3(256), 0, nullptr,
                           part, tab.spec.data(), p.blocks, (unsigned)slots, 1u, (unsigned)n, Sc, 1);
    size_t bad = 0;
    for (size_t q = 0; q < cnt; ++q) bad += Sc[q] != 1.f;
    printf("blocks=%u tiles=%u entries=%zu bad=%zu\n", p.blocks, p.blocks * st::MM_TPB, cnt, bad);
    rc = bad == 0 ? 0 : 4;
    free(part); free(Sc);
#elif defined(CHECK_M2COVER)
    // The tasks of the second moment's strip path and the kept-position rule of its reduce kernel: with every raw
    // accumulator set to 1 and Sc to 0, the reduce kernel in accumulate mode must leave exactly 1 in every unique
    // entry.  One slice: only the first of the kernel's eight slice groups adds anything, so the emulation's
    // sequential threads see what a workgroup would.   args: n
    const int n = (int)a[0];
    const size_t cnt = (size_t)st::count_sym2<int64_t>(n);
    const st::M2WPlan p = st::m2w_plan(4, n);
    if (p.S != 1) return 3;
    float *part = fbuf((size_t)p.ntasks * st::M2W_ACC), *Sc = fbuf(cnt);
    for (size_t q = 0; q < cnt; ++q) Sc[q] = 0.f;
    hipLaunchKernelGGL(st::moment2_strip_reduce_kernel, dim3(p.ntasks * (unsigned)st::M2W_ACC / 32u), dim3(256), 0, nullptr,
                       part, 1u, (unsigned)n, p.nb, p.nbb, p.ntasks, Sc, 1);
    size_t bad = 0;
    for (size_t q = 0; q < cnt; ++q) bad += Sc[q] != 1.f;
    printf("strips=%u tasks=%u entries=%zu bad=%zu\n", p.nb, p.ntasks, cnt, bad);
    rc = bad == 0 ? 0 : 4;
    free(part); free(Sc);
#elif defined(CHECK_MOMENT2) || defined(CHECK_MOMENT4)
    const long N = a[0];
    const int n = (int)a[1], accumulate = (int)a[2];
#if defined(CHECK_MOMENT2)
    const size_t cnt = (size_t)st::count_sym2<int64_t>(n), wsb = st::moment2_workspace(N, n);
#else
    const size_t cnt = (size_t)st::count_sym4<int64_t>(n), wsb = st::moment4_workspace(N, n);
#endif
    float *X = fbuf((size_t)N * n), *Sc = fbuf(cnt);
    void *ws = malloc(wsb ? wsb : 1);
#if defined(CHECK_MOMENT2)
    rc = st::launch_moment2(X, N, n, Sc, accumulate, ws, nullptr);
#else
    rc = st::launch_moment4(X, N, n, Sc, accumulate, ws, nullptr);
#endif
    free(X); free(Sc); free(ws);
#elif defined(CHECK_EXPAND)
    const int n = (int)a[0], order = (int)a[1];
    if (order == 2 || order == 3 || order == 4) {
        const size_t cnt = (size_t)(order == 2   ? st::count_sym2<int64_t>(n)
                                    : order == 3 ? st::count_sym3<int64_t>(n)
                                                 : st::count_sym4<int64_t>(n));
        size_t full = 1;
        for (int i = 0; i < order; ++i) full *= (size_t)n;
        float *Sc = fbuf(cnt), *S = fbuf(full);
        rc = st::launch_expand(Sc, S, n, order, nullptr);
        free(Sc); free(S);
    } else {   // order = 10 + kind: device unrank of `count` positions from p0
        const int kind = order - 10;
        const long w = a[2], p0 = a[3], count = a[4];
        int32_t *out = static_cast<int32_t *>(malloc((size_t)count * (kind == 3 ? 3 : kind == 5 ? 4 : 2) * sizeof(int32_t) + 1));
        rc = st::launch_unrank(kind, n, w, p0, count, out, nullptr);
        free(out);
    }
#elif defined(CHECK_TABLE)
    // op (0 thp, 1 mttkrp with fixed indices, 2 band expand), structure | kind | w, ni, nj | nk, nl, R
    const int op = (int)a[0], sk = (int)a[1], ni = (int)a[2], nj = (int)a[3], nl = (int)a[4], R = (int)a[5];
    if (op == 0) {
        const long pairs = sk == ST_STRUCT_DIAG ? (ni < nj ? ni : nj) : sk == ST_STRUCT_FIXED_I ? nj
                           : sk == ST_STRUCT_FIXED_J ? ni : (long)st::count_sym2<int64_t>(ni);
        const int fixed = sk == ST_STRUCT_FIXED_I ? ni - 1 : sk == ST_STRUCT_FIXED_J ? nj - 1 : 0;
        float *Bc = fbuf((size_t)pairs * nl), *C = fbuf((size_t)ni * nj * nl), *Ac = fbuf((size_t)pairs * nl);
        rc = st::launch_thp(sk, Bc, C, Ac, pairs, nj, nl, fixed, nullptr);
        free(Bc); free(C); free(Ac);
    } else if (op == 1) {
        const int nk = nj;
        const size_t brows = sk == ST_MTTKRP_FIXED_IK ? 1 : sk == ST_MTTKRP_FIXED_I ? nk : ni;
        const size_t arows = sk == ST_MTTKRP_FIXED_K ? ni : 1;
        const size_t wsb = st::mttkrp_fixed_workspace(sk, ni, nk, nl, R);
        float *Bc = fbuf(brows * nl), *C = fbuf((size_t)nk * R), *D = fbuf((size_t)nl * R), *A = fbuf(arows * R);
        void *ws = malloc(wsb ? wsb : 1);
        rc = st::launch_mttkrp_fixed(sk, Bc, C, D, A, ni, nk, nl, R, nk - 1, ws, nullptr);
        free(Bc); free(C); free(D); free(A); free(ws);
    } else {
        const int n = ni, w = sk;
        float *Tc = fbuf((size_t)st::count_band<int64_t>(n, w) * nl), *T = fbuf((size_t)n * n * nl);
        rc = st::launch_expand_band(Tc, T, n, w, nl, nullptr);
        free(Tc); free(T);
    }
#endif
    printf("rc=%d\n", rc);
    return rc == 0 ? 0 : 1;
}
