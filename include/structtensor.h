/*
 * structtensor.h -- C ABI of the structured-tensor kernel library for
 * AMD CDNA4 (gfx950), libstructtensor_hip.so.
 *
 * The library evaluates tensor kernels over only the unique, non-zero
 * iteration space fixed by a tensor's sparsity structure (unique set T_U)
 * and redundancy structure (redundancy map T_R), and reconstructs redundant
 * outputs afterwards, as in "Compiling Structured Tensor Algebra"
 * (StructTensor).  Where the paper leaves a compressed tensor inside a full
 * n-d array (code generation section), this library stores it PACKED.
 *
 * Packed layouts (part of the ABI; 0-based, last index fastest, i.e. the
 * visiting order of the paper's loop nests, code generation section):
 *   sym2 : pairs   0<=i<=j<n      (class S / upper-triangular unique set),
 *          n(n+1)/2 entries, row i holds columns i..n-1.
 *   sym3 : triples 0<=i<=j<=k<n   ("Tensor Structures": unique elements of a
 *          degree-3 interaction tensor), n(n+1)(n+2)/6 entries.
 *   sym4 : quadruples 0<=i<=j<=k<=l<n (the M3 term of the same covariance),
 *          n(n+1)(n+2)(n+3)/24 entries.
 *   band : pairs |i-j|<=w, 0<=i,j<n, row-major; a band 3-tensor stores one
 *          contiguous fibre of length nl per in-band pair.
 *
 * Conventions for every kernel entry point:
 *   - all data pointers are DEVICE pointers to contiguous fp32, 16-byte
 *     aligned (ST_ERR_ALIGN otherwise); dense matrices are row-major;
 *   - the caller owns every buffer, including the workspace `ws` of at least
 *     st_<kernel>_workspace(...) bytes (may be NULL when that is 0);
 *     the library allocates no device memory and no result depends on an
 *     earlier call.  What it does keep, per process and behind locks, are
 *     host-side caches: the CU count and the dynamic-LDS limits it has raised
 *     per device, the tile tables of the table-driven moment kernels (built
 *     at first use, with a copy in pinned host memory), the compiled modules
 *     of descriptors, and the address of the static scratch array of
 *     st_batax_utri_noalloc;
 *   - inputs and outputs must not overlap;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns without synchronising: every
 *     entry point enqueues kernels only (the moment kernels for 64 < n <= 256
 *     bring their tile table into the workspace with a small kernel that
 *     reads the pinned copy);
 *   - arguments are validated on the host before anything is launched: on
 *     ST_ERR_NULL / SHAPE / ALIGN / WORKSPACE / UNSUPPORTED nothing was
 *     launched and outputs are untouched.  ST_ERR_LAUNCH means the HIP
 *     runtime refused a launch: entry points that enqueue several kernels
 *     may then have enqueued the earlier ones, and outputs are undefined;
 *   - results are deterministic: same inputs, same bits (no float atomics).
 */
#ifndef STRUCTTENSOR_H
#define STRUCTTENSOR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int st_status;
enum {
    ST_OK = 0,
    ST_ERR_NULL = 1,        /* a required pointer is NULL                       */
    ST_ERR_SHAPE = 2,       /* a size is out of range, or buffers alias         */
    ST_ERR_ALIGN = 3,       /* a device pointer is not 16-byte aligned          */
    ST_ERR_WORKSPACE = 4,   /* ws is NULL or ws_bytes is below the query        */
    ST_ERR_LAUNCH = 5,      /* the HIP runtime reported an error at launch      */
    ST_ERR_UNSUPPORTED = 6  /* valid arguments outside what is implemented      */
};

/* Static, NUL-terminated description of a status code. */
const char *st_status_string(st_status s);

/* ---- host-side integer utilities (pure functions, no GPU needed) -------- */

/* Sizes of the unique sets.  n(n+1)/2 is what remains of n^2 for an
 * upper-triangular / symmetric matrix ("half of the elements", compressed
 * tensor example); n(n+1)(n+2)/6 is the number of i<=j<=k triples.  w is
 * clamped to n-1.  Return -1 for n < 0 or w < 0. */
int64_t st_count_sym2(int64_t n);
int64_t st_count_sym3(int64_t n);
int64_t st_count_sym4(int64_t n);   /* i<=j<=k<=l quadruples (M3 nest), n(n+1)(n+2)(n+3)/24 */
int64_t st_count_band(int64_t n, int64_t w);

/* Position of an index tuple in packed storage (closed forms, no tables).
 * Return -1 if the tuple is outside the unique set. */
int64_t st_rank_sym2(int64_t n, int64_t i, int64_t j);
int64_t st_rank_sym3(int64_t n, int64_t i, int64_t j, int64_t k);
int64_t st_rank_sym4(int64_t n, int64_t i, int64_t j, int64_t k, int64_t l);
int64_t st_rank_band(int64_t n, int64_t w, int64_t i, int64_t j);

/* Inverse maps.  ST_ERR_SHAPE if p is outside [0, count); ST_ERR_NULL for a
 * NULL result pointer. */
st_status st_unrank_sym2(int64_t n, int64_t p, int64_t *i, int64_t *j);
st_status st_unrank_sym3(int64_t n, int64_t p, int64_t *i, int64_t *j, int64_t *k);
st_status st_unrank_sym4(int64_t n, int64_t p, int64_t *i, int64_t *j, int64_t *k, int64_t *l);
st_status st_unrank_band(int64_t n, int64_t w, int64_t p, int64_t *i, int64_t *j);

/* Batched inverse maps on the host: tuples of positions p0 .. p0+count-1
 * written to HOST memory `out` as int32, 2 (sym2, band), 3 (sym3) or 4 (sym4)
 * per position. */
st_status st_unrank_sym2_batch(int64_t n, int64_t p0, int64_t count, int32_t *out);
st_status st_unrank_sym3_batch(int64_t n, int64_t p0, int64_t count, int32_t *out);
st_status st_unrank_sym4_batch(int64_t n, int64_t p0, int64_t count, int32_t *out);
st_status st_unrank_band_batch(int64_t n, int64_t w, int64_t p0, int64_t count, int32_t *out);

/* The same inverse maps evaluated by the DEVICE code the kernels use (the
 * kernels turn a flat position into indices with these, instead of masks).
 * `out` is a DEVICE pointer to 2*count (kind 2: sym2, kind 4: band, with
 * w), 3*count (kind 3: sym3) or 4*count (kind 5: sym4) int32.  For checking the
 * device index maps. */
st_status st_unrank_device(int kind, int64_t n, int64_t w, int64_t p0, int64_t count,
                           int32_t *out, void *stream);

/* ---- workspace queries (bytes; 0 means ws may be NULL) -------------------- */
size_t st_mttkrp_sym3_workspace(int n, int R);
size_t st_batax_utri_workspace(int n);
size_t st_ttm_band_workspace(int n, int w, int nl, int R);
size_t st_moment3_sym_workspace(int64_t N, int n);
size_t st_moment2_sym_workspace(int64_t N, int n);
size_t st_moment4_sym_workspace(int64_t N, int n);
size_t st_ttm_struct_workspace(int structure, int ni, int nj, int nl, int R);
size_t st_mttkrp_fixed_workspace(int kind, int ni, int nk, int nl, int R);

/* ---- kernels -------------------------------------------------------------- */

/* MTTKRP with a fully symmetric order-3 tensor and equal factors:
 *     M(i,r) = sum_{j,k} T(i,j,k) * B(j,r) * B(k,r)        0<=i<n, 0<=r<R
 * (kernel table, MTTKRP row  A(i,j) := B(i,k,l) * C(k,j) * D(l,j)  with
 * C = D; structure from "Tensor Structures").  Only the unique entries are
 * read: Tc holds the n(n+1)(n+2)/6 sym3-packed values of T; the sum still
 * ranges over the FULL symmetric tensor (each stored entry stands for its 1,
 * 3 or 6 index permutations).  B is n x R, M is n x R, overwritten.
 * n >= 1, R >= 1. */
st_status st_mttkrp_sym3(const float *Tc, const float *B, float *M, int n, int R,
                         void *ws, size_t ws_bytes, void *stream);

/* y = beta * A^T (A x) for an upper-triangular A, A(i,j) = 0 for i > j
 * (unique set 0<=i<=j<n of the upper-triangular compressed-tensor example;
 * matrix-vector products as sum-of-products rules).  Ap holds the n(n+1)/2
 * sym2-packed entries of A, x and y have n entries, y is overwritten.  A is
 * streamed from memory once for n <= 16384 (a row stays on chip between its
 * two uses), twice beyond.  1 <= n <= 65000. */
st_status st_batax_utri(const float *Ap, const float *x, float *y, int n, float beta,
                        void *ws, size_t ws_bytes, void *stream);

/* st_batax_utri for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bit-identical results;
 * the per-workgroup partial results go to a static device array of the library
 * (8 MiB per GPU, held until the process ends) instead of `ws`, and the call
 * allocates nothing.  n <= st_batax_utri_noalloc_max_n() = 8192
 * (ST_ERR_UNSUPPORTED beyond).  All calls on one GPU share that array: calls
 * that overlap in time on the same GPU (different streams or threads) race and
 * give undefined results; calls ordered on one stream are fine. */
int st_batax_utri_noalloc_max_n(void);
st_status st_batax_utri_noalloc(const float *Ap, const float *x, float *y, int n, float beta,
                                void *stream);

/* Tensor-times-matrix along mode 3 of a band tensor:
 *     Y(i,j,r) = sum_l T(i,j,l) * U(l,r)   for |i-j| <= w, zero elsewhere
 * (kernel table, TTM row  A(i,j,k) := B(i,j,l) * C(k,l)  with U(l,r) =
 * C(r,l); w = 0 is the table's "diagonal plane" structure; the output keeps
 * the input's unique set by the product and projection inference rules).
 * Tc is [st_count_band(n,w)][nl], U is nl x R, Yc is
 * [st_count_band(n,w)][R] in the same band order, overwritten.
 * n >= 1, w >= 0 (clamped to n-1), nl >= 1, R >= 1. */
st_status st_ttm_band(const float *Tc, const float *U, float *Yc, int n, int w, int nl,
                      int R, void *ws, size_t ws_bytes, void *stream);

/* Third-moment (degree-3 interaction) accumulation over N samples:
 *     Sc(rank3(i,j,k)) (+)= sum_s X(s,i) * X(s,j) * X(s,k)    for i<=j<=k
 * (the M2 = f (x) vec(f (x) f) term of the degree-2 polynomial-regression
 * covariance, summed over the data: "creation and addition of covariance
 * matrices").  X is N x n row-major.  accumulate = 0 overwrites Sc, 1 adds to
 * it.  Raw sums: no 1/N, no centring.  N >= 0 (N = 0 zero-fills when
 * accumulate = 0), n >= 1.  The workspace can be large (64 < n <= 256: a tile
 * table and the partial sums of every sample slice, up to 2 GB; ask
 * st_moment3_sym_workspace); for those n a small kernel copies the table
 * into it at every call. */
st_status st_moment3_sym(const float *X, int64_t N, int n, float *Sc, int accumulate,
                         void *ws, size_t ws_bytes, void *stream);

/* Second-moment accumulation over N samples, upper half only:
 *     Sc(rank2(i,j)) (+)= sum_s X(s,i) * X(s,j)    for i<=j
 * (the M1 = f (x) f term of the same covariance; its structure is plain
 * symmetry).  Arguments as for st_moment3_sym; Sc has n(n+1)/2 entries.  Up to
 * 1024 features the sum runs on the matrix cores; the workspace holds slice
 * partials (about 50 MB; more only for N in the tens of millions at several
 * hundred features: a slice ends after 131,072 samples).  Between 65 and 1024
 * features N is limited to 2^31 - 1 (ST_ERR_UNSUPPORTED beyond; such an X would
 * be more than half a terabyte). */
st_status st_moment2_sym(const float *X, int64_t N, int n, float *Sc, int accumulate,
                         void *ws, size_t ws_bytes, void *stream);

/* Fourth-moment accumulation over N samples, unique entries only:
 *     Sc(rank4(i,j,k,l)) (+)= sum_s X(s,i) * X(s,j) * X(s,k) * X(s,l)   for i<=j<=k<=l
 * (the M3 = vec(f (x) f) (x) vec(f (x) f) term of the same covariance: about 23 of
 * every 24 dense entries are redundant).  Arguments as for st_moment3_sym; Sc has
 * st_count_sym4(n) entries; n <= 256.  For n >= 56 the workspace holds a tile
 * table (copied in by a small kernel at every call) and slice partials, up to
 * about 2 GB. */
st_status st_moment4_sym(const float *X, int64_t N, int n, float *Sc, int accumulate,
                         void *ws, size_t ws_bytes, void *stream);

/* Covariance of degree-2 polynomial regression over N samples, creation and
 * addition, in the semi-ring form of the end-to-end experiment: the degree-2,
 * degree-3 and degree-4 interaction terms M1 = f (x) f, M2 = f (x) vec(f (x) f)
 * and M3 = vec(f (x) f) (x) vec(f (x) f) are kept apart, each with its unique
 * entries only (for n = 4 features: 10 + 20 + 35 = 65 values instead of 400).
 * One call = st_moment2_sym, st_moment3_sym and st_moment4_sym on the same X,
 * enqueued on `stream` in that order with one shared workspace
 * (st_covar_pr2_workspace); with at most sixteen features all three terms
 * come from ONE pass over X (same results within rounding, its own summation
 * order).  S1, S2, S3 have st_count_sym2/3/4(n) entries; n <= 256. */
size_t st_covar_pr2_workspace(int64_t N, int n);
st_status st_covar_pr2(const float *X, int64_t N, int n, float *S1, float *S2, float *S3, int accumulate,
                       void *ws, size_t ws_bytes, void *stream);

/* Reconstruction through the redundancy map (Property 5:
 * T(x) = T_C(x) + T_R(x,x') * T_C(x')).  order 2: S(i,j) = Sc[rank2(min,max)]
 * (class S: i' = j, j' = i for j < i); order 3: S(i,j,k) = Sc[rank3(sorted
 * triple)]; order 4: S(i,j,k,l) = Sc[rank4(sorted quadruple)] (n <= 256).  S is
 * the dense n^order array, overwritten.  A bit-exact copy. */
st_status st_expand_sym(const float *Sc, float *S, int n, int order, void *stream);

/* ---- the sparsity structures of the paper's kernel table -------------------
 *
 * The table evaluates TTM, THP and MTTKRP with an order-3 operand B(i,j,l)
 * whose unique set restricts the index pair (i,j) and leaves l free.  Packed,
 * such an operand is a list of its non-zero fibres B(i,j,:), `nl` contiguous
 * values each, in the order of the table's unique set (i outer, j inner):
 *   ST_STRUCT_DIAG    "diagonal (plane)", i = j:   fibre p is (p,p), min(ni,nj) fibres
 *   ST_STRUCT_FIXED_I "fixed i",  i = I:           fibre p is (I,p), nj fibres
 *   ST_STRUCT_FIXED_J "fixed j",  j = J:           fibre p is (p,J), ni fibres
 *   ST_STRUCT_UPPER   "upper half cube", i <= j:   fibre p is the p-th sym2 pair,
 *                     ni = nj required, ni(ni+1)/2 fibres
 */
enum { ST_STRUCT_DIAG = 0, ST_STRUCT_FIXED_I = 1, ST_STRUCT_FIXED_J = 2, ST_STRUCT_UPPER = 3 };

/* Number of non-zero fibres of a structure; -1 for an unknown structure, a
 * negative size, or ni != nj with ST_STRUCT_UPPER. */
int64_t st_count_struct(int structure, int64_t ni, int64_t nj);

/* TTM of the kernel table,  A(i,j,k) := B(i,j,l) * C(k,l),  U(l,k) = C(k,l):
 *     Ac(p,r) = sum_l Bc(p,l) * U(l,r)      for every non-zero fibre p of B
 * The output keeps the unique set of B (product and projection inference
 * rules) and is packed the same way: Bc is [fibres][nl], U is nl x R, Ac is
 * [fibres][R], overwritten.  The value of a fixed index does not enter. */
st_status st_ttm_struct(int structure, const float *Bc, const float *U, float *Ac, int ni, int nj,
                        int nl, int R, void *ws, size_t ws_bytes, void *stream);

/* THP of the kernel table,  A(i,j,k) := B(i,j,k) * C(i,j,k):
 *     Ac(p,l) = Bc(p,l) * C(i(p), j(p), l)
 * B is packed ([fibres][nl]); C is a DENSE ni x nj x nl tensor of which only
 * the fibres inside the unique set of B are read; Ac is packed like Bc,
 * overwritten.  `fixed` is the value I or J of the fixed index (ignored for
 * the other structures; ST_ERR_SHAPE if out of range). */
st_status st_thp_struct(int structure, const float *Bc, const float *C, float *Ac, int ni, int nj,
                        int nl, int fixed, void *stream);

/* MTTKRP of the kernel table,  A(i,r) := B(i,k,l) * C(k,r) * D(l,r),  with
 * indices of B fixed (the table names the positions of B (i,j,l): its
 * "fixed j" is the contracted index k here):
 *   ST_MTTKRP_FIXED_IK "fixed i, j": B(I,K,:) only.  Bc is [nl], A is [R] (row I
 *                      of the result, every other row is zero):
 *                      A(r) = C(K,r) * sum_l Bc(l) D(l,r)
 *   ST_MTTKRP_FIXED_I  "fixed i": B(I,:,:) only.  Bc is [nk][nl], A is [R]:
 *                      A(r) = sum_k C(k,r) * sum_l Bc(k,l) D(l,r)
 *   ST_MTTKRP_FIXED_K  "fixed j": B(:,K,:) only.  Bc is [ni][nl], A is [ni][R]:
 *                      A(i,r) = C(K,r) * sum_l Bc(i,l) D(l,r)
 * C is nk x R, D is nl x R; `fixed_k` selects the row of C (ignored for
 * ST_MTTKRP_FIXED_I; ST_ERR_SHAPE if outside [0, nk)). */
enum { ST_MTTKRP_FIXED_IK = 0, ST_MTTKRP_FIXED_I = 1, ST_MTTKRP_FIXED_K = 2 };
st_status st_mttkrp_fixed(int kind, const float *Bc, const float *C, const float *D, float *A, int ni,
                          int nk, int nl, int R, int fixed_k, void *ws, size_t ws_bytes, void *stream);

/* Zero-filled dense form of a packed band tensor (Property 5 restricted to a
 * sparsity structure: T = T_C on the unique set, zero elsewhere):
 *     T(i,j,l) = Tc(rank_band(i,j), l) if |i-j| <= w, else 0
 * Tc is [st_count_band(n,w)][nl], T is n x n x nl, overwritten. */
st_status st_expand_band(const float *Tc, float *T, int n, int w, int nl, void *stream);

/* ---- descriptor-driven structures -------------------------------------------
 *
 * The paper describes a structure by a unique set T_U (a product of
 * comparisons over the index variables) and a redundancy map T_R, and derives
 * loop nests from them: variables in the order written, each from the maximum
 * of its lower bounds to the minimum of its upper bounds (code generation
 * section).  These entry points do that at run time for a descriptor given as
 * text, and run kernels generated and compiled (hiprtc) for that descriptor.
 *
 *   unique_set   "T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)"
 *                NAME(variables): factors joined by '*'; a factor is a chain of
 *                comparisons (<=, <, =, >=, >) of affine expressions over the
 *                variables, the named parameters and integers.  Every
 *                comparison bounds the LAST variable it mentions, which must
 *                have coefficient 1 or -1 there (ST_ERR_UNSUPPORTED otherwise).
 *   redundancy   NULL / "" (none: a sparsity structure, zero elsewhere), "sort"
 *                (all permutations of a stored tuple hold its value; equal
 *                sizes), or terms "(condition factors) -> (e0,e1,..)" joined by
 *                ';': a dense index meeting the condition takes the value
 *                stored at the unique index (e0,e1,..), e.g. "(0<=j<i<n) -> (j,i)".
 *   dims[v]      dense extent of variable v (0 <= x_v < dims[v] always holds);
 *                param_names/values bind the other names of the text.
 *
 * Packed layout: visiting order of the derived nest, last variable fastest.
 * The host object is created without a GPU; the device kernels need the
 * table (st_desc_table_bytes / st_desc_table: HOST buffer to be copied to the
 * device by the caller, 16-byte aligned there) and compile on first use.
 * On a parse error st_desc_create still returns an object whose
 * st_desc_error() says what was wrong; destroy it like any other.
 * A redundancy term whose condition holds for a stored entry is an error
 * (ST_ERR_SHAPE): the unique set and the redundancy map must be disjoint
 * (Property 1 of the semantics, T_U * T_R is empty).
 */
typedef struct st_desc st_desc;
st_status st_desc_create(const char *unique_set, const char *redundancy, const int64_t *dims, int ndims,
                         const char *const *param_names, const int64_t *param_values, int nparams,
                         st_desc **out);
void st_desc_destroy(st_desc *desc);
const char *st_desc_error(const st_desc *desc);
int64_t st_desc_count(const st_desc *desc);         /* entries of the unique set                     */
int64_t st_desc_runs(const st_desc *desc);          /* non-empty innermost runs                      */
const char *st_desc_nest(const st_desc *desc);      /* the derived loop nest, as text                */
const char *st_desc_source(const st_desc *desc);    /* the generated HIP source                      */
size_t st_desc_table_bytes(const st_desc *desc);
st_status st_desc_table(const st_desc *desc, void *host_out);
st_status st_desc_compile(st_desc *desc);           /* compile the source for gfx950 (no GPU needed) */

/* Generated kernels; `table` is the DEVICE copy of st_desc_table.
 * st_desc_list: out[p][v] = value of variable v at packed position p (int32,
 *   st_desc_count x order).
 * st_desc_thp: Ac(p) = Bc(p) * C(x(p)) over the unique set, C dense (the
 *   kernel table's THP for any structure).
 * st_desc_expand: T(x) = Tc(rank(x)) on the unique set, the value of the
 *   unique index given by the redundancy map elsewhere, 0 where neither
 *   applies (Property 5). */
st_status st_desc_list(st_desc *desc, const void *table, int32_t *out, void *stream);
st_status st_desc_thp(st_desc *desc, const void *table, const float *Bc, const float *C, float *Ac,
                      void *stream);
st_status st_desc_expand(st_desc *desc, const void *table, const float *Tc, float *T, void *stream);

/* The kernel table's MTTKRP for ANY sparsity structure of an order-3 operand
 * ("Tensor Kernels": A(i,j) := B(i,k,l) * C(k,j) * D(l,j)), evaluated over the
 * unique set only:
 *     A(x0, r) = sum over the stored (x1, x2) of row x0 of Bc(rank(x)) * C(x1, r) * D(x2, r)
 * Bc is the packed operand (st_desc_count floats), C is dims[1] x R, D is
 * dims[2] x R, A is dims[0] x R (all row-major, DEVICE, 16-byte aligned; rows
 * of A without a stored entry are written as zeros).  Two routes, chosen by
 * the structure: when it leaves the LAST variable free (every run is a whole
 * fibre: diagonal plane, fixed index, band or upper half on (i,k)) the
 * contraction over l runs on the matrix cores through the kernels of
 * st_ttm_band into Y(run, r) in the workspace, and a generated kernel adds
 * C(x1, r) * Y(run, r) over the runs of every row; otherwise a generated
 * vector-ALU kernel, one workgroup per output row and 16 columns.  Sums in a
 * fixed order either way.  st_desc_mttkrp_workspace is 0 for the second route
 * (ws may be NULL then).  ST_ERR_UNSUPPORTED for orders other than 3 and for
 * descriptors with a redundancy map (their operand has entries outside the
 * unique set; the fully symmetric case is st_mttkrp_sym3). */
size_t st_desc_mttkrp_workspace(const st_desc *desc, int R);
st_status st_desc_mttkrp(st_desc *desc, const void *table, const float *Bc, const float *C, const float *D,
                         float *A, int R, void *ws, size_t ws_bytes, void *stream);

/* Structure inference for an element-wise product  A(x) := M(x) * V(x)  of two
 * structured operands of the same shape ("Structure Inference", general rule for
 * products):  A_U = M_U*V_U + M_U*V_R + M_R*V_U,  A_R = M_R*V_R, followed by the
 * logical simplification: summands whose comparisons contradict each other are
 * empty and drop out.  The result is a new descriptor (packed layout = its own
 * derived nest).  E.g. upper-triangular times symmetric gives the upper
 * triangle with no redundancy (the paper's UHS walk-through); symmetric times
 * symmetric stays symmetric.  ST_ERR_UNSUPPORTED when more than one summand of
 * A_U survives (a descriptor holds one product of comparisons), for 'sort'
 * maps of order above 2, or when two surviving redundancy terms disagree.
 * The object is returned on failure too (st_desc_error says why).
 * Destroy it like any other descriptor. */
st_status st_desc_product(const st_desc *m, const st_desc *v, st_desc **out);

/* Values of a structured tensor at a LIST of dense positions, times an
 * optional factor per position:
 *     out[p] = (scale ? scale[p] : 1) * T(idx[p][0], .., idx[p][order-1]) + (addend ? addend[p] : 0)
 * with T(x) the stored value on the unique set, the value at the unique index
 * the redundancy map names elsewhere, 0 where neither applies or x lies
 * outside the dense extents (Property 5, evaluated only where asked).  idx is
 * DEVICE int32 with `idx_stride` ints per position, of which the `order` ints
 * from `idx_offset` on are the position (idx_stride = order, idx_offset = 0
 * for a plain [count][order] list such as st_desc_list gives; an outer
 * product reads the two halves of its own list: ST_ERR_SHAPE unless
 * 0 <= idx_offset and idx_offset + order <= idx_stride <= 64).  Tc is the
 * packed operand of `desc`, scale and addend NULL or DEVICE fp32 [count]
 * (either may be `out` itself: element p is read before out[p] is written, by
 * the same thread).  Two calls
 * evaluate a product of two structured operands on the unique set of the
 * result only:  A_C = gather(V, list(A), scale = gather(M, list(A))). */
st_status st_desc_gather(st_desc *desc, const void *table, const float *Tc, const int32_t *idx, int64_t count,
                         int idx_stride, int idx_offset, const float *scale, const float *addend, float *out,
                         void *stream);

/* Structure inference for a sum  A(x) := M(x) + V(x)  of two structured operands
 * of the same shape ("Unique Set Inference": the unique set of a sum is the
 * union; "Redundancy Map Inference": operands of the same structure keep it,
 * otherwise every non-zero element of an operand, unique or redundant, counts
 * as stored and the result has no redundancy map).  The union has to be one
 * nest: the unique set of an operand without a redundancy map, or the whole
 * box; each candidate is checked point by point against the union of the two
 * supports (box of at most 2^26 elements).  E.g. diagonal + upper triangular
 * is upper triangular, symmetric + symmetric stays symmetric, symmetric +
 * upper triangular is the whole box.  ST_ERR_UNSUPPORTED otherwise (band +
 * a row: a sum of nests).  Values: out = gather(V, list(A), addend =
 * gather(M, list(A))). */
st_status st_desc_sum(const st_desc *m, const st_desc *v, st_desc **out);

/* Marginalization of the LAST variable,  A(x_0..x_{d-2}) := sum over x_{d-1} of
 * B(x)  (a rule whose head leaves a variable of the body out sums over it;
 * "Unique Set Inference", projection: the output is non-zero wherever some
 * value of the dropped variable is stored).  st_desc_project infers the
 * descriptor of A: the bounds of the earlier variables plus, for every pair
 * (lower bound, upper bound) of the dropped variable, the comparison
 * lower <= upper -- exact for the affine integer bounds descriptors have.
 * Its packed order is the run order of B, so st_desc_sum_last(B) writes the
 * packed values of A: out[run] = sum of the entries of the run (DEVICE fp32,
 * st_desc_runs(B) = st_desc_count(A) values, fixed summation order).  The
 * output structure of the kernel table's TTM is
 * st_desc_outer(st_desc_project(B), <range of k>).  ST_ERR_UNSUPPORTED for
 * operands with a redundancy map. */
st_status st_desc_project(const st_desc *b, st_desc **out);
st_status st_desc_sum_last(st_desc *desc, const void *table, const float *Bc, float *out, void *stream);

/* Structure inference for the tensor outer product  T(x, y) := M(x) * V(y)
 * over disjoint index lists, the variables of V behind those of M, total order
 * at most 4 ("Redundancy Map Inference", outer-product rule):
 *     T_U = M_U * V_U,   T_R = M_U * V_R + M_R * V_U + M_R * V_R
 * ('sort' maps of order 2 enter as the class-S term; of higher order:
 * ST_ERR_UNSUPPORTED).  The values on T_U are two st_desc_gather calls on the
 * two halves of st_desc_list(T). */
st_status st_desc_outer(const st_desc *m, const st_desc *v, st_desc **out);

/* Structure inference for the k-fold outer product of a VECTOR with itself,
 * T(x_1..x_k) := v(x_1) * .. * v(x_k), k = 2..4 (the self-multiplication rule
 * and its extension to higher degrees; the vector self-outer-product
 * example): the unique set is v's range on every index and
 * x_1 <= x_2 <= .. <= x_k, the redundancy map is `sort`.  These are the
 * structures of the covariance terms M1, M2, M3 ("Tensor Structures"); with
 * st_desc_moment they give the accumulation over samples.  ST_ERR_UNSUPPORTED
 * for descriptors of order above 1 or with a redundancy map. */
st_status st_desc_power(const st_desc *v, int k, st_desc **out);

/* Structure inference for the direct sum  T := M (+) V  of two operands of the
 * same order ("Redundancy Map Inference", direct-sum rule; "Representation of
 * linear algebra operations", the rule for (+)): with d = dims(M), T has
 * dims(M) + dims(V) on every index and
 *     T_U(x)     = M_U(x) + V_U(y) * (y = x - d),
 *     T_R(x, x') = M_R(x, x') + V_R(y, y') * (y = x - d) * (y' = x' - d).
 * The two summands lie in disjoint boxes, so T_U is a sum of two nests; as in
 * the code generation of the paper every summand gets a nest of its own, and
 * each is returned as an ordinary descriptor over the box of T: *out_m is the
 * structure of M inside that box, *out_v the structure of V moved by d (every
 * bound, condition and map of V read at x - d).  The packed array of T is M_C
 * followed by V_C: each part keeps the packed order of its operand.  The dense
 * T is st_desc_expand of the first part and st_desc_expand_onto of the second
 * on the same array; every other call works on a part as on any descriptor.
 * Both outputs are NULL on ST_ERR_NULL / ST_ERR_SHAPE (different orders);
 * otherwise *out_m is always set and *out_v once *out_m has succeeded; a
 * failed one still has to be destroyed (st_desc_error tells why). */
st_status st_desc_direct_sum(const st_desc *m, const st_desc *v, st_desc **out_m, st_desc **out_v);

/* st_desc_expand that writes ONLY the elements the structure holds (stored, or
 * reached through its redundancy map) and leaves every other element of the
 * dense array T as it was: lays one summand of a sum of nests over what the
 * previous summands wrote.  Arguments, alignment and errors as st_desc_expand. */
st_status st_desc_expand_onto(st_desc *desc, const void *table, const float *Tc, float *T, void *stream);

/* Moment accumulation over the unique set of a descriptor of order 2 or 3 whose
 * variables all range over the n <= 256 features of X (N x n, row-major):
 *     Sc(rank(x)) (+)= sum_s prod_v X(s, x_v)       for every x in the unique set
 * (creation and addition of a covariance term for ANY structure: st_moment2_sym
 * and st_moment3_sym are the cases i<=j and i<=j<=k; a band i<=j<=i+w keeps only
 * the interactions of neighbouring features, and so on).  Generated kernels on
 * the vector ALUs.  accumulate = 0 overwrites Sc (st_desc_count entries), 1 adds;
 * ws of st_desc_moment_workspace(desc, N) bytes.  ST_ERR_UNSUPPORTED for other
 * orders or unequal extents. */
size_t st_desc_moment_workspace(const st_desc *desc, int64_t N);
st_status st_desc_moment(st_desc *desc, const void *table, const float *X, int64_t N, float *Sc,
                         int accumulate, void *ws, size_t ws_bytes, void *stream);

/* TTM of the kernel table along the LAST variable of a descriptor that leaves it
 * free (every run is a whole fibre, e.g. any structure on (i,j) of B(i,j,l)):
 *     Ac(run, r) = sum_l Bc(run, l) * U(l, r)
 * Bc is [st_desc_runs][dims[last]], U is dims[last] x R, Ac is [st_desc_runs][R]:
 * the output keeps the structure of the other variables (product and projection
 * inference rules).  Runs on the matrix cores through the kernels of st_ttm_band;
 * ST_ERR_UNSUPPORTED when the last variable is bounded by the structure. */
st_status st_desc_ttm(st_desc *desc, const float *Bc, const float *U, float *Ac, int R, void *stream);

/* ---- measurement support (no computation) -----------------------------------
 *
 * The floors a short call is judged against: an empty launch of `grid`
 * workgroups of `block` threads, and a plain streaming read of `bytes` bytes
 * at DEVICE pointer `src` in that launch shape (16-byte loads, every byte
 * once, at most 32 loads per thread: ST_ERR_UNSUPPORTED beyond; `sink` is a
 * DEVICE float the kernel never writes in practice).  The benchmark times
 * them beside the kernels so that a kernel time can be split into launch,
 * memory and the rest. */
st_status st_probe_empty(int grid, int block, void *stream);
st_status st_probe_stream(const void *src, size_t bytes, int grid, int block, float *sink, void *stream);

/* The matrix-core floor of the single-precision kernels: 256 workgroups of 512
 * threads (two waves per SIMD) repeat `iters` times a block of `valu` (0, 9 or
 * 13: ST_ERR_SHAPE otherwise) cross-lane vector multiplies followed by 23
 * independent 16x16x4 single-precision MFMAs on register operands, i.e.
 * 256 * 8 * iters * 23 * 2048 flops on the matrix cores.  9 multiplies per 23
 * MFMAs is the instruction mix of the third-moment kernel on its busiest
 * SIMDs (every pair product formed once per K-step and workgroup); 13 is what
 * it was before the tiles were dealt by product.  `sink` is a DEVICE buffer
 * of 256 * 512 floats, overwritten. */
st_status st_probe_mfma_f32(int valu, int iters, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* STRUCTTENSOR_H */
