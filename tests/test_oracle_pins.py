"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- values the paper prints, closed forms, library routines on
independently built dense tensors, special cases and invariants."""
import itertools
import math
import os

import numpy as np
import pytest

import st_workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_counts.txt")


def golden():
    out = {}
    with open(GOLD) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                out[line[0]] = int(line[1])
    return out


# ------------------------------------------------------------------ counts
def test_counts_closed_forms(oracle):
    for n in list(range(0, 41)) + [64, 100]:
        assert oracle.count_sym2(n) == math.comb(n + 1, 2)
        assert oracle.count_sym3(n) == math.comb(n + 2, 3)
    for n in range(0, 25):
        assert oracle.count_sym4(n) == math.comb(n + 3, 4)
    assert oracle.count_sym3(512) == 22_500_864
    assert oracle.count_sym3(64) == 45_760
    assert oracle.count_sym2(8192) == 33_558_528
    assert oracle.count_sym2(64) == 2_080


def test_counts_paper_values(oracle):
    g = golden()
    n = 4
    assert n + n * n == g["pr2_matrix_dim_n4"]
    assert (oracle.count_sym2(n) + oracle.count_sym3(n) + oracle.count_sym4(n)
            == g["pr2_distinct_elements_n4"])
    n = 400
    r3 = (n ** 3 - oracle.count_sym3(n)) / oracle.count_sym3(n)
    assert abs(r3 - g["m2_redundant_over_unique"]) < 0.05
    n = 120
    r4 = (n ** 4 - oracle.count_sym4(n)) / oracle.count_sym4(n)
    assert abs(r4 - g["m3_redundant_over_unique"]) < 1.2 and r4 < 23
    n = 2000
    assert abs(n * n / oracle.count_sym2(n) - g["utri_fraction_inverse"]) < 0.01


def test_band_counts(oracle):
    for n in (1, 2, 5, 9, 33):
        assert oracle.count_band(n, 0) == n
        assert oracle.count_band(n, n - 1) == n * n
        assert oracle.count_band(n, n + 7) == n * n
        for w in range(0, n):
            i, j = np.indices((n, n))
            assert oracle.count_band(n, w) == int((np.abs(i - j) <= w).sum())
    assert oracle.count_band(512, 8) == 8_632


# -------------------------------------------------------------- enumeration
@pytest.mark.parametrize("n", [1, 2, 3, 7, 16, 21])
def test_sym_tables_are_lexicographic(oracle, n):
    combos3 = list(itertools.combinations_with_replacement(range(n), 3))
    tab3 = oracle.table_sym3(n)
    lst3 = oracle.list_sym3(n)
    assert lst3.shape == (len(combos3), 3)
    assert [tuple(int(v) for v in t) for t in lst3] == combos3
    for p, (i, j, k) in enumerate(combos3):
        assert tab3[i, j, k] == p
    assert int((tab3 >= 0).sum()) == len(combos3)
    combos2 = list(itertools.combinations_with_replacement(range(n), 2))
    tab2 = oracle.table_sym2(n)
    assert [tuple(int(v) for v in t) for t in oracle.list_sym2(n)] == combos2
    for p, (i, j) in enumerate(combos2):
        assert tab2[i, j] == p
    assert int((tab2 >= 0).sum()) == len(combos2)
    # numpy's own row-major upper-triangle order is the same packing
    iu = np.triu_indices(n)
    assert np.array_equal(tab2[iu], np.arange(len(combos2)))


@pytest.mark.parametrize("n,w", [(1, 0), (4, 0), (4, 1), (7, 2), (7, 6), (12, 3), (12, 20)])
def test_band_table(oracle, n, w):
    i, j = np.indices((n, n))
    mask = np.abs(i - j) <= w
    expect = np.argwhere(mask)              # row-major order
    got = oracle.list_band(n, w)
    assert np.array_equal(got, expect)
    tab = oracle.table_band(n, w)
    assert np.array_equal(tab[mask], np.arange(expect.shape[0]))
    assert np.all(tab[~mask] == -1)


# ---------------------------------------------------------- materialisation
def _dense_sym3_numpy(Tc, n):
    T = np.zeros((n, n, n))
    for p, (i, j, k) in enumerate(itertools.combinations_with_replacement(range(n), 3)):
        for a, b, c in set(itertools.permutations((i, j, k))):
            T[a, b, c] = float(Tc[p])
    return T


@pytest.mark.parametrize("n", [1, 3, 6, 9])
def test_dense_sym3(oracle, n):
    Tc = W.uniform(11, math.comb(n + 2, 3))
    T = oracle.dense_sym3(Tc, n)
    assert np.array_equal(T, _dense_sym3_numpy(Tc, n))
    for perm in itertools.permutations(range(3)):
        assert np.array_equal(T, np.transpose(T, perm))


# --------------------------------------------------------------------- mttkrp
@pytest.mark.parametrize("n,R", [(1, 1), (2, 3), (5, 4), (8, 16), (13, 5)])
def test_mttkrp_against_einsum(oracle, n, R):
    Tc = W.uniform(21, math.comb(n + 2, 3))
    B = W.uniform(22, n * R).reshape(n, R)
    T = _dense_sym3_numpy(Tc, n)
    ref = np.einsum("ijk,jr,kr->ir", T, B.astype(np.float64), B.astype(np.float64))
    got = oracle.mttkrp_sym3(Tc, B)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-13)
    # mode invariance: contracting modes (1,3) or (1,2) gives the same M
    ref2 = np.einsum("jik,jr,kr->ir", T, B.astype(np.float64), B.astype(np.float64))
    assert np.allclose(got, ref2, rtol=1e-13, atol=1e-13)
    rows = np.array([n - 1, 0, n // 2])
    assert np.array_equal(oracle.mttkrp_sym3(Tc, B, rows=rows), got[rows])


def test_mttkrp_special_cases(oracle):
    n, R = 9, 4
    B = W.uniform(31, n * R).reshape(n, R).astype(np.float64)
    ones = np.ones(math.comb(n + 2, 3), dtype=np.float32)
    M = oracle.mttkrp_sym3(ones, B)
    assert np.allclose(M, np.tile(B.sum(axis=0) ** 2, (n, 1)), rtol=1e-13)
    # rank one: T = a (x) a (x) a  =>  M(i,r) = a_i (a^T b_r)^2, with a exact in fp32
    a = np.array([1, -2, 0.5, 3, 0, -1, 2, 0.25, -4], dtype=np.float64)
    lst = oracle.list_sym3(n)
    Tc = (a[lst[:, 0]] * a[lst[:, 1]] * a[lst[:, 2]]).astype(np.float32)
    M = oracle.mttkrp_sym3(Tc, B)
    assert np.allclose(M, np.outer(a, (a @ B) ** 2), rtol=1e-12, atol=1e-12)


def test_mttkrp_weight_sum(oracle):
    # multiplicities of the packed entries (1, 3 or 6 index permutations) add up to n^3:
    # with B = ones(n,1), sum_i M(i,0) = sum over the full tensor.
    n = 10
    Tc = W.uniform(41, math.comb(n + 2, 3))
    B = np.ones((n, 1), dtype=np.float32)
    M = oracle.mttkrp_sym3(Tc, B)
    mult = np.array([len(set(itertools.permutations(t)))
                     for t in itertools.combinations_with_replacement(range(n), 3)])
    assert mult.sum() == n ** 3
    assert np.isclose(M.sum(), float((mult * Tc.astype(np.float64)).sum()), rtol=1e-12)


# ---------------------------------------------------------------------- batax
@pytest.mark.parametrize("n", [1, 2, 5, 33, 100])
def test_batax_against_numpy(oracle, n):
    Ap = W.uniform(51, math.comb(n + 1, 2))
    x = W.uniform(52, n)
    A = np.zeros((n, n))
    A[np.triu_indices(n)] = Ap
    assert np.array_equal(oracle.dense_utri(Ap, n), A)
    beta = 0.5
    ref = beta * (A.T @ (A @ x.astype(np.float64)))
    got = oracle.batax_utri(Ap, x, beta)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-13)
    assert np.isclose(x.astype(np.float64) @ got, beta * np.sum((A @ x.astype(np.float64)) ** 2))


def test_batax_special_cases(oracle):
    n = 17
    x = W.uniform(53, n)
    eye = np.zeros((n, n))
    eye[np.diag_indices(n)] = 1
    Ap = eye[np.triu_indices(n)].astype(np.float32)
    assert np.allclose(oracle.batax_utri(Ap, x, 0.75), 0.75 * x.astype(np.float64), rtol=1e-15)
    ones = np.ones(math.comb(n + 1, 2), dtype=np.float32)
    t = np.cumsum(x.astype(np.float64)[::-1])[::-1]        # suffix sums
    y = 2.0 * np.cumsum(t)                                 # prefix sums of t
    assert np.allclose(oracle.batax_utri(ones, x, 2.0), y, rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------------ ttm
@pytest.mark.parametrize("n,w,nl,R", [(1, 0, 1, 1), (4, 1, 3, 2), (7, 2, 5, 4), (9, 8, 6, 3), (6, 0, 8, 5)])
def test_ttm_against_numpy(oracle, n, w, nl, R):
    i, j = np.indices((n, n))
    mask = np.abs(i - j) <= w
    nb = int(mask.sum())
    Tc = W.uniform(61, nb * nl).reshape(nb, nl)
    U = W.uniform(62, nl * R).reshape(nl, R)
    T = np.zeros((n, n, nl))
    T[mask] = Tc                               # row-major band order
    assert np.array_equal(oracle.dense_band(Tc, n, w, nl), T)
    ref = T @ U.astype(np.float64)
    Y = oracle.ttm_dense(Tc, U, n, w)
    assert np.allclose(Y, ref, rtol=1e-13, atol=1e-13)
    assert np.all(Y[~mask] == 0.0)             # output keeps the input's band
    Yc = oracle.ttm_band(Tc, U, n, w)
    assert np.array_equal(Yc, Y[mask])
    if w >= n - 1:                             # no structure left: a plain GEMM
        assert np.allclose(Yc, Tc.astype(np.float64) @ U.astype(np.float64), rtol=1e-13)


def test_ttm_identity_factor(oracle):
    n, w, nl = 8, 2, 6
    nb = oracle.count_band(n, w)
    Tc = W.uniform(63, nb * nl).reshape(nb, nl)
    Yc = oracle.ttm_band(Tc, np.eye(nl, dtype=np.float32), n, w)
    assert np.array_equal(Yc, Tc.astype(np.float64))


# -------------------------------------------------------------------- moment3
@pytest.mark.parametrize("N,n", [(1, 1), (1, 5), (7, 4), (50, 9)])
def test_moment3_against_einsum(oracle, N, n):
    X = W.normal(71, N * n).reshape(N, n)
    X64 = X.astype(np.float64)
    ref = np.einsum("si,sj,sk->ijk", X64, X64, X64)
    S = oracle.moment3_dense(X)
    assert np.allclose(S, ref, rtol=1e-13, atol=1e-13)
    for perm in itertools.permutations(range(3)):
        assert np.allclose(S, np.transpose(S, perm), rtol=1e-14, atol=1e-14)
    trip = np.array(list(itertools.product(range(n), repeat=3)), dtype=np.int32)
    assert np.array_equal(oracle.moment3_entries(X, trip), S.reshape(-1))


def test_moment3_special_cases(oracle):
    n, N = 6, 11
    X = np.zeros((N, n), dtype=np.float32)
    X[:, 2] = 1.0
    S = oracle.moment3_dense(X)
    assert S[2, 2, 2] == N and np.count_nonzero(S) == 1
    # N = 1 is the paper's M2 nest: S(i,j,k) = f_i f_j f_k, in dense position [i][j*n+k]
    f = W.normal(72, n)
    S = oracle.moment3_dense(f.reshape(1, n))
    f64 = f.astype(np.float64)
    M2 = np.outer(f64, np.outer(f64, f64).reshape(-1))
    assert np.allclose(S.reshape(n, n * n), M2, rtol=1e-15)
    # sum_p mult(p) * S_C(p) = sum_s (1^T x_s)^3
    X = W.normal(73, 40 * n).reshape(40, n)
    lst = oracle.list_sym3(n)
    Sc = oracle.moment3_entries(X, lst)
    mult = np.array([len(set(itertools.permutations(tuple(t)))) for t in lst.tolist()])
    assert np.isclose((mult * Sc).sum(), (X.astype(np.float64).sum(axis=1) ** 3).sum(), rtol=1e-12)


def test_cross_kernel_identity(oracle):
    # mttkrp(moment3(X), B)(i,r) = sum_s x_s(i) (x_s^T b_r)^2, with X small integers so that
    # the third moments are exact in fp32.
    n, N, R = 7, 5, 3
    X = np.round(W.uniform(81, N * n) * 4).reshape(N, n).astype(np.float32)
    B = W.uniform(82, n * R).reshape(n, R)
    Sc = oracle.moment3_entries(X, oracle.list_sym3(n)).astype(np.float32)
    M = oracle.mttkrp_sym3(Sc, B)
    X64, B64 = X.astype(np.float64), B.astype(np.float64)
    ref = np.einsum("si,sr->ir", X64, (X64 @ B64) ** 2)
    assert np.allclose(M, ref, rtol=1e-12, atol=1e-12)


# --------------------------------------------------------------------- expand
@pytest.mark.parametrize("n", [1, 2, 5, 12])
def test_expand(oracle, n):
    Sc3 = W.uniform(91, math.comb(n + 2, 3))
    S = oracle.expand_sym(Sc3, n, 3)
    assert S.dtype == np.float32
    idx = np.sort(np.indices((n, n, n)).reshape(3, -1), axis=0)
    pos = {t: p for p, t in enumerate(itertools.combinations_with_replacement(range(n), 3))}
    ref = np.array([Sc3[pos[tuple(int(v) for v in idx[:, q])]] for q in range(n ** 3)],
                   dtype=np.float32).reshape(n, n, n)
    assert np.array_equal(S.view(np.uint32), ref.view(np.uint32))
    for perm in itertools.permutations(range(3)):
        assert np.array_equal(S, np.transpose(S, perm))
    Sc2 = W.uniform(92, math.comb(n + 1, 2))
    S2 = oracle.expand_sym(Sc2, n, 2)
    assert np.array_equal(S2, S2.T)                      # y[i][j] = y[j][i] for j < i
    assert np.array_equal(S2[np.triu_indices(n)], Sc2)   # unique half is the packed data


# ------------------------------------------------- order-2 and order-4 moments (M1, M3)
@pytest.mark.parametrize("n", [1, 2, 4, 7])
def test_sym4_listing_is_lexicographic(oracle, n):
    lst = oracle.list_sym4(n)
    ref = np.array(list(itertools.combinations_with_replacement(range(n), 4)), dtype=np.int16).reshape(-1, 4)
    assert np.array_equal(lst, ref)
    assert lst.shape[0] == math.comb(n + 3, 4) == oracle.count_sym4(n)


@pytest.mark.parametrize("N,n", [(1, 1), (1, 5), (9, 4), (60, 11)])
def test_moment2_against_matmul(oracle, N, n):
    X = W.normal(101, N * n).reshape(N, n)
    X64 = X.astype(np.float64)
    S = oracle.moment2_dense(X)
    assert np.allclose(S, X64.T @ X64, rtol=1e-13, atol=1e-13)
    assert np.allclose(S, S.T, rtol=1e-15, atol=1e-15)
    if N == 1:   # the paper's M1 nest: M1[i][j] = f[i]*f[j]
        assert np.allclose(S, np.outer(X64[0], X64[0]), rtol=1e-15)


@pytest.mark.parametrize("N,n", [(1, 1), (1, 4), (6, 3), (25, 6)])
def test_moment4_against_einsum(oracle, N, n):
    X = W.normal(102, N * n).reshape(N, n)
    X64 = X.astype(np.float64)
    ref = np.einsum("si,sj,sk,sl->ijkl", X64, X64, X64, X64)
    S = oracle.moment4_dense(X)
    assert np.allclose(S, ref, rtol=1e-13, atol=1e-13)
    for perm in [(1, 0, 2, 3), (0, 2, 1, 3), (0, 1, 3, 2), (3, 2, 1, 0)]:
        assert np.allclose(S, np.transpose(S, perm), rtol=1e-14, atol=1e-14)
    quad = np.array(list(itertools.product(range(n), repeat=4)), dtype=np.int32)
    assert np.array_equal(oracle.moment4_entries(X, quad), S.reshape(-1))


def test_moment4_special_cases(oracle):
    n, N = 5, 13
    X = np.zeros((N, n), dtype=np.float32)
    X[:, 3] = 1.0
    S = oracle.moment4_dense(X)
    assert S[3, 3, 3, 3] == N and np.count_nonzero(S) == 1
    # N = 1 is the paper's M3 nest: M3[i*n+j][k*n+l] = f_i f_j f_k f_l
    f = W.normal(103, n)
    f64 = f.astype(np.float64)
    S = oracle.moment4_dense(f.reshape(1, n))
    v = np.outer(f64, f64).reshape(-1)
    assert np.allclose(S.reshape(n * n, n * n), np.outer(v, v), rtol=1e-15)
    # sum_p mult(p) * S_C(p) = sum_s (1^T x_s)^4, mult = number of distinct permutations
    X = W.normal(104, 30 * n).reshape(30, n)
    lst = oracle.list_sym4(n)
    Sc = oracle.moment4_entries(X, lst)
    mult = np.array([len(set(itertools.permutations(tuple(t)))) for t in lst.tolist()])
    assert set(mult.tolist()) <= {1, 4, 6, 12, 24} and mult.sum() == n ** 4
    assert np.isclose((mult * Sc).sum(), (X.astype(np.float64).sum(axis=1) ** 4).sum(), rtol=1e-12)
    # the order-4 moment restricted to k = l = a unit direction is the order-2 moment of x scaled by x_a
    a = 2
    Xa = (X.astype(np.float64) * X.astype(np.float64)[:, [a]])
    S4 = oracle.moment4_dense(X)
    assert np.allclose(S4[:, :, a, a], Xa.T @ Xa, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("n", [1, 2, 4, 7])
def test_expand_order4(oracle, n):
    Sc = W.uniform(105, math.comb(n + 3, 4))
    S = oracle.expand_sym(Sc, n, 4)
    assert S.dtype == np.float32 and S.shape == (n, n, n, n)
    idx = np.sort(np.indices((n, n, n, n)).reshape(4, -1), axis=0)
    pos = {t: p for p, t in enumerate(itertools.combinations_with_replacement(range(n), 4))}
    ref = np.array([Sc[pos[tuple(int(v) for v in idx[:, q])]] for q in range(n ** 4)],
                   dtype=np.float32).reshape(n, n, n, n)
    assert np.array_equal(S.view(np.uint32), ref.view(np.uint32))
    for perm in [(1, 0, 2, 3), (0, 2, 1, 3), (0, 1, 3, 2)]:
        assert np.array_equal(S, np.transpose(S, perm))


def test_pr2_covariance_distinct_elements(oracle):
    # the three unique sets together are the distinct elements of the degree-2 polynomial-regression
    # covariance: 65 for four features (golden file), counted here through the listings
    n = 4
    assert oracle.count_sym2(n) + oracle.count_sym3(n) + oracle.list_sym4(n).shape[0] == 65


# ------------------------------------------------- the kernel table on dense operands
def test_kernel_table_dense_definitions(oracle):
    ni, nj, nl, R = 5, 4, 6, 3
    B = W.uniform(111, ni * nj * nl).reshape(ni, nj, nl)
    U = W.uniform(112, nl * R).reshape(nl, R)
    B64, U64 = B.astype(np.float64), U.astype(np.float64)
    assert np.allclose(oracle.ttm_full(B, U), np.einsum("ijl,lr->ijr", B64, U64), rtol=1e-13, atol=1e-14)
    Cd = W.uniform(113, ni * nj * nl).reshape(ni, nj, nl)
    assert np.array_equal(oracle.thp_full(B, Cd), B64 * Cd.astype(np.float64))
    nk = nj
    C = W.uniform(114, nk * R).reshape(nk, R)
    D = W.uniform(115, nl * R).reshape(nl, R)
    ref = np.einsum("ikl,kj,lj->ij", B64, C.astype(np.float64), D.astype(np.float64))
    assert np.allclose(oracle.mttkrp_full(B, C, D), ref, rtol=1e-13, atol=1e-14)
    # the symmetric special case agrees with the packed symmetric oracle
    n = 6
    Tc = W.uniform(116, oracle.count_sym3(n))
    Bf = W.uniform(117, n * R).reshape(n, R)
    T = oracle.dense_sym3(Tc, n).astype(np.float32)   # exact: the values are fp32
    assert np.allclose(oracle.mttkrp_full(T, Bf, Bf), oracle.mttkrp_sym3(Tc, Bf), rtol=1e-12, atol=1e-13)
    # a band TTM is the dense TTM of the zero-filled tensor
    n, w = 7, 2
    Tb = W.uniform(118, oracle.count_band(n, w) * nl)
    Tdense = oracle.dense_band(Tb, n, w, nl).astype(np.float32)
    assert np.allclose(oracle.ttm_full(Tdense, U), oracle.ttm_dense(Tb, U, n, w), rtol=1e-13, atol=1e-14)


# ------------------------------------------------- structures given as predicates (brute force over the box)
# The predicate helpers check the descriptor-driven kernels; here they are pinned to the C oracle's counting-loop
# listings and dense definitions (pinned above), to numpy's own index routines and to the paper's two worked
# examples of a unique set / redundancy map.
@pytest.mark.parametrize("n", [1, 2, 5, 12])
def test_struct_enumerate_symmetric_sets(oracle, n):
    assert np.array_equal(oracle.struct_enumerate((n, n), lambda i, j: i <= j), oracle.list_sym2(n))
    assert np.array_equal(oracle.struct_enumerate((n,) * 3, lambda i, j, k: i <= j <= k), oracle.list_sym3(n))
    if n <= 5:
        assert np.array_equal(oracle.struct_enumerate((n,) * 4, lambda i, j, k, l: i <= j <= k <= l),
                              oracle.list_sym4(n))


@pytest.mark.parametrize("n,w", [(1, 0), (4, 0), (7, 2), (12, 3), (9, 20)])
def test_struct_enumerate_band(oracle, n, w):
    assert np.array_equal(oracle.struct_enumerate((n, n), lambda i, j: abs(i - j) <= w), oracle.list_band(n, w))
    # with a free last index every in-band pair is one run of nl consecutive positions
    nl = 3
    lst = oracle.struct_enumerate((n, n, nl), lambda i, j, l: abs(i - j) <= w)
    pairs = oracle.list_band(n, w)
    assert np.array_equal(lst[:, :2], np.repeat(pairs, nl, axis=0))
    assert np.array_equal(lst[:, 2], np.tile(np.arange(nl), pairs.shape[0]))


def test_struct_chess_board_example(oracle):
    # "Chess Pattern Unique Set": even rows keep the odd columns, odd rows the even columns
    m, n = 6, 8
    pred = lambda i, j: (i % 2 == 0 and j % 2 == 1) or (i % 2 == 1 and j % 2 == 0)
    lst = oracle.struct_enumerate((m, n), pred)
    assert lst.shape[0] == 2 * (m // 2) * (n // 2)
    I, J = np.indices((m, n))
    assert np.array_equal(lst, np.argwhere((I + J) % 2 == 1))
    # written as the example writes it: i = 2i', j = 2j'+1  and  i = 2i'+1, j = 2j'
    want = sorted([(2 * a, 2 * b + 1) for a in range(m // 2) for b in range(n // 2)] +
                  [(2 * a + 1, 2 * b) for a in range(m // 2) for b in range(n // 2)])
    assert [tuple(int(v) for v in t) for t in lst] == want
    # no redundancy map: reconstruction puts the stored values on the pattern and zeros elsewhere
    Tc = W.uniform(201, lst.shape[0])
    T = oracle.struct_expand(Tc, (m, n), pred)
    assert np.array_equal(T[lst[:, 0], lst[:, 1]], Tc)
    assert not T[(I + J) % 2 == 0].any()


def test_struct_identical_rows_example(oracle):
    # "Identical Row Matrix Redundancy Map": T_U = (i=0)*(0<=j<n), T_R: (0<i<m)*(0<=j<n) -> (0, j)
    m, n = 5, 7
    pred = lambda i, j: i == 0
    lst = oracle.struct_enumerate((m, n), pred)
    assert np.array_equal(lst, np.stack([np.zeros(n, dtype=np.int32), np.arange(n, dtype=np.int32)], axis=1))
    Tc = W.uniform(202, n)
    T = oracle.struct_expand(Tc, (m, n), pred, lambda i, j: (0, j) if 0 < i < m else None)
    assert np.array_equal(T, np.tile(Tc, (m, 1)))
    # Property 1: no index is both unique and redundant; without the map only the first row is filled
    assert all(not (pred(i, j) and 0 < i < m) for i in range(m) for j in range(n))
    T0 = oracle.struct_expand(Tc, (m, n), pred)
    assert np.array_equal(T0[0], Tc) and not T0[1:].any()


@pytest.mark.parametrize("n", [1, 2, 5, 9])
def test_struct_expand_is_property5(oracle, n):
    # full symmetry (x' = ascending sort of x) must reproduce the C oracle's reconstruction bit for bit
    order_preds = {2: lambda i, j: i <= j, 3: lambda i, j, k: i <= j <= k, 4: lambda i, j, k, l: i <= j <= k <= l}
    counts = {2: oracle.count_sym2, 3: oracle.count_sym3, 4: oracle.count_sym4}
    for order in (2, 3, 4):
        if order == 4 and n > 5:
            continue
        Sc = W.uniform(210 + order, counts[order](n))
        got = oracle.struct_expand(Sc, (n,) * order, order_preds[order], lambda *x: tuple(sorted(x)))
        assert np.array_equal(got.view(np.uint32), oracle.expand_sym(Sc, n, order).view(np.uint32))
    # the class-S map written out: for j < i the unique index is (j, i)
    Sc = W.uniform(215, oracle.count_sym2(n))
    got = oracle.struct_expand(Sc, (n, n), order_preds[2], lambda i, j: (j, i) if j < i else None)
    assert np.array_equal(got, oracle.expand_sym(Sc, n, 2))
    # a band has no redundancy: zero-filled dense form
    w, nl = min(2, n - 1), 3
    Tb = W.uniform(216, oracle.count_band(n, w) * nl)
    got = oracle.struct_expand(Tb, (n, n, nl), lambda i, j, l: abs(i - j) <= w)
    assert np.array_equal(got.astype(np.float64), oracle.dense_band(Tb, n, w, nl))


def test_struct_thp_on_the_band(oracle):
    n, w, nl = 9, 2, 5
    pred = lambda i, j, l: abs(i - j) <= w
    Bc = W.uniform(221, oracle.count_band(n, w) * nl)
    Cd = W.uniform(222, n * n * nl).reshape(n, n, nl)
    pairs = oracle.list_band(n, w).astype(np.int64)
    ref = oracle.thp_full(Bc.reshape(-1, nl), Cd[pairs[:, 0], pairs[:, 1]])      # gathered fibres, dense THP
    assert np.array_equal(oracle.struct_thp(Bc, Cd, (n, n, nl), pred), ref.reshape(-1))
    # and through the zero-filled dense operand: the product keeps the support of B
    dense = oracle.thp_full(oracle.dense_band(Bc, n, w, nl).astype(np.float32), Cd)
    I, J = np.indices((n, n))
    assert np.array_equal(dense[np.abs(I - J) <= w].reshape(-1), ref.reshape(-1))
    assert not dense[np.abs(I - J) > w].any()


@pytest.mark.parametrize("N,n", [(1, 4), (7, 6), (300, 9)])
def test_struct_moment_against_dense_moments(oracle, N, n):
    X = W.normal(230, N * n).reshape(N, n)
    tol = dict(rtol=1e-12, atol=1e-12)
    # the symmetric unique sets: the C oracle's entry-wise and dense moments
    got3 = oracle.struct_moment(X, (n,) * 3, lambda i, j, k: i <= j <= k)
    assert np.allclose(got3, oracle.moment3_entries(X, oracle.list_sym3(n)), **tol)
    got2 = oracle.struct_moment(X, (n, n), lambda i, j: i <= j)
    assert np.allclose(got2, oracle.moment2_dense(X)[np.triu_indices(n)], **tol)
    if n <= 6:
        got4 = oracle.struct_moment(X, (n,) * 4, lambda i, j, k, l: i <= j <= k <= l)
        assert np.allclose(got4, oracle.moment4_entries(X, oracle.list_sym4(n)), **tol)
    # structures only a descriptor gives: the dense moment read at the listed positions
    S3, S2 = oracle.moment3_dense(X), oracle.moment2_dense(X)
    for pred in (lambda i, j, k: i <= j <= k <= i + 2, lambda i, j, k: i == j == k):
        idx = oracle.struct_enumerate((n,) * 3, pred).astype(np.int64)
        assert np.allclose(oracle.struct_moment(X, (n,) * 3, pred), S3[idx[:, 0], idx[:, 1], idx[:, 2]], **tol)
    for pred in (lambda i, j: i <= j <= i + 3, lambda i, j: True):
        idx = oracle.struct_enumerate((n, n), pred).astype(np.int64)
        assert np.allclose(oracle.struct_moment(X, (n, n), pred), S2[idx[:, 0], idx[:, 1]], **tol)
    # independent of the C oracle altogether
    X64 = X.astype(np.float64)
    idx = oracle.struct_enumerate((n,) * 3, lambda i, j, k: i <= j <= k <= i + 2).astype(np.int64)
    ein = np.einsum("si,sj,sk->ijk", X64, X64, X64)[idx[:, 0], idx[:, 1], idx[:, 2]]
    assert np.allclose(oracle.struct_moment(X, (n,) * 3, lambda i, j, k: i <= j <= k <= i + 2), ein, **tol)


def test_direct_sum_definition(oracle):
    """The direct sum against a library routine for matrices (scipy's block-diagonal stacking), against plain
    concatenation for vectors, and by its defining property at order 3: the two diagonal blocks are the operands,
    everything else is zero."""
    import scipy.linalg
    M, V = W.uniform(240, 12).reshape(3, 4), W.uniform(241, 10).reshape(5, 2)
    assert np.array_equal(oracle.direct_sum(M, V), scipy.linalg.block_diag(M, V))
    a, b = W.uniform(242, 4), W.uniform(243, 7)
    assert np.array_equal(oracle.direct_sum(a, b), np.concatenate([a, b]))
    A, B = W.uniform(244, 24).reshape(2, 3, 4), W.uniform(245, 6).reshape(3, 1, 2)
    T = oracle.direct_sum(A, B)
    assert T.shape == (5, 4, 6)
    assert np.array_equal(T[:2, :3, :4], A) and np.array_equal(T[2:, 3:, 4:], B)
    assert np.count_nonzero(T) == np.count_nonzero(A) + np.count_nonzero(B)
    # not commutative: the operands swap corners
    assert np.array_equal(oracle.direct_sum(V, M), scipy.linalg.block_diag(V, M))
