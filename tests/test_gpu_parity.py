"""Parity of the HIP kernels (through the C ABI) against the fp64 CPU oracle, on
the same seeded inputs.

Bar: bit-exact for index maps and expand; for fp32 results the norm-wise error
max|got - ref| / max|ref| <= 1e-4 per output tensor (the outputs are sums of
zero-mean terms, so element-wise relative error is meaningless near zero), and
beside it the floored element-wise error max|got - ref| / max(|ref|, 1e-3 max|ref|)
<= 1e-3: every entry that reaches a thousandth of the largest one is right to
three digits, so an error confined to the small entries cannot hide behind the
large ones.  (An fp32 sum's rounding error does not shrink with the value of the
sum: at the measured norm-wise errors of 1e-7 .. 4e-6 an entry at the floor is
still within 4e-3 .. 1e-4 of its value in the worst case, well inside in practice.)
"""
import itertools
import sys

import numpy as np
import pytest

import st_workloads as W

pytestmark = pytest.mark.gpu

TOL = 1e-4
ELEM_TOL = 1e-3
ELEM_FLOOR = 1e-3


@pytest.fixture(scope="module")
def st():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2211_10482_amd as lib
    lib.lib()
    return lib


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max()
    if scale == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / scale)


def elem_err(got, ref):
    """Floored element-wise error: |got - ref| / max(|ref|, 1e-3 max|ref|), largest over the tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max()
    if scale == 0.0:
        return float(np.abs(got).max())
    return float((np.abs(got - ref) / np.maximum(np.abs(ref), ELEM_FLOOR * scale)).max())


def check(got, ref, what=None):
    """Both error bars of a floating-point result; prints them when the case is named."""
    e, ee = rel_err(got, ref), elem_err(got, ref)
    if what:
        say("  %s: norm-wise error %.3e, floored element-wise error %.3e" % (what, e, ee))
    assert e <= TOL, (what, e)
    assert ee <= ELEM_TOL, (what, ee)


def inf_pattern_matches(got, ref):
    """Non-finite inputs: the result must be infinite exactly where the definition is (same sign), NaN exactly
    where the definition is NaN, and within the usual bar everywhere else."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(ref)), (int(np.isnan(got).sum()), int(np.isnan(ref).sum()))
    assert np.array_equal(np.isinf(got), np.isinf(ref))
    inf = np.isinf(ref)
    assert np.array_equal(np.sign(got[inf]), np.sign(ref[inf]))
    fin = np.isfinite(ref)
    if fin.any():
        assert np.abs(got[fin] - ref[fin]).max() <= TOL * np.abs(ref[fin]).max()


# ------------------------------------------------------------ device index maps
@pytest.mark.parametrize("n", [1, 2, 7, 40, 64])
def test_device_unrank_small(st, oracle, n):
    say("device unrank n=%d" % n)
    got3 = st.unrank_device(3, n, 0, 0, oracle.count_sym3(n)).cpu().numpy()
    assert np.array_equal(got3, oracle.list_sym3(n))
    got2 = st.unrank_device(2, n, 0, 0, oracle.count_sym2(n)).cpu().numpy()
    assert np.array_equal(got2, oracle.list_sym2(n))
    for w in (0, 1, n // 2, n - 1, n + 3):
        gotb = st.unrank_device(4, n, w, 0, oracle.count_band(n, w)).cpu().numpy()
        assert np.array_equal(gotb, oracle.list_band(n, w))


@pytest.mark.parametrize("n", [1, 3, 17, 64])
def test_device_unrank_sym4(st, oracle, n):
    say("device unrank sym4 n=%d" % n)
    lst = oracle.list_sym4(n)
    got = st.unrank_device(5, n, 0, 0, lst.shape[0]).cpu().numpy()
    assert np.array_equal(got, lst)
    if n == 64:   # the 64-bit device path on a window of a larger set
        n2 = 300
        ref = st.unrank_sym4_batch(n2, 200_000_000, 50_000)
        got = st.unrank_device(5, n2, 0, 200_000_000, 50_000).cpu().numpy()
        assert np.array_equal(got, ref)


def test_device_unrank_full_sizes(st, oracle):
    say("device unrank sym3 n=512 (22.5M), sym2 n=8192 (33.6M), band (512,8)")
    lst = oracle.list_sym3(512)
    got = st.unrank_device(3, 512, 0, 0, lst.shape[0]).cpu().numpy()
    assert np.array_equal(got, lst)
    del got, lst
    lst = oracle.list_sym2(8192)
    got = st.unrank_device(2, 8192, 0, 0, lst.shape[0]).cpu().numpy()
    assert np.array_equal(got, lst)
    del got, lst
    got = st.unrank_device(4, 512, 8, 0, 8632).cpu().numpy()
    assert np.array_equal(got, oracle.list_band(512, 8))
    # 64-bit device path (n above the 32-bit range of the kernels' arithmetic)
    n = 1100
    lst = oracle.list_sym3(n)
    p0 = lst.shape[0] - 300_000
    got = st.unrank_device(3, n, 0, p0, 300_000).cpu().numpy()
    assert np.array_equal(got, lst[p0:])


# ---------------------------------------------------------------------- expand
@pytest.mark.parametrize("n", [1, 2, 5, 12, 33, 64])
def test_expand_order3(st, oracle, n):
    say("expand order 3 n=%d" % n)
    Sc = W.uniform(101, oracle.count_sym3(n))
    ref = oracle.expand_sym(Sc, n, 3)
    got = st.expand_sym(dev(Sc), n, 3).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    for perm in itertools.permutations(range(3)):
        assert np.array_equal(got, np.transpose(got, perm))
    idx = oracle.list_sym3(n).astype(np.int64)
    assert np.array_equal(got[idx[:, 0], idx[:, 1], idx[:, 2]], Sc)


@pytest.mark.parametrize("n", [1, 2, 5, 12, 17, 64])
def test_expand_order4(st, oracle, n):
    say("expand order 4 n=%d" % n)
    Sc = W.uniform(103, oracle.count_sym4(n))
    ref = oracle.expand_sym(Sc, n, 4)
    got = st.expand_sym(dev(Sc), n, 4).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    idx = oracle.list_sym4(n).astype(np.int64)
    assert np.array_equal(got[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]], Sc)


@pytest.mark.parametrize("n", [1, 7, 64, 100, 1001])
def test_expand_order2(st, oracle, n):
    say("expand order 2 n=%d" % n)
    Sc = W.uniform(102, oracle.count_sym2(n))
    ref = oracle.expand_sym(Sc, n, 2)
    got = st.expand_sym(dev(Sc), n, 2).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


# ----------------------------------------------------------------------- batax
@pytest.mark.parametrize("n", [1, 2, 5, 33, 100, 257, 1000, 4096, 4100, 8200, 9001, 12288, 16384, 16500])
def test_batax_small(st, oracle, n):
    say("batax n=%d" % n)
    Ap = W.uniform(201, oracle.count_sym2(n))
    x = W.uniform(202, n)
    ref = oracle.batax_utri(Ap, x, 0.5)
    got = st.batax_utri(dev(Ap), dev(x), 0.5).cpu().numpy()
    check(got, ref)
    got2 = st.batax_utri(dev(Ap), dev(x), 0.5).cpu().numpy()
    assert np.array_equal(got, got2)                      # deterministic


def test_batax_identity(st, oracle):
    n = 300
    eye = np.eye(n, dtype=np.float32)[np.triu_indices(n)]
    x = W.uniform(203, n)
    got = st.batax_utri(dev(eye), dev(x), 0.75).cpu().numpy()
    assert np.array_equal(got, (np.float32(0.75) * x))


def test_batax_full(st, oracle):
    cfg = W.CONFIGS[2]
    say("batax full n=%d" % cfg["n"])
    Ap, x = W.batax_inputs(cfg["n"], cfg["entries"])
    ref = oracle.batax_utri(Ap, x, cfg["beta"])
    got = st.batax_utri(dev(Ap), dev(x), cfg["beta"]).cpu().numpy()
    check(got, ref, "batax full, all %d outputs" % got.size)


# ------------------------------------------------------------------------- ttm
@pytest.mark.parametrize("n,w,nl,R", [(1, 0, 1, 1), (7, 2, 5, 4), (9, 0, 16, 16), (40, 3, 32, 16),
                                      (64, 8, 48, 32), (33, 40, 64, 64), (50, 4, 80, 48),
                                      (30, 2, 1040, 256), (20, 3, 16, 272), (600, 14, 128, 48),
                                      (100, 5, 256, 16), (70, 1, 512, 32), (700, 20, 64, 16),
                                      (1100, 9, 512, 64), (90, 6, 500, 50), (64, 3, 130, 250), (50, 2, 33, 17),
                                      (40, 1, 100, 300),
                                      # one to three row tiles per CU (one-shot kernel), every l-range / column count
                                      (300, 3, 128, 48), (400, 10, 256, 32), (50, 2, 64, 16), (700, 8, 512, 64),
                                      (257, 7, 512, 16), (130, 20, 256, 64), (600, 9, 64, 48), (723, 8, 512, 64)])
def test_ttm_small(st, oracle, n, w, nl, R):
    say("ttm n=%d w=%d nl=%d R=%d" % (n, w, nl, R))
    nb = oracle.count_band(n, w)
    Tc = W.uniform(301, nb * nl).reshape(nb, nl)
    U = W.uniform(302, nl * R).reshape(nl, R)
    ref = oracle.ttm_band(Tc, U, n, w)
    got = st.ttm_band(dev(Tc), dev(U), n, w).cpu().numpy()
    assert got.shape == ref.shape
    check(got, ref)


def test_ttm_identity_factor(st, oracle):
    n, w, nl = 24, 3, 32
    nb = oracle.count_band(n, w)
    Tc = W.uniform(303, nb * nl).reshape(nb, nl)
    got = st.ttm_band(dev(Tc), dev(np.eye(nl, dtype=np.float32)), n, w).cpu().numpy()
    assert np.array_equal(got, Tc)


def test_ttm_full(st, oracle):
    cfg = W.CONFIGS[3]
    say("ttm full", cfg)
    Tc, U = W.ttm_inputs(cfg["band_pairs"], cfg["nl"], cfg["R"])
    ref = oracle.ttm_band(Tc, U, cfg["n"], cfg["w"])
    got = st.ttm_band(dev(Tc), dev(U), cfg["n"], cfg["w"]).cpu().numpy()
    check(got, ref, "ttm full, all %d outputs" % got.size)


# --------------------------------------------------------------------- moment3
@pytest.mark.parametrize("N,n", [(1, 5), (7, 4), (50, 9), (300, 17), (1000, 33), (100, 64), (5000, 64),
                                 (70, 1), (200, 70), (3000, 13), (2500, 6), (257, 40), (400, 48), (300, 129),
                                 (150, 200), (40, 256), (30, 260), (500, 128), (20000, 100), (64, 65), (90, 96),
                                 (9000, 80)])
def test_moment3_small(st, oracle, N, n):
    say("moment3 N=%d n=%d" % (N, n))
    X = W.normal(401, N * n).reshape(N, n)
    lst = oracle.list_sym3(n)
    ref = oracle.moment3_entries(X, lst)
    got = st.moment3_sym(dev(X)).cpu().numpy()
    assert got.shape == ref.shape
    check(got, ref)
    got2 = st.moment3_sym(dev(X)).cpu().numpy()
    assert np.array_equal(got, got2)                      # deterministic


def lex_position3(n, t):
    """Position of the sorted triple t among all non-decreasing triples over 0..n-1 in lexicographic order."""
    from math import comb
    i, j, k = (int(v) for v in t)
    return sum(comb(n - a + 1, 2) for a in range(i)) + sum(n - b for b in range(i, j)) + (k - j)


@pytest.mark.parametrize("N,n", [(300000, 80), (150000, 200), (60000, 256), (100000, 128)])
def test_moment3_wide_long(st, oracle, N, n):
    """More than 64 features and sample slices long enough for the periodic flush of the fp32 chains of the
    matrix-core path: sampled entries (repeated indices and indices of one group of 16 among them), accumulate."""
    say("moment3 wide N=%d n=%d" % (N, n))
    X = W.normal(305, N * n).reshape(N, n)
    rng = np.random.default_rng(13)
    tr = [rng.integers(0, n, 3) for _ in range(800)]
    for _ in range(600):
        base = int(rng.integers(0, n))
        tr.append(np.clip(base + rng.integers(-9, 10, 3), 0, n - 1))
    tr += [np.array([0, 0, 0]), np.array([n - 1] * 3), np.array([0, n - 1, n - 1]), np.array([0, 1, 2])]
    tr = np.unique(np.sort(np.array(tr, dtype=np.int64), axis=1), axis=0)
    pos = np.array([lex_position3(n, t) for t in tr], dtype=np.int64)
    ref = oracle.moment3_entries(X, tr.astype(np.int32))
    h = N // 3
    Sc = st.moment3_sym(dev(X[:h]))
    st.moment3_sym(dev(X[h:]), Sc=Sc, accumulate=True)
    got = Sc.cpu().numpy()
    assert got.shape[0] == lex_position3(n, (n - 1,) * 3) + 1
    err = float(np.abs(got[pos] - ref).max() / np.abs(ref).max())
    say("  norm-wise error on %d sampled entries %.3e" % (pos.size, err))
    assert err <= TOL
    assert np.all(np.isfinite(got))


def test_moment3_accumulate_and_empty(st, oracle):
    import torch
    N, n = 600, 20
    X = W.normal(402, N * n).reshape(N, n)
    ref = oracle.moment3_entries(X, oracle.list_sym3(n))
    Sc = st.moment3_sym(dev(X[:250]))
    Sc = st.moment3_sym(dev(X[250:]), Sc=Sc, accumulate=True)
    check(Sc.cpu().numpy(), ref)
    # N = 0: overwrite gives zeros, accumulate leaves Sc alone
    empty = torch.empty((0, n), dtype=torch.float32, device="cuda")
    keep = Sc.clone()
    st.moment3_sym(empty, Sc=Sc, accumulate=True)
    assert torch.equal(Sc, keep)
    st.moment3_sym(empty, Sc=Sc, accumulate=False)
    assert float(Sc.abs().max()) == 0.0


def test_moment3_unit_vectors(st):
    n, N = 64, 777
    X = np.zeros((N, n), dtype=np.float32)
    X[:, 37] = 1.0
    got = st.moment3_sym(dev(X)).cpu().numpy()
    p = st.rank_sym3(n, 37, 37, 37)
    assert got[p] == N and np.count_nonzero(got) == 1


def test_moment3_full(st, oracle):
    cfg = W.CONFIGS[5]
    N, n = cfg["N"], cfg["n"]
    say("moment3 full N=%d n=%d: generating" % (N, n))
    X = W.moment_inputs(N, n)
    say("  running")
    Sc = st.moment3_sym(dev(X))
    got = Sc.cpu().numpy()
    lst = oracle.list_sym3(n)
    assert got.shape[0] == lst.shape[0] == cfg["entries"]
    # every unique entry against the definition, in blocks so that the run reports its progress
    ref = np.empty(lst.shape[0], dtype=np.float64)
    step = 4096
    for p0 in range(0, lst.shape[0], step):
        ref[p0:p0 + step] = oracle.moment3_entries(X, lst[p0:p0 + step])
        if (p0 // step) % 3 == 0:
            say("  oracle: %d of %d entries" % (min(p0 + step, lst.shape[0]), lst.shape[0]))
    check(got, ref, "moment3 full, all %d unique entries" % ref.size)
    # property that holds at any size: sum_p mult(p) Sc(p) = sum_s (1^T x_s)^3
    i, j, k = lst[:, 0], lst[:, 1], lst[:, 2]
    mult = np.where((i == j) & (j == k), 1, np.where((i == j) | (j == k), 3, 6)).astype(np.float64)
    lhs = float((mult * got.astype(np.float64)).sum())
    rhs = float((X.astype(np.float64).sum(axis=1) ** 3).sum())
    bound = TOL * float((mult * np.abs(got.astype(np.float64))).sum())
    assert abs(lhs - rhs) <= bound
    # expand the result (the second half of this workload) and check it bit-exactly
    S = st.expand_sym(Sc, n, 3).cpu().numpy()
    ref_S = oracle.expand_sym(got, n, 3)
    assert np.array_equal(S.view(np.uint32), ref_S.view(np.uint32))


# ---------------------------------------------------------------------- moment2 (M1)
@pytest.mark.parametrize("N,n", [(1, 1), (7, 5), (100, 64), (4097, 64), (33, 64), (1000, 20), (5000, 63), (300, 70),
                                 (64, 200), (700, 65), (90, 1024), (20, 1100), (300000, 6), (70000, 13), (5000, 16),
                                 (999, 2), (400000, 9), (257, 17), (3000, 128), (1001, 130), (2100, 192), (777, 250),
                                 (1500, 256), (513, 258), (900, 260), (640, 384), (333, 513), (400, 1000), (5000, 180),
                                 (2000, 188), (31, 320), (129, 66)])
def test_moment2_small(st, oracle, N, n):
    say("moment2 N=%d n=%d" % (N, n))
    X = W.normal(301, N * n).reshape(N, n)
    iu = np.triu_indices(n)
    ref = oracle.moment2_dense(X)[iu]
    got = st.moment2_sym(dev(X)).cpu().numpy()
    check(got, ref)
    got2 = st.moment2_sym(dev(X)).cpu().numpy()
    assert np.array_equal(got, got2)                      # deterministic
    # accumulate: two halves added into one result
    h = N // 2
    Sc = st.moment2_sym(dev(X[:h]))
    st.moment2_sym(dev(X[h:]), Sc=Sc, accumulate=True)
    check(Sc.cpu().numpy(), ref)


def test_moment2_special_cases(st, oracle):
    import torch
    n, N = 64, 1000
    X = np.zeros((N, n), dtype=np.float32)
    X[:, 9] = 1.0
    got = st.moment2_sym(dev(X)).cpu().numpy()
    assert got[st.rank_sym2(n, 9, 9)] == N and np.count_nonzero(got) == 1
    # N = 0 zero-fills, or leaves Sc alone when accumulating
    Sc = torch.full((st.count_sym2(n),), 3.0, device="cuda")
    st.moment2_sym(torch.empty((0, n), device="cuda"), Sc=Sc, accumulate=True)
    assert float(Sc.min()) == 3.0
    st.moment2_sym(torch.empty((0, n), device="cuda"), Sc=Sc)
    assert float(Sc.abs().max()) == 0.0


@pytest.mark.parametrize("N,n", [(300000, 128), (100000, 320), (40000, 1024), (150001, 250)])
def test_moment2_wide_long(st, oracle, N, n):
    """64 < n <= 1024: strips of 64 columns on the matrix cores, many slices and long accumulation chains."""
    say("moment2 wide N=%d n=%d" % (N, n))
    X = W.moment_inputs(N, n)
    got = st.moment2_sym(dev(X)).cpu().numpy()
    ref = oracle.moment2_dense(X)[np.triu_indices(n)]
    err = rel_err(got, ref)
    say("  norm-wise error %.3e" % err)
    assert err <= TOL


@pytest.mark.parametrize("n", [128, 190, 200, 258, 1024])
def test_moment2_wide_exact_entries(st, n):
    """Two columns set to 1 and 2, everything else zero: the three entries they reach are exact integers, and no
    other entry may be touched -- for column pairs inside a strip, across strips and across blocks."""
    N = 1000
    cols = sorted({0, 3, 63, 64, 65, 127, 128, n // 2, n - 65, n - 2, n - 1} & set(range(n)))
    for a in cols:
        for b in cols:
            if a >= b:
                continue
            X = np.zeros((N, n), dtype=np.float32)
            X[:, a], X[:, b] = 1.0, 2.0
            got = st.moment2_sym(dev(X)).cpu().numpy()
            assert got[st.rank_sym2(n, a, a)] == N and got[st.rank_sym2(n, a, b)] == 2 * N and got[st.rank_sym2(n, b, b)] == 4 * N, (n, a, b)
            assert np.count_nonzero(got) == 3, (n, a, b)


def test_moment2_full(st, oracle):
    cfg = W.CONFIGS[5]
    N, n = cfg["N"], cfg["n"]
    say("moment2 full N=%d n=%d" % (N, n))
    X = W.moment_inputs(N, n)
    got = st.moment2_sym(dev(X)).cpu().numpy()
    ref = oracle.moment2_dense(X)[np.triu_indices(n)]
    err = rel_err(got, ref)
    say("  norm-wise error %.3e" % err)
    assert err <= TOL


# ---------------------------------------------------------------------- moment4 (M3)
@pytest.mark.parametrize("N,n", [(1, 1), (7, 5), (100, 16), (300, 64), (65, 64), (64, 64), (50, 20), (130, 63),
                                 (40, 70), (70, 65), (33, 100), (200, 53), (90, 57), (3000, 60), (50, 52),
                                 (40, 80), (25, 75), (20, 128), (11, 113), (900, 6), (700, 9), (333, 13), (64, 2),
                                 (1000, 3), (257, 12), (150, 29), (90, 32), (70, 44), (40, 48), (30, 36), (60, 28)])
def test_moment4_small(st, oracle, N, n):
    say("moment4 N=%d n=%d" % (N, n))
    X = W.normal(401, N * n).reshape(N, n)
    lst = oracle.list_sym4(n)
    ref = oracle.moment4_entries(X, lst)
    got = st.moment4_sym(dev(X)).cpu().numpy()
    assert got.shape[0] == lst.shape[0]
    check(got, ref)
    got2 = st.moment4_sym(dev(X)).cpu().numpy()
    assert np.array_equal(got, got2)                      # deterministic
    h = N // 2
    Sc = st.moment4_sym(dev(X[:h]))
    st.moment4_sym(dev(X[h:]), Sc=Sc, accumulate=True)
    check(Sc.cpu().numpy(), ref)


def test_moment4_special_cases(st, oracle):
    import torch
    n, N = 64, 200
    X = np.zeros((N, n), dtype=np.float32)
    X[:, 17] = 1.0
    got = st.moment4_sym(dev(X)).cpu().numpy()
    assert got[st.rank_sym4(n, 17, 17, 17, 17)] == N and np.count_nonzero(got) == 1
    Sc = torch.full((st.count_sym4(n),), 2.0, device="cuda")
    st.moment4_sym(torch.empty((0, n), device="cuda"), Sc=Sc, accumulate=True)
    assert float(Sc.min()) == 2.0
    st.moment4_sym(torch.empty((0, n), device="cuda"), Sc=Sc)
    assert float(Sc.abs().max()) == 0.0
    # sum_p mult(p) * S_C(p) = sum_s (1^T x_s)^4 at a size the oracle does not enumerate densely
    N = 5000
    X = W.normal(402, N * n).reshape(N, n)
    got = st.moment4_sym(dev(X)).cpu().numpy().astype(np.float64)
    lst = oracle.list_sym4(n).astype(np.int64)
    srt = np.sort(lst, axis=1)
    runs = np.concatenate([np.ones((len(srt), 1), dtype=bool), srt[:, 1:] != srt[:, :-1]], axis=1)
    # multiplicity = 4! / prod(run lengths!)
    import math
    mult = np.empty(len(srt))
    for q, row in enumerate(srt):
        _, cnts = np.unique(row, return_counts=True)
        mult[q] = 24 / np.prod([math.factorial(int(c)) for c in cnts])
    lhs = float((mult * got).sum())
    rhs = float((X.astype(np.float64).sum(axis=1) ** 4).sum())
    assert abs(lhs - rhs) <= 1e-4 * abs(rhs)


def lex_position4(n, q):
    """Position of the sorted quadruple q among all non-decreasing quadruples over 0..n-1 in lexicographic
    order, by counting the ones in front of it (combinatorial number system; math.comb only)."""
    from math import comb
    i, j, k, l = (int(v) for v in q)
    return (sum(comb(n - a + 2, 3) for a in range(i)) + sum(comb(n - b + 1, 2) for b in range(i, j))
            + sum(n - c for c in range(j, k)) + (l - k))


@pytest.mark.parametrize("N,n", [(5000, 128), (3000, 200), (700, 256), (9000, 96), (40000, 144), (120000, 80)])
def test_moment4_wide(st, oracle, N, n):
    """Feature counts beyond 64 (the matrix-core path with 6 to 16 index groups): sampled entries, among them
    quadruples with repeated indices and with several indices in one group of 16."""
    say("moment4 wide N=%d n=%d" % (N, n))
    X = W.normal(404, N * n).reshape(N, n)
    got = st.moment4_sym(dev(X)).cpu().numpy()
    rng = np.random.default_rng(11)
    quads = [rng.integers(0, n, 4) for _ in range(700)]
    for _ in range(500):                                   # close together: same group, repeated values
        base = int(rng.integers(0, n))
        quads.append(np.clip(base + rng.integers(-9, 10, 4), 0, n - 1))
    for _ in range(200):                                   # two pairs of neighbours
        a, b = rng.integers(0, n, 2)
        quads.append(np.clip(np.array([a, a + rng.integers(0, 3), b, b + rng.integers(0, 3)]), 0, n - 1))
    quads += [np.array([0, 0, 0, 0]), np.array([n - 1] * 4), np.array([0, 0, n - 1, n - 1]), np.array([0, 1, 2, 3])]
    quads = np.unique(np.sort(np.array(quads, dtype=np.int64), axis=1), axis=0)
    pos = np.array([lex_position4(n, q) for q in quads], dtype=np.int64)
    assert got.shape[0] == lex_position4(n, (n - 1,) * 4) + 1 == oracle.count_sym4(n)
    ref = oracle.moment4_entries(X, quads.astype(np.int32))
    err = float(np.abs(got[pos] - ref).max() / np.abs(ref).max())
    say("  norm-wise error on %d sampled entries %.3e" % (pos.size, err))
    assert err <= TOL
    assert np.all(np.isfinite(got))


def test_moment4_full(st, oracle):
    cfg = W.CONFIGS[5]
    N, n = cfg["N"], cfg["n"]
    say("moment4 full N=%d n=%d" % (N, n))
    X = W.moment_inputs(N, n)
    got = st.moment4_sym(dev(X)).cpu().numpy()
    lst = oracle.list_sym4(n)
    rng = np.random.default_rng(7)
    pick = np.unique(np.concatenate([rng.integers(0, lst.shape[0], 1500), [0, lst.shape[0] - 1]]))
    say("  oracle on %d sampled entries" % pick.size)
    ref = oracle.moment4_entries(X, lst[pick])
    scale = np.abs(ref).max()
    err = float(np.abs(got[pick] - ref).max() / scale)
    say("  norm-wise error on the sample %.3e" % err)
    assert err <= TOL
    assert np.all(np.isfinite(got))


# ------------------------------------------- degree-2 polynomial-regression covariance
@pytest.mark.parametrize("N,n", [(300, 4), (1000, 13), (500, 64), (90, 70), (20000, 6), (777, 5), (64, 1), (5000, 3),
                                 (300000, 2), (1, 6), (700, 7), (5000, 8), (333, 9), (2000, 10), (100, 11), (40000, 13),
                                 (900, 14), (65, 15), (3000, 16), (200, 17)])
def test_covar_pr2(st, oracle, N, n):
    """(M1, M2, M3) in one call, as two half-batches (creation and addition), against the dense definitions;
    n = 4 has the paper's 65 distinct elements, 6 and 13 are the feature counts of its end-to-end data sets."""
    say("covar_pr2 N=%d n=%d" % (N, n))
    X = W.normal(451, N * n).reshape(N, n)
    h = N // 2
    S = st.covar_pr2(dev(X[:h]))
    st.covar_pr2(dev(X[h:]), S=S, accumulate=True)
    if n == 4:
        assert sum(t.numel() for t in S) == 65
    ref1 = oracle.moment2_dense(X)[np.triu_indices(n)]
    ref2 = oracle.moment3_entries(X, oracle.list_sym3(n))
    ref3 = oracle.moment4_entries(X, oracle.list_sym4(n))
    for got, ref in zip(S, (ref1, ref2, ref3)):
        assert got.numel() == ref.size
        check(got.cpu().numpy(), ref)
    # the same three results from the three separate entry points: bit for bit where the call runs those three
    # kernels; up to sixteen features it is one fused pass of its own, with its own summation order
    A = (st.moment2_sym(dev(X[:h])), st.moment3_sym(dev(X[:h])), st.moment4_sym(dev(X[:h])))
    st.moment2_sym(dev(X[h:]), Sc=A[0], accumulate=True)
    st.moment3_sym(dev(X[h:]), Sc=A[1], accumulate=True)
    st.moment4_sym(dev(X[h:]), Sc=A[2], accumulate=True)
    for got, sep, ref in zip(S, A, (ref1, ref2, ref3)):
        if n > 16:
            assert np.array_equal(got.cpu().numpy(), sep.cpu().numpy())
        else:
            check(sep.cpu().numpy(), ref)
    S2 = st.covar_pr2(dev(X))
    S3 = st.covar_pr2(dev(X))
    for u, v in zip(S2, S3):
        assert np.array_equal(u.cpu().numpy(), v.cpu().numpy())          # deterministic


# ---------------------------------------------------------------------- mttkrp
@pytest.mark.parametrize("n,R", [(1, 1), (5, 4), (16, 16), (17, 3), (32, 5), (40, 16), (64, 16), (96, 32),
                                 (100, 20), (130, 64), (48, 80), (160, 20), (208, 7)])
def test_mttkrp_small(st, oracle, n, R):
    say("mttkrp n=%d R=%d" % (n, R))
    Tc, B = W.mttkrp_inputs(n, R, oracle.count_sym3(n), "uniform", config_index=1)
    ref = oracle.mttkrp_sym3(Tc, B)
    got = st.mttkrp_sym3(dev(Tc), dev(B)).cpu().numpy()
    check(got, ref)
    got2 = st.mttkrp_sym3(dev(Tc), dev(B)).cpu().numpy()
    assert np.array_equal(got, got2)                      # deterministic


@pytest.mark.parametrize("n,R", [(70, 8), (80, 8)])
def test_mttkrp_all_ones(st, n, R):
    B = W.uniform(501, n * R).reshape(n, R)
    ones = np.ones(st.count_sym3(n), dtype=np.float32)
    got = st.mttkrp_sym3(dev(ones), dev(B)).cpu().numpy()
    ref = np.tile(B.astype(np.float64).sum(axis=0) ** 2, (n, 1))
    check(got, ref)


def test_mttkrp_one_item_per_pair(st, oracle):
    """n = 496 (31 blocks): the smallest size with one unchunked item per block pair."""
    n, R = 496, 48
    say("mttkrp n=%d R=%d" % (n, R))
    Tc, B = W.mttkrp_inputs(n, R, oracle.count_sym3(n), "normal", config_index=4)
    got = st.mttkrp_sym3(dev(Tc), dev(B)).cpu().numpy()
    rows = np.array([0, 7, 16, 100, 239, 240, 241, 255, 256, 300, 479, 480, 495], dtype=np.int64)
    ref = oracle.mttkrp_sym3(Tc, B, rows=rows)
    err = float(np.abs(got[rows] - ref).max() / np.abs(ref).max())
    say("  norm-wise error on the sampled rows %.3e" % err)
    assert err <= TOL
    got2 = st.mttkrp_sym3(dev(Tc), dev(B)).cpu().numpy()
    assert np.array_equal(got, got2)


def test_mttkrp_full(st, oracle):
    cfg = W.CONFIGS[4]
    n, R = cfg["n"], cfg["R"]
    say("mttkrp full n=%d R=%d: generating" % (n, R))
    Tc, B = W.mttkrp_inputs(n, R, cfg["entries"], cfg["b_dist"], config_index=4)
    got = st.mttkrp_sym3(dev(Tc), dev(B)).cpu().numpy()
    say("  oracle on all %d rows" % n)
    ref = np.empty((n, R), dtype=np.float64)
    for r0 in range(0, n, 64):
        ref[r0:r0 + 64] = oracle.mttkrp_sym3(Tc, B, rows=np.arange(r0, min(n, r0 + 64), dtype=np.int64))
        say("  oracle: rows %d .. %d" % (r0, min(n, r0 + 64) - 1))
    check(got, ref, "mttkrp full, all %d x %d outputs" % (n, R))
    got2 = st.mttkrp_sym3(dev(Tc), dev(B)).cpu().numpy()
    assert np.array_equal(got, got2)                      # deterministic


# ------------------------------------------------------------ non-finite inputs
@pytest.mark.parametrize("N,n,c", [(1001, 128, 5), (1003, 190, 189), (999, 64, 63), (1002, 250, 77), (513, 513, 512)])
def test_moment2_infinite_sample(st, oracle, N, n, c):
    """An infinite value in the LAST row of X, with N not a multiple of four: a kernel that pads its last group of
    rows by re-reading a valid row and multiplying by zero would turn that value into NaN.  The definition gives
    +-inf in every entry that involves column c and leaves the others finite."""
    say("moment2 with an infinite sample N=%d n=%d column %d" % (N, n, c))
    X = W.normal(471, N * n).reshape(N, n).copy()
    X[N - 1, c] = np.inf
    ref = oracle.moment2_dense(X)[np.triu_indices(n)]
    assert np.isinf(ref).sum() == n and not np.isnan(ref).any()
    inf_pattern_matches(st.moment2_sym(dev(X)).cpu().numpy(), ref)


@pytest.mark.parametrize("N,n,c", [(1001, 64, 63), (777, 64, 0), (301, 40, 7), (203, 100, 99)])
def test_moment3_infinite_sample(st, oracle, N, n, c):
    say("moment3 with an infinite sample N=%d n=%d column %d" % (N, n, c))
    X = W.normal(472, N * n).reshape(N, n).copy()
    X[N - 1, c] = np.inf
    ref = oracle.moment3_entries(X, oracle.list_sym3(n))
    assert np.isinf(ref).sum() == n * (n + 1) // 2 and not np.isnan(ref).any()
    inf_pattern_matches(st.moment3_sym(dev(X)).cpu().numpy(), ref)


@pytest.mark.parametrize("n,i", [(300, 7), (1000, 998), (4100, 2000), (8192, 8190)])
def test_batax_infinite_entry(st, oracle, n, i):
    """The last entry of packed row i is infinite: the next row's leading 16-byte group starts before that row
    and reads it, so it must be dropped by selection, never by a multiplication with zero.  t_i is infinite,
    so y_j is infinite for j >= i; for j < i the dense definition multiplies the structural zero A(i,j) by the
    infinite t_i, which is NaN in IEEE arithmetic -- in the definition and in the kernel alike."""
    say("batax with an infinite entry n=%d row %d" % (n, i))
    Ap = W.uniform(473, oracle.count_sym2(n)).copy()
    x = W.uniform(474, n)
    row_end = sum(n - a for a in range(i + 1)) - 1          # position of A(i, n-1)
    Ap[row_end] = np.inf
    ref = oracle.batax_utri(Ap, x, 0.5)
    assert np.isinf(ref[i:]).all() and np.isnan(ref[:i]).all()
    inf_pattern_matches(st.batax_utri(dev(Ap), dev(x), 0.5).cpu().numpy(), ref)


@pytest.mark.parametrize("n,R,t", [(64, 16, (3, 17, 40)), (100, 20, (5, 50, 99)), (128, 64, (15, 16, 127)),
                                   (128, 64, (40, 41, 42))])
def test_mttkrp_infinite_entry(st, oracle, n, R, t):
    """One stored entry (a < b < c) is infinite: rows a, b and c of the result are infinite in every column
    (B has no zeros), every other row stays finite."""
    say("mttkrp with an infinite entry n=%d R=%d at %s" % (n, R, t))
    Tc, B = W.mttkrp_inputs(n, R, oracle.count_sym3(n), "uniform", config_index=1)
    Tc = Tc.copy()
    Tc[lex_position3(n, t)] = np.inf
    ref = oracle.mttkrp_sym3(Tc, B)
    assert np.isinf(ref).sum() == 3 * R and not np.isnan(ref).any()
    inf_pattern_matches(st.mttkrp_sym3(dev(Tc), dev(B)).cpu().numpy(), ref)


# ------------------------------------------- the kernel table's sparsity structures
def _struct_support(st, structure, ni, nj, fixed):
    """(i, j) of every packed fibre, in packed order (built here from the table's unique sets)."""
    if structure == st.STRUCT_DIAG:
        return [(p, p) for p in range(min(ni, nj))]
    if structure == st.STRUCT_FIXED_I:
        return [(fixed, j) for j in range(nj)]
    if structure == st.STRUCT_FIXED_J:
        return [(i, fixed) for i in range(ni)]
    return [(i, j) for i in range(ni) for j in range(i, nj)]


def _scatter(Bc, support, ni, nj, nl):
    B = np.zeros((ni, nj, nl), dtype=np.float32)
    for p, (i, j) in enumerate(support):
        B[i, j] = Bc[p]
    return B


@pytest.mark.parametrize("structure,ni,nj,nl,R,fixed", [
    (0, 9, 9, 16, 16, 0), (0, 40, 33, 64, 32, 0), (0, 300, 300, 128, 64, 0),
    (2, 50, 7, 20, 5, 3), (2, 200, 9, 256, 48, 8), (1, 4, 77, 512, 16, 2),
    (3, 12, 12, 24, 8, 0), (3, 40, 40, 64, 64, 0), (3, 1, 1, 1, 1, 0)])
def test_ttm_struct(st, oracle, structure, ni, nj, nl, R, fixed):
    say("ttm_struct s=%d ni=%d nj=%d nl=%d R=%d" % (structure, ni, nj, nl, R))
    sup = _struct_support(st, structure, ni, nj, fixed)
    assert st.count_struct(structure, ni, nj) == len(sup)
    Bc = W.uniform(601, len(sup) * nl).reshape(len(sup), nl)
    U = W.uniform(602, nl * R).reshape(nl, R)
    full = oracle.ttm_full(_scatter(Bc, sup, ni, nj, nl), U)          # dense definition on the zero-filled B
    ii, jj = np.array(sup).T
    ref = full[ii, jj]
    mask = np.ones((ni, nj), dtype=bool)
    mask[ii, jj] = False
    assert not full[mask].any()                                       # the output keeps the unique set of B
    got = st.ttm_struct(structure, dev(Bc), dev(U), ni, nj).cpu().numpy()
    assert got.shape == ref.shape
    check(got, ref)


@pytest.mark.parametrize("structure,ni,nj,nl,fixed", [
    (0, 9, 9, 16, 0), (0, 40, 33, 7, 0), (0, 200, 200, 128, 0),
    (1, 4, 77, 64, 2), (1, 9, 300, 5, 8), (2, 50, 7, 20, 3), (2, 300, 9, 256, 0),
    (3, 12, 12, 24, 0), (3, 70, 70, 33, 0), (3, 1, 1, 1, 0)])
def test_thp_struct(st, oracle, structure, ni, nj, nl, fixed):
    say("thp_struct s=%d ni=%d nj=%d nl=%d" % (structure, ni, nj, nl))
    sup = _struct_support(st, structure, ni, nj, fixed)
    Bc = W.uniform(611, len(sup) * nl).reshape(len(sup), nl)
    Cd = W.uniform(612, ni * nj * nl).reshape(ni, nj, nl)
    full = oracle.thp_full(_scatter(Bc, sup, ni, nj, nl), Cd)
    ii, jj = np.array(sup).T
    ref = full[ii, jj]
    got = st.thp_struct(structure, dev(Bc), dev(Cd), fixed).cpu().numpy()
    assert got.shape == ref.shape
    # one fp32 product: the correctly rounded fp64 product is the only right answer
    assert np.array_equal(got, ref.astype(np.float32))
    assert np.count_nonzero(full) == np.count_nonzero(ref)            # nothing outside the unique set


@pytest.mark.parametrize("kind,ni,nk,nl,R,fi,fk", [
    (0, 5, 7, 33, 70, 2, 6), (0, 3, 3, 512, 64, 0, 0),
    (1, 5, 100, 64, 48, 4, 0), (1, 3, 9, 7, 300, 1, 0), (1, 2, 512, 512, 64, 0, 0),
    (2, 77, 6, 128, 32, 0, 5), (2, 9, 4, 10, 3, 0, 1), (2, 512, 3, 512, 64, 0, 2)])
def test_mttkrp_fixed(st, oracle, kind, ni, nk, nl, R, fi, fk):
    say("mttkrp_fixed kind=%d ni=%d nk=%d nl=%d R=%d" % (kind, ni, nk, nl, R))
    C = W.uniform(621, nk * R).reshape(nk, R)
    D = W.uniform(622, nl * R).reshape(nl, R)
    B = np.zeros((ni, nk, nl), dtype=np.float32)
    if kind == st.MTTKRP_FIXED_IK:
        Bc = W.uniform(623, nl)
        B[fi, fk] = Bc
    elif kind == st.MTTKRP_FIXED_I:
        Bc = W.uniform(623, nk * nl).reshape(nk, nl)
        B[fi] = Bc
    else:
        Bc = W.uniform(623, ni * nl).reshape(ni, nl)
        B[:, fk] = Bc
    full = oracle.mttkrp_full(B, C, D)                                # dense definition on the zero-filled B
    if kind == st.MTTKRP_FIXED_K:
        ref = full
    else:
        ref = full[fi]
        assert not np.delete(full, fi, axis=0).any()                  # only row I of the output is non-zero
    got = st.mttkrp_fixed(kind, dev(Bc), dev(C), dev(D), ni, fk).cpu().numpy()
    assert got.shape == ref.shape
    check(got, ref)
    got2 = st.mttkrp_fixed(kind, dev(Bc), dev(C), dev(D), ni, fk).cpu().numpy()
    assert np.array_equal(got, got2)                                  # deterministic


@pytest.mark.parametrize("n,w,nl", [(1, 0, 1), (9, 0, 5), (20, 3, 8), (13, 40, 4), (64, 8, 64), (100, 5, 3)])
def test_expand_band(st, oracle, n, w, nl):
    say("expand_band n=%d w=%d nl=%d" % (n, w, nl))
    Tc = W.uniform(631, oracle.count_band(n, w) * nl)
    ref = oracle.dense_band(Tc, n, w, nl).astype(np.float32)
    got = st.expand_band(dev(Tc), n, w, nl).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_table_full_sizes(st, oracle):
    """The kernel table at the size of the band workload (512 x 512 x 512, R = 64): sampled fibres."""
    ni = nj = nl = 512
    R = 64
    rng = np.random.default_rng(11)
    U = W.uniform(642, nl * R).reshape(nl, R)
    # TTM, upper half cube: 131,328 fibres
    pairs = st.count_struct(st.STRUCT_UPPER, ni, nj)
    say("table full: ttm upper half cube, %d fibres" % pairs)
    Bc = W.uniform(641, pairs * nl).reshape(pairs, nl)
    got = st.ttm_struct(st.STRUCT_UPPER, dev(Bc), dev(U), ni, nj).cpu().numpy()
    pick = np.unique(np.concatenate([rng.integers(0, pairs, 500), [0, pairs - 1]]))
    ref = oracle.ttm_full(Bc[pick][None], U)[0]                        # each fibre is independent
    assert float(np.abs(got[pick] - ref).max() / np.abs(ref).max()) <= TOL
    # THP, diagonal plane against a dense 512^3 operand
    say("table full: thp diagonal plane")
    Cd = W.uniform(643, ni * nj * nl).reshape(ni, nj, nl)
    Bd = Bc[:ni]
    got = st.thp_struct(st.STRUCT_DIAG, dev(Bd), dev(Cd)).cpu().numpy()
    ref = oracle.thp_full(Bd, Cd[np.arange(ni), np.arange(ni)])
    assert np.array_equal(got, ref.astype(np.float32))
    # THP, upper half cube (every fibre of the dense operand above the diagonal is gathered)
    say("table full: thp upper half cube")
    got = st.thp_struct(st.STRUCT_UPPER, dev(Bc), dev(Cd)).cpu().numpy()
    lst = oracle.list_sym2(ni).astype(np.int64)
    ref = oracle.thp_full(Bc, Cd[lst[:, 0], lst[:, 1]])
    assert np.array_equal(got, ref.astype(np.float32))
    # band expansion of the band workload
    say("table full: expand_band")
    cfg = W.CONFIGS[3]
    Tb, _ = W.ttm_inputs(cfg["band_pairs"], cfg["nl"], cfg["R"])
    got = st.expand_band(dev(Tb), cfg["n"], cfg["w"], cfg["nl"]).cpu().numpy()
    ref = oracle.dense_band(Tb, cfg["n"], cfg["w"], cfg["nl"]).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


# ------------------------------------------------------------ calls enqueue kernels only
@pytest.mark.parametrize("order,n,N", [(3, 128, 3000), (4, 80, 600), (3, 64, 5000)])
def test_moment_calls_can_be_captured(st, oracle, order, n, N):
    """A call enqueues kernels only (the table-driven paths bring their tile table into the workspace with a
    kernel), so it can be captured in a HIP graph: captured once, replayed three times on changing inputs with
    eager work and synchronisations in between, every replay compared with the eager result."""
    import torch
    say("graph capture of moment%d n=%d" % (order, n))
    f = st.moment3_sym if order == 3 else st.moment4_sym
    count = st.count_sym3(n) if order == 3 else st.count_sym4(n)
    X = dev(W.normal(481, N * n).reshape(N, n))
    Sc = torch.empty(count, device="cuda")
    ws = torch.empty(max(16, st.workspace_bytes("moment%d_sym" % order, N=N, n=n)), dtype=torch.uint8, device="cuda")
    f(X, Sc=Sc, ws=ws)                                     # first use outside the capture (builds the table)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        f(X, Sc=Sc, ws=ws)
    for rep in range(3):
        X.copy_(dev(W.normal(482 + rep, N * n).reshape(N, n)))
        want = f(X.clone()).clone()                        # eager, its own workspace and output
        torch.cuda.synchronize()
        Sc.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Sc, want), (order, n, rep)


def test_whole_step_can_be_captured(st, oracle):
    """The six calls of one step (both MTTKRP paths, the one-pass BATAX, the one-shot TTM, the third moment and
    its reconstruction) recorded into ONE HIP graph and replayed three times on changing inputs, with eager work
    and synchronisations between the replays: every output of every replay equals the eager result bit for bit
    (all reductions are in a fixed order), and the first replay is also compared with the oracle."""
    import torch
    say("graph capture of a whole step (small shapes)")
    n1, R1, n2, nb, w, nl, R3, n4, R4, N, n5 = 64, 16, 1000, 96, 3, 512, 64, 96 + 16, 64, 9000, 64
    pairs = oracle.count_band(nb, w)
    def inputs(seed):
        u = lambda k, c: dev(W.uniform(seed * 16 + k, c))
        return dict(T1=u(0, oracle.count_sym3(n1)), B1=u(1, n1 * R1).reshape(n1, R1), Ap=u(2, oracle.count_sym2(n2)), x=u(3, n2),
                    T3=u(4, pairs * nl).reshape(pairs, nl), U=u(5, nl * R3).reshape(nl, R3), T4=u(6, oracle.count_sym3(n4)),
                    B4=dev(W.normal(seed * 16 + 7, n4 * R4, std=0.1).reshape(n4, R4)), X=dev(W.normal(seed * 16 + 8, N * n5).reshape(N, n5)))
    buf = inputs(700)
    f32 = dict(dtype=torch.float32, device="cuda")
    out = dict(M1=torch.empty((n1, R1), **f32), y=torch.empty(n2, **f32), Yc=torch.empty((pairs, R3), **f32),
               M4=torch.empty((n4, R4), **f32), Sc=torch.empty(oracle.count_sym3(n5), **f32), S=torch.empty((n5,) * 3, **f32))
    wsb = max(st.workspace_bytes("mttkrp_sym3", n=n1, R=R1), st.workspace_bytes("batax_utri", n=n2),
              st.workspace_bytes("ttm_band", n=nb, w=w, nl=nl, R=R3), st.workspace_bytes("mttkrp_sym3", n=n4, R=R4),
              st.workspace_bytes("moment3_sym", N=N, n=n5), 16)
    def step(o, ws):
        st.mttkrp_sym3(buf["T1"], buf["B1"], M=o["M1"], ws=ws)
        st.batax_utri(buf["Ap"], buf["x"], 0.5, y=o["y"], ws=ws)
        st.ttm_band(buf["T3"], buf["U"], nb, w, Yc=o["Yc"], ws=ws)
        st.mttkrp_sym3(buf["T4"], buf["B4"], M=o["M4"], ws=ws)
        st.moment3_sym(buf["X"], Sc=o["Sc"], ws=ws)
        st.expand_sym(o["Sc"], n5, 3, S=o["S"])
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    step(out, ws)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(out, ws)
    ws2 = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    for rep in range(3):
        for k, v in inputs(701 + rep).items():
            buf[k].copy_(v)
        want = {k: torch.empty_like(v) for k, v in out.items()}
        step(want, ws2)                                    # eager, its own outputs and workspace
        torch.cuda.synchronize()
        for v in out.values():
            v.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for k in out:
            assert torch.equal(out[k], want[k]), (k, rep)
        if rep == 0:
            check(out["M4"].cpu().numpy(), oracle.mttkrp_sym3(buf["T4"].cpu().numpy(), buf["B4"].cpu().numpy()), "captured mttkrp")
            check(out["y"].cpu().numpy(), oracle.batax_utri(buf["Ap"].cpu().numpy(), buf["x"].cpu().numpy(), 0.5), "captured batax")


def test_random_shapes_against_the_oracle(st, oracle):
    """A seeded sweep over shapes no other case names: the launchers choose kernels by shape (row kernel, pair items
    and repacked tensors for MTTKRP; one- and two-pass BATAX; five contraction kernels behind the band TTM; the
    lane-per-sample, matrix-core and register-tile moment kernels), and every choice must agree with the oracle."""
    import random
    rng = random.Random(20221118)
    say("random shapes against the oracle")
    for _ in range(24):
        n = rng.choice([rng.randint(1, 40), rng.randint(41, 100), rng.choice([16, 32, 48, 64, 96, 112])])
        R = rng.choice([1, 3, 16, 20, 32, 33, 64, 80])
        Tc, B = W.uniform(rng.randrange(1 << 30), oracle.count_sym3(n)), W.uniform(rng.randrange(1 << 30), n * R).reshape(n, R)
        check(st.mttkrp_sym3(dev(Tc), dev(B)).cpu().numpy(), oracle.mttkrp_sym3(Tc, B), None)
    for _ in range(12):
        n = rng.choice([rng.randint(1, 300), rng.randint(1000, 3000)])
        Ap, x = W.uniform(rng.randrange(1 << 30), oracle.count_sym2(n)), W.uniform(rng.randrange(1 << 30), n)
        check(st.batax_utri(dev(Ap), dev(x), 0.5).cpu().numpy(), oracle.batax_utri(Ap, x, 0.5), None)
    for _ in range(24):
        n, w = rng.randint(1, 60), rng.randint(0, 9)
        nl, R = rng.choice([64, 128, 192, 256, 512, 33, 100, 7, 1]), rng.choice([16, 32, 48, 64, 5, 20, 63, 1, 130])
        pairs = oracle.count_band(n, w)
        Tc, U = W.uniform(rng.randrange(1 << 30), pairs * nl).reshape(pairs, nl), W.uniform(rng.randrange(1 << 30), nl * R).reshape(nl, R)
        check(st.ttm_band(dev(Tc), dev(U), n, w).cpu().numpy(), oracle.ttm_band(Tc.reshape(-1), U, n, w), None)
    for _ in range(24):
        n, N = rng.choice([rng.randint(1, 64), rng.randint(65, 100)]), rng.choice([1, 3, 63, 64, 65, 257, 1000])
        X = W.normal(rng.randrange(1 << 30), N * n).reshape(N, n)
        check(st.moment3_sym(dev(X)).cpu().numpy(), oracle.moment3_entries(X, oracle.list_sym3(n)), None)
        check(st.moment2_sym(dev(X)).cpu().numpy(), oracle.moment2_dense(X)[np.triu_indices(n)], None)
        if n <= 40:
            check(st.moment4_sym(dev(X)).cpu().numpy(), oracle.moment4_entries(X, oracle.list_sym4(n)), None)
