"""Closed-form index maps of the library (host side) against the oracle's
counting-loop enumeration: bit-exact, exhaustive."""
import numpy as np
import pytest

import paper_2211_10482_amd as st


def test_counts(oracle):
    for n in list(range(0, 41)) + [64, 512]:
        assert st.count_sym2(n) == oracle.count_sym2(n)
        assert st.count_sym3(n) == oracle.count_sym3(n)
    assert st.count_sym2(8192) == oracle.count_sym2(8192) == 33_558_528
    for n in (1, 2, 3, 7, 12, 33):
        for w in range(0, n + 3):
            assert st.count_band(n, w) == oracle.count_band(n, w)
    assert st.count_band(512, 8) == 8_632
    assert st.count_sym2(-1) == -1 and st.count_sym3(-3) == -1 and st.count_band(4, -1) == -1


@pytest.mark.parametrize("n", list(range(1, 41)) + [64])
def test_sym_rank_unrank_exhaustive(oracle, n):
    tab2, tab3 = oracle.table_sym2(n), oracle.table_sym3(n)
    for i in range(n):
        for j in range(n):
            assert st.rank_sym2(n, i, j) == tab2[i, j]
    if n <= 24 or n == 64:
        idx = np.argwhere(tab3 >= 0)
        got = np.array([st.rank_sym3(n, int(i), int(j), int(k)) for i, j, k in idx[:: max(1, len(idx) // 4000)]])
        assert np.array_equal(got, tab3[tuple(idx[:: max(1, len(idx) // 4000)].T)])
    assert st.rank_sym3(n, 0, 0, 0) == 0
    assert st.rank_sym3(n, n - 1, n - 1, n - 1) == oracle.count_sym3(n) - 1
    assert st.rank_sym3(n, 1, 0, 0) == -1 and st.rank_sym2(n, 0, n) == -1
    assert np.array_equal(st.unrank_sym2_batch(n, 0, oracle.count_sym2(n)), oracle.list_sym2(n))
    assert np.array_equal(st.unrank_sym3_batch(n, 0, oracle.count_sym3(n)), oracle.list_sym3(n))
    p = oracle.count_sym3(n) // 2
    assert st.rank_sym3(n, *st.unrank_sym3(n, p)) == p


@pytest.mark.parametrize("n", [1, 2, 3, 7, 16, 33, 64])
def test_sym4_rank_unrank(oracle, n):
    lst = oracle.list_sym4(n)
    cnt = lst.shape[0]
    assert st.count_sym4(n) == cnt == oracle.count_sym4(n)
    assert np.array_equal(st.unrank_sym4_batch(n, 0, cnt), lst)
    step = max(1, cnt // 3000)
    for p in list(range(0, cnt, step)) + [cnt - 1]:
        i, j, k, l = (int(v) for v in lst[p])
        assert st.rank_sym4(n, i, j, k, l) == p
        assert st.unrank_sym4(n, p) == (i, j, k, l)
    assert st.rank_sym4(n, 0, 0, 0, 0) == 0 and st.rank_sym4(n, n - 1, n - 1, n - 1, n - 1) == cnt - 1
    assert st.rank_sym4(n, 1, 0, 0, 0) == -1 and st.rank_sym4(n, 0, 0, 0, n) == -1
    assert st.count_sym4(-2) == -1


def test_sym4_large_n():
    # 64-bit arithmetic far above the kernels' range: the ends and a few interior points
    import math
    for n in (300, 2000, 50000):
        cnt = st.count_sym4(n)
        assert cnt == math.comb(n + 3, 4)
        assert st.unrank_sym4(n, 0) == (0, 0, 0, 0) and st.unrank_sym4(n, cnt - 1) == (n - 1,) * 4
        for p in (1, n, cnt // 3, cnt // 2 + 12345, cnt - 2):
            t = st.unrank_sym4(n, p)
            assert t[0] <= t[1] <= t[2] <= t[3] < n and st.rank_sym4(n, *t) == p
        # first entry with first index i sits right after all entries with smaller first index
        i = n // 2
        assert st.rank_sym4(n, i, i, i, i) == cnt - math.comb(n - i + 3, 4)


def test_sym3_rank_all_small(oracle):
    for n in (1, 2, 3, 5, 9):
        tab3 = oracle.table_sym3(n)
        for i in range(n):
            for j in range(n):
                for k in range(n):
                    assert st.rank_sym3(n, i, j, k) == tab3[i, j, k]


def test_sym3_unrank_n512(oracle):
    n = 512
    lst = oracle.list_sym3(n)
    assert lst.shape[0] == 22_500_864
    got = st.unrank_sym3_batch(n, 0, lst.shape[0])
    assert np.array_equal(got, lst)
    # rank of a strided sample agrees with the position in the listing
    for p in range(0, lst.shape[0], 999_983):
        i, j, k = (int(v) for v in lst[p])
        assert st.rank_sym3(n, i, j, k) == p


def test_sym2_unrank_n8192(oracle):
    n = 8192
    lst = oracle.list_sym2(n)
    got = st.unrank_sym2_batch(n, 0, lst.shape[0])
    assert np.array_equal(got, lst)
    for p in range(0, lst.shape[0], 1_999_993):
        assert st.rank_sym2(n, int(lst[p, 0]), int(lst[p, 1])) == p


@pytest.mark.parametrize("n,w", [(1, 0), (2, 0), (2, 1), (5, 1), (5, 4), (5, 9), (12, 3), (33, 7), (33, 16),
                                 (33, 31), (40, 20), (512, 8), (512, 0)])
def test_band_rank_unrank(oracle, n, w):
    tab = oracle.table_band(n, w)
    lst = oracle.list_band(n, w)
    assert np.array_equal(st.unrank_band_batch(n, w, 0, lst.shape[0]), lst)
    step = max(1, n // 40)
    for i in range(0, n, step):
        for j in range(n):
            assert st.rank_band(n, w, i, j) == tab[i, j]
    assert st.rank_band(n, w, n - 1, n - 1) == lst.shape[0] - 1


def test_unrank_errors():
    with pytest.raises(st.StructTensorError) as e:
        st.unrank_sym3(4, 20)
    assert e.value.status == 2
    with pytest.raises(st.StructTensorError):
        st.unrank_sym2(4, -1)
    with pytest.raises(st.StructTensorError):
        st.unrank_band(4, 1, 10)
