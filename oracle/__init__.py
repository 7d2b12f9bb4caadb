"""fp64 CPU oracle of the structured-tensor kernels -- TEST INFRASTRUCTURE.

Thin ctypes wrapper over ``st_oracle.c`` (plain C, dense definitions, its own
index enumeration by counting loops).  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; the product never does.
It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build import LIB, build

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        _lib = C.CDLL(LIB)
        i64, p = C.c_int64, C.c_void_p
        sig = {
            "so_enum_sym2": (i64, [i64, p]),
            "so_enum_sym3": (i64, [i64, p]),
            "so_count_sym4": (i64, [i64]),
            "so_enum_band": (i64, [i64, i64, p]),
            "so_list_sym2": (i64, [i64, p]),
            "so_list_sym3": (i64, [i64, p]),
            "so_list_sym4": (i64, [i64, p]),
            "so_list_band": (i64, [i64, i64, p]),
            "so_dense_sym3": (None, [p, i64, p]),
            "so_dense_utri": (None, [p, i64, p]),
            "so_dense_band": (None, [p, i64, i64, i64, p]),
            "so_mttkrp_sym3": (None, [p, p, i64, i64, p, i64, p]),
            "so_batax_utri": (None, [p, p, i64, C.c_double, p]),
            "so_ttm_dense": (None, [p, p, i64, i64, i64, i64, p]),
            "so_ttm_band": (None, [p, p, i64, i64, i64, i64, p]),
            "so_ttm_full": (None, [p, p, i64, i64, i64, i64, p]),
            "so_thp_full": (None, [p, p, i64, p]),
            "so_mttkrp_full": (None, [p, p, p, i64, i64, i64, i64, p]),
            "so_moment3_dense": (None, [p, i64, i64, p]),
            "so_moment3_entries": (None, [p, i64, i64, p, i64, p]),
            "so_moment2_dense": (None, [p, i64, i64, p]),
            "so_moment4_dense": (None, [p, i64, i64, p]),
            "so_moment4_entries": (None, [p, i64, i64, p, i64, p]),
            "so_expand_sym": (C.c_int, [p, i64, C.c_int, p]),
            "so_num_threads": (C.c_int, []),
            "so_set_num_threads": (None, [C.c_int]),
        }
        for name, (res, args) in sig.items():
            f = getattr(_lib, name)
            f.restype, f.argtypes = res, args
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data


def num_threads():
    return int(lib().so_num_threads())


def set_num_threads(threads):
    """Threads of the parallel loops from now on (results do not depend on it)."""
    lib().so_set_num_threads(int(threads))


# ---- enumeration ---------------------------------------------------------
def count_sym2(n):
    return int(lib().so_enum_sym2(n, None))


def count_sym3(n):
    return int(lib().so_enum_sym3(n, None))


def count_sym4(n):
    return int(lib().so_count_sym4(n))


def count_band(n, w):
    return int(lib().so_enum_band(n, w, None))


def table_sym2(n):
    tab = np.empty((n, n), dtype=np.int64)
    lib().so_enum_sym2(n, tab.ctypes.data)
    return tab


def table_sym3(n):
    tab = np.empty((n, n, n), dtype=np.int64)
    lib().so_enum_sym3(n, tab.ctypes.data)
    return tab


def table_band(n, w):
    tab = np.empty((n, n), dtype=np.int64)
    lib().so_enum_band(n, w, tab.ctypes.data)
    return tab


def list_sym2(n):
    out = np.empty((count_sym2(n), 2), dtype=np.int32)
    lib().so_list_sym2(n, out.ctypes.data)
    return out


def list_sym3(n):
    out = np.empty((count_sym3(n), 3), dtype=np.int16)
    lib().so_list_sym3(n, out.ctypes.data)
    return out


def list_sym4(n):
    out = np.empty((count_sym4(n), 4), dtype=np.int16)
    lib().so_list_sym4(n, out.ctypes.data)
    return out


def list_band(n, w):
    out = np.empty((count_band(n, w), 2), dtype=np.int32)
    lib().so_list_band(n, w, out.ctypes.data)
    return out


# ---- dense materialisation -------------------------------------------------
def dense_sym3(Tc, n):
    Tc, pT = _f32(Tc)
    assert Tc.size == count_sym3(n)
    T = np.empty((n, n, n), dtype=np.float64)
    lib().so_dense_sym3(pT, n, T.ctypes.data)
    return T


def dense_utri(Ap, n):
    Ap, pA = _f32(Ap)
    assert Ap.size == count_sym2(n)
    A = np.empty((n, n), dtype=np.float64)
    lib().so_dense_utri(pA, n, A.ctypes.data)
    return A


def dense_band(Tc, n, w, nl):
    Tc, pT = _f32(Tc)
    assert Tc.size == count_band(n, w) * nl
    T = np.empty((n, n, nl), dtype=np.float64)
    lib().so_dense_band(pT, n, w, nl, T.ctypes.data)
    return T


# ---- the five operations -----------------------------------------------------
def mttkrp_sym3(Tc, B, rows=None):
    """M(i,r) = sum_jk T(i,j,k) B(j,r) B(k,r); optional subset of rows."""
    B, pB = _f32(B)
    n, R = B.shape
    Tc, pT = _f32(Tc)
    assert Tc.size == count_sym3(n)
    if rows is None:
        M = np.empty((n, R), dtype=np.float64)
        lib().so_mttkrp_sym3(pT, pB, n, R, None, n, M.ctypes.data)
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        assert rows.size == 0 or (rows.min() >= 0 and rows.max() < n)
        M = np.empty((rows.size, R), dtype=np.float64)
        lib().so_mttkrp_sym3(pT, pB, n, R, rows.ctypes.data, rows.size, M.ctypes.data)
    return M


def batax_utri(Ap, x, beta):
    x, px = _f32(x)
    n = x.size
    Ap, pA = _f32(Ap)
    assert Ap.size == count_sym2(n)
    y = np.empty(n, dtype=np.float64)
    lib().so_batax_utri(pA, px, n, float(beta), y.ctypes.data)
    return y


def ttm_dense(Tc, U, n, w):
    U, pU = _f32(U)
    nl, R = U.shape
    Tc, pT = _f32(Tc)
    assert Tc.size == count_band(n, w) * nl
    Y = np.empty((n, n, R), dtype=np.float64)
    lib().so_ttm_dense(pT, pU, n, w, nl, R, Y.ctypes.data)
    return Y


def ttm_band(Tc, U, n, w):
    U, pU = _f32(U)
    nl, R = U.shape
    Tc, pT = _f32(Tc)
    nb = count_band(n, w)
    assert Tc.size == nb * nl
    Yc = np.empty((nb, R), dtype=np.float64)
    lib().so_ttm_band(pT, pU, n, w, nl, R, Yc.ctypes.data)
    return Yc


def ttm_full(B, U):
    """A(i,j,r) = sum_l B(i,j,l) U(l,r) on a dense B (ni x nj x nl)."""
    B, pB = _f32(B)
    U, pU = _f32(U)
    ni, nj, nl = B.shape
    assert U.shape[0] == nl
    R = U.shape[1]
    A = np.empty((ni, nj, R), dtype=np.float64)
    lib().so_ttm_full(pB, pU, ni, nj, nl, R, A.ctypes.data)
    return A


def thp_full(B, C):
    """A = B * C elementwise (dense operands of equal shape)."""
    B, pB = _f32(B)
    C, pC = _f32(C)
    assert B.shape == C.shape
    A = np.empty(B.shape, dtype=np.float64)
    lib().so_thp_full(pB, pC, B.size, A.ctypes.data)
    return A


def mttkrp_full(B, C, D):
    """A(i,j) = sum_kl B(i,k,l) C(k,j) D(l,j) on a dense B (ni x nk x nl)."""
    B, pB = _f32(B)
    C, pC = _f32(C)
    D, pD = _f32(D)
    ni, nk, nl = B.shape
    R = C.shape[1]
    assert C.shape[0] == nk and D.shape == (nl, R)
    A = np.empty((ni, R), dtype=np.float64)
    lib().so_mttkrp_full(pB, pC, pD, ni, nk, nl, R, A.ctypes.data)
    return A


def moment3_dense(X):
    X, pX = _f32(X)
    N, n = X.shape
    S = np.empty((n, n, n), dtype=np.float64)
    lib().so_moment3_dense(pX, N, n, S.ctypes.data)
    return S


def moment3_entries(X, ijk):
    X, pX = _f32(X)
    N, n = X.shape
    ijk = np.ascontiguousarray(ijk, dtype=np.int32).reshape(-1, 3)
    assert ijk.size == 0 or (ijk.min() >= 0 and ijk.max() < n)
    out = np.empty(ijk.shape[0], dtype=np.float64)
    lib().so_moment3_entries(pX, N, n, ijk.ctypes.data, ijk.shape[0], out.ctypes.data)
    return out


def moment2_dense(X):
    """S(i,j) = sum_s x_s(i) x_s(j), all n^2 positions."""
    X, pX = _f32(X)
    N, n = X.shape
    S = np.empty((n, n), dtype=np.float64)
    lib().so_moment2_dense(pX, N, n, S.ctypes.data)
    return S


def moment4_dense(X):
    """S(i,j,k,l) = sum_s x_s(i) x_s(j) x_s(k) x_s(l), all n^4 positions (small n only)."""
    X, pX = _f32(X)
    N, n = X.shape
    S = np.empty((n, n, n, n), dtype=np.float64)
    lib().so_moment4_dense(pX, N, n, S.ctypes.data)
    return S


def moment4_entries(X, ijkl):
    X, pX = _f32(X)
    N, n = X.shape
    ijkl = np.ascontiguousarray(ijkl, dtype=np.int32).reshape(-1, 4)
    assert ijkl.size == 0 or (ijkl.min() >= 0 and ijkl.max() < n)
    out = np.empty(ijkl.shape[0], dtype=np.float64)
    lib().so_moment4_entries(pX, N, n, ijkl.ctypes.data, ijkl.shape[0], out.ctypes.data)
    return out


def expand_sym(Sc, n, order):
    Sc, pS = _f32(Sc)
    assert order in (2, 3, 4)
    assert Sc.size == {2: count_sym2, 3: count_sym3, 4: count_sym4}[order](n)
    S = np.empty((n,) * order, dtype=np.float32)
    rc = lib().so_expand_sym(pS, n, order, S.ctypes.data)
    assert rc == 0
    return S


# ---- structures given as predicates: brute force over the whole index box ----------------
# (test infrastructure for the descriptor-driven kernels: nothing here parses a descriptor;
# a test states the unique set and the redundancy map as plain Python functions)
def struct_enumerate(dims, in_unique):
    """Index tuples of the unique set in packed order: every tuple of the box, visited as nested
    loops in the order the variables are written with the last one fastest (the visiting order of
    the paper's generated nests, code generation section), kept when it satisfies the unique set."""
    import itertools
    return np.array([x for x in itertools.product(*[range(int(n)) for n in dims]) if in_unique(*x)],
                    dtype=np.int32).reshape(-1, len(dims))


def struct_expand(Tc, dims, in_unique, unique_of=None):
    """Property 5, T(x) = T_C(x) + T_R(x,x') * T_C(x'): the stored value on the unique set, the
    value stored at the unique index x' = unique_of(x) where the redundancy map gives one, zero
    elsewhere.  Positions come from a dictionary built by the enumeration above."""
    import itertools
    Tc = np.asarray(Tc)
    pos = {tuple(int(v) for v in x): p for p, x in enumerate(struct_enumerate(dims, in_unique))}
    T = np.zeros(tuple(int(n) for n in dims), dtype=Tc.dtype)
    for x in itertools.product(*[range(int(n)) for n in dims]):
        if x in pos:
            T[x] = Tc[pos[x]]
        elif unique_of is not None:
            y = unique_of(*x)
            if y is not None and tuple(y) in pos:
                T[x] = Tc[pos[tuple(y)]]
    return T


def struct_thp(Bc, C, dims, in_unique):
    """THP of the kernel table, A(x) = B(x) * C(x), evaluated on the unique set of B only (fp64)."""
    idx = struct_enumerate(dims, in_unique).astype(np.int64)
    Cv = np.asarray(C, dtype=np.float64)[tuple(idx[:, v] for v in range(idx.shape[1]))]
    return np.asarray(Bc, dtype=np.float64) * Cv


def struct_moment(X, dims, in_unique):
    """Sc(p) = sum_s prod_v X(s, x_v(p)) over the unique set in packed order (fp64): the covariance term of
    the overview's M1 / M2 nests ("creation and addition of covariance matrices") restricted to a structure.
    One sample at a time, in sample order: the product of the sample's values at the indices of every unique
    tuple, added to the running sum."""
    idx = struct_enumerate(dims, in_unique).astype(np.int64)
    Xd = np.asarray(X, dtype=np.float64)
    out = np.zeros(idx.shape[0], dtype=np.float64)
    for s in range(Xd.shape[0]):
        prod = np.ones(idx.shape[0], dtype=np.float64)
        for v in range(idx.shape[1]):
            prod = prod * Xd[s, idx[:, v]]
        out += prod
    return out


def direct_sum(M, V):
    """T = M (+) V for two dense arrays of the same order ("Representation of linear algebra operations", the
    rule for the direct sum; "Redundancy Map Inference", direct-sum rule): with d = dims(M), element x of the
    result is M(x) where every index lies below d, V(x - d) where every index lies at or above d, zero
    elsewhere.  Written as that case distinction, one element at a time."""
    import itertools
    M, V = np.asarray(M), np.asarray(V)
    assert M.ndim == V.ndim and M.dtype == V.dtype
    d = M.shape
    T = np.zeros(tuple(a + b for a, b in zip(M.shape, V.shape)), dtype=M.dtype)
    for x in itertools.product(*[range(n) for n in T.shape]):
        if all(x[v] < d[v] for v in range(M.ndim)):
            T[x] = M[x]
        elif all(x[v] >= d[v] for v in range(M.ndim)):
            T[x] = V[tuple(x[v] - d[v] for v in range(M.ndim))]
    return T
