"""ctypes binding of libstructtensor_hip.so: same names as the C ABI, argument
marshalling only (pointers, sizes, the current torch stream, a torch-allocated
workspace)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libstructtensor_hip.so")

_lib = None


class StructTensorError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s failed: status %d (%s)" % (what, status, _status_string(status)))


# names and signatures of include/structtensor.h
_I64, _I32, _P, _SZ, _F = C.c_int64, C.c_int, C.c_void_p, C.c_size_t, C.c_float
SIGNATURES = {
    "st_status_string": (C.c_char_p, [_I32]),
    "st_count_sym2": (_I64, [_I64]),
    "st_count_sym3": (_I64, [_I64]),
    "st_count_sym4": (_I64, [_I64]),
    "st_count_band": (_I64, [_I64, _I64]),
    "st_rank_sym2": (_I64, [_I64, _I64, _I64]),
    "st_rank_sym3": (_I64, [_I64, _I64, _I64, _I64]),
    "st_rank_sym4": (_I64, [_I64, _I64, _I64, _I64, _I64]),
    "st_rank_band": (_I64, [_I64, _I64, _I64, _I64]),
    "st_unrank_sym2": (_I32, [_I64, _I64, _P, _P]),
    "st_unrank_sym3": (_I32, [_I64, _I64, _P, _P, _P]),
    "st_unrank_sym4": (_I32, [_I64, _I64, _P, _P, _P, _P]),
    "st_unrank_band": (_I32, [_I64, _I64, _I64, _P, _P]),
    "st_unrank_sym2_batch": (_I32, [_I64, _I64, _I64, _P]),
    "st_unrank_sym3_batch": (_I32, [_I64, _I64, _I64, _P]),
    "st_unrank_sym4_batch": (_I32, [_I64, _I64, _I64, _P]),
    "st_unrank_band_batch": (_I32, [_I64, _I64, _I64, _I64, _P]),
    "st_unrank_device": (_I32, [_I32, _I64, _I64, _I64, _I64, _P, _P]),
    "st_mttkrp_sym3_workspace": (_SZ, [_I32, _I32]),
    "st_batax_utri_workspace": (_SZ, [_I32]),
    "st_ttm_band_workspace": (_SZ, [_I32, _I32, _I32, _I32]),
    "st_moment3_sym_workspace": (_SZ, [_I64, _I32]),
    "st_moment2_sym_workspace": (_SZ, [_I64, _I32]),
    "st_moment4_sym_workspace": (_SZ, [_I64, _I32]),
    "st_mttkrp_sym3": (_I32, [_P, _P, _P, _I32, _I32, _P, _SZ, _P]),
    "st_batax_utri": (_I32, [_P, _P, _P, _I32, _F, _P, _SZ, _P]),
    "st_batax_utri_noalloc_max_n": (_I32, []),
    "st_batax_utri_noalloc": (_I32, [_P, _P, _P, _I32, _F, _P]),
    "st_ttm_band": (_I32, [_P, _P, _P, _I32, _I32, _I32, _I32, _P, _SZ, _P]),
    "st_moment3_sym": (_I32, [_P, _I64, _I32, _P, _I32, _P, _SZ, _P]),
    "st_moment2_sym": (_I32, [_P, _I64, _I32, _P, _I32, _P, _SZ, _P]),
    "st_moment4_sym": (_I32, [_P, _I64, _I32, _P, _I32, _P, _SZ, _P]),
    "st_expand_sym": (_I32, [_P, _P, _I32, _I32, _P]),
    "st_count_struct": (_I64, [_I32, _I64, _I64]),
    "st_ttm_struct_workspace": (_SZ, [_I32, _I32, _I32, _I32, _I32]),
    "st_mttkrp_fixed_workspace": (_SZ, [_I32, _I32, _I32, _I32, _I32]),
    "st_ttm_struct": (_I32, [_I32, _P, _P, _P, _I32, _I32, _I32, _I32, _P, _SZ, _P]),
    "st_thp_struct": (_I32, [_I32, _P, _P, _P, _I32, _I32, _I32, _I32, _P]),
    "st_mttkrp_fixed": (_I32, [_I32, _P, _P, _P, _P, _I32, _I32, _I32, _I32, _I32, _P, _SZ, _P]),
    "st_expand_band": (_I32, [_P, _P, _I32, _I32, _I32, _P]),
    "st_desc_create": (_I32, [C.c_char_p, C.c_char_p, _P, _I32, _P, _P, _I32, _P]),
    "st_desc_destroy": (None, [_P]),
    "st_desc_error": (C.c_char_p, [_P]),
    "st_desc_count": (_I64, [_P]),
    "st_desc_runs": (_I64, [_P]),
    "st_desc_nest": (C.c_char_p, [_P]),
    "st_desc_source": (C.c_char_p, [_P]),
    "st_desc_table_bytes": (_SZ, [_P]),
    "st_desc_table": (_I32, [_P, _P]),
    "st_desc_compile": (_I32, [_P]),
    "st_desc_list": (_I32, [_P, _P, _P, _P]),
    "st_desc_thp": (_I32, [_P, _P, _P, _P, _P, _P]),
    "st_desc_mttkrp_workspace": (_SZ, [_P, _I32]),
    "st_desc_mttkrp": (_I32, [_P, _P, _P, _P, _P, _P, _I32, _P, _SZ, _P]),
    "st_desc_expand": (_I32, [_P, _P, _P, _P, _P]),
    "st_desc_ttm": (_I32, [_P, _P, _P, _P, _I32, _P]),
    "st_desc_product": (_I32, [_P, _P, _P]),
    "st_desc_gather": (_I32, [_P, _P, _P, _P, _I64, _I32, _I32, _P, _P, _P, _P]),
    "st_desc_sum": (_I32, [_P, _P, _P]),
    "st_desc_project": (_I32, [_P, _P]),
    "st_desc_sum_last": (_I32, [_P, _P, _P, _P, _P]),
    "st_desc_outer": (_I32, [_P, _P, _P]),
    "st_desc_power": (_I32, [_P, _I32, _P]),
    "st_desc_direct_sum": (_I32, [_P, _P, _P, _P]),
    "st_desc_expand_onto": (_I32, [_P, _P, _P, _P, _P]),
    "st_desc_moment_workspace": (_SZ, [_P, _I64]),
    "st_desc_moment": (_I32, [_P, _P, _P, _I64, _P, _I32, _P, _SZ, _P]),
    "st_probe_empty": (_I32, [_I32, _I32, _P]),
    "st_probe_stream": (_I32, [_P, _SZ, _I32, _I32, _P, _P]),
    "st_probe_mfma_f32": (_I32, [_I32, _I32, _P, _P]),
    "st_covar_pr2_workspace": (_SZ, [_I64, _I32]),
    "st_covar_pr2": (_I32, [_P, _I64, _I32, _P, _P, _P, _I32, _P, _SZ, _P]),
}

# structures of the kernel table (values of include/structtensor.h)
STRUCT_DIAG, STRUCT_FIXED_I, STRUCT_FIXED_J, STRUCT_UPPER = 0, 1, 2, 3
MTTKRP_FIXED_IK, MTTKRP_FIXED_I, MTTKRP_FIXED_K = 0, 1, 2


def lib():
    """Load the HIP library (built in-tree by ``build.py``).  No fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libstructtensor_hip.so is not built: run `python -m paper_2211_10482_amd.build` "
                "(there is no CPU fallback)")
        # The device pointers and streams this binding passes come from PyTorch, so both must talk to ONE HIP
        # runtime: PyTorch loads the copy it ships, and a library loaded after it binds to that copy.  Loaded
        # the other way round, the library would pull in the system's runtime and every launch would fail.
        import torch  # noqa: F401
        _lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            f = getattr(_lib, name)
            f.restype, f.argtypes = res, args
    return _lib


def _status_string(status: int) -> str:
    return lib().st_status_string(status).decode()


def _check(status: int, what: str):
    if status != 0:
        raise StructTensorError(status, what)


# ---- host index utilities --------------------------------------------------------
def count_sym2(n): return int(lib().st_count_sym2(n))
def count_sym3(n): return int(lib().st_count_sym3(n))
def count_sym4(n): return int(lib().st_count_sym4(n))
def count_band(n, w): return int(lib().st_count_band(n, w))
def rank_sym2(n, i, j): return int(lib().st_rank_sym2(n, i, j))
def rank_sym3(n, i, j, k): return int(lib().st_rank_sym3(n, i, j, k))
def rank_sym4(n, i, j, k, l): return int(lib().st_rank_sym4(n, i, j, k, l))
def rank_band(n, w, i, j): return int(lib().st_rank_band(n, w, i, j))


def count_struct(structure, ni, nj): return int(lib().st_count_struct(structure, ni, nj))


def unrank_sym2(n, p):
    i, j = _I64(), _I64()
    _check(lib().st_unrank_sym2(n, p, C.byref(i), C.byref(j)), "st_unrank_sym2")
    return i.value, j.value


def unrank_sym3(n, p):
    i, j, k = _I64(), _I64(), _I64()
    _check(lib().st_unrank_sym3(n, p, C.byref(i), C.byref(j), C.byref(k)), "st_unrank_sym3")
    return i.value, j.value, k.value


def unrank_sym4(n, p):
    i, j, k, l = _I64(), _I64(), _I64(), _I64()
    _check(lib().st_unrank_sym4(n, p, C.byref(i), C.byref(j), C.byref(k), C.byref(l)), "st_unrank_sym4")
    return i.value, j.value, k.value, l.value


def unrank_band(n, w, p):
    i, j = _I64(), _I64()
    _check(lib().st_unrank_band(n, w, p, C.byref(i), C.byref(j)), "st_unrank_band")
    return i.value, j.value


def unrank_sym2_batch(n, p0, count):
    out = np.empty((count, 2), dtype=np.int32)
    _check(lib().st_unrank_sym2_batch(n, p0, count, out.ctypes.data), "st_unrank_sym2_batch")
    return out


def unrank_sym3_batch(n, p0, count):
    out = np.empty((count, 3), dtype=np.int32)
    _check(lib().st_unrank_sym3_batch(n, p0, count, out.ctypes.data), "st_unrank_sym3_batch")
    return out


def unrank_sym4_batch(n, p0, count):
    out = np.empty((count, 4), dtype=np.int32)
    _check(lib().st_unrank_sym4_batch(n, p0, count, out.ctypes.data), "st_unrank_sym4_batch")
    return out


def unrank_band_batch(n, w, p0, count):
    out = np.empty((count, 2), dtype=np.int32)
    _check(lib().st_unrank_band_batch(n, w, p0, count, out.ctypes.data), "st_unrank_band_batch")
    return out


# ---- device entry points -----------------------------------------------------------
def _torch():
    import torch
    return torch


def _stream():
    return C.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _dev_f32(t, what):
    torch = _torch()
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous float32 CUDA tensor" % what)
    return C.c_void_p(t.data_ptr())


def _expect(t, numel, what, at_least=False):
    """The C ABI takes bare pointers, so a tensor of the wrong length would become an out-of-bounds device
    access: every packed operand and caller-supplied output is checked against the size of its unique set
    here, before anything is marshalled."""
    if not isinstance(t, _torch().Tensor):
        raise TypeError("%s must be a contiguous float32 CUDA tensor" % what)
    have = int(t.numel())
    if have != int(numel) and not (at_least and have > int(numel)):
        raise ValueError("%s holds %d elements, expected %s%d" % (what, have, "at least " if at_least else "", numel))


def _matrix(t, what):
    if not isinstance(t, _torch().Tensor):
        raise TypeError("%s must be a contiguous float32 CUDA tensor" % what)
    if t.dim() != 2:
        raise ValueError("%s must be a matrix, got %d dimensions" % (what, t.dim()))
    return int(t.shape[0]), int(t.shape[1])


def _workspace(nbytes, like, ws):
    torch = _torch()
    if ws is None:
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=like.device)
    if not (ws.is_cuda and ws.is_contiguous()):
        raise TypeError("workspace must be a contiguous CUDA tensor")
    return ws, C.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def workspace_bytes(kernel: str, **kw) -> int:
    L = lib()
    if kernel == "mttkrp_sym3":
        return int(L.st_mttkrp_sym3_workspace(kw["n"], kw["R"]))
    if kernel == "batax_utri":
        return int(L.st_batax_utri_workspace(kw["n"]))
    if kernel == "ttm_band":
        return int(L.st_ttm_band_workspace(kw["n"], kw["w"], kw["nl"], kw["R"]))
    if kernel == "moment3_sym":
        return int(L.st_moment3_sym_workspace(kw["N"], kw["n"]))
    if kernel == "moment4_sym":
        return int(L.st_moment4_sym_workspace(kw["N"], kw["n"]))
    if kernel == "moment2_sym":
        return int(L.st_moment2_sym_workspace(kw["N"], kw["n"]))
    if kernel == "covar_pr2":
        return int(L.st_covar_pr2_workspace(kw["N"], kw["n"]))
    if kernel == "ttm_struct":
        return int(L.st_ttm_struct_workspace(kw["structure"], kw["ni"], kw["nj"], kw["nl"], kw["R"]))
    if kernel == "mttkrp_fixed":
        return int(L.st_mttkrp_fixed_workspace(kw["kind"], kw["ni"], kw["nk"], kw["nl"], kw["R"]))
    raise KeyError(kernel)


def unrank_device(kind, n, w, p0, count):
    torch = _torch()
    width = {3: 3, 5: 4}.get(kind, 2)
    out = torch.empty((max(count, 1), width), dtype=torch.int32, device="cuda")
    _check(lib().st_unrank_device(kind, n, w, p0, count, C.c_void_p(out.data_ptr()), _stream()),
           "st_unrank_device")
    return out[:count]


def mttkrp_sym3(Tc, B, M=None, ws=None):
    torch = _torch()
    n, R = _matrix(B, "B")
    _expect(Tc, count_sym3(n), "Tc")
    if M is None:
        M = torch.empty((n, R), dtype=torch.float32, device=B.device)
    _expect(M, n * R, "M")
    ws, pws, wsb = _workspace(workspace_bytes("mttkrp_sym3", n=n, R=R), B, ws)
    _check(lib().st_mttkrp_sym3(_dev_f32(Tc, "Tc"), _dev_f32(B, "B"), _dev_f32(M, "M"), n, R, pws, wsb,
                                _stream()), "st_mttkrp_sym3")
    return M


def batax_utri(Ap, x, beta, y=None, ws=None):
    torch = _torch()
    n = x.numel()
    _expect(Ap, count_sym2(n), "Ap")
    if y is None:
        y = torch.empty(n, dtype=torch.float32, device=x.device)
    _expect(y, n, "y")
    ws, pws, wsb = _workspace(workspace_bytes("batax_utri", n=n), x, ws)
    _check(lib().st_batax_utri(_dev_f32(Ap, "Ap"), _dev_f32(x, "x"), _dev_f32(y, "y"), n, float(beta), pws,
                               wsb, _stream()), "st_batax_utri")
    return y


def batax_utri_noalloc(Ap, x, beta, y):
    """st_batax_utri through the library's static scratch array: the call allocates nothing, so the caller
    passes the output as well."""
    n = x.numel()
    _expect(Ap, count_sym2(n), "Ap")
    _expect(y, n, "y")
    _check(lib().st_batax_utri_noalloc(_dev_f32(Ap, "Ap"), _dev_f32(x, "x"), _dev_f32(y, "y"), n, float(beta),
                                       _stream()), "st_batax_utri_noalloc")
    return y


def ttm_band(Tc, U, n, w, Yc=None, ws=None):
    torch = _torch()
    nl, R = _matrix(U, "U")
    rows = count_band(n, w)
    if rows < 0:
        raise ValueError("n and w must be non-negative")
    _expect(Tc, rows * nl, "Tc")
    if Yc is None:
        Yc = torch.empty((rows, R), dtype=torch.float32, device=U.device)
    _expect(Yc, rows * R, "Yc")
    ws, pws, wsb = _workspace(workspace_bytes("ttm_band", n=n, w=w, nl=nl, R=R), U, ws)
    _check(lib().st_ttm_band(_dev_f32(Tc, "Tc"), _dev_f32(U, "U"), _dev_f32(Yc, "Yc"), n, w, nl, R, pws, wsb,
                             _stream()), "st_ttm_band")
    return Yc


def moment3_sym(X, Sc=None, accumulate=False, ws=None):
    torch = _torch()
    N, n = _matrix(X, "X")
    if Sc is None:
        if accumulate:
            raise ValueError("accumulate needs an existing Sc")
        Sc = torch.empty(count_sym3(n), dtype=torch.float32, device=X.device)
    _expect(Sc, count_sym3(n), "Sc")
    ws, pws, wsb = _workspace(workspace_bytes("moment3_sym", N=N, n=n), X, ws)
    px = _dev_f32(X, "X") if N > 0 else C.c_void_p(X.data_ptr() if X.numel() else 0)
    _check(lib().st_moment3_sym(px, N, n, _dev_f32(Sc, "Sc"), 1 if accumulate else 0, pws, wsb, _stream()),
           "st_moment3_sym")
    return Sc


def _moment(order, X, Sc, accumulate, ws):
    torch = _torch()
    N, n = _matrix(X, "X")
    name = "moment%d_sym" % order
    count = {2: count_sym2, 3: count_sym3, 4: count_sym4}[order](n)
    if Sc is None:
        if accumulate:
            raise ValueError("accumulate needs an existing Sc")
        Sc = torch.empty(count, dtype=torch.float32, device=X.device)
    _expect(Sc, count, "Sc")
    ws, pws, wsb = _workspace(workspace_bytes(name, N=N, n=n), X, ws)
    px = _dev_f32(X, "X") if N > 0 else C.c_void_p(X.data_ptr() if X.numel() else 0)
    _check(getattr(lib(), "st_" + name)(px, N, n, _dev_f32(Sc, "Sc"), 1 if accumulate else 0, pws, wsb, _stream()),
           "st_" + name)
    return Sc


def covar_pr2(X, S=None, accumulate=False, ws=None):
    """(S1, S2, S3): unique entries of the degree-2, -3 and -4 interaction terms of the samples X."""
    torch = _torch()
    N, n = _matrix(X, "X")
    if S is None:
        if accumulate:
            raise ValueError("accumulate needs existing outputs")
        S = tuple(torch.empty(c(n), dtype=torch.float32, device=X.device) for c in (count_sym2, count_sym3, count_sym4))
    if len(S) != 3:
        raise ValueError("S must hold the three terms (S1, S2, S3)")
    for t, c, what in zip(S, (count_sym2, count_sym3, count_sym4), ("S1", "S2", "S3")):
        _expect(t, c(n), what)
    ws, pws, wsb = _workspace(workspace_bytes("covar_pr2", N=N, n=n), X, ws)
    px = _dev_f32(X, "X") if N > 0 else C.c_void_p(X.data_ptr() if X.numel() else 0)
    _check(lib().st_covar_pr2(px, N, n, _dev_f32(S[0], "S1"), _dev_f32(S[1], "S2"), _dev_f32(S[2], "S3"),
                              1 if accumulate else 0, pws, wsb, _stream()), "st_covar_pr2")
    return S


def moment2_sym(X, Sc=None, accumulate=False, ws=None):
    return _moment(2, X, Sc, accumulate, ws)


def moment4_sym(X, Sc=None, accumulate=False, ws=None):
    return _moment(4, X, Sc, accumulate, ws)


def expand_sym(Sc, n, order, S=None):
    torch = _torch()
    if order not in (2, 3, 4) or n < 1:
        raise ValueError("order must be 2, 3 or 4 and n positive")
    _expect(Sc, {2: count_sym2, 3: count_sym3, 4: count_sym4}[order](n), "Sc")
    if S is None:
        S = torch.empty((n,) * order, dtype=torch.float32, device=Sc.device)
    _expect(S, n ** order, "S")
    _check(lib().st_expand_sym(_dev_f32(Sc, "Sc"), _dev_f32(S, "S"), n, order, _stream()), "st_expand_sym")
    return S


# ---- the kernel table's sparsity structures ---------------------------------------------
def ttm_struct(structure, Bc, U, ni, nj, Ac=None, ws=None):
    torch = _torch()
    nl, R = _matrix(U, "U")
    rows = count_struct(structure, ni, nj)
    if rows < 0:
        raise ValueError("unknown structure, or extents it does not allow")
    _expect(Bc, rows * nl, "Bc")
    if Ac is None:
        Ac = torch.empty((max(rows, 0), R), dtype=torch.float32, device=U.device)
    _expect(Ac, rows * R, "Ac")
    ws, pws, wsb = _workspace(workspace_bytes("ttm_struct", structure=structure, ni=ni, nj=nj, nl=nl, R=R), U, ws)
    _check(lib().st_ttm_struct(structure, _dev_f32(Bc, "Bc"), _dev_f32(U, "U"), _dev_f32(Ac, "Ac"), ni, nj, nl, R,
                               pws, wsb, _stream()), "st_ttm_struct")
    return Ac


def thp_struct(structure, Bc, C, fixed=0, Ac=None):
    torch = _torch()
    if C.dim() != 3:
        raise ValueError("C must be a dense order-3 tensor")
    ni, nj, nl = (int(v) for v in C.shape)
    rows = count_struct(structure, ni, nj)
    if rows < 0:
        raise ValueError("unknown structure, or extents it does not allow")
    _expect(Bc, rows * nl, "Bc")
    if Ac is None:
        Ac = torch.empty((max(rows, 0), nl), dtype=torch.float32, device=C.device)
    _expect(Ac, rows * nl, "Ac")
    _check(lib().st_thp_struct(structure, _dev_f32(Bc, "Bc"), _dev_f32(C, "C"), _dev_f32(Ac, "Ac"), ni, nj, nl,
                               int(fixed), _stream()), "st_thp_struct")
    return Ac


def mttkrp_fixed(kind, Bc, C, D, ni, fixed_k=0, A=None, ws=None):
    torch = _torch()
    nk, R = _matrix(C, "C")
    nl, RD = _matrix(D, "D")
    if RD != R:
        raise ValueError("C and D must have the same number of columns")
    if kind not in (MTTKRP_FIXED_IK, MTTKRP_FIXED_I, MTTKRP_FIXED_K):
        raise ValueError("unknown kind")
    _expect(Bc, {MTTKRP_FIXED_IK: 1, MTTKRP_FIXED_I: nk, MTTKRP_FIXED_K: ni}[kind] * nl, "Bc")
    if A is None:
        shape = (ni, R) if kind == MTTKRP_FIXED_K else (R,)
        A = torch.empty(shape, dtype=torch.float32, device=C.device)
    _expect(A, (ni if kind == MTTKRP_FIXED_K else 1) * R, "A")
    ws, pws, wsb = _workspace(workspace_bytes("mttkrp_fixed", kind=kind, ni=ni, nk=nk, nl=nl, R=R), C, ws)
    _check(lib().st_mttkrp_fixed(kind, _dev_f32(Bc, "Bc"), _dev_f32(C, "C"), _dev_f32(D, "D"), _dev_f32(A, "A"),
                                 ni, nk, nl, R, int(fixed_k), pws, wsb, _stream()), "st_mttkrp_fixed")
    return A


def expand_band(Tc, n, w, nl, T=None):
    torch = _torch()
    rows = count_band(n, w)
    if rows < 0 or nl < 1:
        raise ValueError("n, w must be non-negative and nl positive")
    _expect(Tc, rows * nl, "Tc")
    if T is None:
        T = torch.empty((n, n, nl), dtype=torch.float32, device=Tc.device)
    _expect(T, n * n * nl, "T")
    _check(lib().st_expand_band(_dev_f32(Tc, "Tc"), _dev_f32(T, "T"), n, w, nl, _stream()), "st_expand_band")
    return T


def hadamard_struct(dm, Mc, dv, Vc):
    """A(x) := M(x) * V(x) for two structured operands: the descriptor of the result (inferred) and its packed
    values, evaluated on the unique set of the result only."""
    da = dm.product(dv)
    if da.count == 0:
        return da, _torch().empty(0, dtype=_torch().float32, device=Mc.device)
    idx = da.list().contiguous()
    return da, dv.gather(Vc, idx, scale=dm.gather(Mc, idx))


def add_struct(dm, Mc, dv, Vc):
    """A(x) := M(x) + V(x) for two structured operands of the same shape: the inferred descriptor of the result
    and its packed values (each operand read through its own unique set and redundancy map)."""
    da = dm.sum(dv)
    if da.count == 0:
        return da, _torch().empty(0, dtype=_torch().float32, device=Mc.device)
    idx = da.list().contiguous()
    return da, dv.gather(Vc, idx, addend=dm.gather(Mc, idx))


def outer_struct(dm, Mc, dv, Vc):
    """T(x, y) := M(x) * V(y) for two structured operands: the inferred descriptor of the result and its packed
    values, from the two halves of the result's own index list."""
    dt = dm.outer(dv)
    if dt.count == 0:
        return dt, _torch().empty(0, dtype=_torch().float32, device=Mc.device)
    idx = dt.list().contiguous()
    return dt, dv.gather(Vc, idx, scale=dm.gather(Mc, idx), offset=len(dm.dims))


# ---- measurement support ----------------------------------------------------------------
def probe_empty(grid, block):
    _check(lib().st_probe_empty(int(grid), int(block), _stream()), "st_probe_empty")


def probe_stream(src, grid, block, sink):
    _check(lib().st_probe_stream(C.c_void_p(src.data_ptr()), src.numel() * src.element_size(), int(grid), int(block),
                                 _dev_f32(sink, "sink"), _stream()), "st_probe_stream")


def probe_mfma_f32(valu, iters, sink):
    """256 x 512 threads repeat `iters` times: `valu` (0 or 13) cross-lane multiplies, then 23 MFMAs 16x16x4 (fp32).
    Returns the flops the launch performs on the matrix cores."""
    _expect(sink, 256 * 512, "sink", at_least=True)
    _check(lib().st_probe_mfma_f32(int(valu), int(iters), _dev_f32(sink, "sink"), _stream()), "st_probe_mfma_f32")
    return 256 * 8 * int(iters) * 23 * 2048


# ---- descriptor-driven structures -------------------------------------------------------
class Descriptor:
    """Host object of ``st_desc_create`` plus (lazily) the device copy of its table."""

    def __init__(self, unique_set, dims, redundancy=None, _handle=None, **params):
        if _handle is not None:                       # an object the library made (st_desc_product)
            self._h = _handle
            self.dims = tuple(int(v) for v in dims)
            self._table_dev = None
            return
        self._h = C.c_void_p()
        dims = [int(v) for v in dims]
        da = (C.c_int64 * len(dims))(*dims)
        names = sorted(params)
        na = (C.c_char_p * max(len(names), 1))(*[k.encode() for k in names])
        va = (C.c_int64 * max(len(names), 1))(*[int(params[k]) for k in names])
        rc = lib().st_desc_create(unique_set.encode(), redundancy.encode() if redundancy else None, da, len(dims),
                                  na, va, len(names), C.byref(self._h))
        if rc != 0:
            msg = lib().st_desc_error(self._h).decode() if self._h else ""
            self.close()
            raise StructTensorError(rc, "st_desc_create (%s)" % msg)
        self.dims = tuple(dims)
        self._table_dev = None

    def close(self):
        if getattr(self, "_h", None):
            lib().st_desc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def count(self): return int(lib().st_desc_count(self._h))
    @property
    def runs(self): return int(lib().st_desc_runs(self._h))
    @property
    def nest(self): return lib().st_desc_nest(self._h).decode()
    @property
    def source(self): return lib().st_desc_source(self._h).decode()

    def table(self):
        out = np.empty(int(lib().st_desc_table_bytes(self._h)) // 4, dtype=np.int32)
        _check(lib().st_desc_table(self._h, out.ctypes.data), "st_desc_table")
        return out

    def compile(self):
        rc = lib().st_desc_compile(self._h)
        if rc != 0:
            raise StructTensorError(rc, "st_desc_compile (%s)" % lib().st_desc_error(self._h).decode())

    def _tab(self):
        if self._table_dev is None:
            self._table_dev = _torch().from_numpy(self.table()).cuda()
        return C.c_void_p(self._table_dev.data_ptr())

    def _call(self, rc, what):
        if rc != 0:
            raise StructTensorError(rc, "%s (%s)" % (what, lib().st_desc_error(self._h).decode()))

    def list(self):
        torch = _torch()
        out = torch.empty((max(self.count, 1), len(self.dims)), dtype=torch.int32, device="cuda")
        self._call(lib().st_desc_list(self._h, self._tab(), C.c_void_p(out.data_ptr()), _stream()), "st_desc_list")
        return out[:self.count]

    def thp(self, Bc, Cd, Ac=None):
        torch = _torch()
        _expect(Bc, self.count, "Bc", at_least=True)
        _expect(Cd, int(np.prod(self.dims)), "C")
        if Ac is None:
            Ac = torch.empty(max(self.count, 4), dtype=torch.float32, device=Cd.device)
        _expect(Ac, self.count, "Ac", at_least=True)
        self._call(lib().st_desc_thp(self._h, self._tab(), _dev_f32(Bc, "Bc"), _dev_f32(Cd, "C"),
                                     _dev_f32(Ac, "Ac"), _stream()), "st_desc_thp")
        return Ac[:self.count]

    def mttkrp(self, Bc, Cm, Dm, A=None, ws=None):
        """A(x0, r) = sum over the stored (x1, x2) of Bc(rank(x)) C(x1, r) D(x2, r) (order 3, no redundancy map)."""
        torch = _torch()
        _expect(Bc, self.count, "Bc", at_least=True)
        if len(self.dims) != 3:
            raise StructTensorError(6, "st_desc_mttkrp (order 3 only)")
        _matrix(Cm, "C")
        _matrix(Dm, "D")
        R = int(Cm.shape[1])
        _expect(Cm, self.dims[1] * R, "C")
        _expect(Dm, self.dims[2] * R, "D")
        if A is None:
            A = torch.empty((self.dims[0], R), dtype=torch.float32, device=Cm.device)
        _expect(A, self.dims[0] * R, "A")
        need = int(lib().st_desc_mttkrp_workspace(self._h, R))
        ws, wsp, wsb = _workspace(need, Cm, ws)
        self._call(lib().st_desc_mttkrp(self._h, self._tab(), _dev_f32(Bc, "Bc"), _dev_f32(Cm, "C"), _dev_f32(Dm, "D"),
                                        _dev_f32(A, "A"), R, wsp, wsb, _stream()), "st_desc_mttkrp")
        return A

    def expand(self, Tc, T=None):
        torch = _torch()
        _expect(Tc, self.count, "Tc", at_least=True)
        if T is None:
            T = torch.empty(self.dims, dtype=torch.float32, device=Tc.device)
        _expect(T, int(np.prod(self.dims)), "T")
        self._call(lib().st_desc_expand(self._h, self._tab(), _dev_f32(Tc, "Tc"), _dev_f32(T, "T"), _stream()),
                   "st_desc_expand")
        return T

    def expand_onto(self, Tc, T):
        """Write the elements this structure holds into the dense array T; every other element of T stays."""
        _expect(Tc, self.count, "Tc", at_least=True)
        _expect(T, int(np.prod(self.dims)), "T")
        self._call(lib().st_desc_expand_onto(self._h, self._tab(), _dev_f32(Tc, "Tc"), _dev_f32(T, "T"), _stream()),
                   "st_desc_expand_onto")
        return T

    def direct_sum(self, other):
        """The two summands of the direct sum self (+) other, each a descriptor over the box of the result
        (structure inference); the packed array of the result is self's followed by other's."""
        if len(self.dims) != len(other.dims):
            raise ValueError("the operands of a direct sum have the same order")
        dims = tuple(a + b for a, b in zip(self.dims, other.dims))
        hm, hv = C.c_void_p(), C.c_void_p()
        rc = lib().st_desc_direct_sum(self._h, other._h, C.byref(hm), C.byref(hv))
        if rc != 0:
            msg = "; ".join(lib().st_desc_error(h).decode() for h in (hm, hv) if h)
            for h in (hm, hv):
                if h:
                    lib().st_desc_destroy(h)
            raise StructTensorError(rc, "st_desc_direct_sum (%s)" % msg)
        return Descriptor(None, dims, _handle=hm), Descriptor(None, dims, _handle=hv)

    def product(self, other):
        """Descriptor of the element-wise product of two structured operands (structure inference)."""
        h = C.c_void_p()
        rc = lib().st_desc_product(self._h, other._h, C.byref(h))
        if rc != 0:
            msg = lib().st_desc_error(h).decode() if h else ""
            if h:
                lib().st_desc_destroy(h)
            raise StructTensorError(rc, "st_desc_product (%s)" % msg)
        return Descriptor(None, self.dims, _handle=h)

    def _derived(self, rc, h, what, dims):
        if rc != 0:
            msg = lib().st_desc_error(h).decode() if h else ""
            if h:
                lib().st_desc_destroy(h)
            raise StructTensorError(rc, "%s (%s)" % (what, msg))
        return Descriptor(None, dims, _handle=h)

    def outer(self, other):
        """Descriptor of the tensor outer product T(x, y) = self(x) * other(y) (structure inference)."""
        h = C.c_void_p()
        return self._derived(lib().st_desc_outer(self._h, other._h, C.byref(h)), h, "st_desc_outer",
                             tuple(self.dims) + tuple(other.dims))

    def power(self, k):
        """Descriptor of the k-fold outer product of a vector with itself: x_1 <= .. <= x_k, redundancy map sort."""
        h = C.c_void_p()
        return self._derived(lib().st_desc_power(self._h, int(k), C.byref(h)), h, "st_desc_power",
                             tuple(self.dims) * int(k))

    def project(self):
        """Descriptor of A(x_0..x_{d-2}) = sum over the last variable of this tensor (structure inference)."""
        h = C.c_void_p()
        return self._derived(lib().st_desc_project(self._h, C.byref(h)), h, "st_desc_project", self.dims[:-1])

    def sum_last(self, Bc, out=None):
        """Packed values of the projection: the sum of every run of the unique set (in run order)."""
        torch = _torch()
        _expect(Bc, self.count, "Bc", at_least=True)
        if out is None:
            out = torch.empty(max(self.runs, 4), dtype=torch.float32, device=Bc.device)
        _expect(out, self.runs, "out", at_least=True)
        self._call(lib().st_desc_sum_last(self._h, self._tab(), _dev_f32(Bc, "Bc"), _dev_f32(out, "out"), _stream()),
                   "st_desc_sum_last")
        return out[:self.runs]

    def sum(self, other):
        """Descriptor of the sum of two structured operands of the same shape (structure inference)."""
        h = C.c_void_p()
        return self._derived(lib().st_desc_sum(self._h, other._h, C.byref(h)), h, "st_desc_sum", self.dims)

    def gather(self, Tc, idx, scale=None, out=None, offset=0, addend=None):
        """Values of the structured tensor at the dense positions idx[:, offset:offset+order] (int32), times scale."""
        torch = _torch()
        if not (isinstance(idx, torch.Tensor) and idx.is_cuda and idx.dtype == torch.int32 and idx.is_contiguous()):
            raise TypeError("idx must be a contiguous int32 CUDA tensor")
        if idx.dim() != 2 or offset < 0 or idx.shape[1] < offset + len(self.dims):
            raise ValueError("idx must be [count][>= offset + order]")
        count, stride = int(idx.shape[0]), int(idx.shape[1])
        _expect(Tc, self.count, "Tc", at_least=True)
        if scale is not None:
            _expect(scale, count, "scale", at_least=True)
        if addend is not None:
            _expect(addend, count, "addend", at_least=True)
        if out is None:
            out = torch.empty(max(count, 4), dtype=torch.float32, device=Tc.device)
        _expect(out, count, "out", at_least=True)
        self._call(lib().st_desc_gather(self._h, self._tab(), _dev_f32(Tc, "Tc"), C.c_void_p(idx.data_ptr()), count,
                                        stride, int(offset), _dev_f32(scale, "scale") if scale is not None else None,
                                        _dev_f32(addend, "addend") if addend is not None else None,
                                        _dev_f32(out, "out"), _stream()), "st_desc_gather")
        return out[:count]

    def ttm(self, Bc, U, Ac=None):
        torch = _torch()
        nl, R = _matrix(U, "U")
        if nl != self.dims[-1]:
            raise ValueError("U must have as many rows as the last extent of the descriptor")
        _expect(Bc, self.count, "Bc", at_least=True)      # = runs * nl when the last variable is free (else the library refuses)
        if Ac is None:
            Ac = torch.empty((max(self.runs, 1), R), dtype=torch.float32, device=U.device)
        _expect(Ac, self.runs * R, "Ac", at_least=True)
        self._call(lib().st_desc_ttm(self._h, _dev_f32(Bc, "Bc"), _dev_f32(U, "U"), _dev_f32(Ac, "Ac"), R, _stream()),
                   "st_desc_ttm")
        return Ac[:self.runs]

    def moment(self, X, Sc=None, accumulate=False, ws=None):
        torch = _torch()
        N, n = _matrix(X, "X")
        if len(set(self.dims)) == 1 and n != self.dims[0]:     # (unequal extents: the library refuses the call)
            raise ValueError("X must have one column per feature of the descriptor")
        if Sc is None:
            if accumulate:
                raise ValueError("accumulate needs an existing Sc")
            Sc = torch.empty(max(self.count, 4), dtype=torch.float32, device=X.device)
        _expect(Sc, self.count, "Sc", at_least=True)
        ws, pws, wsb = _workspace(int(lib().st_desc_moment_workspace(self._h, N)), X, ws)
        px = _dev_f32(X, "X") if N > 0 else C.c_void_p(X.data_ptr() if X.numel() else 0)
        self._call(lib().st_desc_moment(self._h, self._tab(), px, N, _dev_f32(Sc, "Sc"), 1 if accumulate else 0, pws,
                                        wsb, _stream()), "st_desc_moment")
        return Sc[:self.count]
