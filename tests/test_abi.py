"""The C-ABI library loads without a GPU, exports every symbol the header
declares, and turns invalid arguments into status codes on the host (nothing is
launched on any of these paths)."""
import ctypes as C
import os
import re

import paper_2211_10482_amd as st
from paper_2211_10482_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "structtensor.h")

OK, NULL, SHAPE, ALIGN, WORKSPACE, LAUNCH, UNSUPPORTED = range(7)
P = 0x7F0000001000      # an aligned, never dereferenced, fake device address


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(st_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_symbols()
    assert "st_mttkrp_sym3" in names and "st_expand_sym" in names and len(names) >= 20
    lib = st.lib()
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(binding.SIGNATURES)


def test_status_strings():
    lib = st.lib()
    for s in range(0, 7):
        assert len(lib.st_status_string(s)) > 0
    assert lib.st_status_string(0) == b"ok"


def test_null_and_shape_errors():
    L = st.lib()
    assert L.st_mttkrp_sym3(None, P, P + 0x100000, 4, 2, None, 0, None) == NULL
    assert L.st_mttkrp_sym3(P, P + 0x10000, P + 0x20000, 0, 2, None, 0, None) == SHAPE
    assert L.st_mttkrp_sym3(P, P + 0x10000, P + 0x20000, 4, 0, None, 0, None) == SHAPE
    assert L.st_mttkrp_sym3(P, P + 0x10000, P + 0x20000, 5000, 4, None, 0, None) == UNSUPPORTED
    assert L.st_batax_utri(P, None, P + 0x10000, 4, 0.5, None, 0, None) == NULL
    assert L.st_batax_utri(P, P + 0x10000, P + 0x20000, -1, 0.5, None, 0, None) == SHAPE
    assert L.st_ttm_band(P, P + 0x100000, None, 4, 1, 4, 4, None, 0, None) == NULL
    assert L.st_ttm_band(P, P + 0x100000, P + 0x200000, 4, -1, 4, 4, None, 0, None) == SHAPE
    assert L.st_ttm_band(P, P + 0x100000, P + 0x200000, 4, 1, 0, 4, None, 0, None) == SHAPE
    assert L.st_moment3_sym(P, 10, 4, None, 0, None, 0, None) == NULL
    assert L.st_moment3_sym(None, 10, 4, P, 0, None, 0, None) == NULL
    assert L.st_moment3_sym(P, -1, 4, P + 0x100000, 0, None, 0, None) == SHAPE
    assert L.st_moment3_sym(P, 10, 4, P + 0x100000, 2, None, 0, None) == SHAPE
    assert L.st_expand_sym(None, P, 4, 3, None) == NULL
    assert L.st_expand_sym(P, P + 0x100000, 4, 5, None) == SHAPE
    assert L.st_expand_sym(P, P + 0x40000000, 300, 4, None) == UNSUPPORTED
    assert L.st_expand_sym(P, P + 0x100000, 0, 3, None) == SHAPE
    assert L.st_unrank_device(6, 4, 0, 0, 1, P, None) == SHAPE
    assert L.st_unrank_device(5, 4, 0, 34, 2, P, None) == SHAPE
    assert L.st_unrank_device(3, 4, 0, 19, 2, P, None) == SHAPE
    # measurement support: shapes are checked before anything is launched
    assert L.st_probe_empty(0, 64, None) == SHAPE
    assert L.st_probe_empty(4, 2048, None) == SHAPE
    assert L.st_probe_stream(None, 1024, 4, 64, P, None) == NULL
    assert L.st_probe_stream(P, 8, 4, 64, P + 0x1000, None) == SHAPE
    assert L.st_probe_stream(P + 4, 1024, 4, 64, P + 0x1000, None) == ALIGN
    assert L.st_probe_stream(P, 1 << 30, 4, 64, P + 0x40000000, None) == UNSUPPORTED      # more than 32 loads per thread
    assert L.st_probe_mfma_f32(0, 10, None, None) == NULL
    assert L.st_probe_mfma_f32(5, 10, P, None) == SHAPE
    assert L.st_probe_mfma_f32(13, 0, P, None) == SHAPE


def test_alignment_overlap_workspace_errors():
    L = st.lib()
    assert L.st_batax_utri(P + 4, P + 0x10000, P + 0x20000, 8, 0.5, None, 0, None) == ALIGN
    assert L.st_expand_sym(P, P + 0x100008, 4, 3, None) == ALIGN
    # output aliases an input
    assert L.st_batax_utri(P, P + 0x10000, P + 0x10000, 8, 0.5, None, 0, None) == SHAPE
    assert L.st_expand_sym(P, P + 16, 4, 3, None) == SHAPE
    assert L.st_mttkrp_sym3(P, P + 0x10000, P, 4, 2, None, 0, None) == SHAPE
    # workspace missing / too small / misaligned
    need = L.st_batax_utri_workspace(100)
    assert need > 0
    assert L.st_batax_utri(P, P + 0x100000, P + 0x200000, 100, 0.5, None, 0, None) == WORKSPACE
    assert L.st_batax_utri(P, P + 0x100000, P + 0x200000, 100, 0.5, P + 0x300000, need - 1, None) == WORKSPACE
    assert L.st_batax_utri(P, P + 0x100000, P + 0x200000, 100, 0.5, P + 0x300004, need, None) == ALIGN
    need = L.st_moment3_sym_workspace(1000, 8)
    assert need > 0
    assert L.st_moment3_sym(P, 1000, 8, P + 0x100000, 0, None, 0, None) == WORKSPACE
    assert L.st_mttkrp_sym3_workspace(20, 4) == 0          # one launch, no partial results
    need = L.st_mttkrp_sym3_workspace(112, 48)
    assert need > 0
    assert L.st_mttkrp_sym3(P, P + 0x1000000, P + 0x2000000, 112, 48, P + 0x3000000, need - 4, None) == WORKSPACE
    assert L.st_moment3_sym_workspace(0, 8) == 0 and L.st_ttm_band_workspace(8, 1, 8, 8) == 0


def test_binding_refuses_host_tensors():
    import numpy as np
    import pytest
    import torch
    with pytest.raises(TypeError):
        st.expand_sym(torch.zeros(20), 4, 3, S=torch.zeros(4, 4, 4))
    with pytest.raises(TypeError):
        st.expand_sym(np.zeros(20, dtype=np.float32), 4, 3, S=torch.zeros(4, 4, 4))


def test_kernel_table_errors():
    L = st.lib()
    assert L.st_count_struct(0, 5, 7) == 5 and L.st_count_struct(1, 5, 7) == 7 and L.st_count_struct(2, 5, 7) == 5
    assert L.st_count_struct(3, 6, 6) == 21 and L.st_count_struct(3, 5, 7) == -1 and L.st_count_struct(4, 5, 5) == -1
    assert L.st_count_struct(0, -1, 5) == -1
    Q = P + 0x1000000
    assert L.st_ttm_struct(0, None, Q, Q + 0x1000000, 4, 4, 4, 4, None, 0, None) == NULL
    assert L.st_ttm_struct(7, P, Q, Q + 0x1000000, 4, 4, 4, 4, None, 0, None) == SHAPE
    assert L.st_ttm_struct(3, P, Q, Q + 0x1000000, 4, 5, 4, 4, None, 0, None) == SHAPE
    assert L.st_ttm_struct(0, P, Q, Q + 0x1000000, 4, 4, 0, 4, None, 0, None) == SHAPE
    assert L.st_ttm_struct(0, P + 4, Q, Q + 0x1000000, 4, 4, 4, 4, None, 0, None) == ALIGN
    assert L.st_ttm_struct(0, P, Q, P, 4, 4, 4, 4, None, 0, None) == SHAPE            # output aliases B
    assert L.st_thp_struct(1, P, Q, None, 4, 4, 4, 0, None) == NULL
    assert L.st_thp_struct(1, P, Q, Q + 0x1000000, 4, 4, 4, 4, None) == SHAPE           # fixed i out of range
    assert L.st_thp_struct(2, P, Q, Q + 0x1000000, 4, 6, 4, 6, None) == SHAPE           # fixed j out of range
    assert L.st_thp_struct(0, P, Q, Q + 0x1000000, 4, 4, -1, 0, None) == SHAPE
    assert L.st_thp_struct(0, P, Q, Q + 0x1000000, 70000, 4, 4, 0, None) == UNSUPPORTED
    R3 = Q + 0x2000000
    assert L.st_mttkrp_fixed(0, P, Q, None, R3, 4, 4, 4, 4, 0, None, 0, None) == NULL
    assert L.st_mttkrp_fixed(3, P, Q, Q + 0x1000000, R3, 4, 4, 4, 4, 0, None, 0, None) == SHAPE
    assert L.st_mttkrp_fixed(0, P, Q, Q + 0x1000000, R3, 4, 4, 4, 4, 4, None, 0, None) == SHAPE   # fixed k out of range
    assert L.st_mttkrp_fixed(1, P, Q, Q + 0x1000000, R3, 4, 4, 4, 4, 9, None, 0, None) == WORKSPACE
    assert L.st_mttkrp_fixed(2, P, Q, Q + 0x1000000, R3, 4, 4, 4, 4, 1, None, 0, None) == WORKSPACE
    assert L.st_mttkrp_fixed_workspace(2, 4, 4, 8, 16) == 8 * 16 * 4
    assert L.st_mttkrp_fixed_workspace(1, 4, 9, 8, 16) == 9 * 16 * 4
    assert L.st_mttkrp_fixed_workspace(0, 4, 9, 8, 16) == 0
    assert L.st_expand_band(None, P, 4, 1, 4, None) == NULL
    assert L.st_expand_band(P, Q, 4, -1, 4, None) == SHAPE
    assert L.st_expand_band(P, Q, 50000, 1, 4, None) == UNSUPPORTED
    assert L.st_expand_band(P, P + 16, 4, 1, 4, None) == SHAPE                       # buffers overlap


def test_descriptor_errors():
    L = st.lib()
    h = C.c_void_p()
    dims = (C.c_int64 * 2)(4, 4)
    names = (C.c_char_p * 1)(b"n")
    vals = (C.c_int64 * 1)(4)
    assert L.st_desc_create(None, None, dims, 2, names, vals, 1, C.byref(h)) == NULL
    assert L.st_desc_create(b"S(i,j): (0<=i<=j<n)", None, dims, 2, names, vals, 1, None) == NULL
    assert L.st_desc_create(b"S(i,j): (0<=i<=j<n)", None, dims, 5, names, vals, 1, C.byref(h)) == SHAPE
    assert L.st_desc_create(b"S(i,j): (0<=i<=j<q)", None, dims, 2, names, vals, 1, C.byref(h)) == SHAPE
    assert b"unknown name" in L.st_desc_error(h)
    assert L.st_desc_list(h, P, P + 0x10000, None) == SHAPE          # nothing was generated for a failed parse
    L.st_desc_destroy(h)
    assert L.st_desc_create(b"S(i,j): (0<=i<=j<n)", None, dims, 2, names, vals, 1, C.byref(h)) == OK
    assert L.st_desc_count(h) == 10 and L.st_desc_runs(h) == 4 and L.st_desc_table_bytes(h) == (4 + 4 + 2) * 4
    assert L.st_desc_list(h, None, P, None) == NULL
    assert L.st_desc_list(h, P + 4, P + 0x10000, None) == ALIGN
    assert L.st_desc_thp(h, P, P + 0x10000, None, P + 0x20000, None) == NULL
    assert L.st_desc_thp(h, P, P + 0x10000, P + 0x20000, P + 0x10000, None) == SHAPE      # output aliases B
    assert L.st_desc_expand(h, P, None, P + 0x10000, None) == NULL
    assert L.st_desc_expand(h, P, P + 0x10000, P + 0x10010, None) == SHAPE                # buffers overlap
    assert L.st_desc_table(h, None) == NULL
    assert L.st_desc_moment(h, P, None, 10, P + 0x10000, 0, None, 0, None) == NULL
    assert L.st_desc_moment(h, P, P + 0x20000, 10, P + 0x10000, 0, None, 0, None) == WORKSPACE
    assert L.st_desc_moment(h, P, P + 0x20000, -1, P + 0x10000, 0, None, 0, None) == SHAPE
    assert L.st_desc_moment_workspace(h, 10) == 1 * 1 * 64 * 4        # one slice, one 8 x 8 block pair
    assert L.st_desc_ttm(h, P, None, P + 0x10000, 4, None) == NULL
    assert L.st_desc_ttm(h, P, P + 0x10000, P + 0x20000, 4, None) == UNSUPPORTED   # last variable is bounded by i <= j
    assert L.st_desc_ttm(h, P, P + 0x10000, P + 0x20000, 0, None) == SHAPE
    assert L.st_desc_mttkrp(h, P, P + 0x10000, P + 0x20000, P + 0x30000, P + 0x40000, 4, None, 0, None) == UNSUPPORTED    # order 2
    assert L.st_desc_count(None) == -1
    L.st_desc_destroy(h)
    L.st_desc_destroy(None)
    # the generated MTTKRP: order 3 without a redundancy map
    dims3 = (C.c_int64 * 3)(4, 4, 4)
    assert L.st_desc_create(b"B(i,j,l): (0<=i<n)*(i<=j<n)*(0<=l<n)", None, dims3, 3, names, vals, 1, C.byref(h)) == OK
    assert L.st_desc_mttkrp(h, P, None, P + 0x20000, P + 0x30000, P + 0x40000, 4, None, 0, None) == NULL
    assert L.st_desc_mttkrp(h, P, P + 0x10000, P + 0x20000, P + 0x30000, P + 0x40000, 0, None, 0, None) == SHAPE
    assert L.st_desc_mttkrp(h, P, P + 0x10000, P + 0x20004, P + 0x30000, P + 0x40000, 4, None, 0, None) == ALIGN
    assert L.st_desc_mttkrp(h, P, P + 0x10000, P + 0x20000, P + 0x30000, P + 0x20000, 4, None, 0, None) == SHAPE  # A aliases C
    # the last variable is free: ten runs of four entries, Y(run, r) in the workspace
    assert L.st_desc_mttkrp_workspace(h, 4) == 256 and L.st_desc_mttkrp_workspace(h, 0) == 0
    assert L.st_desc_mttkrp(h, P, P + 0x10000, P + 0x20000, P + 0x30000, P + 0x40000, 4, None, 0, None) == WORKSPACE
    assert L.st_desc_mttkrp(h, P, P + 0x10000, P + 0x20000, P + 0x30000, P + 0x40000, 4, P + 0x50000, 16, None) == WORKSPACE
    assert L.st_desc_mttkrp(h, P, P + 0x10000, P + 0x20000, P + 0x30000, P + 0x40000, 4, P + 0x40000, 256, None) == SHAPE  # ws aliases A
    L.st_desc_destroy(h)
    assert L.st_desc_create(b"T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)", b"sort", dims3, 3, names, vals, 1, C.byref(h)) == OK
    assert L.st_desc_mttkrp(h, P, P + 0x10000, P + 0x20000, P + 0x30000, P + 0x40000, 4, None, 0, None) == UNSUPPORTED    # redundancy map
    assert L.st_desc_mttkrp_workspace(h, 4) == 0
    L.st_desc_destroy(h)


def test_covar_pr2_errors():
    L = st.lib()
    a, b, c, x = P, P + 0x1000000, P + 0x2000000, P + 0x3000000
    assert L.st_covar_pr2(x, 10, 4, None, b, c, 0, None, 0, None) == NULL
    assert L.st_covar_pr2(None, 10, 4, a, b, c, 0, None, 0, None) == NULL
    assert L.st_covar_pr2(x, 10, 300, a, b, c, 0, None, 0, None) == UNSUPPORTED
    assert L.st_covar_pr2(x, 10, 4, a, b, c, 2, None, 0, None) == SHAPE
    assert L.st_covar_pr2(x, 10, 4, a, a, c, 0, None, 0, None) == SHAPE               # outputs alias
    assert L.st_covar_pr2(x, 5000, 64, a, b, c, 0, None, 0, None) == WORKSPACE
    need = L.st_covar_pr2_workspace(5000, 64)
    assert need == max(L.st_moment2_sym_workspace(5000, 64), L.st_moment3_sym_workspace(5000, 64),
                       L.st_moment4_sym_workspace(5000, 64)) > 0
    assert L.st_covar_pr2_workspace(10, 300) == 0


def test_binding_rejects_wrong_sized_tensors():
    """The binding compares every packed operand and caller-supplied output with the size of its unique set
    before it marshals anything: a wrong length is a ValueError, raised on the host (CPU tensors suffice: the
    size check comes before the device check, and a right-sized CPU tensor then fails as 'not a CUDA tensor')."""
    import pytest
    import torch
    z = lambda *shape: torch.zeros(*shape)
    n, R = 6, 3
    bad = [
        lambda: st.mttkrp_sym3(z(st.count_sym3(n) - 1), z(n, R)),
        lambda: st.mttkrp_sym3(z(st.count_sym3(n)), z(n, R), M=z(n, R + 1)),
        lambda: st.mttkrp_sym3(z(st.count_sym3(n)), z(n * R)),
        lambda: st.batax_utri(z(st.count_sym2(n) + 4), z(n), 0.5),
        lambda: st.batax_utri(z(st.count_sym2(n)), z(n), 0.5, y=z(n - 1)),
        lambda: st.ttm_band(z(st.count_band(n, 1), 8)[:-1], z(8, R), n, 1),
        lambda: st.ttm_band(z(st.count_band(n, 1), 8), z(8, R), n, 1, Yc=z(st.count_band(n, 1), R - 1)),
        lambda: st.moment3_sym(z(10, n), Sc=z(st.count_sym3(n) - 1)),
        lambda: st.moment2_sym(z(10, n), Sc=z(st.count_sym2(n) + 1)),
        lambda: st.moment4_sym(z(10, n), Sc=z(st.count_sym4(n) - 1)),
        lambda: st.moment3_sym(z(10 * n)),
        lambda: st.covar_pr2(z(10, n), S=(z(st.count_sym2(n)), z(st.count_sym3(n)), z(st.count_sym4(n) - 2))),
        lambda: st.expand_sym(z(st.count_sym3(n) - 1), n, 3),
        lambda: st.expand_sym(z(st.count_sym3(n)), n, 3, S=z(n, n, n - 1)),
        lambda: st.expand_sym(z(st.count_sym2(n)), n, 3),
        lambda: st.ttm_struct(st.STRUCT_UPPER, z(st.count_sym2(n), 8)[1:], z(8, R), n, n),
        lambda: st.ttm_struct(st.STRUCT_DIAG, z(n, 8), z(8, R), n, n, Ac=z(n - 1, R)),
        lambda: st.ttm_struct(st.STRUCT_UPPER, z(n, 8), z(8, R), n, n + 1),
        lambda: st.thp_struct(st.STRUCT_FIXED_I, z(n - 1, 8), z(4, n, 8)),
        lambda: st.thp_struct(st.STRUCT_DIAG, z(n, 8), z(n, n, 8), Ac=z(n, 7)),
        lambda: st.mttkrp_fixed(st.MTTKRP_FIXED_K, z(5, 8)[:-1], z(4, R), z(8, R), 5),
        lambda: st.mttkrp_fixed(st.MTTKRP_FIXED_I, z(4, 8), z(4, R), z(8, R + 1), 5),
        lambda: st.mttkrp_fixed(st.MTTKRP_FIXED_I, z(4, 8), z(4, R), z(8, R), 5, A=z(R + 1)),
        lambda: st.expand_band(z(st.count_band(n, 2) * 4 - 1), n, 2, 4),
        lambda: st.expand_band(z(st.count_band(n, 2) * 4), n, 2, 4, T=z(n, n, 3)),
    ]
    for q, f in enumerate(bad):
        with pytest.raises(ValueError):
            f()
            raise AssertionError("case %d was accepted" % q)
    # right sizes pass the size checks and stop at the device check: nothing was launched
    with pytest.raises(TypeError):
        st.mttkrp_sym3(z(st.count_sym3(n)), z(n, R), ws=torch.zeros(1 << 20, dtype=torch.uint8))
    with pytest.raises(TypeError):
        st.expand_sym(z(st.count_sym2(n)), n, 2)
    # descriptor calls
    d = st.Descriptor("T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)", (n, n, n), "sort", n=n)
    for f in (lambda: d.expand(z(d.count - 1)), lambda: d.expand(z(d.count), T=z(n, n, n + 1)),
              lambda: d.thp(z(d.count), z(n, n, n - 1)), lambda: d.thp(z(d.count - 3), z(n, n, n)),
              lambda: d.moment(z(10, n + 1)), lambda: d.moment(z(10, n), Sc=z(d.count - 1))):
        with pytest.raises(ValueError):
            f()
    d.close()
    db = st.Descriptor("B(i,j,l): (0<=i<n)*(i-1<=j<=i+1)*(0<=l<m)", (n, n, 4), n=n, m=4)
    for f in (lambda: db.ttm(z(db.runs, 4), z(5, R)), lambda: db.ttm(z(db.runs - 1, 4), z(4, R)),
              lambda: db.ttm(z(db.runs, 4), z(4, R), Ac=z(db.runs - 1, R))):
        with pytest.raises(ValueError):
            f()
    db.close()
