"""Descriptor-driven structures on the CPU: the parsed unique set / redundancy map against brute force
over the index box (predicates written out by hand here), the derived nests against the paper's printed
ones, the host tables against the closed-form index maps, and the GENERATED kernel source both compiled
with hiprtc for gfx950 (no GPU needed) and run on the CPU through the host stand-in of the HIP runtime."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import paper_2211_10482_amd as st
import st_workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EMUL = os.path.join(ROOT, "tests", "emul")
CLANG = shutil.which("clang++", path="/opt/rocm/llvm/bin") or shutil.which("clang++")


def _sorted(*x):
    return tuple(sorted(x))


# name -> (unique set text, dims, redundancy text, parameters, predicate, unique_of)
CASES = {
    # "Tensor Structures": unique elements of a symmetric matrix / degree-3 / degree-4 interaction tensor
    "sym2": ("S(i,j): (0<=i<=j<n)", (7, 7), "(0<=j<i<n) -> (j,i)", dict(n=7),
             lambda i, j: i <= j, lambda i, j: (j, i) if j < i else None),
    "sym3": ("T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)", (6, 6, 6), "sort", dict(n=6),
             lambda i, j, k: i <= j <= k, _sorted),
    "sym4": ("Q(i,j,k,l): (0<=i<=j<n)*(j<=k<=l<n)", (4, 4, 4, 4), "sort", dict(n=4),
             lambda i, j, k, l: i <= j <= k <= l, _sorted),
    # band |i-j| <= w with a free last index (the band tensor of the TTM workload)
    "band": ("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", (9, 9, 5), None, dict(n=9, w=2, m=5),
             lambda i, j, l: abs(i - j) <= 2, None),
    # the kernel table: diagonal plane, fixed i, fixed j, upper half cube
    "diag": ("B(i,j,l): (0<=i<n)*(i=j)*(0<=l<m)", (6, 6, 3), None, dict(n=6, m=3),
             lambda i, j, l: i == j, None),
    "fixed_i": ("B(i,j,l): (i=I)*(0<=j<n)*(0<=l<m)", (5, 6, 3), None, dict(I=2, n=6, m=3),
                lambda i, j, l: i == 2, None),
    "fixed_j": ("B(i,j,l): (0<=i<n)*(j=J)*(0<=l<m)", (5, 6, 3), None, dict(J=4, n=5, m=3),
                lambda i, j, l: j == 4, None),
    "upper_cube": ("B(i,j,l): (0<=i<n)*(i<=j<n)*(0<=l<m)", (6, 6, 4), None, dict(n=6, m=4),
                   lambda i, j, l: i <= j, None),
    # the paper's identical-rows example: only row 0 is stored, every other row repeats it
    "same_rows": ("M(i,j): (i=0)*(0<=j<m)", (5, 7), "(1<=i<n) -> (0,j)", dict(n=5, m=7),
                  lambda i, j: i == 0, lambda i, j: (0, j) if i >= 1 else None),
    # strictly lower triangle; an anti-diagonal band (two bounds from both sides on the last variable)
    "lower": ("L(i,j): (0<=j<i<n)", (6, 6), None, dict(n=6), lambda i, j: j < i, None),
    "anti": ("A(i,j): (0<=i<n)*(n-2<=i+j<=n)", (7, 7), None, dict(n=7), lambda i, j: 5 <= i + j <= 7, None),
    "order1": ("v(i): (2<=i<n)", (9,), None, dict(n=6), lambda i: 2 <= i < 6, None),
    "sym3_vec": ("T(i,j,k): (0<=i<=j<n)*(j<=k<n)", (8, 8, 8), "sort", dict(n=8), lambda i, j, k: i <= j <= k, _sorted),
    "order1_vec": ("v(i): (3<=i<=9)", (12,), None, dict(), lambda i: 3 <= i <= 9, None),
    "empty": ("E(i,j): (0<=i<n)*(j<i)*(j>i)", (4, 4), None, dict(n=4), lambda i, j: False, None),
    "none_by_param": ("E(i,j): (0<=i<n)*(n<=3)*(0<=j<n)", (4, 4), None, dict(n=4), lambda i, j: False, None),
}


@pytest.fixture(scope="module")
def descs():
    out = {}
    for name, (text, dims, red, params, _, _) in CASES.items():
        out[name] = st.Descriptor(text, dims, red, **params)
    yield out
    for d in out.values():
        d.close()


@pytest.mark.parametrize("name", sorted(CASES))
def test_counts_and_tables_against_brute_force(descs, oracle, name):
    text, dims, red, params, pred, _ = CASES[name]
    d = descs[name]
    lst = oracle.struct_enumerate(dims, pred)
    assert d.count == lst.shape[0]
    tab = d.table()
    nprefix = int(np.prod(dims[:-1])) if len(dims) > 1 else 1
    # orders 2 and 3 over one extent <= 256 also carry the block tuples (8 x 8, 4 x 4 x 4) that hold unique entries
    tiles = np.zeros((0, len(dims)), dtype=np.int64)
    if len(dims) in (2, 3) and len(set(dims)) == 1 and dims[0] <= 256 and lst.shape[0] > 0:
        tiles = np.unique(lst.astype(np.int64) // (8 if len(dims) == 2 else 4), axis=0)
    assert tab.size == nprefix + d.runs + tiles.size
    assert np.array_equal(tab[nprefix + d.runs:].reshape(-1, len(dims)), tiles)
    # run starts: position of the first entry of every prefix that has one, -1 for the others
    want = np.full(nprefix, -1, dtype=np.int64)
    for p in range(lst.shape[0] - 1, -1, -1):
        pf = 0
        for v in range(len(dims) - 1):
            pf = pf * dims[v] + int(lst[p, v])
        want[pf] = p
    assert np.array_equal(tab[:nprefix], want)
    assert np.array_equal(tab[nprefix:nprefix + d.runs], np.flatnonzero(want >= 0))


def test_tables_match_the_closed_form_index_maps(oracle):
    n, w, m = 40, 5, 3
    d3 = st.Descriptor("T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)", (n, n, n), "sort", n=n)
    assert d3.count == st.count_sym3(n) == oracle.count_sym3(n)
    tab = d3.table()[: n * n].reshape(n, n)
    for i in range(n):
        for j in range(n):
            assert tab[i, j] == (st.rank_sym3(n, i, j, j) if i <= j else -1)
    db = st.Descriptor("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", (n, n, m), n=n, w=w, m=m)
    assert db.count == st.count_band(n, w) * m
    tab = db.table()[: n * n].reshape(n, n)
    for i in range(n):
        for j in range(n):
            assert tab[i, j] == (st.rank_band(n, w, i, j) * m if abs(i - j) <= w else -1)
    d4 = st.Descriptor("Q(i,j,k,l): (0<=i<=j<n)*(j<=k<=l<n)", (9, 9, 9, 9), "sort", n=9)
    assert d4.count == st.count_sym4(9)
    # the distinct elements of the degree-2 polynomial-regression covariance of four features (golden file)
    n = 4
    total = sum(st.Descriptor(t, (n,) * o, n=n).count for t, o in (
        ("S(i,j): (0<=i<=j<n)", 2), ("T(i,j,k): (0<=i<=j<n)*(j<=k<n)", 3), ("Q(i,j,k,l): (0<=i<=j<n)*(j<=k<=l<n)", 4)))
    golden = dict(l.split()[:2] for l in open(os.path.join(ROOT, "tests", "golden", "paper_counts.txt"))
                  if l.strip() and not l.startswith("#"))
    assert total == int(golden["pr2_distinct_elements_n4"]) == 65


def test_derived_nests(descs):
    # the overview's M1, M2 and M3 nests: for i; for j = i; for k = j; for l = k
    assert descs["sym3"].nest.splitlines()[:3] == [
        "for (i = 0; i <= 5; ++i)", "  for (j = i; j <= 5; ++j)", "    for (k = j; k <= 5; ++k)"]
    assert descs["sym4"].nest.splitlines()[:4] == [
        "for (i = 0; i <= 3; ++i)", "  for (j = i; j <= 3; ++j)", "    for (k = j; k <= 3; ++k)",
        "      for (l = k; l <= 3; ++l)"]
    assert descs["sym2"].nest.splitlines()[:2] == ["for (i = 0; i <= 6; ++i)", "  for (j = i; j <= 6; ++j)"]
    # bounds are the maximum of the lower and the minimum of the upper bounds
    assert descs["band"].nest.splitlines()[1] == "  for (j = max(0, i - 2); j <= min(8, i + 2); ++j)"
    assert descs["anti"].nest.splitlines()[1] == "  for (j = max(0, -i + 5); j <= min(6, -i + 7); ++j)"
    assert descs["diag"].nest.splitlines()[1] == "  for (j = i; j <= i; ++j)"
    assert descs["fixed_j"].nest.splitlines()[1] == "  for (j = 4; j <= 4; ++j)"
    assert descs["lower"].nest.splitlines()[:2] == ["for (i = 0; i <= 5; ++i)", "  for (j = 0; j <= i - 1; ++j)"]


def test_parse_errors():
    bad = [
        ("S(i,j) (0<=i<n)", (4, 4), None, dict(n=4)),                       # no colon
        ("S(i,j): (0<=i<n)*(2*j<=i)", (4, 4), None, dict(n=4)),             # non-unit coefficient
        ("S(i,j): (0<=i<q)", (4, 4), None, dict(n=4)),                      # unknown name
        ("S(i,j): (0<=i<n)", (4,), None, dict(n=4)),                        # sizes / variables mismatch
        ("S(i,i): (0<=i<n)", (4, 4), None, dict(n=4)),                      # variable twice
        ("S(i,j): (0<=i<n) junk", (4, 4), None, dict(n=4)),                 # trailing text
        ("S(i,j): (0<=i<=j<n)", (4, 5), "sort", dict(n=4)),                 # sort needs equal sizes
        ("S(i,j): (0<=i<=j<n)", (4, 4), "(0<=j<i<n) -> (j)", dict(n=4)),    # target arity
        ("S(i,j): (0<=i<=j<n)", (4, 4), "(0<=j<i<n) (j,i)", dict(n=4)),     # no arrow
        ("S(i,j,k,l,m): (0<=i<n)", (4,) * 5, None, dict(n=4)),              # order > 4
    ]
    for text, dims, red, params in bad:
        with pytest.raises(st.StructTensorError):
            st.Descriptor(text, dims, red, **params)


@pytest.mark.parametrize("name", sorted(CASES))
def test_generated_source_compiles_for_gfx950(descs, name):
    descs[name].compile()
    src = descs[name].source
    assert "st_gen_list" in src and "st_gen_thp" in src and "st_gen_expand" in src


@pytest.mark.parametrize("name", sorted(CASES))
def test_generated_kernels_on_the_cpu(descs, oracle, tmp_path, name):
    if CLANG is None:
        pytest.skip("no clang++ for the host build")
    text, dims, red, params, pred, unique_of = CASES[name]
    d = descs[name]
    box = int(np.prod(dims))
    src = tmp_path / "generated.hip"
    src.write_text(d.source)
    exe = str(tmp_path / "driver")
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fno-omit-frame-pointer",
           '-DGEN_SRC="%s"' % src, "-I", EMUL, "-x", "c++", os.path.join(EMUL, "desc_driver.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    Bc = W.uniform(701, max(d.count, 1))[: d.count]
    Cd = W.uniform(702, box).reshape(dims)
    d.table().tofile(str(tmp_path / "table.i32"))
    Bc.tofile(str(tmp_path / "bc.f32"))
    Cd.tofile(str(tmp_path / "c.f32"))
    has_moment = "st_gen_moment" in d.source
    N = 7
    X = W.normal(703, N * dims[0]).reshape(N, dims[0])
    X.tofile(str(tmp_path / "x.f32"))
    has_mttkrp = len(dims) == 3 and red is None          # the kernel table's MTTKRP: order 3, sparsity only
    R = 24 if name in ("band", "diag") else 21          # two column blocks, the second one ragged; 24: 16-byte row loads
    if has_mttkrp:
        assert "st_gen_mttkrp" in d.source
        Cm, Dm = W.uniform(704, dims[1] * R).reshape(dims[1], R), W.uniform(705, dims[2] * R).reshape(dims[2], R)
        np.array([R], dtype=np.int32).tofile(str(tmp_path / "mk_r.i32"))
        Cm.tofile(str(tmp_path / "mk_c.f32"))
        Dm.tofile(str(tmp_path / "mk_d.f32"))
    r = subprocess.run([exe, str(tmp_path), str(d.count), str(box), str(len(dims)), str(d.runs), str(dims[-1])]
                       + ([str(N)] if has_moment else []), capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "rc=0" in r.stdout, r.stderr[-3000:]
    lst = np.fromfile(str(tmp_path / "list.i32"), dtype=np.int32).reshape(-1, len(dims))
    assert np.array_equal(lst, oracle.struct_enumerate(dims, pred))
    thp = np.fromfile(str(tmp_path / "thp.f32"), dtype=np.float32)
    assert np.array_equal(thp, oracle.struct_thp(Bc, Cd, dims, pred).astype(np.float32))
    ex = np.fromfile(str(tmp_path / "expand.f32"), dtype=np.float32).reshape(dims)
    ref = oracle.struct_expand(Bc, dims, pred, unique_of)
    assert np.array_equal(ex.view(np.uint32), ref.view(np.uint32))
    # every run summed (marginalization of the last variable): against the zero-filled dense operand summed over
    # its last axis, at the prefixes that hold a run, in nest order
    if red is None and d.count:
        sums = np.fromfile(str(tmp_path / "sum_last.f32"), dtype=np.float32)
        Bz = np.zeros(dims, dtype=np.float64)
        Bz[tuple(lst[:, v].astype(np.int64) for v in range(len(dims)))] = Bc
        tot, hit = Bz.sum(axis=-1).reshape(-1), np.zeros(dims, dtype=bool)
        hit[tuple(lst[:, v].astype(np.int64) for v in range(len(dims)))] = True
        want = tot[hit.any(axis=-1).reshape(-1)]
        assert sums.size == d.runs == want.size and float(np.abs(sums - want).max()) <= 1e-5 * max(float(np.abs(want).max()), 1.0)
    if has_mttkrp:
        # against the dense definition on the zero-filled operand (the C oracle), row by row
        got = np.fromfile(str(tmp_path / "mttkrp.f32"), dtype=np.float32).reshape(dims[0], R)
        Bd = np.zeros(dims, dtype=np.float32)
        Bd[tuple(lst[:, v].astype(np.int64) for v in range(3))] = Bc
        refa = oracle.mttkrp_full(Bd, Cm, Dm)
        assert float(np.abs(got - refa).max()) <= 1e-5 * max(float(np.abs(refa).max()), 1.0)
        empty_rows = ~Bd.reshape(dims[0], -1).any(axis=1)
        assert not got[empty_rows].any()                  # rows without a stored entry are written as zeros
        if name in ("band", "diag", "fixed_i", "fixed_j", "upper_cube"):       # last variable free: the second route
            got2 = np.fromfile(str(tmp_path / "mttkrp_combine.f32"), dtype=np.float32).reshape(dims[0], R)
            assert float(np.abs(got2 - refa).max()) <= 1e-5 * max(float(np.abs(refa).max()), 1.0)
            assert not got2[empty_rows].any()
    if has_moment:
        mom = np.fromfile(str(tmp_path / "moment.f32"), dtype=np.float32)
        refm = oracle.struct_moment(X, dims, pred)
        assert mom.size == refm.size and float(np.abs(mom - refm).max()) <= 1e-5 * max(float(np.abs(refm).max()), 1.0)


# ------------------------------------------------------------------ Property 1: T_U * T_R is empty
def test_redundancy_term_must_not_meet_the_unique_set():
    """The unique set and the redundancy map are disjoint ("Properties" of the semantics, property 1): a term
    whose condition holds for a stored entry is refused, with the first such entry in the message."""
    bad = [
        ("S(i,j): (0<=i<=j<n)", (5, 5), "(0<=j<=i<n) -> (j,i)", dict(n=5), "(0,0)"),          # meets the diagonal
        ("M(i,j): (i=0)*(0<=j<m)", (4, 6), "(0<=i<n) -> (0,j)", dict(n=4, m=6), "(0,0)"),      # row 0 is stored
        ("B(i,j,l): (0<=i<n)*(i-1<=j<=i+1)*(0<=l<m)", (5, 5, 3), "(0<=i<n)*(j=i+1)*(l=2) -> (i,i,l)", dict(n=5, m=3), "(0,1,2)"),
    ]
    for text, dims, red, params, where in bad:
        with pytest.raises(st.StructTensorError) as e:
            st.Descriptor(text, dims, red, **params)
        assert e.value.status == 2 and where in str(e.value) and "disjoint" in str(e.value), str(e.value)
    # the hand-wired maps of the library's own structures are disjoint by the same check
    for text, dims, red, params in (("S(i,j): (0<=i<=j<n)", (9, 9), "(0<=j<i<n) -> (j,i)", dict(n=9)),
                                    ("M(i,j): (i=0)*(0<=j<m)", (4, 6), "(1<=i<n) -> (0,j)", dict(n=4, m=6))):
        st.Descriptor(text, dims, red, **params).close()


# ------------------------------------------------------------------ structure inference for element-wise products
SYM_RED = "(0<=j<i<n) -> (j,i)"
_swap = lambda i, j: (j, i) if j < i else None
# name -> (M: text, redundancy, predicate, unique_of), (V: ...), dims, params, expected (predicate, unique_of) or None
PRODUCTS = {
    # the paper's walk-through: upper triangular (.) symmetric = upper triangular, no redundancy
    "uhs": (("M(i,j): (0<=i<=j<n)", None, lambda i, j: i <= j, None),
            ("N(i,j): (0<=i<=j<n)", "sort", lambda i, j: i <= j, _swap), (7, 7), dict(n=7),
            (lambda i, j: i <= j, None), ["for (i = 0; i <= 6; ++i)", "  for (j = i; j <= 6; ++j)"]),
    "sym_sym": (("M(i,j): (0<=i<=j<n)", SYM_RED, lambda i, j: i <= j, _swap),
                ("N(i,j): (0<=i<=j<n)", "sort", lambda i, j: i <= j, _swap), (6, 6), dict(n=6),
                (lambda i, j: i <= j, _swap), None),
    "band_upper": (("M(i,j): (0<=i<n)*(i-w<=j<=i+w)", None, lambda i, j: abs(i - j) <= 2, None),
                   ("N(i,j): (0<=i<=j<n)", None, lambda i, j: i <= j, None), (8, 8), dict(n=8, w=2),
                   (lambda i, j: i <= j <= i + 2, None), ["for (i = 0; i <= 7; ++i)", "  for (j = i; j <= min(7, i + 2); ++j)"]),
    "rows_rows": (("M(i,j): (i=0)*(0<=j<m)", "(1<=i<n) -> (0,j)", lambda i, j: i == 0, lambda i, j: (0, j) if i >= 1 else None),
                  ("N(i,j): (i=0)*(0<=j<m)", "(1<=i<n) -> (0,j)", lambda i, j: i == 0, lambda i, j: (0, j) if i >= 1 else None),
                  (4, 5), dict(n=4, m=5), (lambda i, j: i == 0, lambda i, j: (0, j) if i >= 1 else None), None),
    "diag_sym": (("M(i,j): (0<=i<n)*(i=j)", None, lambda i, j: i == j, None),
                 ("N(i,j): (0<=i<=j<n)", SYM_RED, lambda i, j: i <= j, _swap), (5, 5), dict(n=5),
                 (lambda i, j: i == j, None), None),
    "disjoint": (("M(i,j): (0<=j<i<n)", None, lambda i, j: j < i, None),
                 ("N(i,j): (0<=i<j<n)", None, lambda i, j: i < j, None), (5, 5), dict(n=5),
                 (lambda i, j: False, None), None),
    "band3_cube": (("M(i,j,l): (0<=i<n)*(i-1<=j<=i+1)*(0<=l<m)", None, lambda i, j, l: abs(i - j) <= 1, None),
                   ("N(i,j,l): (0<=i<n)*(i<=j<n)*(0<=l<m)", None, lambda i, j, l: i <= j, None), (6, 6, 4), dict(n=6, m=4),
                   (lambda i, j, l: i <= j <= i + 1, None), None),
    # lower triangle (.) symmetric: the diagonal comes from M_U * N_U, the strict lower part from M_U * N_R: two summands
    "lower_sym": (("M(i,j): (0<=j<=i<n)", None, lambda i, j: j <= i, None),
                  ("N(i,j): (0<=i<=j<n)", SYM_RED, lambda i, j: i <= j, _swap), (5, 5), dict(n=5), None, None),
}


def _run_generated(d, workdir, dims, Tc, gather_idx=None, scale=None, addend=None, onto=None):
    """Compile the generated source of descriptor d against the host stand-in and run the driver in workdir."""
    os.makedirs(workdir, exist_ok=True)
    src = os.path.join(workdir, "generated.hip")
    open(src, "w").write(d.source)
    exe = os.path.join(workdir, "driver")
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fno-omit-frame-pointer",
           '-DGEN_SRC="%s"' % src, "-I", EMUL, "-x", "c++", os.path.join(EMUL, "desc_driver.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    box = int(np.prod(dims))
    d.table().tofile(os.path.join(workdir, "table.i32"))
    np.asarray(Tc, dtype=np.float32).tofile(os.path.join(workdir, "bc.f32"))
    np.zeros(box, dtype=np.float32).tofile(os.path.join(workdir, "c.f32"))
    if gather_idx is not None:
        np.ascontiguousarray(gather_idx, dtype=np.int32).tofile(os.path.join(workdir, "gather.i32"))
        if scale is not None:
            np.asarray(scale, dtype=np.float32).tofile(os.path.join(workdir, "gather_scale.f32"))
        if addend is not None:
            np.asarray(addend, dtype=np.float32).tofile(os.path.join(workdir, "gather_addend.f32"))
    if onto is not None:
        np.ascontiguousarray(onto, dtype=np.float32).tofile(os.path.join(workdir, "onto.f32"))
    r = subprocess.run([exe, workdir, str(d.count), str(box), str(len(dims)), str(d.runs), str(dims[-1])],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "rc=0" in r.stdout, r.stderr[-3000:]
    return np.fromfile(os.path.join(workdir, "gather.f32"), dtype=np.float32) if gather_idx is not None else None


@pytest.mark.parametrize("name", sorted(PRODUCTS))
def test_product_inference(oracle, tmp_path, name):
    """A(x) := M(x) * V(x): the inferred unique set and redundancy map against predicates written out by hand
    (brute force over the box), and the values -- the generated gather kernels run on the CPU -- against the
    product of the two reconstructed dense operands: bit for bit on the unique set, and Property 5 for the
    result (reconstructing A from A_C through the inferred map gives the dense product everywhere)."""
    if CLANG is None:
        pytest.skip("no clang++ for the host build")
    (mt, mred, mpred, muniq), (vt, vred, vpred, vuniq), dims, params, want, nest = PRODUCTS[name]
    dm, dv = st.Descriptor(mt, dims, mred, **params), st.Descriptor(vt, dims, vred, **params)
    if want is None:
        with pytest.raises(st.StructTensorError) as e:
            dm.product(dv)
        assert e.value.status == 6 and "sum of 2" in str(e.value)
        return
    apred, auniq = want
    da = dm.product(dv)
    lst = oracle.struct_enumerate(dims, apred)
    assert da.count == lst.shape[0]
    if nest is not None:
        assert da.nest.splitlines()[:len(nest)] == nest
    Mc, Vc = W.uniform(771, max(dm.count, 1))[: dm.count], W.uniform(772, max(dv.count, 1))[: dv.count]
    Md = oracle.struct_expand(Mc, dims, mpred, muniq)
    Vd = oracle.struct_expand(Vc, dims, vpred, vuniq)
    dense = Md * Vd                                              # fp32 products, correctly rounded
    if da.count == 0:
        assert not dense.any()
        return
    gm = _run_generated(dm, str(tmp_path / "m"), dims, Mc, gather_idx=lst)
    ac = _run_generated(dv, str(tmp_path / "v"), dims, Vc, gather_idx=lst, scale=gm)
    cols = tuple(lst[:, v].astype(np.int64) for v in range(len(dims)))
    assert np.array_equal(gm, Md[cols])
    assert np.array_equal(ac.view(np.uint32), dense[cols].view(np.uint32))
    # Property 5 for the result, through the library's own reconstruction of A_C (CPU run of A's expand kernel)
    _run_generated(da, str(tmp_path / "a"), dims, ac)
    ex = np.fromfile(str(tmp_path / "a" / "expand.f32"), dtype=np.float32).reshape(dims)
    # (by value: a structural zero times a negative entry is -0 in the dense product, +0 in a reconstruction)
    assert np.array_equal(ex, dense)
    assert np.array_equal(oracle.struct_expand(ac, dims, apred, auniq), dense)
    # positions outside the dense extents read as zero
    out = _run_generated(dm, str(tmp_path / "o"), dims, Mc, gather_idx=np.array([[-1] * len(dims), list(dims)], dtype=np.int32))
    assert np.array_equal(out, np.zeros(2, dtype=np.float32))
    for d in (dm, dv, da):
        d.close()


# ------------------------------------------------------------------ structure inference for outer products
_rows = lambda i, j: (0, j) if i >= 1 else None
# name -> (M: text, dims, redundancy, params, predicate, unique_of), (V: ...), expected unique_of of the result or "none"
OUTERS = {
    # the shape of the paper's walk-through of the outer-product rule: no redundancy x symmetric
    "lower_x_sym": (("M(a,b): (0<=b<a<n)", (5, 5), None, dict(n=5), lambda a, b: b < a, None),
                    ("V(c,d): (0<=c<=d<m)", (4, 4), "(0<=d<c<m) -> (d,c)", dict(m=4), lambda c, d: c <= d, _swap)),
    # both redundant: all three summands of T_R
    "sym_x_sym": (("M(i,j): (0<=i<=j<n)", (4, 4), "sort", dict(n=4), lambda i, j: i <= j, _swap),
                  ("N(i,j): (0<=i<=j<m)", (3, 3), "(0<=j<i<m) -> (j,i)", dict(m=3), lambda i, j: i <= j, _swap)),
    "rows_x_vec": (("M(i,j): (i=0)*(0<=j<m)", (3, 5), "(1<=i<n) -> (0,j)", dict(n=3, m=5), lambda i, j: i == 0, _rows),
                   ("v(k): (1<=k<n)", (6,), None, dict(n=6), lambda k: 1 <= k, None)),
    "vec_x_band": (("v(i): (0<=i<n)", (4,), None, dict(n=4), lambda i: True, None),
                   ("B(j,l): (0<=j<n)*(j-1<=l<=j+1)", (6, 6), None, dict(n=6), lambda j, l: abs(j - l) <= 1, None)),
    # same variable names in both operands: the result renames
    "vec_x_vec": (("v(i): (2<=i<n)", (7,), None, dict(n=7), lambda i: i >= 2, None),
                  ("w(i): (0<=i<=m)", (5,), None, dict(m=2), lambda i: i <= 2, None)),
}


@pytest.mark.parametrize("name", sorted(OUTERS))
def test_outer_product_inference(oracle, tmp_path, name):
    """T(x, y) := M(x) * V(y): T_U = M_U * V_U and T_R = M_U*V_R + M_R*V_U + M_R*V_R against predicates written out
    by hand (brute force over the box); values on T_U from the two operands' generated gather kernels (CPU run)
    against the dense outer product, bit for bit; Property 5 for the result through its own generated
    reconstruction."""
    if CLANG is None:
        pytest.skip("no clang++ for the host build")
    (mt, mdims, mred, mpar, mpred, muniq), (vt, vdims, vred, vpar, vpred, vuniq) = OUTERS[name]
    dm, dv = st.Descriptor(mt, mdims, mred, **mpar), st.Descriptor(vt, vdims, vred, **vpar)
    k = len(mdims)
    dims = tuple(mdims) + tuple(vdims)
    dt = dm.outer(dv)
    pred = lambda *x: mpred(*x[:k]) and vpred(*x[k:])
    def unique_of(*x):
        a = (muniq(*x[:k]) if muniq and not mpred(*x[:k]) else None) or x[:k]
        b = (vuniq(*x[k:]) if vuniq and not vpred(*x[k:]) else None) or x[k:]
        return tuple(a) + tuple(b) if tuple(a) + tuple(b) != tuple(x) else None
    lst = oracle.struct_enumerate(dims, pred)
    assert dt.count == lst.shape[0] == dm.count * dv.count
    Mc, Vc = W.uniform(781, dm.count), W.uniform(782, dv.count)
    Md, Vd = oracle.struct_expand(Mc, mdims, mpred, muniq), oracle.struct_expand(Vc, vdims, vpred, vuniq)
    dense = (Md.reshape(mdims + (1,) * len(vdims)) * Vd.reshape((1,) * k + vdims)).astype(np.float32)
    gm = _run_generated(dm, str(tmp_path / "m"), mdims, Mc, gather_idx=lst[:, :k])
    tc = _run_generated(dv, str(tmp_path / "v"), vdims, Vc, gather_idx=lst[:, k:], scale=gm)
    cols = tuple(lst[:, v].astype(np.int64) for v in range(len(dims)))
    assert np.array_equal(tc.view(np.uint32), dense[cols].view(np.uint32))
    _run_generated(dt, str(tmp_path / "t"), dims, tc)
    got = np.fromfile(str(tmp_path / "t" / "list.i32"), dtype=np.int32).reshape(-1, len(dims))
    assert np.array_equal(got, lst)
    ex = np.fromfile(str(tmp_path / "t" / "expand.f32"), dtype=np.float32).reshape(dims)
    assert np.array_equal(ex, dense)
    assert np.array_equal(oracle.struct_expand(tc, dims, pred, unique_of), dense)      # the same map, written by hand


def test_outer_product_limits():
    a = st.Descriptor("B(i,j,l): (0<=i<n)*(i<=j<n)*(0<=l<n)", (3, 3, 3), None, n=3)
    b = st.Descriptor("S(i,j): (0<=i<=j<n)", (3, 3), "sort", n=3)
    with pytest.raises(st.StructTensorError) as e:
        a.outer(b)                                                   # order 5
    assert e.value.status == 6
    t = st.Descriptor("T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)", (3, 3, 3), "sort", n=3)
    v = st.Descriptor("v(i): (0<=i<n)", (3,), None, n=3)
    with pytest.raises(st.StructTensorError) as e:
        t.outer(v)                                                   # a sort map of order 3 is a sum of conditions
    assert e.value.status == 6 and "sort" in str(e.value)


# ------------------------------------------------------------------ the self-multiplication rule and its extension
@pytest.mark.parametrize("k", [2, 3, 4])
def test_vector_self_product_inference(oracle, tmp_path, k):
    """x (x) x (x) .. (k factors) of a vector: the inferred structure is the one the moment kernels are written
    for -- the nests of the overview (for i; for j = i; for k = j), the closed-form counts, the packed order of
    the C oracle, and a reconstruction that equals the oracle's bit for bit."""
    if CLANG is None:
        pytest.skip("no clang++ for the host build")
    n = 6
    v = st.Descriptor("x(i): (0<=i<n)", (n,), None, n=n)
    p = v.power(k)
    names = "ijkl"
    want = ["for (i = 0; i <= 5; ++i)"] + ["%sfor (%s = %s; %s <= 5; ++%s)" % ("  " * t, names[t], names[t - 1], names[t], names[t])
                                             for t in range(1, k)]
    assert p.nest.splitlines()[:k] == want
    ref = {2: oracle.list_sym2, 3: oracle.list_sym3, 4: oracle.list_sym4}[k](n)
    assert p.count == ref.shape[0] == {2: 21, 3: 56, 4: 126}[k]
    Tc = W.uniform(791, p.count)
    _run_generated(p, str(tmp_path / "p"), (n,) * k, Tc)
    lst = np.fromfile(str(tmp_path / "p" / "list.i32"), dtype=np.int32).reshape(-1, k)
    assert np.array_equal(lst, ref.astype(np.int32))
    ex = np.fromfile(str(tmp_path / "p" / "expand.f32"), dtype=np.float32).reshape((n,) * k)
    assert np.array_equal(ex.view(np.uint32), oracle.expand_sym(Tc, n, k).view(np.uint32))
    # a vector whose unique set is a sub-range: the same structure on that range
    w = st.Descriptor("x(i): (2<=i<n)", (n,), None, n=n).power(k)
    sub = {2: oracle.list_sym2, 3: oracle.list_sym3, 4: oracle.list_sym4}[k](n - 2) + 2
    assert w.count == sub.shape[0]
    _run_generated(w, str(tmp_path / "w"), (n,) * k, W.uniform(792, w.count))
    assert np.array_equal(np.fromfile(str(tmp_path / "w" / "list.i32"), dtype=np.int32).reshape(-1, k), sub.astype(np.int32))


def test_vector_self_product_limits():
    s = st.Descriptor("S(i,j): (0<=i<=j<n)", (3, 3), None, n=3)
    with pytest.raises(st.StructTensorError) as e:
        s.power(2)
    assert e.value.status == 6
    v = st.Descriptor("x(i): (0<=i<n)", (3,), None, n=3)
    for k in (1, 5):
        with pytest.raises(st.StructTensorError) as e:
            v.power(k)
        assert e.value.status == 2


# ------------------------------------------------------------------ structure inference for sums
# name -> (M: text, redundancy, predicate, unique_of), (V: ...), dims, params, expected (predicate, unique_of) or None
SUMS = {
    # the same structure on both sides is kept, redundancy map included
    "sym_sym": (("M(i,j): (0<=i<=j<n)", SYM_RED, lambda i, j: i <= j, _swap),
                ("N(i,j): (0<=i<=j<n)", "sort", lambda i, j: i <= j, _swap), (6, 6), dict(n=6), (lambda i, j: i <= j, _swap)),
    "rows_rows": (("M(i,j): (i=0)*(0<=j<m)", "(1<=i<n) -> (0,j)", lambda i, j: i == 0, _rows),
                  ("N(i,j): (i=0)*(0<=j<m)", "(1<=i<n) -> (0,j)", lambda i, j: i == 0, _rows), (4, 5), dict(n=4, m=5),
                  (lambda i, j: i == 0, _rows)),
    # one support inside the other: the larger unique set, no redundancy
    "diag_upper": (("D(i,j): (0<=i<n)*(i=j)", None, lambda i, j: i == j, None),
                   ("U(i,j): (0<=i<=j<n)", None, lambda i, j: i <= j, None), (7, 7), dict(n=7), (lambda i, j: i <= j, None)),
    "band_diag3": (("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", None, lambda i, j, l: abs(i - j) <= 2, None),
                   ("D(i,j,l): (0<=i<n)*(i=j)*(0<=l<m)", None, lambda i, j, l: i == j, None), (8, 8, 3), dict(n=8, w=2, m=3),
                   (lambda i, j, l: abs(i - j) <= 2, None)),
    # different structures with a redundancy map: the maps are dropped, every non-zero element counts: the whole box
    "sym_upper": (("M(i,j): (0<=i<=j<n)", "sort", lambda i, j: i <= j, _swap),
                  ("U(i,j): (0<=i<=j<n)", None, lambda i, j: i <= j, None), (5, 5), dict(n=5), (lambda i, j: True, None)),
    "upper_lower": (("U(i,j): (0<=i<=j<n)", None, lambda i, j: i <= j, None),
                    ("L(i,j): (0<=j<i<n)", None, lambda i, j: j < i, None), (6, 6), dict(n=6), (lambda i, j: True, None)),
    # the union is a sum of nests: refused
    "band_row": (("B(i,j): (0<=i<n)*(i-1<=j<=i+1)", None, lambda i, j: abs(i - j) <= 1, None),
                 ("R(i,j): (i=0)*(0<=j<n)", None, lambda i, j: i == 0, None), (6, 6), dict(n=6), None),
}


@pytest.mark.parametrize("name", sorted(SUMS))
def test_sum_inference(oracle, tmp_path, name):
    """A(x) := M(x) + V(x): the inferred structure against predicates written out by hand, the values (two generated
    gather kernels run on the CPU, the second with the first as its addend) against the sum of the two reconstructed
    dense operands, bit for bit, and Property 5 for the result."""
    if CLANG is None:
        pytest.skip("no clang++ for the host build")
    (mt, mred, mpred, muniq), (vt, vred, vpred, vuniq), dims, params, want = SUMS[name]
    dm, dv = st.Descriptor(mt, dims, mred, **params), st.Descriptor(vt, dims, vred, **params)
    if want is None:
        with pytest.raises(st.StructTensorError) as e:
            dm.sum(dv)
        assert e.value.status == 6 and "sum of nests" in str(e.value)
        return
    apred, auniq = want
    da = dm.sum(dv)
    lst = oracle.struct_enumerate(dims, apred)
    assert da.count == lst.shape[0]
    Mc, Vc = W.uniform(801, dm.count), W.uniform(802, dv.count)
    dense = oracle.struct_expand(Mc, dims, mpred, muniq) + oracle.struct_expand(Vc, dims, vpred, vuniq)     # fp32 sums
    gm = _run_generated(dm, str(tmp_path / "m"), dims, Mc, gather_idx=lst)
    ac = _run_generated(dv, str(tmp_path / "v"), dims, Vc, gather_idx=lst, addend=gm)
    cols = tuple(lst[:, v].astype(np.int64) for v in range(len(dims)))
    assert np.array_equal(ac, dense[cols])
    _run_generated(da, str(tmp_path / "a"), dims, ac)
    got = np.fromfile(str(tmp_path / "a" / "list.i32"), dtype=np.int32).reshape(-1, len(dims))
    assert np.array_equal(got, lst)
    ex = np.fromfile(str(tmp_path / "a" / "expand.f32"), dtype=np.float32).reshape(dims)
    assert np.array_equal(ex, dense)
    assert np.array_equal(oracle.struct_expand(ac, dims, apred, auniq), dense)


# ------------------------------------------------------------------ projection: a rule head that drops the last variable
# name -> (text, dims, params, predicate, expected nest lines of the projection or None)
PROJECTIONS = {
    # the band tensor of the TTM workload: the last variable is free, the projection is the band on (i,j)
    "band": ("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", (9, 9, 5), dict(n=9, w=2, m=5), lambda i, j, l: abs(i - j) <= 2,
             ["for (i = 0; i <= 8; ++i)", "  for (j = max(0, i - 2); j <= min(8, i + 2); ++j)"]),
    # a tetrahedron of non-zeros: some l >= j exists for every j
    "tetra": ("B(i,j,l): (0<=i<n)*(i<=j<n)*(j<=l<n)", (6, 6, 6), dict(n=6), lambda i, j, l: i <= j <= l,
              ["for (i = 0; i <= 5; ++i)", "  for (j = i; j <= 5; ++j)"]),
    # the run of (i,j) is i-j <= l < m: not empty only when i - j <= m - 1, a comparison the dropped variable leaves behind
    "staircase": ("B(i,j,l): (0<=i<n)*(0<=j<=i)*(i-j<=l<m)", (7, 7, 3), dict(n=7, m=3), lambda i, j, l: j <= i and i - j <= l < 3,
                  ["for (i = 0; i <= 6; ++i)", "  for (j = max(0, i - 2); j <= i; ++j)"]),
    # two bounds on both sides of the last variable (an anti-diagonal band): every row keeps some column
    "anti": ("A(i,j): (0<=i<n)*(n-2<=i+j<=n)", (7, 7), dict(n=7), lambda i, j: 5 <= i + j <= 7, ["for (i = 0; i <= 6; ++i)"]),
    # nothing stored below a threshold of the first variable
    "late": ("L(i,j): (0<=i<n)*(0<=j<=i-3)", (8, 8), dict(n=8), lambda i, j: j <= i - 3, ["for (i = 3; i <= 7; ++i)"]),
    "diag": ("D(i,j): (0<=i<n)*(i=j)", (6, 6), dict(n=6), lambda i, j: i == j, ["for (i = 0; i <= 5; ++i)"]),
}


@pytest.mark.parametrize("name", sorted(PROJECTIONS))
def test_projection_inference(oracle, name):
    """A(x') := sum over the last variable of B(x', l): the inferred unique set is "some l is stored" (brute force),
    its nest is the expected one, and its packed order is the run order of B."""
    text, dims, params, pred, nest = PROJECTIONS[name]
    b = st.Descriptor(text, dims, None, **params)
    a = b.project()
    exists = lambda *x: any(pred(*x, l) for l in range(dims[-1]))
    lst = oracle.struct_enumerate(dims[:-1], exists)
    assert a.count == lst.shape[0] == b.runs
    assert a.nest.splitlines()[:len(nest)] == nest, a.nest
    full = oracle.struct_enumerate(dims, pred)
    heads = np.unique(full[:, :-1], axis=0)                          # prefixes that hold a run, sorted = nest order
    assert np.array_equal(heads.reshape(lst.shape), lst)
    a.close()
    b.close()


def test_projection_limits():
    s = st.Descriptor("S(i,j): (0<=i<=j<n)", (4, 4), "sort", n=4)
    with pytest.raises(st.StructTensorError) as e:
        s.project()
    assert e.value.status == 6
    v = st.Descriptor("v(i): (0<=i<n)", (4,), None, n=4)
    with pytest.raises(st.StructTensorError) as e:
        v.project()
    assert e.value.status == 2


def test_constant_range_rule_written_as_text(oracle, tmp_path):
    """The constant-range rule (T(x) := b <= x < c: only x = b is stored, every other element of the range takes its
    value): one redundancy term per variable, each excluding b itself so that Property 1 holds; a single stored
    value reconstructs the whole range, zero outside it."""
    if CLANG is None:
        pytest.skip("no clang++ for the host build")
    dims = (5, 6)
    d = st.Descriptor("T(i,j): (i=1)*(j=2)", dims, "(1<i<4)*(2<=j<5) -> (1,2); (i=1)*(2<j<5) -> (1,2)")
    assert d.count == 1
    _run_generated(d, str(tmp_path / "c"), dims, np.array([3.25], dtype=np.float32))
    ex = np.fromfile(str(tmp_path / "c" / "expand.f32"), dtype=np.float32).reshape(dims)
    want = np.zeros(dims, dtype=np.float32)
    want[1:4, 2:5] = 3.25
    assert np.array_equal(ex, want)
    with pytest.raises(st.StructTensorError) as e:                  # the range itself as the condition meets (1,2)
        st.Descriptor("T(i,j): (i=1)*(j=2)", dims, "(1<=i<4)*(2<=j<5) -> (1,2)")
    assert e.value.status == 2 and "disjoint" in str(e.value)
    d.close()


# ------------------------------------------------------------------ direct sum: a unique set that is a sum of two nests
_rows_n = lambda n: (lambda i, j: (0, j) if 1 <= i < n else None)
# name -> ((text, dims, redundancy, params, predicate, unique_of) of M, the same of V, nest lines of V's part or None)
DIRECT_SUMS = {
    "upper_sym": (("U(i,j): (0<=i<=j<n)", (4, 4), None, dict(n=4), lambda i, j: i <= j, None),
                  ("S(i,j): (0<=i<=j<n)", (5, 5), "sort", dict(n=5), lambda i, j: i <= j, _swap),
                  ["for (i = 4; i <= 8; ++i)", "  for (j = i; j <= 8; ++j)"]),
    # different offsets on the two indices, written-out terms on both sides (class S; identical rows)
    "sym_rows": (("S(i,j): (0<=i<=j<n)", (3, 3), SYM_RED, dict(n=3), lambda i, j: i <= j, _swap),
                 ("M(i,j): (i=0)*(0<=j<m)", (4, 6), "(1<=i<n) -> (0,j)", dict(n=4, m=6), lambda i, j: i == 0, _rows_n(4)),
                 ["for (i = 3; i <= 3; ++i)", "  for (j = 3; j <= 8; ++j)"]),
    "vectors": (("v(i): (2<=i<n)", (9,), None, dict(n=6), lambda i: 2 <= i < 6, None),
                ("w(i): (1<=i<=3)", (5,), None, dict(), lambda i: 1 <= i <= 3, None),
                ["for (i = 10; i <= 12; ++i)"]),
    "band3_diag3": (("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", (5, 5, 2), None, dict(n=5, w=1, m=2),
                     lambda i, j, l: abs(i - j) <= 1, None),
                    ("D(i,j,l): (0<=i<n)*(i=j)*(0<=l<m)", (4, 4, 3), None, dict(n=4, m=3), lambda i, j, l: i == j, None),
                    ["for (i = 5; i <= 8; ++i)", "  for (j = i; j <= i; ++j)", "    for (l = 2; l <= 4; ++l)"]),
    "sym3_lower": (("T(i,j,k): (0<=i<=j<n)*(j<=k<n)", (3, 3, 3), "sort", dict(n=3), lambda i, j, k: i <= j <= k, _sorted),
                   ("T(i,j,k): (0<=i<=j<n)*(j<=k<n)", (4, 4, 4), "sort", dict(n=4), lambda i, j, k: i <= j <= k, _sorted),
                   None),
    "empty_upper": (("E(i,j): (0<=i<n)*(j<i)*(j>i)", (3, 3), None, dict(n=3), lambda i, j: False, None),
                    ("U(i,j): (0<=i<=j<n)", (4, 4), None, dict(n=4), lambda i, j: i <= j, None), None),
}


@pytest.mark.parametrize("name", sorted(DIRECT_SUMS))
def test_direct_sum_inference(oracle, tmp_path, name):
    """T := M (+) V ("Redundancy Map Inference", direct-sum rule): the two summands of T_U and T_R come back as two
    descriptors over the box of T.  Each is checked against the operand's predicate moved by hand (brute force over
    the box), its packed order must be the operand's, and the reconstruction -- the first part expanded, the second
    laid over it, both generated kernels run on the CPU -- must equal the dense direct sum of the two reconstructed
    operands bit for bit."""
    if CLANG is None:
        pytest.skip("no clang++ for the host build")
    (mt, mdims, mred, mpar, mpred, muniq), (vt, vdims, vred, vpar, vpred, vuniq), nest = DIRECT_SUMS[name]
    dm, dv = st.Descriptor(mt, mdims, mred, **mpar), st.Descriptor(vt, vdims, vred, **vpar)
    pm, pv = dm.direct_sum(dv)
    dims = tuple(a + b for a, b in zip(mdims, vdims))
    assert pm.dims == dims and pv.dims == dims
    assert pm.count == dm.count and pv.count == dv.count
    order = len(dims)
    in_m = lambda *x: all(x[q] < mdims[q] for q in range(order)) and mpred(*x)
    in_v = lambda *x: all(x[q] >= mdims[q] for q in range(order)) and vpred(*[x[q] - mdims[q] for q in range(order)])
    lm, lv = oracle.struct_enumerate(dims, in_m), oracle.struct_enumerate(dims, in_v)
    assert lm.shape[0] == dm.count and lv.shape[0] == dv.count
    # the packed order of each part is the operand's: the operand's own listing, moved
    assert np.array_equal(lm, oracle.struct_enumerate(mdims, mpred))
    assert np.array_equal(lv, oracle.struct_enumerate(vdims, vpred) + np.asarray(mdims, dtype=np.int32))
    if nest is not None:
        assert pv.nest.splitlines()[:len(nest)] == nest
    Mc, Vc = W.uniform(811, max(dm.count, 1))[: dm.count], W.uniform(812, max(dv.count, 1))[: dv.count]
    dense = oracle.direct_sum(oracle.struct_expand(Mc, mdims, mpred, muniq), oracle.struct_expand(Vc, vdims, vpred, vuniq))
    _run_generated(pm, str(tmp_path / "m"), dims, Mc)
    got = np.fromfile(str(tmp_path / "m" / "list.i32"), dtype=np.int32).reshape(-1, order)
    assert np.array_equal(got, lm)
    first = np.fromfile(str(tmp_path / "m" / "expand.f32"), dtype=np.float32).reshape(dims)
    assert np.array_equal(first, oracle.direct_sum(oracle.struct_expand(Mc, mdims, mpred, muniq),
                                                   np.zeros(vdims, dtype=np.float32)))
    _run_generated(pv, str(tmp_path / "v"), dims, Vc, onto=first)
    got = np.fromfile(str(tmp_path / "v" / "list.i32"), dtype=np.int32).reshape(-1, order)
    assert np.array_equal(got, lv)
    both = np.fromfile(str(tmp_path / "v" / "expand_onto.f32"), dtype=np.float32).reshape(dims)
    assert np.array_equal(both.view(np.uint32), dense.view(np.uint32))
    # laid over a marker instead: only the elements of V's part change
    marker = np.full(dims, -3.0, dtype=np.float32)
    _run_generated(pv, str(tmp_path / "k"), dims, Vc, onto=marker)
    kept = np.fromfile(str(tmp_path / "k" / "expand_onto.f32"), dtype=np.float32).reshape(dims)
    vd = oracle.direct_sum(np.zeros(mdims, dtype=np.float32), np.ones(vdims, dtype=np.float32)) > 0
    held = oracle.direct_sum(np.zeros(mdims, dtype=np.float32),
                             oracle.struct_expand(np.ones(max(dv.count, 1), dtype=np.float32)[: dv.count], vdims, vpred, vuniq)) > 0
    assert np.array_equal(kept[~held], marker[~held]) and np.array_equal(kept[held], dense[held]) and not (held & ~vd).any()
    for d in (dm, dv, pm, pv):
        d.close()


def test_direct_sum_limits():
    """Operands of different orders are refused; a 'sort' map cannot be moved by different amounts on its indices."""
    a = st.Descriptor("v(i): (0<=i<n)", (4,), None, n=4)
    b = st.Descriptor("U(i,j): (0<=i<=j<n)", (4, 4), None, n=4)
    with pytest.raises(ValueError):
        a.direct_sum(b)
    m = st.Descriptor("G(i,j): (0<=i<n)*(0<=j<m)", (3, 5), None, n=3, m=5)
    s = st.Descriptor("S(i,j): (0<=i<=j<n)", (4, 4), "sort", n=4)
    with pytest.raises(st.StructTensorError) as e:
        m.direct_sum(s)
    assert e.value.status == 6 and "same offset" in str(e.value)
    # the other way round the symmetric operand stays in place and the general one moves: fine
    ps, pg = s.direct_sum(m)
    assert ps.count == 10 and pg.count == 15 and pg.nest.splitlines()[0] == "for (i = 4; i <= 6; ++i)"
