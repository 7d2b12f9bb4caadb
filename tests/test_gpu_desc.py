"""Descriptor-driven structures on the GPU: kernels generated for a textual unique set / redundancy map,
compiled with hiprtc and run through the C ABI, against brute force over the index box (small cases) and
against the hand-written kernels of the same structures (full sizes)."""
import sys

import numpy as np
import pytest

import st_workloads as W
from test_desc import CASES, OUTERS, PROJECTIONS, SUMS

pytestmark = pytest.mark.gpu


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


@pytest.mark.parametrize("name", sorted(CASES))
def test_generated_kernels_small(st, oracle, name):
    say("descriptor", name)
    text, dims, red, params, pred, unique_of = CASES[name]
    d = st.Descriptor(text, dims, red, **params)
    lst = oracle.struct_enumerate(dims, pred)
    assert np.array_equal(d.list().cpu().numpy(), lst)
    Bc = W.uniform(711, max(d.count, 4))
    Cd = W.uniform(712, int(np.prod(dims))).reshape(dims)
    got = d.thp(dev(Bc), dev(Cd)).cpu().numpy()[: d.count]
    assert np.array_equal(got, oracle.struct_thp(Bc[: d.count], Cd, dims, pred).astype(np.float32))
    ex = d.expand(dev(Bc)).cpu().numpy()
    ref = oracle.struct_expand(Bc[: d.count], dims, pred, unique_of)
    assert np.array_equal(ex.view(np.uint32), ref.view(np.uint32))
    d.close()


def test_generated_against_handwritten_sym3(st, oracle):
    n = 64
    say("descriptor sym3 n=%d against st_expand_sym / the closed-form unrank" % n)
    d = st.Descriptor("T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)", (n, n, n), "sort", n=n)
    assert d.count == st.count_sym3(n)
    assert np.array_equal(d.list().cpu().numpy(), oracle.list_sym3(n).astype(np.int32))
    Sc = dev(W.uniform(721, d.count))
    got = d.expand(Sc).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), st.expand_sym(Sc, n, 3).cpu().numpy().view(np.uint32))
    assert np.array_equal(got.view(np.uint32), oracle.expand_sym(Sc.cpu().numpy(), n, 3).view(np.uint32))
    d.close()


def test_generated_against_handwritten_sym4(st, oracle):
    n = 24
    d = st.Descriptor("Q(i,j,k,l): (0<=i<=j<n)*(j<=k<=l<n)", (n,) * 4, "sort", n=n)
    assert d.count == st.count_sym4(n)
    assert np.array_equal(d.list().cpu().numpy(), oracle.list_sym4(n).astype(np.int32))
    Sc = dev(W.uniform(722, d.count))
    got = d.expand(Sc).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), oracle.expand_sym(Sc.cpu().numpy(), n, 4).view(np.uint32))
    d.close()


def test_generated_against_handwritten_band_full(st, oracle):
    cfg = W.CONFIGS[3]
    n, w, nl = cfg["n"], cfg["w"], cfg["nl"]
    say("descriptor band n=%d w=%d nl=%d against st_expand_band / the band oracle" % (n, w, nl))
    d = st.Descriptor("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", (n, n, nl), n=n, w=w, m=nl)
    assert d.count == cfg["band_pairs"] * nl and d.runs == cfg["band_pairs"]
    Tb, _ = W.ttm_inputs(cfg["band_pairs"], nl, cfg["R"])
    Tbd = dev(Tb.reshape(-1))
    got = d.expand(Tbd).cpu().numpy()
    ref = oracle.dense_band(Tb, n, w, nl).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    assert np.array_equal(got, st.expand_band(Tbd, n, w, nl).cpu().numpy())
    # THP over the band against a dense operand: every in-band fibre times the matching fibre of C
    Cd = W.uniform(731, n * n * nl).reshape(n, n, nl)
    thp = d.thp(Tbd, dev(Cd)).cpu().numpy().reshape(-1, nl)
    pairs = oracle.list_band(n, w).astype(np.int64)
    ref = oracle.thp_full(Tb.reshape(-1, nl), Cd[pairs[:, 0], pairs[:, 1]])
    assert np.array_equal(thp, ref.astype(np.float32))
    d.close()


def test_generated_against_handwritten_upper_cube(st, oracle):
    n, nl = 200, 64
    d = st.Descriptor("B(i,j,l): (0<=i<n)*(i<=j<n)*(0<=l<m)", (n, n, nl), n=n, m=nl)
    pairs = st.count_struct(st.STRUCT_UPPER, n, n)
    assert d.count == pairs * nl
    Bc = W.uniform(741, pairs * nl).reshape(pairs, nl)
    Cd = W.uniform(742, n * n * nl).reshape(n, n, nl)
    got = d.thp(dev(Bc.reshape(-1)), dev(Cd)).cpu().numpy().reshape(pairs, nl)
    hand = st.thp_struct(st.STRUCT_UPPER, dev(Bc), dev(Cd)).cpu().numpy()
    assert np.array_equal(got, hand)
    d.close()


@pytest.mark.parametrize("name,R", [("band", 16), ("diag", 5), ("fixed_j", 32), ("upper_cube", 48)])
def test_descriptor_ttm_small(st, oracle, name, R):
    say("descriptor ttm", name)
    text, dims, red, params, pred, _ = CASES[name]
    d = st.Descriptor(text, dims, red, **params)
    nl = dims[-1]
    lst = oracle.struct_enumerate(dims, pred)
    Bc = W.uniform(751, d.count)
    U = W.uniform(752, nl * R).reshape(nl, R)
    B = np.zeros(dims, dtype=np.float32)
    B[tuple(lst[:, v] for v in range(len(dims)))] = Bc            # zero-filled dense operand
    full = oracle.ttm_full(B, U)                                   # dense definition
    heads = lst[::nl, :-1]                                         # one (i,j) per run, in packed order
    ref = full[heads[:, 0], heads[:, 1]]
    mask = np.ones(dims[:2], dtype=bool)
    mask[heads[:, 0], heads[:, 1]] = False
    assert not full[mask].any()                                    # the output keeps the structure of (i,j)
    got = d.ttm(dev(Bc.reshape(-1, nl)), dev(U)).cpu().numpy()
    assert got.shape == ref.shape
    assert float(np.abs(got - ref).max() / np.abs(ref).max()) <= 1e-4
    d.close()


# the kernel table's MTTKRP over ANY sparsity structure of an order-3 operand, generated from the descriptor
MTTKRP_CASES = {
    # name: (unique set, dims, parameters, predicate, R)
    "band": ("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", (40, 40, 33), dict(n=40, w=3, m=33), lambda i, j, l: abs(i - j) <= 3, 21),
    "diag": ("B(i,j,l): (0<=i<n)*(i=j)*(0<=l<m)", (50, 50, 70), dict(n=50, m=70), lambda i, j, l: i == j, 64),
    "fixed_i": ("B(i,j,l): (i=I)*(0<=j<n)*(0<=l<m)", (9, 30, 65), dict(I=4, n=30, m=65), lambda i, j, l: i == 4, 16),
    "fixed_j": ("B(i,j,l): (0<=i<n)*(j=J)*(0<=l<m)", (37, 12, 129), dict(J=7, n=37, m=129), lambda i, j, l: j == 7, 48),
    "upper_cube": ("B(i,j,l): (0<=i<n)*(i<=j<n)*(0<=l<m)", (33, 33, 40), dict(n=33, m=40), lambda i, j, l: i <= j, 5),
    # an empty unique set (the factors contradict each other through a parameter): every row comes back as zeros
    "empty": ("B(i,j,l): (0<=i<n)*(n<=3)*(0<=j<n)*(0<=l<n)", (6, 6, 6), dict(n=6), lambda i, j, l: False, 8),
    # a structure on all three indices, which no hand-written kernel here has: the tetrahedron as a SPARSITY pattern
    "tetra": ("B(i,j,l): (0<=i<n)*(i<=j<n)*(j<=l<n)", (30, 30, 30), dict(n=30), lambda i, j, l: i <= j <= l, 33),
    "staircase": ("B(i,j,l): (0<=i<n)*(0<=j<=i)*(i-j<=l<m)", (25, 25, 31), dict(n=25, m=31), lambda i, j, l: j <= i and l >= i - j, 17),
}


@pytest.mark.parametrize("name", sorted(MTTKRP_CASES))
def test_descriptor_mttkrp_small(st, oracle, name):
    """A(i,r) = sum_kl B(i,k,l) C(k,r) D(l,r) over the unique set only, against the dense definition (C oracle) on
    the zero-filled operand; rows without a stored entry come back as zeros."""
    say("descriptor mttkrp", name)
    text, dims, params, pred, R = MTTKRP_CASES[name]
    d = st.Descriptor(text, dims, None, **params)
    lst = oracle.struct_enumerate(dims, pred)
    assert d.count == lst.shape[0]
    Bc = W.uniform(761, max(d.count, 4))[: max(d.count, 4)]
    Cm, Dm = W.uniform(762, dims[1] * R).reshape(dims[1], R), W.uniform(763, dims[2] * R).reshape(dims[2], R)
    B = np.zeros(dims, dtype=np.float32)
    B[tuple(lst[:, v].astype(np.int64) for v in range(3))] = Bc[: d.count]
    ref = oracle.mttkrp_full(B, Cm, Dm)
    import torch
    A = torch.full((dims[0], R), float("nan"), device="cuda")
    got = d.mttkrp(dev(Bc), dev(Cm), dev(Dm), A=A).cpu().numpy()
    assert float(np.abs(got - ref).max()) <= 1e-4 * max(float(np.abs(ref).max()), 1e-30)
    empty = ~B.reshape(dims[0], -1).any(axis=1)
    assert not got[empty].any()
    again = d.mttkrp(dev(Bc), dev(Cm), dev(Dm)).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), again.view(np.uint32))          # fixed summation order
    d.close()


def test_descriptor_mttkrp_against_handwritten_fixed_k(st, oracle):
    """The kernel table's "fixed j" structure at full size (n = 512): the generated kernel against the hand-written
    st_mttkrp_fixed, and sampled rows against the oracle."""
    n, nl, R, K = 512, 512, 64, 100
    say("descriptor mttkrp fixed k n=%d against st_mttkrp_fixed" % n)
    d = st.Descriptor("B(i,k,l): (0<=i<n)*(k=K)*(0<=l<m)", (n, n, nl), None, n=n, K=K, m=nl)
    Bc = W.uniform(771, n * nl).reshape(n, nl)
    Cm, Dm = W.uniform(772, n * R).reshape(n, R), W.uniform(773, nl * R).reshape(nl, R)
    got = d.mttkrp(dev(Bc.reshape(-1)), dev(Cm), dev(Dm)).cpu().numpy()
    hand = st.mttkrp_fixed(st.MTTKRP_FIXED_K, dev(Bc), dev(Cm), dev(Dm), n, fixed_k=K).cpu().numpy()
    assert float(np.abs(got - hand).max()) <= 1e-4 * float(np.abs(hand).max())
    rows = np.array([0, 1, 77, 255, 256, 511])
    ref = (Bc[rows].astype(np.float64) @ Dm.astype(np.float64)) * Cm[K].astype(np.float64)
    assert float(np.abs(got[rows] - ref).max()) <= 1e-4 * float(np.abs(ref).max())
    d.close()


def test_descriptor_mttkrp_refuses_what_it_does_not_cover(st):
    import torch
    z = torch.zeros(4096, device="cuda")
    d = st.Descriptor("T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)", (8, 8, 8), "sort", n=8)        # redundancy map
    with pytest.raises(st.StructTensorError) as e:
        d.mttkrp(z[:d.count], z[:64].reshape(8, 8), z[:64].reshape(8, 8))
    assert e.value.status == 6
    d.close()
    d = st.Descriptor("S(i,j): (0<=i<=j<n)", (8, 8), None, n=8)                               # order 2
    with pytest.raises(st.StructTensorError) as e:
        d.mttkrp(z[:d.count], z[:64].reshape(8, 8), z[:64].reshape(8, 8))
    assert e.value.status == 6
    d.close()


def test_descriptor_ttm_needs_a_free_last_variable(st):
    d = st.Descriptor("T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)", (8, 8, 8), "sort", n=8)
    import torch
    z = torch.zeros(4096, device="cuda")
    with pytest.raises(st.StructTensorError):
        d.ttm(z[:d.count], z[:64].reshape(8, 8))
    d.close()


def test_descriptor_ttm_band_full(st, oracle):
    cfg = W.CONFIGS[3]
    n, w, nl, R = cfg["n"], cfg["w"], cfg["nl"], cfg["R"]
    d = st.Descriptor("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", (n, n, nl), n=n, w=w, m=nl)
    Tb, U = W.ttm_inputs(cfg["band_pairs"], nl, R)
    got = d.ttm(dev(Tb), dev(U)).cpu().numpy()
    ref = oracle.ttm_band(Tb, U, n, w)
    assert float(np.abs(got - ref).max() / np.abs(ref).max()) <= 1e-4
    assert np.array_equal(got, st.ttm_band(dev(Tb), dev(U), n, w).cpu().numpy())
    d.close()


MOMENT_CASES = {
    # name -> (text, order, n, params, predicate)
    "sym2": ("S(i,j): (0<=i<=j<n)", 2, 40, {}, lambda i, j: i <= j),
    "sym3": ("T(i,j,k): (0<=i<=j<n)*(j<=k<n)", 3, 22, {}, lambda i, j, k: i <= j <= k),
    "near2": ("S(i,j): (0<=i<n)*(i<=j<=i+w)", 2, 70, dict(w=3), lambda i, j: i <= j <= i + 3),
    "near3": ("T(i,j,k): (0<=i<=j<n)*(j<=k<=i+w)", 3, 30, dict(w=5), lambda i, j, k: i <= j <= k <= i + 5),
    "full2": ("G(i,j): (0<=i<n)*(0<=j<n)", 2, 9, {}, lambda i, j: True),
    "diag3": ("D(i,j,k): (0<=i<n)*(i=j)*(j=k)", 3, 33, {}, lambda i, j, k: i == j == k),
}


@pytest.mark.parametrize("name", sorted(MOMENT_CASES))
@pytest.mark.parametrize("N", [1, 257, 1500])
def test_descriptor_moment(st, oracle, name, N):
    say("descriptor moment", name, N)
    text, order, n, params, pred = MOMENT_CASES[name]
    d = st.Descriptor(text, (n,) * order, None, n=n, **params)
    X = W.normal(761, N * n).reshape(N, n)
    ref = oracle.struct_moment(X, (n,) * order, pred)
    assert d.count == ref.size
    got = d.moment(dev(X)).cpu().numpy()
    scale = np.abs(ref).max()
    assert float(np.abs(got - ref).max() / scale) <= 1e-4
    # creation and addition: two batches
    h = N // 2
    Sc = d.moment(dev(X[:h])).clone() if h > 0 else None
    if Sc is not None:
        import torch
        buf = torch.empty(max(d.count, 4), device="cuda")
        buf[: d.count] = Sc
        got2 = d.moment(dev(X[h:]), Sc=buf, accumulate=True).cpu().numpy()
        assert float(np.abs(got2 - ref).max() / scale) <= 1e-4
    d.close()


def test_descriptor_moment_against_handwritten(st, oracle):
    import torch
    n, N = 64, 20000
    X = dev(W.normal(762, N * n).reshape(N, n))
    d3 = st.Descriptor("T(i,j,k): (0<=i<=j<n)*(j<=k<n)", (n, n, n), "sort", n=n)
    a, b = d3.moment(X).cpu().numpy(), st.moment3_sym(X).cpu().numpy()
    assert float(np.abs(a - b).max() / np.abs(b).max()) <= 2e-5
    d2 = st.Descriptor("S(i,j): (0<=i<=j<n)", (n, n), None, n=n)
    a, b = d2.moment(X).cpu().numpy(), st.moment2_sym(X).cpu().numpy()
    assert float(np.abs(a - b).max() / np.abs(b).max()) <= 2e-5
    # N = 0: overwrite gives zeros, accumulate leaves Sc alone
    buf = torch.full((d2.count,), 3.0, device="cuda")
    empty = torch.empty((0, n), device="cuda")
    d2.moment(empty, Sc=buf, accumulate=True)
    assert float(buf.min()) == 3.0
    d2.moment(empty, Sc=buf)
    assert float(buf.abs().max()) == 0.0
    # unsupported: unequal extents
    db = st.Descriptor("B(i,j,l): (0<=i<n)*(i-1<=j<=i+1)*(0<=l<m)", (8, 8, 4), n=8, m=4)
    with pytest.raises(st.StructTensorError):
        db.moment(torch.zeros((5, 8), device="cuda"))
    for d in (d2, d3, db):
        d.close()


# ------------------------------------------------------------ element-wise products of two structured operands
from test_desc import PRODUCTS


@pytest.mark.parametrize("name", sorted(k for k, v in PRODUCTS.items() if v[4] is not None))
def test_product_of_structured_operands_small(st, oracle, name):
    say("descriptor product", name)
    (mt, mred, mpred, muniq), (vt, vred, vpred, vuniq), dims, params, (apred, auniq), _ = PRODUCTS[name]
    dm, dv = st.Descriptor(mt, dims, mred, **params), st.Descriptor(vt, dims, vred, **params)
    Mc, Vc = W.uniform(771, max(dm.count, 4)), W.uniform(772, max(dv.count, 4))
    da, Ac = st.hadamard_struct(dm, dev(Mc), dv, dev(Vc))
    lst = oracle.struct_enumerate(dims, apred)
    assert da.count == lst.shape[0] == Ac.numel()
    dense = oracle.struct_expand(Mc[: dm.count], dims, mpred, muniq) * oracle.struct_expand(Vc[: dv.count], dims, vpred, vuniq)
    if da.count:
        assert np.array_equal(da.list().cpu().numpy(), lst)
        cols = tuple(lst[:, v].astype(np.int64) for v in range(len(dims)))
        got = Ac.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), dense[cols].view(np.uint32))
        import torch
        buf = torch.zeros(max(da.count, 4), device="cuda")
        buf[: da.count] = Ac
        assert np.array_equal(da.expand(buf).cpu().numpy(), dense)          # Property 5 for the result
    else:
        assert not dense.any()
    for d in (dm, dv, da):
        d.close()


def test_upper_triangular_times_symmetric_full(st, oracle):
    """The paper's UHS walk-through at n = 2048: the inferred structure is the upper triangle with no redundancy,
    the values are the products of the stored entries (both operands share the packing), checked against the C
    oracle's dense forms of the two operands."""
    n = 2048
    say("descriptor product: upper triangular (.) symmetric, n=%d" % n)
    dm = st.Descriptor("M(i,j): (0<=i<=j<n)", (n, n), None, n=n)
    dv = st.Descriptor("N(i,j): (0<=i<=j<n)", (n, n), "sort", n=n)
    cnt = oracle.count_sym2(n)
    Mc, Vc = W.uniform(781, cnt), W.uniform(782, cnt)
    da, Ac = st.hadamard_struct(dm, dev(Mc), dv, dev(Vc))
    assert da.count == cnt and da.nest.splitlines()[1].strip() == "for (j = i; j <= %d; ++j)" % (n - 1)
    dense = oracle.dense_utri(Mc, n).astype(np.float32) * oracle.expand_sym(Vc, n, 2)
    iu = np.triu_indices(n)
    assert np.array_equal(Ac.cpu().numpy(), dense[iu])
    assert not np.tril(dense, -1).any()                    # nothing below the diagonal: no redundancy map needed
    # the other order of the operands gives the same structure and values
    db, Bc = st.hadamard_struct(dv, dev(Vc), dm, dev(Mc))
    assert db.count == cnt and np.array_equal(Bc.cpu().numpy(), Ac.cpu().numpy())
    for d in (dm, dv, da, db):
        d.close()


@pytest.mark.parametrize("name", sorted(OUTERS))
def test_outer_product_of_structured_operands(st, oracle, name):
    """T(x, y) := M(x) * V(y) on the GPU: inferred descriptor, values from two gathers over the two halves of the
    result's own index list, against the dense outer product (bit for bit), and Property 5 through the generated
    reconstruction of the result."""
    say("descriptor outer product", name)
    (mt, mdims, mred, mpar, mpred, muniq), (vt, vdims, vred, vpar, vpred, vuniq) = OUTERS[name]
    dm, dv = st.Descriptor(mt, mdims, mred, **mpar), st.Descriptor(vt, vdims, vred, **vpar)
    k, dims = len(mdims), tuple(mdims) + tuple(vdims)
    Mc, Vc = W.uniform(781, max(dm.count, 4)), W.uniform(782, max(dv.count, 4))
    dt, Tc = st.outer_struct(dm, dev(Mc), dv, dev(Vc))
    lst = oracle.struct_enumerate(dims, lambda *x: mpred(*x[:k]) and vpred(*x[k:]))
    assert dt.count == lst.shape[0] == Tc.numel()
    assert np.array_equal(dt.list().cpu().numpy(), lst)
    Md = oracle.struct_expand(Mc[: dm.count], mdims, mpred, muniq)
    Vd = oracle.struct_expand(Vc[: dv.count], vdims, vpred, vuniq)
    dense = (Md.reshape(mdims + (1,) * len(vdims)) * Vd.reshape((1,) * k + vdims)).astype(np.float32)
    cols = tuple(lst[:, v].astype(np.int64) for v in range(len(dims)))
    assert np.array_equal(Tc.cpu().numpy().view(np.uint32), dense[cols].view(np.uint32))
    import torch
    buf = torch.zeros(max(dt.count, 4), device="cuda")
    buf[: dt.count] = Tc
    assert np.array_equal(dt.expand(buf).cpu().numpy(), dense)
    for d in (dm, dv, dt):
        d.close()


@pytest.mark.parametrize("k", [2, 3])
def test_self_product_structure_drives_the_moment_kernels(st, oracle, k):
    """The covariance terms as the inference gives them: the k-fold self product of the feature vector has the
    structure x_1 <= .. <= x_k with a sort map; accumulating over samples on that descriptor equals the hand-written
    moment kernels (same packed order) and the oracle, and its reconstruction equals st_expand_sym."""
    n, N = 64, 3000
    say("self product of a vector, degree %d, n=%d: moments through the inferred descriptor" % (k, n))
    v = st.Descriptor("f(i): (0<=i<n)", (n,), None, n=n)
    p = v.power(k)
    assert p.count == (st.count_sym2(n) if k == 2 else st.count_sym3(n))
    X = W.normal(795, N * n).reshape(N, n)
    got = p.moment(dev(X)).cpu().numpy()
    hand = (st.moment2_sym if k == 2 else st.moment3_sym)(dev(X)).cpu().numpy()
    ref = oracle.moment2_dense(X)[np.triu_indices(n)] if k == 2 else oracle.moment3_entries(X, oracle.list_sym3(n))
    scale = float(np.abs(ref).max())
    assert float(np.abs(got - ref).max()) <= 1e-4 * scale and float(np.abs(got - hand).max()) <= 1e-4 * scale
    Sc = dev(W.uniform(796, p.count))
    assert np.array_equal(p.expand(Sc).cpu().numpy().view(np.uint32), st.expand_sym(Sc, n, k).cpu().numpy().view(np.uint32))
    v.close()
    p.close()


@pytest.mark.parametrize("name", sorted(k for k, v in SUMS.items() if v[4] is not None))
def test_sum_of_structured_operands(st, oracle, name):
    """A(x) := M(x) + V(x) on the GPU: inferred descriptor, values from two gathers (the second adds the first),
    against the sum of the two reconstructed dense operands, and Property 5 for the result."""
    say("descriptor sum", name)
    (mt, mred, mpred, muniq), (vt, vred, vpred, vuniq), dims, params, (apred, auniq) = SUMS[name]
    dm, dv = st.Descriptor(mt, dims, mred, **params), st.Descriptor(vt, dims, vred, **params)
    Mc, Vc = W.uniform(801, max(dm.count, 4)), W.uniform(802, max(dv.count, 4))
    da, Ac = st.add_struct(dm, dev(Mc), dv, dev(Vc))
    lst = oracle.struct_enumerate(dims, apred)
    assert da.count == lst.shape[0] == Ac.numel()
    assert np.array_equal(da.list().cpu().numpy(), lst)
    dense = oracle.struct_expand(Mc[: dm.count], dims, mpred, muniq) + oracle.struct_expand(Vc[: dv.count], dims, vpred, vuniq)
    cols = tuple(lst[:, v].astype(np.int64) for v in range(len(dims)))
    assert np.array_equal(Ac.cpu().numpy(), dense[cols])
    import torch
    buf = torch.zeros(max(da.count, 4), device="cuda")
    buf[: da.count] = Ac
    assert np.array_equal(da.expand(buf).cpu().numpy(), dense)
    for d in (dm, dv, da):
        d.close()


@pytest.mark.parametrize("name", sorted(PROJECTIONS))
def test_projection_of_a_structured_operand(st, oracle, name):
    """A(x') := sum_l B(x', l) on the GPU: inferred descriptor (packed order = run order of B) and the run sums of
    the generated kernel against the zero-filled dense operand summed over its last axis; bit-identical twice."""
    say("descriptor projection", name)
    text, dims, params, pred, _ = PROJECTIONS[name]
    b = st.Descriptor(text, dims, None, **params)
    a = b.project()
    lst = oracle.struct_enumerate(dims, pred)
    Bc = W.uniform(811, max(b.count, 4))
    Bz = np.zeros(dims, dtype=np.float64)
    cols = tuple(lst[:, v].astype(np.int64) for v in range(len(dims)))
    Bz[cols] = Bc[: b.count]
    alst = a.list().cpu().numpy()
    want = Bz.sum(axis=-1)[tuple(alst[:, v].astype(np.int64) for v in range(len(dims) - 1))]
    got = b.sum_last(dev(Bc)).cpu().numpy()
    assert got.shape == want.shape and float(np.abs(got - want).max()) <= 1e-5 * max(float(np.abs(want).max()), 1.0)
    assert np.array_equal(got, b.sum_last(dev(Bc)).cpu().numpy())
    a.close()
    b.close()


def test_ttm_output_structure_is_projection_times_range(st, oracle):
    """The kernel table's TTM, A(i,j,k) := B(i,j,l) * C(k,l): its output structure by inference is the projection of
    B's over l, outer product with the range of k -- and that is the packed layout st_desc_ttm writes: row p of its
    output is entry (i,j) number p of the projected descriptor, all k."""
    n, w, nl, R = 40, 3, 64, 16
    b = st.Descriptor("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", (n, n, nl), None, n=n, w=w, m=nl)
    k = st.Descriptor("k(r): (0<=r<R)", (R,), None, R=R)
    a = b.project().outer(k)
    assert a.count == b.runs * R and a.dims == (n, n, R)
    pairs = oracle.list_band(n, w).astype(np.int32)
    want = np.concatenate([np.repeat(pairs, R, axis=0), np.tile(np.arange(R, dtype=np.int32), pairs.shape[0])[:, None]], axis=1)
    assert np.array_equal(a.list().cpu().numpy(), want)
    Bc, U = W.uniform(821, b.count).reshape(-1, nl), W.uniform(822, nl * R).reshape(nl, R)
    Ac = b.ttm(dev(Bc), dev(U))                                       # [runs][R] = the packed values of A
    dense = a.expand(Ac.reshape(-1)).cpu().numpy()                    # reconstruction through the inferred descriptor
    ref = oracle.ttm_dense(Bc.reshape(-1), U, n, w)
    assert float(np.abs(dense - ref).max()) <= 1e-4 * float(np.abs(ref).max())
    for d in (a, b, k):
        d.close()


from test_desc import DIRECT_SUMS


@pytest.mark.parametrize("name", sorted(DIRECT_SUMS))
def test_direct_sum_of_structured_operands(st, oracle, name):
    """T := M (+) V on the GPU: the two parts list the operands' unique sets moved into the box of T, and the first
    part expanded with the second laid over it is the dense direct sum of the two reconstructed operands, bit for bit."""
    say("descriptor direct sum", name)
    import torch
    (mt, mdims, mred, mpar, mpred, muniq), (vt, vdims, vred, vpar, vpred, vuniq), _ = DIRECT_SUMS[name]
    dm, dv = st.Descriptor(mt, mdims, mred, **mpar), st.Descriptor(vt, vdims, vred, **vpar)
    pm, pv = dm.direct_sum(dv)
    off = np.asarray(mdims, dtype=np.int32)
    assert np.array_equal(pm.list().cpu().numpy(), oracle.struct_enumerate(mdims, mpred))
    assert np.array_equal(pv.list().cpu().numpy(), oracle.struct_enumerate(vdims, vpred) + off)
    # one packed array for T: M_C followed by V_C (the second part starts at a 16-byte boundary of its own copy here)
    Mc, Vc = W.uniform(811, max(dm.count, 4)), W.uniform(812, max(dv.count, 4))
    T = pm.expand(dev(Mc))
    pv.expand_onto(dev(Vc), T)
    dense = oracle.direct_sum(oracle.struct_expand(Mc[: dm.count], mdims, mpred, muniq),
                              oracle.struct_expand(Vc[: dv.count], vdims, vpred, vuniq))
    assert np.array_equal(T.cpu().numpy().view(np.uint32), dense.view(np.uint32))
    # a part is an ordinary descriptor: the Hadamard product with a dense operand on V's part alone
    Cd = W.uniform(813, int(np.prod(dense.shape))).reshape(dense.shape)
    if dv.count:
        got = pv.thp(dev(Vc), dev(Cd)).cpu().numpy()
        lv = pv.list().cpu().numpy().astype(np.int64)
        assert np.array_equal(got, Vc[: dv.count] * Cd[tuple(lv[:, q] for q in range(lv.shape[1]))])
    for d in (dm, dv, pm, pv):
        d.close()


def test_direct_sum_of_large_blocks(st, oracle):
    """A symmetric 300 x 300 block and an upper-triangular 212 x 212 block: 512 x 512 in all, checked through the
    block property of the dense definition (the oracle's element-by-element loop is too slow here)."""
    say("descriptor direct sum, 300 + 212")
    import torch
    ds = st.Descriptor("S(i,j): (0<=i<=j<n)", (300, 300), "sort", n=300)
    du = st.Descriptor("U(i,j): (0<=i<=j<n)", (212, 212), None, n=212)
    ps, pu = ds.direct_sum(du)
    Sc, Uc = W.uniform(821, ds.count), W.uniform(822, du.count)
    T = ps.expand(dev(Sc))
    pu.expand_onto(dev(Uc), T)
    T = T.cpu().numpy()
    S = np.zeros((300, 300), dtype=np.float32)
    iu = np.triu_indices(300)
    S[iu] = Sc
    S.T[iu] = Sc
    U = np.zeros((212, 212), dtype=np.float32)
    U[np.triu_indices(212)] = Uc
    assert np.array_equal(T[:300, :300], S) and np.array_equal(T[300:, 300:], U)
    assert not T[:300, 300:].any() and not T[300:, :300].any()
    for d in (ds, du, ps, pu):
        d.close()
