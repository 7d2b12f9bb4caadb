"""The entry point that allocates nothing (st_batax_utri_noalloc: partial results in a static device array of the
library) against st_batax_utri, through the C ABI: same kernels, so the results must be bit-identical.  Two
calls in a row, the second with a smaller input, so that what the first call left in the shared array is there
when the second runs."""
import sys

import numpy as np
import pytest

import st_workloads as W

pytestmark = pytest.mark.gpu


def test_noalloc_matches_workspace_entry_point(oracle):
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    import paper_2211_10482_amd as st
    st.lib()
    assert st.lib().st_batax_utri_noalloc_max_n() == 8192
    for n in (8192, 1000, 4100, 257, 5, 8192):
        print("batax without allocation n=%d" % n, flush=True)
        sys.stdout.flush()
        Ap = torch.from_numpy(W.uniform(811, oracle.count_sym2(n))).cuda()
        x = torch.from_numpy(W.uniform(812, n)).cuda()
        want = st.batax_utri(Ap, x, 0.5)
        y = torch.full((n,), float("nan"), device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        st.batax_utri_noalloc(Ap, x, 0.5, y)
        assert torch.cuda.memory_allocated() == before           # nothing came from torch's allocator either
        torch.cuda.synchronize()
        assert torch.equal(y, want), n
        ref = oracle.batax_utri(Ap.cpu().numpy(), x.cpu().numpy(), 0.5)
        assert float(np.abs(y.cpu().numpy() - ref).max() / np.abs(ref).max()) <= 1e-4
    # beyond the static array: a clear error, nothing launched
    n = 8193
    Ap = torch.zeros(oracle.count_sym2(n), device="cuda")
    x = torch.zeros(n, device="cuda")
    y = torch.zeros(n, device="cuda")
    with pytest.raises(st.StructTensorError) as e:
        st.batax_utri_noalloc(Ap, x, 0.5, y)
    assert e.value.status == 6
