"""fasth_forward_static (the entry point that allocates nothing) against fasth_forward, through the C ABI:
two calls in a row on the same GPU, the second with a smaller input, so stale contents of the shared
scratch array would show."""
import ctypes

import numpy as np
import pytest

from helpers import REL_TOL, rel_err, to_gpu
from oracle import householder as orc
from paper_2009_13977_amd import synthetic


def _both(d, n, m, k, seed, transpose):
    import torch
    from paper_2009_13977_amd import binding as B
    p = synthetic.householder_problem(d, n, m, seed=seed)
    V, X = to_gpu(p["V"]), to_gpu(p["X"])
    A_ref = torch.empty_like(X)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))
    B.fasth_forward(V, X, A_ref, ws, k, transpose)
    A = torch.full_like(X, float("nan"))
    B.fasth_forward_static(V, X, A, k, transpose)
    torch.cuda.synchronize()
    return p, A.cpu().numpy(), A_ref.cpu().numpy()


@pytest.mark.gpu
@pytest.mark.parametrize("transpose", [False, True])
def test_static_forward_matches_forward_twice_in_a_row(transpose):
    for (d, n, m, k, seed) in ((1024, 1024, 32, 32, 91), (192, 128, 12, 16, 92)):
        p, A, A_ref = _both(d, n, m, k, seed, transpose)
        assert np.isfinite(A).all()
        assert rel_err(A, A_ref) <= REL_TOL
        want = orc.product_apply(p["V"], p["X"], transpose=transpose)
        assert rel_err(A, want) <= REL_TOL


@pytest.mark.gpu
def test_static_forward_larger_blocks_then_smaller():
    for (d, n, m, k, seed) in ((2048, 512, 64, 128, 93), (64, 64, 32, 32, 94)):
        p, A, A_ref = _both(d, n, m, k, seed, False)
        assert rel_err(A, A_ref) <= REL_TOL
        assert rel_err(A, orc.product_apply(p["V"], p["X"])) <= REL_TOL


@pytest.mark.gpu
def test_static_forward_falls_back_to_the_layout_without_shared_columns():
    """d = 2048 with 4096 reflections and 8 columns: the kernels in which workgroups share a column would need 25 MiB
    for the partial matrices of their 64-row factors, more than the array holds; the call then uses the caller's block
    size and the per-column kernels, 10 MiB. A shape beyond that too is refused."""
    from paper_2009_13977_amd import binding as B
    p, A, A_ref = _both(2048, 4096, 8, 32, 95, False)
    assert rel_err(A, A_ref) <= REL_TOL
    assert rel_err(A, orc.product_apply(p["V"], p["X"])) <= REL_TOL
    shape = B.fasth_shape(8192, 8192, 8, 128, 0)
    assert B.load_library().fasth_forward_static(ctypes.byref(shape), 256, 256, 256, None) == B.FASTH_EUNSUPPORTED

