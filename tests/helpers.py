"""Shared test helpers: error metric and GPU marshalling (no method arithmetic)."""
import numpy as np

REL_TOL = 1e-4  # relative Frobenius error bar for fp32 GPU results against the fp64 checker
# A Frobenius norm over a whole output would hide an error confined to a few entries or to one row, so every
# parity check also bounds the largest single deviation, against the output's largest entry, and (for
# gradients of Householder vectors, whose rows scale like 1 / ||v_j||) every row's own relative error. The
# fp32 kernels measure 1e-7 .. 2e-6 on all three; the bounds leave the same two orders of headroom.
MAX_TOL = 1e-4
ROW_TOL = 1e-4
ROW_FLOOR = 1e-3  # a row far smaller than the largest is held to this fraction of the largest row's norm


def rel_err(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / (den if den > 0 else 1.0))


def max_err(got, ref) -> float:
    """Largest deviation of one entry, relative to the largest entry of the reference."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(got - ref)) / (den if den > 0 else 1.0))


def row_err(got, ref) -> float:
    """Largest relative error of one row of a matrix (rows much smaller than the largest row are measured
    against ROW_FLOOR times the largest row's norm)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.ndim != 2 or ref.size == 0:
        return rel_err(got, ref)
    norms = np.linalg.norm(ref, axis=1)
    if not norms.max() > 0:  # an all-zero reference (d = 1: every reflection is -1): absolute deviation
        return float(np.max(np.linalg.norm(got - ref, axis=1)))
    den = np.maximum(norms, ROW_FLOOR * float(norms.max()))
    return float(np.max(np.linalg.norm(got - ref, axis=1) / den))


def assert_close(got, ref, what="", rows=False) -> None:
    """The parity bar: relative Frobenius error, largest single deviation and (rows=True) every row."""
    got = np.asarray(got)
    ref = np.asarray(ref)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), (what, "non-finite values")
    fro, mx = rel_err(got, ref), max_err(got, ref)
    assert fro <= REL_TOL, (what, "relative Frobenius error", fro)
    assert mx <= MAX_TOL, (what, "largest deviation / largest entry", mx)
    if rows:
        rw = row_err(got, ref)
        assert rw <= ROW_TOL, (what, "worst row's relative error", rw)


def to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_fasth(V, X, G, k, transpose=False):
    """Run fasth_forward + fasth_backward through the C ABI; returns numpy A, dV, dX."""
    import torch
    from paper_2009_13977_amd import binding as B
    n, d = V.shape
    m = X.shape[1]
    Vd, Xd, Gd = to_gpu(V), to_gpu(X), to_gpu(G)
    A = torch.empty_like(Xd); dX = torch.empty_like(Xd); dV = torch.empty_like(Vd)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))
    B.fasth_forward(Vd, Xd, A, ws, k, transpose)
    B.fasth_backward(Vd, Gd, dV, dX, ws, k, transpose)
    torch.cuda.synchronize()
    return A.cpu().numpy(), dV.cpu().numpy(), dX.cpu().numpy()


def gpu_sequential(V, X, G, transpose=False):
    import torch
    from paper_2009_13977_amd import binding as B
    n, d = V.shape
    m = X.shape[1]
    Vd, Xd, Gd = to_gpu(V), to_gpu(X), to_gpu(G)
    A = torch.empty_like(Xd); dX = torch.empty_like(Xd); dV = torch.empty_like(Vd)
    ws = B.new_workspace(B.fasth_sequential_workspace_bytes(d, n, m))
    B.fasth_sequential_forward(Vd, Xd, A, transpose)
    B.fasth_sequential_backward(Vd, A, Gd, dV, dX, ws, transpose)
    torch.cuda.synchronize()
    return A.cpu().numpy(), dV.cpu().numpy(), dX.cpu().numpy()


def gpu_svd_layer(Uv, sigma, Vv, X, G, k, inverse=False):
    import torch
    from paper_2009_13977_amd import binding as B
    n, d = Uv.shape
    m = X.shape[1]
    Ud, sd, Vd, Xd, Gd = (to_gpu(a) for a in (Uv, sigma, Vv, X, G))
    Y = torch.empty_like(Xd); dX = torch.empty_like(Xd)
    dU = torch.empty_like(Ud); dVv = torch.empty_like(Vd); ds = torch.empty_like(sd)
    ws = B.new_workspace(B.svd_layer_workspace_bytes(d, n, m, k))
    if inverse:
        B.svd_layer_inverse_apply(Ud, sd, Vd, Xd, Y, ws, k)
        B.svd_layer_inverse_apply_backward(Ud, sd, Vd, Gd, dU, ds, dVv, dX, ws, k)
    else:
        B.svd_layer_apply(Ud, sd, Vd, Xd, Y, ws, k)
        B.svd_layer_apply_backward(Ud, sd, Vd, Gd, dU, ds, dVv, dX, ws, k)
    torch.cuda.synchronize()
    return tuple(t.cpu().numpy() for t in (Y, dU, ds, dVv, dX))


def gpu_svd_sym(Uv, sigma, X, G, k, function="identity"):
    import torch
    from paper_2009_13977_amd import binding as B
    n, d = Uv.shape
    m = X.shape[1]
    Ud, sd, Xd, Gd = (to_gpu(a) for a in (Uv, sigma, X, G))
    Y = torch.empty_like(Xd); dX = torch.empty_like(Xd); dU = torch.empty_like(Ud); ds = torch.empty_like(sd)
    ws = B.new_workspace(B.svd_layer_workspace_bytes(d, n, m, k))
    B.svd_sym_apply(Ud, sd, Xd, Y, ws, k, function)
    B.svd_sym_apply_backward(Ud, sd, Gd, dU, ds, dX, ws, k, function)
    torch.cuda.synchronize()
    return tuple(t.cpu().numpy() for t in (Y, dU, ds, dX))


def gpu_svd_rect(Uv, sigma, Vv, X, G, k):
    import torch
    from paper_2009_13977_amd import binding as B
    (n_u, rows), (n_v, cols), m = Uv.shape, Vv.shape, X.shape[1]
    Ud, sd, Vd, Xd, Gd = (to_gpu(a) for a in (Uv, sigma, Vv, X, G))
    Y = torch.empty_like(Gd); dX = torch.empty_like(Xd)
    dU = torch.empty_like(Ud); dVv = torch.empty_like(Vd); ds = torch.empty_like(sd)
    ws = B.new_workspace(B.svd_rect_workspace_bytes(rows, cols, n_u, n_v, m, k))
    B.svd_rect_apply(Ud, sd, Vd, Xd, Y, ws, k)
    B.svd_rect_apply_backward(Ud, sd, Vd, Gd, dU, ds, dVv, dX, ws, k)
    torch.cuda.synchronize()
    return tuple(t.cpu().numpy() for t in (Y, dU, ds, dVv, dX))
