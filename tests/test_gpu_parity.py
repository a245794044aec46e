"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU checker on the same
seeded inputs. Bar: relative Frobenius error <= 1e-4 for every output (fp32 kernels vs fp64)."""
import sys

import numpy as np
import pytest

from oracle import householder as orc
from paper_2009_13977_amd import synthetic
from helpers import REL_TOL, assert_close, gpu_fasth, gpu_sequential, gpu_svd_layer, gpu_svd_rect, gpu_svd_sym, rel_err

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


# (d, n, m, k): small cases the checker finishes in well under a second. They span several 16-wide
# matrix-core tiles, ragged tails in every dimension, k = 1, one single block, m = 1 and n != d.
SMALL = [
    (64, 64, 32, 32),
    (256, 256, 32, 32),
    (100, 60, 5, 12),
    (33, 16, 1, 16),
    (130, 128, 7, 128),
    (64, 64, 32, 1),
    (257, 96, 3, 48),
    (70, 70, 33, 70),
    (48, 80, 9, 20),
    (300, 300, 40, 100),
    (1, 4, 3, 2),
]


@pytest.mark.parametrize("transpose", [False, True])
@pytest.mark.parametrize("d,n,m,k", SMALL)
def test_fasth_small_cases(d, n, m, k, transpose):
    _say(f"fasth small d={d} n={n} m={m} k={k} transpose={transpose}")
    p = synthetic.householder_problem(d, n, m, seed=1000 + d + n + m + k)
    A, dV, dX = gpu_fasth(p["V"], p["X"], p["G"], k, transpose)
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"], transpose=transpose)
    assert_close(A, A0, "A")
    assert_close(dX, dX0, "dX")
    assert_close(dV, dV0, "dV", rows=True)


# One case per chain-kernel variant the launcher can pick: blocks held in registers and applied whole or
# as steps of 8, 16 or 32 rows (with a short last step when k is not a multiple of the step), at every
# workgroup size including shapes that leave whole waves without work, vector lengths that are not a
# multiple of 4 (rows not 16-byte aligned, last chunk hanging over the row's end), and the general
# kernel for very long vectors. Few reflections and columns keep the checker fast.
DISPATCH = [
    (1024, 32, 3, 16), (2048, 32, 3, 16),
    (256, 64, 3, 32), (512, 64, 3, 32), (1024, 96, 3, 32), (2048, 64, 3, 32), (1500, 64, 3, 32),
    (256, 128, 3, 64), (512, 128, 3, 64), (1024, 128, 3, 64), (1000, 128, 2, 64),
    (1024, 256, 3, 128), (2048, 128, 2, 64), (4096, 64, 2, 32), (3000, 48, 2, 24),
    (2046, 32, 2, 32), (1022, 40, 2, 8), (1023, 32, 2, 16), (777, 21, 2, 7),
    (4100, 32, 2, 16), (5001, 16, 2, 8),
    (3072, 64, 3, 32), (2304, 48, 2, 24), (4096, 56, 2, 28), (4096, 256, 1, 128), (2052, 10, 2, 5),
    (1024, 56, 3, 28), (784, 112, 2, 56), (1024, 36, 2, 12), (1024, 15, 2, 5), (1024, 40, 2, 8),
    (2048, 40, 2, 8), (2048, 20, 2, 5), (1536, 72, 2, 24), (1280, 200, 2, 100),
    (512, 256, 3, 128), (256, 256, 2, 128), (256, 48, 3, 16), (512, 48, 3, 16), (200, 40, 3, 8), (400, 40, 3, 8),
    (2046, 14, 2, 7), (9000, 16, 2, 8), (12290, 8, 1, 8),
    # blocks of 32 / 64 / 128 rows, d a multiple of 4 up to 1024: 2, 4 or 8 waves per column, lane pairs; chains of one to five steps
    (1024, 32, 4, 32), (1024, 64, 3, 32), (516, 96, 2, 32), (1000, 160, 33, 32), (768, 128, 5, 64), (1024, 256, 3, 128),
    (640, 128, 200, 128), (512, 128, 9, 64), (260, 64, 7, 32), (384, 96, 2, 32), (8, 32, 3, 32), (132, 256, 40, 128),
    (512, 64, 300, 32), (256, 128, 700, 64), (384, 128, 1024, 128),  # the same with several workgroups per compute unit
    (1024, 64, 200, 32), (1000, 128, 180, 64), (1024, 128, 256, 128),  # d > 896, 177 .. 256 columns: four waves, 32-row steps
    # the lane-pair kernel with a short last step per block (17 <= k <= 127, not 32 or 64)
    (784, 56, 4, 28), (1000, 200, 3, 100), (512, 192, 5, 96), (300, 40, 3, 20), (1024, 66, 2, 33), (640, 126, 2, 63),
    (256, 34, 300, 17), (1024, 127, 2, 127), (512, 80, 3, 40), (768, 160, 2, 80),
    # the same block sizes where the 4-wave kernel serves (d > 896 from 177 columns, d > 512 from 257)
    (1024, 160, 200, 80), (1024, 56, 200, 28), (640, 80, 300, 40), (1000, 200, 180, 100),
    # the lane-pair kernel with rows that are not 16-byte aligned (d not a multiple of 4)
    (1023, 64, 3, 32), (1021, 100, 2, 50), (515, 96, 5, 32), (510, 128, 33, 128), (255, 60, 2, 20), (131, 64, 300, 64),
    (1022, 192, 2, 96), (769, 34, 7, 17),
    (1023, 64, 200, 32), (701, 40, 300, 20),  # ... where the 4-wave kernel serves such rows
]


@pytest.mark.parametrize("transpose", [False, True])
@pytest.mark.parametrize("d,n,m,k", DISPATCH)
def test_fasth_every_chain_kernel(d, n, m, k, transpose):
    _say(f"fasth dispatch d={d} n={n} m={m} k={k} transpose={transpose}")
    p = synthetic.householder_problem(d, n, m, seed=4000 + d + n + m + k)
    A, dV, dX = gpu_fasth(p["V"], p["X"], p["G"], k, transpose)
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"], transpose=transpose)
    assert_close(A, A0, "A")
    assert_close(dX, dX0, "dX")
    assert_close(dV, dV0, "dV", rows=True)


# Wide mini-batches (more than 1024 columns) take the matrix-core chain kernel: 16 columns per workgroup, rows in
# steps of 16. Cases: every groups-per-wave variant (d <= 256, 512, 768, 1024; 1536, 2048), d and m with ragged tails, blocks
# of one and of several steps, n != d; few reflections keep the checker fast.
WIDE = [
    (256, 64, 1040, 32), (512, 32, 1030, 16), (768, 96, 1026, 48), (1024, 64, 1036, 32), (1000, 128, 1100, 64),
    (100, 32, 1025, 16), (320, 256, 1056, 128),
    (2048, 32, 1036, 16), (1500, 48, 1026, 48), (1280, 64, 1040, 64),  # 8 waves per workgroup
    (125, 128, 800, 64), (125, 256, 800, 128),  # odd d: per-column chain in rounds, dV with 4-byte fetches reading Z
    # more columns than compute units, fewer than the matrix-core kernel takes: 16-row steps, several workgroups per unit
    (1024, 64, 300, 32), (768, 128, 260, 64), (1024, 128, 780, 128), (1024, 32, 1024, 32), (516, 96, 770, 32),
    # 449 .. 1024 columns at 512 < d <= 1024 (897 .. 2048 at 256 < d <= 512, 640 .. 1024 at 1024 < d <= 2048) with blocks of
    # 32 (an even number where d <= 1024), 64 or 128: tiles of 16 columns on the matrix cores, each shared by two to four workgroups; other block sizes from 769
    # columns on (608 at d > 896): four columns per workgroup on the matrix cores;
    # one and several steps per block, ragged d and m, n != d; and neighbours that stay with the per-column kernels
    (1024, 64, 800, 32), (1000, 128, 771, 64), (640, 256, 1023, 128), (900, 64, 610, 32), (516, 64, 1024, 32),
    (1024, 96, 900, 96), (768, 64, 768, 32), (1024, 64, 607, 32),
    # the shared tiles again: the fewest and the most columns, two, three and four parts, a last part of 4 and of 44
    # elements, one to four steps, two steps per block of 128, a ragged last tile
    (1024, 128, 449, 32), (1024, 256, 1024, 64), (512, 128, 2048, 32), (300, 64, 1000, 64), (512, 256, 897, 128),
    (1020, 192, 500, 64), (768, 64, 1280, 32), (600, 128, 999, 128), (1024, 64, 448, 32),
    # columns of 1025 .. 2048 elements: parts of 512, steps of 32 rows (one, two and four per block), three and four
    # parts, a last part of 4 elements, the fewest and the most columns
    (2048, 64, 640, 32), (1536, 128, 1024, 64), (1028, 256, 700, 128), (2044, 96, 1000, 32), (1280, 64, 639, 64),
]


@pytest.mark.parametrize("transpose", [False, True])
@pytest.mark.parametrize("d,n,m,k", WIDE)
def test_fasth_wide_minibatch(d, n, m, k, transpose):
    _say(f"fasth wide d={d} n={n} m={m} k={k} transpose={transpose}")
    p = synthetic.householder_problem(d, n, m, seed=5000 + d + n + m + k)
    A, dV, dX = gpu_fasth(p["V"], p["X"], p["G"], k, transpose)
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"], transpose=transpose)
    assert_close(A, A0, "A")
    assert_close(dX, dX0, "dX")
    assert_close(dV, dV0, "dV", rows=True)


# Few columns of 513 .. 4096 elements are shared by workgroups that hand each other every step's partial inner products
# through the workspace. A team of 2 to 8 workgroups with steps of 64 rows (blocks of 32 merged in pairs, of 64, of
# 128 as two steps) while every workgroup has a compute unit of its own: the three block sizes over the team sizes,
# parts that are full, nearly empty (d = 516, 1028, 2052) and ragged, one column, the most columns a team size takes, n != d;
# steps of 128 rows (two blocks of 64 joined through the product of their rows) where d is 513 .. 2048 and n a multiple
# of 128: one to five steps (the kernel's loop takes three at a time), 4 to 8 parts, full, ragged and nearly empty
# last parts, the most columns;
# two workgroups per column with steps of 32 rows beyond that (d > 1024, up to 128 columns); and neighbours that stay
# with one workgroup per column (an odd number of blocks of 32, a block size with a short last step, 129 columns).
SHARED = [
    (1024, 128, 8, 32), (1024, 128, 5, 64), (1024, 256, 3, 128), (600, 64, 128, 32), (516, 64, 2, 64), (768, 128, 1, 128),
    (1280, 64, 5, 32), (1536, 64, 1, 64), (1028, 128, 8, 64), (1540, 192, 80, 64), (1300, 128, 85, 128),
    (2048, 128, 13, 32), (2048, 256, 64, 128), (1544, 128, 33, 64),
    (2560, 128, 5, 32), (3072, 128, 42, 64), (4096, 256, 32, 128), (3600, 64, 3, 32), (2052, 128, 7, 64), (4096, 64, 33, 32),
    (2044, 96, 128, 32), (2048, 128, 65, 64), (1032, 256, 100, 128),
    (1024, 96, 7, 32), (2048, 64, 129, 32), (2048, 96, 16, 48),
    (1024, 256, 32, 32), (772, 128, 3, 32), (1792, 384, 9, 64), (2048, 512, 32, 128), (1280, 640, 2, 32), (900, 128, 64, 32),
    (1024, 384, 64, 64), (2048, 256, 1, 32), (1284, 256, 40, 128), (1000, 512, 7, 64),
]


@pytest.mark.parametrize("transpose", [False, True])
@pytest.mark.parametrize("d,n,m,k", SHARED)
def test_fasth_shared_columns(d, n, m, k, transpose):
    from paper_2009_13977_amd import binding as B
    _say(f"fasth shared columns d={d} n={n} m={m} k={k} transpose={transpose}")
    p = synthetic.householder_problem(d, n, m, seed=6000 + d + n + m + k)
    A, dV, dX = gpu_fasth(p["V"], p["X"], p["G"], k, transpose)
    assert B.fasth_wait_status() == B.FASTH_OK
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"], transpose=transpose)
    assert_close(A, A0, "A")
    assert_close(dX, dX0, "dX")
    assert_close(dV, dV0, "dV", rows=True)


@pytest.mark.parametrize("d,n,m,k", [(2048, 64, 16, 32), (1024, 256, 16, 32), (768, 128, 500, 64)])  # steps of 64 rows, of 128; shared tiles
def test_shared_columns_wait_gives_up_and_recovers(d, n, m, k):
    """A wait between the workgroups of a column that runs out of polls ends the kernel normally and raises the
    status word; the next call with the ordinary limit is correct again. The limit is forced to zero from the host,
    so the very first unsuccessful poll gives up: nothing on the GPU hangs or faults."""
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    _say(f"shared columns: wait limit 0, d={d} n={n} m={m} k={k}")
    p = synthetic.householder_problem(d, n, m, seed=6100)
    Vd, Xd, Gd = (to_gpu(p[a]) for a in ("V", "X", "G"))
    A = torch.empty_like(Xd); dX = torch.empty_like(Xd); dV = torch.empty_like(Vd)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))
    assert B.fasth_wait_status() == B.FASTH_OK
    B.fasth_set_wait_limit(0)
    try:
        B.fasth_forward(Vd, Xd, A, ws, k)
        assert B.fasth_wait_status() == B.FASTH_ETIMEOUT   # some workgroup saw its partner's word late
        assert B.fasth_wait_status() == B.FASTH_OK         # reading the status clears it
    finally:
        B.fasth_set_wait_limit(-1)
    _say("shared columns: default limit again")
    for _ in range(2):  # the second pass continues the tag counters of the first
        B.fasth_forward(Vd, Xd, A, ws, k)
        B.fasth_backward(Vd, Gd, dV, dX, ws, k)
    assert B.fasth_wait_status() == B.FASTH_OK
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"])
    assert_close(A.cpu().numpy(), A0, "A")
    assert_close(dX.cpu().numpy(), dX0, "dX")
    assert_close(dV.cpu().numpy(), dV0, "dV", rows=True)


@pytest.mark.parametrize("d,n,m,k", [(1024, 128, 8, 32), (2048, 128, 5, 64), (1536, 256, 3, 128), (2048, 64, 100, 32), (1024, 128, 450, 32)])
def test_shared_columns_captured_and_replayed(d, n, m, k):
    """Forward + backward captured into a HIP graph and replayed with new V, X and G each time, with eager work on the
    same workspace in between: the tags of the hand-offs count on in the workspace, the ready words of the factor
    kernel are cleared by their reader, and no replay may see anything of the one before."""
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    _say(f"shared columns under graph capture d={d} n={n} m={m} k={k}")
    probs = [synthetic.householder_problem(d, n, m, seed=6600 + r) for r in range(4)]
    Vd, Xd, Gd = (to_gpu(probs[0][a]) for a in ("V", "X", "G"))
    A = torch.empty_like(Xd); dX = torch.empty_like(Xd); dV = torch.empty_like(Vd)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # once eagerly: everything the library sets up on first use is done before capture
        B.fasth_forward(Vd, Xd, A, ws, k)
        B.fasth_backward(Vd, Gd, dV, dX, ws, k)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.fasth_forward(Vd, Xd, A, ws, k)
        B.fasth_backward(Vd, Gd, dV, dX, ws, k)
    for r in (1, 2, 3, 1):
        p = probs[r]
        Vd.copy_(to_gpu(p["V"])); Xd.copy_(to_gpu(p["X"])); Gd.copy_(to_gpu(p["G"]))
        graph.replay()
        torch.cuda.synchronize()
        assert B.fasth_wait_status() == B.FASTH_OK
        A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"])
        assert_close(A.cpu().numpy(), A0, f"A, replay with inputs {r}")
        assert_close(dX.cpu().numpy(), dX0, f"dX, replay with inputs {r}")
        assert_close(dV.cpu().numpy(), dV0, f"dV, replay with inputs {r}", rows=True)
        # eager work on the same workspace between replays (other inputs, transposed order)
        q = probs[0]
        A2, dV2, dX2 = gpu_fasth(q["V"], q["X"], q["G"], k, True)
        B.fasth_forward(to_gpu(q["V"]), to_gpu(q["X"]), torch.empty_like(Xd), ws, k, True)
        torch.cuda.synchronize()


def test_shared_columns_in_the_layers():
    """The SVD layer, a symmetric form (one set of factors serving two products) and the rectangular layer at sizes
    whose chains run two workgroups per column; prepared factors applied repeatedly."""
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    _say("shared columns: svd layer d=1536")
    p = synthetic.svd_layer_problem(1536, 64, 8, seed=6200)
    for inverse in (False, True):
        got = gpu_svd_layer(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], 32, inverse)
        fn = orc.svd_layer_inverse_gradients if inverse else orc.svd_layer_gradients
        for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got, fn(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])):
            assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))
    _say("shared columns: symmetric form d=1280")
    rng = np.random.default_rng(6300)
    Uv = rng.standard_normal((64, 1280)).astype(np.float32)
    sigma = rng.uniform(-0.8, 0.9, 1280).astype(np.float32)
    X = rng.standard_normal((1280, 6)).astype(np.float32)
    G = rng.standard_normal((1280, 6)).astype(np.float32)
    for name, g, r in zip(("Y", "dUv", "dsigma", "dX"), gpu_svd_sym(Uv, sigma, X, G, 32, "exp"),
                          orc.symmetric_gradients(Uv, sigma, X, G, "exp")):
        assert_close(g, r, name, rows=name == "dUv")
    _say("shared columns: rectangular layer 2048 x 1100")
    p = synthetic.rect_layer_problem(2048, 1100, 64, 32, 7, seed=6400)
    got = gpu_svd_rect(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], 32)
    for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got,
                          orc.rectangular_gradients(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])):
        assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))
    _say("shared columns, steps of 128 rows: svd layer d=1024")
    p = synthetic.svd_layer_problem(1024, 256, 6, seed=6210)
    for inverse in (False, True):
        got = gpu_svd_layer(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], 32, inverse)
        fn = orc.svd_layer_inverse_gradients if inverse else orc.svd_layer_gradients
        for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got, fn(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])):
            assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))
    _say("shared columns, steps of 128 rows: symmetric form d=1100")
    rng = np.random.default_rng(6310)
    Uv = rng.standard_normal((128, 1100)).astype(np.float32)
    sigma = rng.uniform(-0.8, 0.9, 1100).astype(np.float32)
    X = rng.standard_normal((1100, 5)).astype(np.float32)
    G = rng.standard_normal((1100, 5)).astype(np.float32)
    for name, g, r in zip(("Y", "dUv", "dsigma", "dX"), gpu_svd_sym(Uv, sigma, X, G, 64, "exp"),
                          orc.symmetric_gradients(Uv, sigma, X, G, "exp")):
        assert_close(g, r, name, rows=name == "dUv")
    _say("shared columns, steps of 128 rows: rectangular layer 1024 x 900")
    p = synthetic.rect_layer_problem(1024, 900, 128, 128, 5, seed=6410)
    got = gpu_svd_rect(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], 32)
    for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got,
                          orc.rectangular_gradients(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])):
        assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))
    _say("shared tiles of 16 columns: svd layer d=768, 512 columns")
    p = synthetic.svd_layer_problem(768, 128, 512, seed=6220)
    for inverse in (False, True):
        got = gpu_svd_layer(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], 64, inverse)
        fn = orc.svd_layer_inverse_gradients if inverse else orc.svd_layer_gradients
        for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got, fn(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])):
            assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))
    _say("shared tiles of 16 columns: rectangular layer 1024 x 600, 460 columns")
    p = synthetic.rect_layer_problem(1024, 600, 128, 64, 460, seed=6420)
    got = gpu_svd_rect(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], 32)
    for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got,
                          orc.rectangular_gradients(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])):
        assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))
    _say("shared columns: prepared factors")
    d, n, m, k = 2048, 64, 24, 32
    p = synthetic.householder_problem(d, n, m, seed=6500)
    Vd, Xd = to_gpu(p["V"]), to_gpu(p["X"])
    Y1 = torch.empty_like(Xd); Y2 = torch.empty_like(Xd)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))
    B.fasth_prepare(Vd, m, ws, k)
    for _ in range(3):
        B.fasth_apply(Vd, Xd, Y1, ws, k)
        B.fasth_apply(Vd, Y1, Y2, ws, k, transpose=True)
    assert B.fasth_wait_status() == B.FASTH_OK
    assert_close(Y1.cpu().numpy(), orc.product_apply(p["V"], p["X"]), "H X")
    assert_close(Y2.cpu().numpy(), p["X"].astype(np.float64), "H^T H X")
    for (d, n, m, k) in ((1000, 192, 470, 64), (2048, 96, 650, 32)):
        _say(f"shared tiles of 16 columns: prepared factors d={d} m={m}")
        p = synthetic.householder_problem(d, n, m, seed=6520 + d)
        Vd, Xd = to_gpu(p["V"]), to_gpu(p["X"])
        Y1 = torch.empty_like(Xd); Y2 = torch.empty_like(Xd)
        ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))
        B.fasth_prepare(Vd, m, ws, k)
        for _ in range(2):
            B.fasth_apply(Vd, Xd, Y1, ws, k)
            B.fasth_apply(Vd, Y1, Y2, ws, k, transpose=True)
        assert B.fasth_wait_status() == B.FASTH_OK
        assert_close(Y1.cpu().numpy(), orc.product_apply(p["V"], p["X"]), "H X")
        assert_close(Y2.cpu().numpy(), p["X"].astype(np.float64), "H^T H X")
    _say("shared columns, steps of 128 rows: prepared factors")
    d, n, m, k = 1536, 384, 20, 64
    p = synthetic.householder_problem(d, n, m, seed=6510)
    Vd, Xd = to_gpu(p["V"]), to_gpu(p["X"])
    Y1 = torch.empty_like(Xd); Y2 = torch.empty_like(Xd)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))
    B.fasth_prepare(Vd, m, ws, k)
    for _ in range(3):
        B.fasth_apply(Vd, Xd, Y1, ws, k)
        B.fasth_apply(Vd, Y1, Y2, ws, k, transpose=True)
    assert B.fasth_wait_status() == B.FASTH_OK
    assert_close(Y1.cpu().numpy(), orc.product_apply(p["V"], p["X"]), "H X")
    assert_close(Y2.cpu().numpy(), p["X"].astype(np.float64), "H^T H X")


def test_fasth_wide_benchmark_config():
    """The wide workload at full size (4096 columns) against the checker on every output."""
    name = "d1024_m4096_k32"
    w = synthetic.WORKLOADS[name]
    _say(f"fasth config {name}")
    p = synthetic.workload_inputs(name)
    A, dV, dX = gpu_fasth(p["V"], p["X"], p["G"], w.k)
    _say("  checker")
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"])
    errs = (rel_err(A, A0), rel_err(dV, dV0), rel_err(dX, dX0))
    _say(f"  rel errors A/dV/dX: {errs}")
    assert_close(A, A0, "A")
    assert_close(dV, dV0, "dV", rows=True)
    assert_close(dX, dX0, "dX")


def test_fasth_widest_benchmark_config():
    """The 16384-column workload at full size, in the launch configuration the benchmark times (its saved block
    inputs come to 2 GiB per chain, the limit of the kernels' 32-bit byte offsets). The checker would need minutes
    for all columns, so it computes sampled outputs one by one: columns of A and dX are independent of each other,
    and with G zero outside a sample of columns dV is the sum of those columns' Eq. 5 terms alone (every term
    carries a factor from its column of G). The sample holds the first and last columns, the neighbours of 16-column
    tile boundaries and random ones."""
    name = "d1024_m16384_k32"
    w = synthetic.WORKLOADS[name]
    _say(f"fasth config {name}")
    p = synthetic.workload_inputs(name)
    rng = np.random.default_rng(20261128)
    cols = np.unique(np.concatenate([np.arange(4), np.arange(w.m - 4, w.m), [15, 16, 17, 8191, 8192, 16367, 16368],
                                     rng.choice(w.m, size=40, replace=False)]))
    A, dV, dX = gpu_fasth(p["V"], p["X"], p["G"], w.k)
    _say("  properties that hold at any size")
    nx, ng = np.linalg.norm(p["X"].astype(np.float64)), np.linalg.norm(p["G"].astype(np.float64))
    assert abs(np.linalg.norm(A.astype(np.float64)) - nx) <= 1e-5 * nx       # H is orthogonal
    assert abs(np.linalg.norm(dX.astype(np.float64)) - ng) <= 1e-5 * ng
    lhs = float(np.sum(p["G"].astype(np.float64) * A)); rhs = float(np.sum(dX.astype(np.float64) * p["X"]))
    assert abs(lhs - rhs) <= 1e-5 * nx * ng                                  # <G, H X> = <H^T G, X>
    row = np.abs(np.sum(dV.astype(np.float64) * p["V"], axis=1))
    assert np.max(row / (np.linalg.norm(dV, axis=1) * np.linalg.norm(p["V"], axis=1))) < 1e-5  # grad v_j is orthogonal to v_j
    _say(f"  checker on {len(cols)} sampled columns of A and dX")
    assert_close(A[:, cols], orc.product_apply(p["V"], p["X"][:, cols]), "A[:, sample]")
    assert_close(dX[:, cols], orc.product_apply(p["V"], p["G"][:, cols], transpose=True), "dX[:, sample]")
    _say("  dV with G zero outside the sample")
    Gs = np.zeros_like(p["G"])
    Gs[:, cols] = p["G"][:, cols]
    _, dVs, dXs = gpu_fasth(p["V"], p["X"], Gs, w.k)
    _, dV0, dX0 = orc.product_gradients(p["V"], p["X"][:, cols], p["G"][:, cols])
    assert_close(dVs, dV0, "dV", rows=True)
    assert_close(dXs[:, cols], dX0, "dX[:, sample]")
    other = np.setdiff1d(np.arange(w.m), cols)
    assert not dXs[:, other].any()


def test_layers_wide_minibatch():
    """The layers on the matrix-core chain kernel: the diagonal factor fused into its input fetch (every mode),
    a rectangular Sigma (rows of the chain's input that do not exist), and the gradient of sigma from a launch of
    its own."""
    d, n, m, k = 256, 128, 1040, 64  # k >= 64, k m >= 32768: the dV kernel reads Z formed by a launch of its own
    p = synthetic.svd_layer_problem(d, n, m, seed=5100)
    for inverse in (False, True):
        _say(f"svd layer wide inverse={inverse}")
        got = gpu_svd_layer(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], k, inverse)
        fn = orc.svd_layer_inverse_gradients if inverse else orc.svd_layer_gradients
        ref = fn(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])
        for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got, ref):
            assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))
    rng = np.random.default_rng(5200)
    sigma = rng.uniform(-0.8, 0.9, d).astype(np.float32)
    for function in ("exp", "cayley"):
        _say(f"svd sym wide f={function}")
        got = gpu_svd_sym(p["Uv"], sigma, p["X"], p["G"], k, function)
        ref = orc.symmetric_gradients(p["Uv"], sigma, p["X"], p["G"], function)
        for name, g, r in zip(("Y", "dUv", "dsigma", "dX"), got, ref):
            assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))
    # (2048, 64): the two factors differ in how the dV mini-batch is split, so their dV launches stay separate
    for rows, cols in ((256, 192), (192, 256), (2048, 64)):
        _say(f"svd rect wide rows={rows} cols={cols}")
        q = synthetic.rect_layer_problem(rows, cols, 32 if rows < 2048 else 128, 32, 1040, seed=5300 + rows)
        got = gpu_svd_rect(q["Uv"], q["sigma"], q["Vv"], q["X"], q["G"], 16)  # k m < 32768: Z rebuilt per workgroup
        ref = orc.rectangular_gradients(q["Uv"], q["sigma"], q["Vv"], q["X"], q["G"])
        for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got, ref):
            assert g.shape == r.shape, name
            assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))


def _random_shapes(count, seed):
    """Seeded shapes over the whole supported range: any d (multiples of 4 and not), block sizes that do and do not
    divide into 8/16/32-row steps, narrow and wide mini-batches, n != d. Few reflections keep the checker fast."""
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(count):
        d = int(rng.choice([rng.integers(1, 64), rng.integers(64, 600), rng.integers(600, 2100), rng.integers(2100, 4200)]))
        if rng.random() < 0.7:
            d = max(4, d // 4 * 4)
        k = int(rng.choice([1, 2, 3, 5, 7, 8, 12, 16, 20, 24, 28, 32, 40, 48, 56, 64, 96, 100, 128]))
        nb = int(rng.integers(1, 4))
        m = int(rng.choice([1, 2, 5, 16, 31, 32, 33, 64, 100, 1030, 1100])) if d <= 2100 else int(rng.choice([1, 3, 32, 40]))
        if m > 700 and d > 1100:
            nb = 1
        shapes.append((d, nb * k, m, k, bool(rng.integers(0, 2))))
    return shapes


@pytest.mark.parametrize("d,n,m,k,transpose", _random_shapes(48, seed=20260927))
def test_fasth_random_shapes(d, n, m, k, transpose):
    _say(f"fasth random d={d} n={n} m={m} k={k} transpose={transpose}")
    p = synthetic.householder_problem(d, n, m, seed=12000 + d + n + m + k)
    A, dV, dX = gpu_fasth(p["V"], p["X"], p["G"], k, transpose)
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"], transpose=transpose)
    assert_close(A, A0, "A")
    assert_close(dX, dX0, "dX")
    assert_close(dV, dV0, "dV", rows=True)


def _random_pair_shapes(count, seed):
    """Seeded shapes in the range of the lane-pair chain kernel: d a multiple of 4 up to 1024, 17 <= k <= 128
    (multiples of 32 and not), one to six blocks, narrow and crowded mini-batches."""
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(count):
        d = int(rng.integers(1, 257)) * 4
        k = int(rng.integers(17, 129))
        nb = int(rng.integers(1, 7))
        m = int(rng.choice([1, 2, 7, 32, 33, 100, 177, 256, 300]))
        if d * nb * k * m > 2e8:
            m = 7
        shapes.append((d, nb * k, m, k, bool(rng.integers(0, 2))))
    return shapes


@pytest.mark.parametrize("d,n,m,k,transpose", _random_pair_shapes(24, seed=20261128))
def test_fasth_random_shapes_lane_pairs(d, n, m, k, transpose):
    _say(f"fasth random (lane pairs) d={d} n={n} m={m} k={k} transpose={transpose}")
    p = synthetic.householder_problem(d, n, m, seed=13000 + d + n + m + k)
    A, dV, dX = gpu_fasth(p["V"], p["X"], p["G"], k, transpose)
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"], transpose=transpose)
    assert_close(A, A0, "A")
    assert_close(dX, dX0, "dX")
    assert_close(dV, dV0, "dV", rows=True)


@pytest.mark.parametrize("name", ["d64_m32_k32", "d256_m32_k32", "d1024_m32_k32",
                                  "d2048_m64_k32", "d2048_m64_k64", "d2048_m64_k128"])
def test_fasth_benchmark_configs(name):
    w = synthetic.WORKLOADS[name]
    _say(f"fasth config {name}")
    p = synthetic.workload_inputs(name)
    A, dV, dX = gpu_fasth(p["V"], p["X"], p["G"], w.k)
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"])
    errs = (rel_err(A, A0), rel_err(dV, dV0), rel_err(dX, dX0))
    _say(f"  rel errors A/dV/dX: {errs}")
    assert_close(A, A0, "A")
    assert_close(dV, dV0, "dV", rows=True)
    assert_close(dX, dX0, "dX")
    # properties that hold at any size
    assert abs(np.linalg.norm(A.astype(np.float64)) - np.linalg.norm(p["X"].astype(np.float64))) <= 1e-5 * np.linalg.norm(p["X"])
    # H does not depend on the length of v_j, so the gradient of v_j is orthogonal to it (follows from Eq. 1)
    row = np.abs(np.sum(dV.astype(np.float64) * p["V"], axis=1))
    scale = np.linalg.norm(dV, axis=1) * np.linalg.norm(p["V"], axis=1)
    assert np.max(row / scale) < 1e-5


def test_limits_of_the_supported_range():
    """Longest supported vector (generic chain kernel, 1024 threads x 16 elements), the largest block
    size, and a mini-batch wider than several LDS chunks of the dV kernel."""
    for (d, n, m, k) in [(16384, 16, 1, 16), (16384, 8, 2, 8), (200, 128, 3, 128), (64, 64, 100, 32), (48, 32, 257, 16)]:
        _say(f"limits d={d} n={n} m={m} k={k}")
        p = synthetic.householder_problem(d, n, m, seed=6000 + d + n + m + k)
        got = gpu_fasth(p["V"], p["X"], p["G"], k)
        ref = orc.product_gradients(p["V"], p["X"], p["G"])
        for name, g, r in zip(("A", "dV", "dX"), got, ref):
            assert_close(g, r, name, rows=name == "dV")


def test_workspace_reuse_and_repeated_backward():
    """One workspace serves calls of different shapes; backward may be called again with a new G."""
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    ws = B.new_workspace(B.fasth_workspace_bytes(256, 256, 32, 32))
    for (d, n, m, k) in [(256, 256, 32, 32), (100, 60, 5, 12), (256, 128, 16, 16)]:
        assert B.fasth_workspace_bytes(d, n, m, k) <= ws.numel()
        p = synthetic.householder_problem(d, n, m, seed=7000 + d)
        Vd, Xd = to_gpu(p["V"]), to_gpu(p["X"])
        A = torch.empty_like(Xd); dX = torch.empty_like(Xd); dV = torch.empty_like(Vd)
        B.fasth_forward(Vd, Xd, A, ws, k)
        for seed in (1, 2):
            G = np.random.default_rng(seed).standard_normal((d, m)).astype(np.float32)
            B.fasth_backward(Vd, to_gpu(G), dV, dX, ws, k)
            torch.cuda.synchronize()
            A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], G)
            assert_close(A.cpu().numpy(), A0, "A")
            assert_close(dV.cpu().numpy(), dV0, "dV", rows=True)
            assert_close(dX.cpu().numpy(), dX0, "dX")


def test_runs_on_a_side_stream():
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    p = synthetic.householder_problem(128, 128, 8, seed=11)
    Vd, Xd, Gd = (to_gpu(p[a]) for a in ("V", "X", "G"))
    A = torch.empty_like(Xd); dX = torch.empty_like(Xd); dV = torch.empty_like(Vd)
    ws = B.new_workspace(B.fasth_workspace_bytes(128, 128, 8, 32))
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        B.fasth_forward(Vd, Xd, A, ws, 32)
        B.fasth_backward(Vd, Gd, dV, dX, ws, 32)
    side.synchronize()
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"])
    assert_close(A.cpu().numpy(), A0, "A")
    assert_close(dV.cpu().numpy(), dV0, "dV", rows=True)
    assert_close(dX.cpu().numpy(), dX0, "dX")


def test_prepare_once_apply_many():
    """Section 3.3 "Recurrent Layers": the block factors are built once and the same H is applied
    r times (here H, then H^T, then H twice, then a saved apply followed by backward)."""
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    d = n = 256; m = 32; k = 32
    p = synthetic.householder_problem(d, n, m, seed=21)
    Vd, Xd, Gd = (to_gpu(p[a]) for a in ("V", "X", "G"))
    Y1 = torch.empty_like(Xd); Y2 = torch.empty_like(Xd); Y3 = torch.empty_like(Xd)
    dX = torch.empty_like(Xd); dV = torch.empty_like(Vd)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))
    B.fasth_prepare(Vd, m, ws, k)
    B.fasth_apply(Vd, Xd, Y1, ws, k)                      # H X
    B.fasth_apply(Vd, Y1, Y2, ws, k, transpose=True)      # H^T H X = X
    B.fasth_apply(Vd, Y1, Y3, ws, k)                      # H H X
    torch.cuda.synchronize()
    HX = orc.product_apply(p["V"], p["X"])
    assert rel_err(Y1.cpu().numpy(), HX) <= REL_TOL
    assert rel_err(Y2.cpu().numpy(), p["X"]) <= REL_TOL
    assert rel_err(Y3.cpu().numpy(), orc.product_apply(p["V"], HX)) <= REL_TOL
    B.fasth_apply(Vd, Xd, Y1, ws, k, save_for_backward=True)
    B.fasth_backward(Vd, Gd, dV, dX, ws, k)
    torch.cuda.synchronize()
    _, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"])
    assert_close(dV.cpu().numpy(), dV0, "dV", rows=True)
    assert_close(dX.cpu().numpy(), dX0, "dX")


@pytest.mark.parametrize("d,n,m,k,spread", [(256, 256, 32, 32, 3), (1024, 128, 8, 64, 4), (512, 64, 1040, 32, 3), (96, 96, 8, 48, 5)])
def test_row_scales_over_many_orders_of_magnitude(d, n, m, k, spread):
    """H_j does not depend on the length of v_j (Eq. 1), but the block factors are built from unnormalised vectors:
    rows scaled by 10^U(-spread, spread) must not cost accuracy. dV rows scale like 1/|v_j|, so they are compared
    after scaling back, which makes the short rows count."""
    _say(f"row scales d={d} n={n} m={m} k={k} spread=1e+-{spread}")
    p = synthetic.householder_problem(d, n, m, seed=99)
    scale = (10.0 ** np.random.default_rng(7).uniform(-spread, spread, n)).astype(np.float32)
    V = (p["V"] * scale[:, None]).astype(np.float32)
    A, dV, dX = gpu_fasth(V, p["X"], p["G"], k)
    A0, dV0, dX0 = orc.product_gradients(V, p["X"], p["G"])
    assert rel_err(A, A0) <= REL_TOL and rel_err(dX, dX0) <= REL_TOL
    assert rel_err(dV * scale[:, None], dV0 * scale[:, None]) <= REL_TOL


def test_nearly_parallel_vectors_within_a_block():
    """Three of every four vectors differ from their predecessor by a thousandth: the block's Gram matrix is close
    to singular while every reflection stays well defined."""
    d, n, m, k = 256, 64, 8, 32
    p = synthetic.householder_problem(d, n, m, seed=98)
    V = p["V"].copy()
    for j in range(1, n):
        if j % 4:
            V[j] = V[j - 1] + 1e-3 * V[j]
    got = gpu_fasth(V, p["X"], p["G"], k)
    ref = orc.product_gradients(V, p["X"], p["G"])
    for g, r in zip(got, ref):
        assert rel_err(g, r) <= REL_TOL


def test_block_size_independence():
    """Theorem 1 correctness: the result does not depend on how reflections are grouped."""
    p = synthetic.householder_problem(96, 96, 8, seed=77)
    ref = orc.product_gradients(p["V"], p["X"], p["G"])
    for k in (1, 2, 3, 8, 32, 48, 96):
        _say(f"block-size independence k={k}")
        got = gpu_fasth(p["V"], p["X"], p["G"], k)
        for g, r in zip(got, ref):
            assert rel_err(g, r) <= REL_TOL


@pytest.mark.parametrize("d,n,m,k", [(256, 256, 32, 32), (128, 64, 1040, 32), (1024, 64, 1040, 64), (1001, 48, 5, 24)])
def test_bitwise_repeatable(d, n, m, k):
    """Every sum runs in a fixed order (no atomics), also where the mini-batch is split over workgroups and on the
    matrix-core chain kernel: two runs give the same bits."""
    p = synthetic.householder_problem(d, n, m, seed=5)
    a = gpu_fasth(p["V"], p["X"], p["G"], k)
    b = gpu_fasth(p["V"], p["X"], p["G"], k)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_prepare_once_apply_many_wide():
    """The same on the matrix-core chain kernel (4096 columns): factors once, H then H^T gives X back."""
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    d, n, m, k = 512, 64, 4096, 32
    p = synthetic.householder_problem(d, n, m, seed=22)
    Vd, Xd = to_gpu(p["V"]), to_gpu(p["X"])
    Y1 = torch.empty_like(Xd); Y2 = torch.empty_like(Xd)
    ws = B.new_workspace(B.fasth_workspace_bytes(d, n, m, k))
    B.fasth_prepare(Vd, m, ws, k)
    B.fasth_apply(Vd, Xd, Y1, ws, k)
    B.fasth_apply(Vd, Y1, Y2, ws, k, transpose=True)
    torch.cuda.synchronize()
    assert rel_err(Y1.cpu().numpy(), orc.product_apply(p["V"], p["X"])) <= REL_TOL
    assert rel_err(Y2.cpu().numpy(), p["X"]) <= REL_TOL


@pytest.mark.parametrize("transpose", [False, True])
@pytest.mark.parametrize("d,n,m", [(64, 64, 32), (100, 60, 5), (300, 300, 3), (1024, 256, 4), (5000, 12, 2), (9000, 8, 2)])
def test_sequential_kernels(d, n, m, transpose):
    _say(f"sequential d={d} n={n} m={m} transpose={transpose}")
    p = synthetic.householder_problem(d, n, m, seed=2000 + d + n + m)
    A, dV, dX = gpu_sequential(p["V"], p["X"], p["G"], transpose)
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"], transpose=transpose)
    assert_close(A, A0, "A")
    assert_close(dX, dX0, "dX")
    assert_close(dV, dV0, "dV", rows=True)


@pytest.mark.parametrize("inverse", [False, True])
@pytest.mark.parametrize("d,n,m,k", [(64, 64, 32, 32), (100, 60, 5, 12), (256, 256, 32, 32)])
def test_svd_layer_small(d, n, m, k, inverse):
    _say(f"svd layer d={d} n={n} m={m} k={k} inverse={inverse}")
    p = synthetic.svd_layer_problem(d, n, m, seed=3000 + d + n + m + k)
    got = gpu_svd_layer(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], k, inverse)
    fn = orc.svd_layer_inverse_gradients if inverse else orc.svd_layer_gradients
    ref = fn(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])
    for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got, ref):
        assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))


@pytest.mark.parametrize("inverse", [False, True])
def test_svd_layer_benchmark_config(inverse):
    name = "svd_d1024_m32_k32"
    w = synthetic.WORKLOADS[name]
    _say(f"svd layer config {name} inverse={inverse}")
    p = synthetic.workload_inputs(name)
    got = gpu_svd_layer(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], w.k, inverse)
    fn = orc.svd_layer_inverse_gradients if inverse else orc.svd_layer_gradients
    ref = fn(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])
    errs = {nm: rel_err(g, r) for nm, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got, ref)}
    _say(f"  rel errors: {errs}")
    assert max(errs.values()) <= REL_TOL


def _random_layer_shapes(count, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(count):
        d = int(rng.choice([rng.integers(4, 64), rng.integers(64, 600), rng.integers(600, 1500)]))
        if rng.random() < 0.7:
            d = max(4, d // 4 * 4)
        k = int(rng.choice([1, 3, 8, 12, 16, 24, 32, 48, 64]))
        nb = int(rng.integers(1, 3))
        m = int(rng.choice([1, 5, 32, 33, 100, 1040]))
        shapes.append((d, nb * k, m, k, bool(rng.integers(0, 2))))
    return shapes


@pytest.mark.parametrize("d,n,m,k,inverse", _random_layer_shapes(16, seed=20260928))
def test_svd_layer_random_shapes(d, n, m, k, inverse):
    """Every chain-kernel family under the layer: fused diagonal factor, gradient of sigma riding along or launched
    on its own, both factors' launches shared or separate."""
    _say(f"svd layer random d={d} n={n} m={m} k={k} inverse={inverse}")
    p = synthetic.svd_layer_problem(d, n, m, seed=13000 + d + n + m + k)
    got = gpu_svd_layer(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], k, inverse)
    fn = orc.svd_layer_inverse_gradients if inverse else orc.svd_layer_gradients
    ref = fn(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])
    for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got, ref):
        assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))


def test_svd_layer_inverse_round_trip():
    """Table 1: W^-1 (W X) = X."""
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    p = synthetic.svd_layer_problem(256, 256, 32, seed=9)
    Ud, sd, Vd, Xd = (to_gpu(p[a]) for a in ("Uv", "sigma", "Vv", "X"))
    Y = torch.empty_like(Xd); Xr = torch.empty_like(Xd)
    ws = B.new_workspace(B.svd_layer_workspace_bytes(256, 256, 32, 32))
    B.svd_layer_apply(Ud, sd, Vd, Xd, Y, ws, 32)
    B.svd_layer_inverse_apply(Ud, sd, Vd, Y, Xr, ws, 32)
    torch.cuda.synchronize()
    assert rel_err(Xr.cpu().numpy(), p["X"]) <= REL_TOL


@pytest.mark.parametrize("function", ["identity", "exp", "cayley"])
@pytest.mark.parametrize("d,n,m,k", [(64, 64, 32, 32), (100, 60, 5, 12), (256, 256, 32, 32), (1024, 1024, 32, 32)])
def test_symmetric_forms(d, n, m, k, function):
    """Table 1: U f(Sigma) U^T X for f = identity, exp, Cayley, with gradients wrt U (both uses), sigma, X."""
    _say(f"svd sym d={d} n={n} m={m} k={k} f={function}")
    rng = np.random.default_rng(8000 + d + n + m + k)
    Uv = rng.standard_normal((n, d)).astype(np.float32)
    sigma = rng.uniform(-0.8, 0.9, d).astype(np.float32)
    X = rng.standard_normal((d, m)).astype(np.float32)
    G = rng.standard_normal((d, m)).astype(np.float32)
    got = gpu_svd_sym(Uv, sigma, X, G, k, function)
    ref = orc.symmetric_gradients(Uv, sigma, X, G, function)
    for name, g, r in zip(("Y", "dUv", "dsigma", "dX"), got, ref):
        assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))


RECT = [  # rows, cols, n_u, n_v, m, k: both orientations, every family of chain kernel, ragged min(rows, cols)
    (64, 48, 64, 48, 8, 16), (96, 256, 96, 256, 32, 32), (1024, 512, 1024, 512, 32, 32),
    (512, 1024, 512, 1024, 32, 32), (100, 37, 60, 24, 5, 12), (3000, 1000, 64, 64, 3, 32),
    (1024, 510, 64, 64, 4, 32), (5001, 64, 24, 32, 2, 8), (7, 7, 7, 7, 1, 7),
]


@pytest.mark.parametrize("rows,cols,n_u,n_v,m,k", RECT)
def test_rectangular_layer(rows, cols, n_u, n_v, m, k):
    """Section 3.3 "Rectangular Matrices": W = U Sigma V^T with a rows x cols diagonal Sigma."""
    _say(f"svd rect rows={rows} cols={cols} n_u={n_u} n_v={n_v} m={m} k={k}")
    p = synthetic.rect_layer_problem(rows, cols, n_u, n_v, m, seed=11000 + rows + cols + m + k)
    got = gpu_svd_rect(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"], k)
    ref = orc.rectangular_gradients(p["Uv"], p["sigma"], p["Vv"], p["X"], p["G"])
    for name, g, r in zip(("Y", "dUv", "dsigma", "dVv", "dX"), got, ref):
        assert g.shape == r.shape, name
        assert_close(g, r, name, rows=name.startswith("d") and name.endswith("v"))


def test_log_abs_det():
    """Table 1: sum_i log|sigma_i| and its gradient."""
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    for d in (1, 7, 256, 1024, 5000):
        rng = np.random.default_rng(9000 + d)
        sigma = (rng.uniform(0.5, 2.0, d) * rng.choice([-1.0, 1.0], d)).astype(np.float32)
        sd = to_gpu(sigma)
        out = torch.zeros(4, dtype=torch.float32, device="cuda"); ds = torch.empty_like(sd)
        B.svd_layer_log_abs_det(sd, out, ds)
        torch.cuda.synchronize()
        ref = orc.log_abs_det(sigma)
        assert abs(float(out[0]) - ref) <= 1e-5 * max(1.0, abs(ref)) + 1e-4
        assert rel_err(ds.cpu().numpy(), 1.0 / sigma.astype(np.float64)) <= 1e-6


def test_block_size_search():
    """Section 3.3: the search tries the candidates once and returns the fastest; the paper's own
    example size d = 784 (all divisors of 784 up to 128)."""
    import time
    import torch
    from paper_2009_13977_amd import binding as B
    from helpers import to_gpu
    d = n = 784; m = 32
    p = synthetic.householder_problem(d, n, m, seed=31)
    Vd, Xd, Gd = (to_gpu(p[a]) for a in ("V", "X", "G"))
    A = torch.empty_like(Xd); dX = torch.empty_like(Xd); dV = torch.empty_like(Vd)
    divisors = [k for k in range(2, 129) if n % k == 0]
    ws = B.new_workspace(max(B.fasth_workspace_bytes(d, n, m, k) for k in divisors))
    t0 = time.perf_counter()
    k, ms = B.fasth_tune_block_size(Vd, Xd, Gd, A, dV, dX, ws, repetitions=3)
    elapsed = time.perf_counter() - t0
    _say(f"  block-size search at d=784: best k={k}, {ms * 1e3:.1f} us per pass, search took {elapsed:.3f} s")
    assert k in divisors and ms > 0
    A0, dV0, dX0 = orc.product_gradients(p["V"], p["X"], p["G"])
    assert_close(A.cpu().numpy(), A0, "A")
    assert_close(dV.cpu().numpy(), dV0, "dV", rows=True)
    assert_close(dX.cpu().numpy(), dX0, "dX")
    k2, _ = B.fasth_tune_block_size(Vd, Xd, Gd, A, dV, dX, ws, candidates=[5, 16, 28, 300], repetitions=2)
    assert k2 in (16, 28)
