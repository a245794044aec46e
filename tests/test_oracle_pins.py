"""Pins for the fp64 CPU checker: facts fixed by the paper or by mathematics,
none of them computed by re-calling the checker's own formulae.

Each test names the passage it pins. A plausible mistake in the checker (a
dropped term, a wrong sign, the wrong product order, input/output of a
reflection swapped, a transposed operand) fails at least one of them.
"""
import json
import os

import numpy as np
import pytest
import scipy.linalg

from oracle import householder as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _dense_reflection(v):
    v = np.asarray(v, dtype=np.float64)
    return np.eye(v.size) - 2.0 * np.outer(v, v) / (v @ v)


def _dense_product(V):
    """H_1 H_2 ... H_n by explicit d x d matrix products (independent route)."""
    d = V.shape[1]
    H = np.eye(d)
    for j in range(V.shape[0]):
        H = H @ _dense_reflection(V[j])
    return H


# ------------------------------------------------------------------ forward

def test_golden_two_reflections_exact_rationals():
    """Eq. 1 and the product order of Section 2.2, hand-worked rationals."""
    with open(os.path.join(GOLDEN, "two_reflections_3x3.json")) as f:
        gold = json.load(f)
    V = np.array([gold["v1"], gold["v2"]], dtype=np.float64)
    den = gold["denominator"]
    I = np.eye(3)
    np.testing.assert_allclose(orc.reflect(V[0], I) * den, gold["H1_times_9"], atol=1e-14)
    np.testing.assert_allclose(orc.reflect(V[1], I) * den, gold["H2_times_9"], atol=1e-14)
    np.testing.assert_allclose(orc.product_apply(V, I) * den, gold["H1H2_times_9"], atol=1e-14)
    # the two orders differ, so this also pins which end touches X first
    np.testing.assert_allclose(orc.product_apply(V[::-1], I) * den, gold["H2H1_times_9"], atol=1e-14)
    np.testing.assert_allclose(orc.product_apply(V, I, transpose=True) * den,
                               np.array(gold["H1H2_times_9"]).T, atol=1e-14)


@pytest.mark.parametrize("d,n", [(16, 16), (64, 64), (40, 17)])
def test_orthogonality_by_applying_to_identity(d, n):
    """Section 2.2: every product of Householder matrices is orthogonal."""
    V = _rng(1).standard_normal((n, d))
    H = orc.dense_matrix(V)
    assert np.max(np.abs(H.T @ H - np.eye(d))) < 1e-12
    assert np.max(np.abs(H @ H.T - np.eye(d))) < 1e-12


def test_norm_preserved_and_determinant_sign():
    V = _rng(2).standard_normal((13, 24))
    X = _rng(3).standard_normal((24, 7))
    A = orc.product_apply(V, X)
    assert abs(np.linalg.norm(A) - np.linalg.norm(X)) < 1e-12 * np.linalg.norm(X)
    # each reflection has determinant -1
    sign, logdet = np.linalg.slogdet(orc.dense_matrix(V))
    assert sign == (-1.0) ** 13 and abs(logdet) < 1e-12


def test_reflection_textbook_properties():
    """Eq. 1: H v = -v, H u = u for u orthogonal to v, H(c v) = H(v), H H = I."""
    r = _rng(4)
    v = r.standard_normal(9)
    u = r.standard_normal(9)
    u -= v * (u @ v) / (v @ v)
    np.testing.assert_allclose(orc.reflect(v, v[:, None])[:, 0], -v, atol=1e-14)
    np.testing.assert_allclose(orc.reflect(v, u[:, None])[:, 0], u, atol=1e-14)
    X = r.standard_normal((9, 4))
    np.testing.assert_allclose(orc.reflect(-3.7 * v, X), orc.reflect(v, X), atol=1e-14)
    np.testing.assert_allclose(orc.reflect(v, orc.reflect(v, X)), X, atol=1e-14)


@pytest.mark.parametrize("d", [2, 5, 16])
def test_matches_explicit_dense_product(d):
    """H X equals the explicitly multiplied d x d matrices times X (d <= 16)."""
    r = _rng(5 + d)
    V = r.standard_normal((d, d))
    X = r.standard_normal((d, 6))
    H = _dense_product(V)
    np.testing.assert_allclose(orc.product_apply(V, X), H @ X, atol=1e-13)
    np.testing.assert_allclose(orc.product_apply(V, X, transpose=True), H.T @ X, atol=1e-13)


def test_ordering_against_lapack_reflectors():
    """Section 2.2: any orthogonal matrix is a product of Householder matrices
    (QR). LAPACK's geqrf stores Q = H_1 H_2 ... with H_j = I - tau_j v_j v_j^T,
    tau_j = 2/||v_j||^2; feeding its reflectors must reproduce LAPACK's own Q.
    This pins H_1 as the LEFTMOST factor against a library."""
    d = 48
    M = _rng(6).standard_normal((d, d))
    (h, tau), _ = scipy.linalg.qr(M, mode="raw")
    Q, _ = scipy.linalg.qr(M, mode="full")
    V = np.zeros((d - 1, d))
    for j in range(d - 1):  # the d-th LAPACK reflector has tau = 0 (identity)
        V[j, j] = 1.0
        V[j, j + 1:] = h[j + 1:, j]
        assert abs(tau[j] - 2.0 / (V[j] @ V[j])) < 1e-12
    np.testing.assert_allclose(orc.dense_matrix(V), Q, atol=1e-13)


def test_special_cases():
    d = 8
    I = np.eye(d)
    # v_j = e_j for every j: each H_j flips one coordinate, H = -I
    np.testing.assert_allclose(orc.dense_matrix(I), -I, atol=0)
    v = _rng(7).standard_normal(d)
    # all vectors equal: H_j H_j = I, so an even count is the identity and an
    # odd count is one reflection
    np.testing.assert_allclose(orc.dense_matrix(np.tile(v, (6, 1))), I, atol=1e-14)
    np.testing.assert_allclose(orc.dense_matrix(np.tile(v, (5, 1))), _dense_reflection(v), atol=1e-14)
    with pytest.raises(ZeroDivisionError):
        orc.reflect(np.zeros(d), I)


# ---------------------------------------------------------------- gradients

def _loss(V, X, G, transpose=False):
    """L = <G, H X> evaluated through explicit dense matrices (not the checker)."""
    H = _dense_product(V)
    if transpose:
        H = H.T
    return float(np.sum(G * (H @ X)))


def _fd_grad_V(V, X, G, entries, h=1e-6, transpose=False):
    out = []
    for (j, i) in entries:
        Vp = V.copy(); Vp[j, i] += h
        Vm = V.copy(); Vm[j, i] -= h
        out.append((_loss(Vp, X, G, transpose) - _loss(Vm, X, G, transpose)) / (2 * h))
    return np.array(out)


def test_golden_single_vector_gradient():
    """Eq. 5, hand-worked 2-d case."""
    with open(os.path.join(GOLDEN, "single_vector_gradient_2d.json")) as f:
        gold = json.load(f)
    got = orc.vector_gradient(np.array(gold["v"], float), np.array(gold["a_in"], float),
                              np.array(gold["g_out"], float))
    np.testing.assert_allclose(got, gold["grad_v"], atol=1e-15)


@pytest.mark.parametrize("transpose", [False, True])
@pytest.mark.parametrize("d,n,m", [(6, 6, 3), (12, 12, 5), (16, 9, 4)])
def test_dV_against_central_differences_all_entries(d, n, m, transpose):
    """Eq. 5 (all three terms, their signs and factors) and the input/output
    roles of a and g: central differences of L in fp64 on every entry."""
    r = _rng(100 + d + n)
    V = r.standard_normal((n, d)); X = r.standard_normal((d, m)); G = r.standard_normal((d, m))
    _, dV, _ = orc.product_gradients(V, X, G, transpose=transpose)
    entries = [(j, i) for j in range(n) for i in range(d)]
    fd = _fd_grad_V(V, X, G, entries, transpose=transpose).reshape(n, d)
    assert np.linalg.norm(dV - fd) <= 1e-6 * np.linalg.norm(fd)
    assert np.max(np.abs(dV - fd)) <= 1e-6 * np.max(np.abs(fd))


def test_dV_against_central_differences_sampled_d64():
    r = _rng(8)
    d = n = 64; m = 8
    V = r.standard_normal((n, d)); X = r.standard_normal((d, m)); G = r.standard_normal((d, m))
    _, dV, _ = orc.product_gradients(V, X, G)
    entries = [(int(a), int(b)) for a, b in zip(r.integers(0, n, 40), r.integers(0, d, 40))]
    entries += [(0, 0), (n - 1, d - 1), (0, d - 1), (n - 1, 0)]
    fd = _fd_grad_V(V, X, G, entries)
    got = np.array([dV[j, i] for (j, i) in entries])
    assert np.max(np.abs(got - fd)) <= 1e-6 * np.max(np.abs(fd))


def test_dX_is_transposed_product_of_G():
    """Supplement 8.1: dL/dX = H_n^T ... H_1^T dL/dA_1; and dense H^T G."""
    r = _rng(9)
    d = n = 16; m = 5
    V = r.standard_normal((n, d)); X = r.standard_normal((d, m)); G = r.standard_normal((d, m))
    A, _, dX = orc.product_gradients(V, X, G)
    H = _dense_product(V)
    np.testing.assert_allclose(A, H @ X, atol=1e-13)
    np.testing.assert_allclose(dX, H.T @ G, atol=1e-13)
    _, _, dXt = orc.product_gradients(V, X, G, transpose=True)
    np.testing.assert_allclose(dXt, H @ G, atol=1e-13)


def test_dV_invariants():
    """H is homogeneous of degree 0 in each v_j (Eq. 1), hence v_j^T dL/dv_j = 0
    and scaling v_j by c scales its gradient by 1/c."""
    r = _rng(10)
    d = n = 20; m = 6
    V = r.standard_normal((n, d)); X = r.standard_normal((d, m)); G = r.standard_normal((d, m))
    _, dV, _ = orc.product_gradients(V, X, G)
    scale = np.linalg.norm(dV, axis=1) * np.linalg.norm(V, axis=1)
    assert np.max(np.abs(np.sum(V * dV, axis=1)) / scale) < 1e-12
    c = np.linspace(0.3, 2.9, n) * np.where(np.arange(n) % 2 == 0, 1.0, -1.0)
    _, dVc, _ = orc.product_gradients(V * c[:, None], X, G)
    np.testing.assert_allclose(dVc * c[:, None], dV, rtol=1e-11, atol=1e-13)


def test_reversible_walk_equals_stored_activations():
    """Eq. 4: recovering inputs by H_j^-1 = H_j^T gives the same gradients as
    keeping every intermediate."""
    r = _rng(11)
    d = n = 48; m = 7
    V = r.standard_normal((n, d)); X = r.standard_normal((d, m)); G = r.standard_normal((d, m))
    A1, dV1, dX1 = orc.product_gradients(V, X, G)
    A2, dV2, dX2 = orc.product_gradients_stored(V, X, G)
    np.testing.assert_allclose(A1, A2, atol=1e-12)
    np.testing.assert_allclose(dX1, dX2, atol=1e-12)
    assert np.linalg.norm(dV1 - dV2) <= 1e-12 * np.linalg.norm(dV2)


# ---------------------------------------------------------------- SVD layer

def _dense_layer(Uv, sigma, Vv):
    return _dense_product(Uv) @ np.diag(sigma) @ _dense_product(Vv).T


def test_svd_layer_against_dense_and_solve():
    """Section 2.2 W = U Sigma V^T; Table 1: W^-1 = V Sigma^-1 U^T and
    sum log|sigma_i| = log|det W|."""
    r = _rng(12)
    d = 12; m = 5
    Uv = r.standard_normal((d, d)); Vv = r.standard_normal((d, d))
    sigma = r.uniform(0.5, 2.0, d); X = r.standard_normal((d, m))
    W = _dense_layer(Uv, sigma, Vv)
    Y = orc.svd_layer_apply(Uv, sigma, Vv, X)
    np.testing.assert_allclose(Y, W @ X, atol=1e-12)
    np.testing.assert_allclose(orc.svd_layer_inverse_apply(Uv, sigma, Vv, X), np.linalg.solve(W, X), atol=1e-11)
    np.testing.assert_allclose(orc.svd_layer_inverse_apply(Uv, sigma, Vv, Y), X, atol=1e-11)
    np.testing.assert_allclose(np.linalg.svd(W, compute_uv=False), np.sort(sigma)[::-1], atol=1e-12)
    assert abs(orc.log_abs_det(sigma) - np.linalg.slogdet(W)[1]) < 1e-11


@pytest.mark.parametrize("inverse", [False, True])
def test_svd_layer_gradients_against_central_differences(inverse):
    r = _rng(13)
    d = 8; m = 3
    Uv = r.standard_normal((d, d)); Vv = r.standard_normal((d, d))
    sigma = r.uniform(0.5, 2.0, d); X = r.standard_normal((d, m)); G = r.standard_normal((d, m))

    def loss(Uv_, sigma_, Vv_, X_):
        W = _dense_layer(Uv_, sigma_, Vv_)
        Y = np.linalg.solve(W, X_) if inverse else W @ X_
        return float(np.sum(G * Y))

    fn = orc.svd_layer_inverse_gradients if inverse else orc.svd_layer_gradients
    Y, dUv, dsigma, dVv, dX = fn(Uv, sigma, Vv, X, G)
    W = _dense_layer(Uv, sigma, Vv)
    np.testing.assert_allclose(Y, np.linalg.solve(W, X) if inverse else W @ X, atol=1e-11)
    h = 1e-6
    args = [Uv, sigma, Vv, X]
    for idx, grad in ((0, dUv), (1, dsigma), (2, dVv), (3, dX)):
        fd = np.zeros_like(grad)
        it = np.nditer(grad, flags=["multi_index"])
        for _ in it:
            p = [a.copy() for a in args]; q = [a.copy() for a in args]
            p[idx][it.multi_index] += h; q[idx][it.multi_index] -= h
            fd[it.multi_index] = (loss(*p) - loss(*q)) / (2 * h)
        assert np.linalg.norm(grad - fd) <= 1e-6 * np.linalg.norm(fd), idx


# ------------------------------------------------------- symmetric forms (Table 1)

def _dense_symmetric(Uv, sigma):
    U = _dense_product(Uv)
    return U @ np.diag(sigma) @ U.T


def test_symmetric_forms_against_dense_expm_and_cayley():
    """Table 1: e^W = U e^Sigma U^T and (I - W)(I + W)^-1 = U (I - Sigma)(I + Sigma)^-1 U^T for
    W = U Sigma U^T, against scipy's Pade expm and a dense solve."""
    r = _rng(14)
    d = 10; m = 4
    Uv = r.standard_normal((d, d)); sigma = r.uniform(-0.8, 0.9, d); X = r.standard_normal((d, m))
    W = _dense_symmetric(Uv, sigma)
    np.testing.assert_allclose(orc.symmetric_apply(Uv, sigma, X), W @ X, atol=1e-12)
    np.testing.assert_allclose(orc.symmetric_apply(Uv, sigma, X, "exp"), scipy.linalg.expm(W) @ X, atol=1e-11)
    cay = np.linalg.solve(np.eye(d) + W, (np.eye(d) - W) @ X)
    np.testing.assert_allclose(orc.symmetric_apply(Uv, sigma, X, "cayley"), cay, atol=1e-11)
    # the Cayley map of a symmetric matrix is its own inverse map: applying it twice returns W X
    s_c, _ = orc.diagonal_function(sigma, "cayley")
    np.testing.assert_allclose(orc.symmetric_apply(Uv, s_c, X, "cayley"), W @ X, atol=1e-11)


@pytest.mark.parametrize("kind", ["identity", "exp", "cayley"])
def test_symmetric_gradients_against_central_differences(kind):
    r = _rng(15)
    d = 7; m = 3
    Uv = r.standard_normal((d, d)); sigma = r.uniform(-0.6, 0.8, d)
    X = r.standard_normal((d, m)); G = r.standard_normal((d, m))

    def loss(Uv_, sigma_, X_):
        W = _dense_symmetric(Uv_, sigma_)
        if kind == "exp":
            M = scipy.linalg.expm(W)
        elif kind == "cayley":
            M = np.linalg.solve(np.eye(d) + W, np.eye(d) - W)
        else:
            M = W
        return float(np.sum(G * (M @ X_)))

    Y, dUv, dsigma, dX = orc.symmetric_gradients(Uv, sigma, X, G, kind)
    h = 1e-6
    args = [Uv, sigma, X]
    for idx, grad in ((0, dUv), (1, dsigma), (2, dX)):
        fd = np.zeros_like(grad)
        it = np.nditer(grad, flags=["multi_index"])
        for _ in it:
            p = [a.copy() for a in args]; q = [a.copy() for a in args]
            p[idx][it.multi_index] += h; q[idx][it.multi_index] -= h
            fd[it.multi_index] = (loss(*p) - loss(*q)) / (2 * h)
        assert np.linalg.norm(grad - fd) <= 2e-6 * np.linalg.norm(fd), (kind, idx)


# ----------------------------------------------------------- rectangular W (Section 3.3)

def _dense_rect(Uv, sigma, Vv):
    p, q = Uv.shape[1], Vv.shape[1]
    S = np.zeros((p, q))
    S[np.arange(sigma.size), np.arange(sigma.size)] = sigma
    return _dense_product(Uv) @ S @ _dense_product(Vv).T


@pytest.mark.parametrize("p,q", [(9, 5), (5, 9), (7, 7)])
def test_rectangular_layer_against_dense(p, q):
    """Section 3.3: W = U Sigma V^T with a rectangular diagonal Sigma; its singular values are sigma."""
    r = _rng(16 + p + q)
    Uv = r.standard_normal((p, p)); Vv = r.standard_normal((q, q))
    sigma = r.uniform(0.5, 2.0, min(p, q)); X = r.standard_normal((q, 4)); G = r.standard_normal((p, 4))
    W = _dense_rect(Uv, sigma, Vv)
    assert W.shape == (p, q)
    np.testing.assert_allclose(orc.rectangular_apply(Uv, sigma, Vv, X), W @ X, atol=1e-12)
    np.testing.assert_allclose(np.linalg.svd(W, compute_uv=False), np.sort(sigma)[::-1], atol=1e-12)

    def loss(Uv_, sigma_, Vv_, X_):
        return float(np.sum(G * (_dense_rect(Uv_, sigma_, Vv_) @ X_)))

    Y, dUv, dsigma, dVv, dX = orc.rectangular_gradients(Uv, sigma, Vv, X, G)
    np.testing.assert_allclose(dX, W.T @ G, atol=1e-12)
    h = 1e-6
    args = [Uv, sigma, Vv, X]
    for idx, grad in ((0, dUv), (1, dsigma), (2, dVv), (3, dX)):
        fd = np.zeros_like(grad)
        it = np.nditer(grad, flags=["multi_index"])
        for _ in it:
            a = [x.copy() for x in args]; b = [x.copy() for x in args]
            a[idx][it.multi_index] += h; b[idx][it.multi_index] -= h
            fd[it.multi_index] = (loss(*a) - loss(*b)) / (2 * h)
        assert np.linalg.norm(grad - fd) <= 1e-6 * np.linalg.norm(fd), idx
