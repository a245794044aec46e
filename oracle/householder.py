"""fp64 CPU checker for products of Householder reflections and their gradients.

TEST INFRASTRUCTURE ONLY. Nothing in the product path may import this module;
it exists so that tests, the smoke check and the benchmark's CPU-baseline leg
have an independent, obviously correct answer to compare the HIP kernels with.
It shares no code with the HIP path.

The method under test (FastH, Algorithms 1 and 2 of the paper) reaches exactly
the result of the sequential algorithm it replaces (Section 4.1, last
paragraph; Theorem 1 and Theorem 2 "Correctness"), so this file is the plain
definition written out, one reflection at a time, in numpy fp64:

* Eq. 1:           H_j = I - 2 v_j v_j^T / ||v_j||^2
* Section 2.2:     H X = H_1 (H_2 ( ... (H_n X)))   (H_n touches X first)
* Supplement 8.1:  dL/dX = H_n^T ... H_1^T dL/dA_1
* Eq. 4:           the input of H_j is recovered from its output, H_j^-1 = H_j^T
* Eq. 5:           dL/dv_j, summed over the m columns of the mini-batch
* Section 2.2 / Table 1:  W = U diag(sigma) V^T,  W^-1 = V diag(1/sigma) U^T,
                          exp(U S U^T) = U e^S U^T,  Cayley(U S U^T) = U (I - S)(I + S)^-1 U^T
* Section 3.3 "Rectangular Matrices":  W (p x q) = U Sigma V^T with U p x p, V q x q, Sigma p x q

Layout: V is [n][d], row j-1 holding v_j; X, A, G are [d][m], one sample per
column. Every function promotes its inputs to float64.

Readings of the paper taken here (each one is pinned by a test):
* Eq. 5's leading factor -2/||v||^2 multiplies all three terms of the sum, and
  the third term carries one more factor 2/||v||^2.
* In Eq. 5, a is a column of the INPUT of H_j and g a column of the gradient at
  its OUTPUT.
* The gradient is a sum over the mini-batch, not a mean.
* No epsilon is added to ||v||^2; a zero vector is an error.

Parity pins: all functions are pinned (see tests/test_oracle_pins.py); none is
"parity unpinned".
"""
from __future__ import annotations

import numpy as np


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


def reflect(v, A) -> np.ndarray:
    """Eq. 1 applied to a d x m matrix: A - 2 v (v^T A) / (v^T v)."""
    v = _f64(v)
    A = _f64(A)
    s = float(v @ v)
    if s == 0.0:
        raise ZeroDivisionError("Householder vector is zero: Eq. 1 is undefined")
    return A - np.outer(v, (2.0 / s) * (v @ A))


def product_apply(V, X, transpose: bool = False) -> np.ndarray:
    """H X with H = H_1 ... H_n (Section 2.2 "Multiplication"): H_n is applied
    first. With transpose=True, H^T X = H_n ... H_1 X (each H_j is symmetric),
    so H_1 is applied first."""
    V = _f64(V)
    A = _f64(X).copy()
    n = V.shape[0]
    order = range(n) if transpose else range(n - 1, -1, -1)
    for j in order:
        A = reflect(V[j], A)
    return A


def vector_gradient(v, a_in, g_out) -> np.ndarray:
    """Eq. 5: gradient of L wrt one Householder vector, summed over columns.

    a_in  : input of H_j  (d x m), called A-hat_{j+1} in Section 3.2
    g_out : dL/d(output of H_j) (d x m), called dL/dA-hat_j
    """
    v = _f64(v)
    s = float(v @ v)
    alpha = v @ a_in          # v^T a^(l), one per column
    gamma = v @ g_out         # v^T g^(l)
    total = g_out @ alpha + a_in @ gamma - (2.0 / s) * float(alpha @ gamma) * v
    return -(2.0 / s) * total


def product_gradients(V, X, G, transpose: bool = False):
    """A = H X (or H^T X), and the gradients of L = <G, A> wrt V and X.

    Follows Section 3.2 with blocks of one reflection: walk j = 1..n from the
    output side holding (output of H_j, dL/d output of H_j); recover the input
    of H_j by Eq. 4 (H_j is its own inverse), emit dL/dv_j by Eq. 5, then move
    the gradient through H_j^T = H_j. The last gradient is dL/dX.

    The transposed product H^T = H_n ... H_1 is the same product with the
    vectors taken in the opposite order, so it is handled by reversal.
    """
    V = _f64(V)
    X = _f64(X)
    G = _f64(G)
    if transpose:
        A, dV_rev, dX = product_gradients(V[::-1], X, G, transpose=False)
        return A, dV_rev[::-1].copy(), dX
    n = V.shape[0]
    A = product_apply(V, X)
    dV = np.zeros_like(V)
    a_out = A
    g = G.copy()
    for j in range(n):
        a_in = reflect(V[j], a_out)            # Eq. 4, left
        dV[j] = vector_gradient(V[j], a_in, g)  # Eq. 5
        g = reflect(V[j], g)                   # Eq. 4, right
        a_out = a_in
    return A, dV, g


def product_gradients_stored(V, X, G):
    """Same gradients as product_gradients(transpose=False), but keeping every
    intermediate input on the way forward instead of recomputing it by Eq. 4.
    Used only as a cross-check of the reversible walk."""
    V = _f64(V)
    X = _f64(X)
    G = _f64(G)
    n = V.shape[0]
    inputs = [None] * n
    A = X.copy()
    for j in range(n - 1, -1, -1):
        inputs[j] = A
        A = reflect(V[j], A)
    dV = np.zeros_like(V)
    g = G.copy()
    for j in range(n):
        dV[j] = vector_gradient(V[j], inputs[j], g)
        g = reflect(V[j], g)
    return A, dV, g


def dense_matrix(V, transpose: bool = False) -> np.ndarray:
    """The d x d matrix H (or H^T), by applying the product to the identity."""
    V = _f64(V)
    return product_apply(V, np.eye(V.shape[1]), transpose=transpose)


# --------------------------------------------------------------------------
# SVD-reparameterised layer (Section 2.2; Table 1 row "Inverse")
# --------------------------------------------------------------------------

def svd_layer_apply(Uv, sigma, Vv, X) -> np.ndarray:
    """W X with W = U diag(sigma) V^T, U and V Householder products."""
    sigma = _f64(sigma)
    Z1 = product_apply(Vv, X, transpose=True)
    Z2 = sigma[:, None] * Z1
    return product_apply(Uv, Z2)


def svd_layer_inverse_apply(Uv, sigma, Vv, X) -> np.ndarray:
    """W^-1 X = V diag(1/sigma) U^T X (Table 1)."""
    sigma = _f64(sigma)
    Z1 = product_apply(Uv, X, transpose=True)
    Z2 = Z1 / sigma[:, None]
    return product_apply(Vv, Z2)


def svd_layer_gradients(Uv, sigma, Vv, X, G):
    """Y = W X and the gradients of L = <G, Y> wrt (Uv, sigma, Vv, X), by the
    chain rule through the three stages Z1 = V^T X, Z2 = sigma * Z1, Y = U Z2."""
    sigma = _f64(sigma)
    Z1 = product_apply(Vv, X, transpose=True)
    Z2 = sigma[:, None] * Z1
    Y, dUv, dZ2 = product_gradients(Uv, Z2, G)
    dsigma = np.sum(dZ2 * Z1, axis=1)
    dZ1 = sigma[:, None] * dZ2
    _, dVv, dX = product_gradients(Vv, X, dZ1, transpose=True)
    return Y, dUv, dsigma, dVv, dX


def svd_layer_inverse_gradients(Uv, sigma, Vv, X, G):
    """Y = W^-1 X and the gradients of L = <G, Y> wrt (Uv, sigma, Vv, X).
    With rho = 1/sigma: Z1 = U^T X, Z2 = rho * Z1, Y = V Z2, and
    d sigma = -d rho / sigma^2."""
    sigma = _f64(sigma)
    rho = 1.0 / sigma
    Z1 = product_apply(Uv, X, transpose=True)
    Z2 = rho[:, None] * Z1
    Y, dVv, dZ2 = product_gradients(Vv, Z2, G)
    drho = np.sum(dZ2 * Z1, axis=1)
    dsigma = -drho / (sigma * sigma)
    dZ1 = rho[:, None] * dZ2
    _, dUv, dX = product_gradients(Uv, X, dZ1, transpose=True)
    return Y, dUv, dsigma, dVv, dX


def log_abs_det(sigma) -> float:
    """Table 1 row "Determinant": sum_i log |sigma_i| = log |det W|."""
    return float(np.sum(np.log(np.abs(_f64(sigma)))))


# --------------------------------------------------------------------------
# Symmetric forms of Table 1 (rows "Matrix Exponential" and "Cayley map"): one
# orthogonal factor U and a diagonal, W = U diag(sigma) U^T.
# --------------------------------------------------------------------------

def diagonal_function(sigma, kind: str):
    """f(sigma) and f'(sigma) for the diagonal of U f(Sigma) U^T.
    'identity': W itself; 'exp': e^W = U e^Sigma U^T; 'cayley': (I - W)(I + W)^-1 =
    U (I - Sigma)(I + Sigma)^-1 U^T."""
    sigma = _f64(sigma)
    if kind == "identity":
        return sigma.copy(), np.ones_like(sigma)
    if kind == "exp":
        e = np.exp(sigma)
        return e, e
    if kind == "cayley":
        return (1.0 - sigma) / (1.0 + sigma), -2.0 / (1.0 + sigma) ** 2
    raise ValueError(kind)


def symmetric_apply(Uv, sigma, X, kind: str = "identity") -> np.ndarray:
    """U f(Sigma) U^T X."""
    s, _ = diagonal_function(sigma, kind)
    Z1 = product_apply(Uv, X, transpose=True)
    return product_apply(Uv, s[:, None] * Z1)


def symmetric_gradients(Uv, sigma, X, G, kind: str = "identity"):
    """Y = U f(Sigma) U^T X and the gradients of L = <G, Y> wrt (Uv, sigma, X). U enters twice
    (as U^T on X and as U on the scaled result); its two gradient contributions add."""
    s, ds_dsigma = diagonal_function(sigma, kind)
    Z1 = product_apply(Uv, X, transpose=True)
    Z2 = s[:, None] * Z1
    Y, dU_outer, dZ2 = product_gradients(Uv, Z2, G)
    dsigma = np.sum(dZ2 * Z1, axis=1) * ds_dsigma
    dZ1 = s[:, None] * dZ2
    _, dU_inner, dX = product_gradients(Uv, X, dZ1, transpose=True)
    return Y, dU_outer + dU_inner, dsigma, dX


# --------------------------------------------------------------------------
# Rectangular W (Section 3.3 "Rectangular Matrices"): W in R^{p x q}, U in R^{p x p},
# V in R^{q x q}, Sigma in R^{p x q} with sigma on its main diagonal (min(p, q) values).
# --------------------------------------------------------------------------

def _rect_scale(sigma, Z, p):
    """Sigma Z for Z with q rows: row i < min(p, q) is scaled by sigma_i, the result has p rows."""
    sigma = _f64(sigma)
    r = sigma.shape[0]
    out = np.zeros((p, Z.shape[1]))
    out[:r] = sigma[:, None] * Z[:r]
    return out


def rectangular_apply(Uv, sigma, Vv, X) -> np.ndarray:
    p = _f64(Uv).shape[1]
    Z1 = product_apply(Vv, X, transpose=True)
    return product_apply(Uv, _rect_scale(sigma, Z1, p))


def rectangular_gradients(Uv, sigma, Vv, X, G):
    """Y = U Sigma V^T X and the gradients of L = <G, Y> wrt (Uv, sigma, Vv, X)."""
    sigma = _f64(sigma)
    p = _f64(Uv).shape[1]
    q = _f64(Vv).shape[1]
    r = sigma.shape[0]
    Z1 = product_apply(Vv, X, transpose=True)
    Z2 = _rect_scale(sigma, Z1, p)
    Y, dUv, dZ2 = product_gradients(Uv, Z2, G)
    dsigma = np.sum(dZ2[:r] * Z1[:r], axis=1)
    dZ1 = _rect_scale(sigma, dZ2, q)  # Sigma^T dZ2
    _, dVv, dX = product_gradients(Vv, X, dZ1, transpose=True)
    return Y, dUv, dsigma, dVv, dX
