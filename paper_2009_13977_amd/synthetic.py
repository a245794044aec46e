"""Seeded synthetic inputs for the FastH workloads.

This module only draws random numbers. It holds none of the method's
arithmetic, so both the fp64 CPU checker and the HIP path can be fed from it
without sharing any computation.

The paper's timing experiment (Section 4.1 and its supplement "Comparing
Running Time") uses a dummy input X and a dummy upstream gradient G with
i.i.d. N(0,1) entries, mini-batch m = 32, and one d x d matrix of Householder
vectors; it does not state how the vectors are drawn, so they are N(0,1) too.
The SVD layer adds singular values drawn uniformly from [0.5, 2] so that the
inverse is well conditioned.

Every array is drawn in fp64 with numpy's PCG64 `default_rng(seed)` in a fixed
order and rounded to fp32 once. A consumer that computes in fp64 promotes
those fp32 values, so both sides see bit-identical inputs.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict

import numpy as np

SEED_BASE = 13977000


@dataclass(frozen=True)
class Workload:
    """One named problem size: n reflections of length d, m columns, block k."""

    name: str
    d: int
    n: int
    m: int
    k: int
    seed: int
    svd_layer: bool = False


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in (
        Workload("d64_m32_k32", 64, 64, 32, 32, SEED_BASE + 1),
        Workload("d256_m32_k32", 256, 256, 32, 32, SEED_BASE + 2),
        Workload("d1024_m32_k32", 1024, 1024, 32, 32, SEED_BASE + 3),
        Workload("d2048_m64_k32", 2048, 2048, 64, 32, SEED_BASE + 4),
        Workload("d2048_m64_k64", 2048, 2048, 64, 64, SEED_BASE + 4),
        Workload("d2048_m64_k128", 2048, 2048, 64, 128, SEED_BASE + 4),
        Workload("svd_d1024_m32_k32", 1024, 1024, 32, 32, SEED_BASE + 5, True),
        # Section 3.3, convolutional and recurrent uses: one V applied to m * h * w (or m * r) columns
        Workload("d1024_m4096_k32", 1024, 1024, 4096, 32, SEED_BASE + 6),
        Workload("d1024_m16384_k32", 1024, 1024, 16384, 32, SEED_BASE + 7),
        Workload("d1024_m1024_k32", 1024, 1024, 1024, 32, SEED_BASE + 8),
    )
}

HEADLINE = "d1024_m32_k32"


def _f32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a.astype(np.float32))


def householder_problem(d: int, n: int, m: int, seed: int) -> Dict[str, np.ndarray]:
    """V [n][d] (row j is the j-th Householder vector), X [d][m], G [d][m]."""
    rng = np.random.default_rng(seed)
    V = rng.standard_normal((n, d))
    X = rng.standard_normal((d, m))
    G = rng.standard_normal((d, m))
    return {"V": _f32(V), "X": _f32(X), "G": _f32(G)}


def svd_layer_problem(d: int, n: int, m: int, seed: int) -> Dict[str, np.ndarray]:
    """Uv, Vv [n][d] Householder vectors of the two orthogonal factors,
    sigma [d] in [0.5, 2], X [d][m], G [d][m]."""
    rng = np.random.default_rng(seed)
    Uv = rng.standard_normal((n, d))
    Vv = rng.standard_normal((n, d))
    sigma = rng.uniform(0.5, 2.0, size=d)
    X = rng.standard_normal((d, m))
    G = rng.standard_normal((d, m))
    return {"Uv": _f32(Uv), "Vv": _f32(Vv), "sigma": _f32(sigma), "X": _f32(X), "G": _f32(G)}


def rect_layer_problem(rows: int, cols: int, n_u: int, n_v: int, m: int, seed: int) -> Dict[str, np.ndarray]:
    """Uv [n_u][rows], Vv [n_v][cols], sigma [min(rows, cols)] in [0.5, 2], X [cols][m], G [rows][m]."""
    rng = np.random.default_rng(seed)
    Uv = rng.standard_normal((n_u, rows))
    Vv = rng.standard_normal((n_v, cols))
    sigma = rng.uniform(0.5, 2.0, size=min(rows, cols))
    X = rng.standard_normal((cols, m))
    G = rng.standard_normal((rows, m))
    return {"Uv": _f32(Uv), "Vv": _f32(Vv), "sigma": _f32(sigma), "X": _f32(X), "G": _f32(G)}


def workload_inputs(name: str) -> Dict[str, np.ndarray]:
    w = WORKLOADS[name]
    if w.svd_layer:
        return svd_layer_problem(w.d, w.n, w.m, w.seed)
    return householder_problem(w.d, w.n, w.m, w.seed)
