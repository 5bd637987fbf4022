"""Seeded synthetic inputs for the compensated quantized GEMM.

Only input generation lives here (no quantization, selection or product
arithmetic), so that the HIP path's tests/bench and the CPU oracle's tests can
draw identical matrices.  All draws use ``numpy.random.default_rng(seed)``,
A first, then B, in float32.

The paper itself measures on synthetic random matrices (uniform(0,1) for the
speed tables, five distributions for the precision figure, Sec. 4.1), so these
recipes stand in for no external dataset.
"""
from __future__ import annotations

import dataclasses
from typing import Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    M: int
    N: int
    K: int
    seed: int
    densities: Tuple[float, ...]     # target densities of the reduced operands
    recipe: str


WORKLOADS = {
    "C1": Workload("C1", 256, 256, 256, 0, (0.05,), "uniform[-1,1)"),
    "C2": Workload("C2", 2048, 2048, 2048, 1, (0.01, 0.05, 0.20), "normal(0,1)"),
    "C3": Workload("C3", 8192, 8192, 8192, 2, (0.05,),
                   "normal(0,1), 0.1% of entries at random distinct positions x100"),
    "C4": Workload("C4", 4096, 14336, 4096, 3, (0.02,),
                   "A normal(0,1) with 16 random columns x50; B normal(0,0.02)"),
    "C5": Workload("C5", 16384, 16384, 16384, 4, (0.05, 0.20, 0.50),
                   "sign * 2^e * uniform[1,2), e integer uniform in [-10,10]"),
}


def _normal(rng, shape):
    return rng.standard_normal(shape, dtype=np.float32)


def _scale_random_entries(rng, X, fraction, factor):
    n = int(round(X.size * fraction))
    if n:
        pos = rng.choice(X.size, size=n, replace=False)
        X.reshape(-1)[pos] *= np.float32(factor)


def _wide_range(rng, shape):
    e = rng.integers(-10, 11, size=shape).astype(np.float32)
    mant = (rng.random(shape, dtype=np.float32) + np.float32(1.0))
    sign = np.where(rng.integers(0, 2, size=shape) == 0, np.float32(-1), np.float32(1))
    return (sign * np.exp2(e) * mant).astype(np.float32)


def make_inputs(name: str, M: int = None, N: int = None, K: int = None, seed: int = None):
    """Return (A[M,K], B[K,N]) float32 for the named recipe.  M, N, K and seed
    default to the workload's own; smaller shapes give same-distribution cases
    for quick tests."""
    w = WORKLOADS[name]
    M = w.M if M is None else M
    N = w.N if N is None else N
    K = w.K if K is None else K
    rng = np.random.default_rng(w.seed if seed is None else seed)
    if name == "C1":
        A = rng.random((M, K), dtype=np.float32) * np.float32(2) - np.float32(1)
        B = rng.random((K, N), dtype=np.float32) * np.float32(2) - np.float32(1)
    elif name == "C2":
        A = _normal(rng, (M, K))
        B = _normal(rng, (K, N))
    elif name == "C3":
        A = _normal(rng, (M, K))
        _scale_random_entries(rng, A, 1e-3, 100.0)
        B = _normal(rng, (K, N))
        _scale_random_entries(rng, B, 1e-3, 100.0)
    elif name == "C4":
        A = _normal(rng, (M, K))
        cols = rng.choice(K, size=min(16, K), replace=False)
        A[:, cols] *= np.float32(50.0)
        B = _normal(rng, (K, N)) * np.float32(0.02)
    elif name == "C5":
        A = _wide_range(rng, (M, K))
        B = _wide_range(rng, (K, N))
    else:
        raise KeyError(name)
    return np.ascontiguousarray(A), np.ascontiguousarray(B)


def paper_distribution(kind: str, shape, seed: int):
    """The five input distributions of the paper's precision test (caption of
    the precision figure, Sec. 4.1.1), all non-negative."""
    rng = np.random.default_rng(seed)
    if kind == "uniform":
        X = rng.random(shape)
    elif kind == "normal":
        X = rng.normal(10.0, np.sqrt(3.0), shape)      # "mean 10, variance 3"
    elif kind == "exponential":
        X = rng.exponential(1.0 / 4.0, shape)          # rate lambda = 4
    elif kind == "poisson":
        X = rng.poisson(10.0, shape)
    elif kind == "chisquare":
        X = rng.chisquare(1.0, shape)
    else:
        raise KeyError(kind)
    return np.ascontiguousarray(X.astype(np.float32))


def qr_factors(kind: str, n: int, seed: int):
    """Inputs of the paper's QR experiment (Sec. 4.2): a square matrix drawn from one of the
    precision-test distributions and its Householder QR factors, all float32.  The experiment
    multiplies Q by R with the quantized product and compares with the matrix itself.
    Returns (X, Q, R) with Q orthogonal (n x n) and R upper triangular."""
    X = paper_distribution(kind, (n, n), seed)
    Q, R = np.linalg.qr(X.astype(np.float64))
    return X, np.ascontiguousarray(Q.astype(np.float32)), np.ascontiguousarray(R.astype(np.float32))


def theta_for_density(X, dvec, axis, density: float) -> float:
    """Harness-side calibration: the threshold factor theta such that about
    ``density`` of the entries of X satisfy |x| > theta * dvec[v].

    This is the (1-density)-quantile of |x| / dvec[v]; it is not part of the
    method (the paper sweeps theta and reports the density it gets).  X and dvec
    are numpy arrays or torch tensors (the quantile is then taken on the tensor's
    device); axis is "row" (or 0) when dvec holds one value per row of X, "col"
    (or 1) for one per column.  The one copy of this helper: bench.py, the sweep
    harnesses and the tests all call it."""
    by_row = axis in ("row", 0)
    if hasattr(X, "detach"):                            # torch tensors
        import torch
        d = dvec.view(-1, 1) if by_row else dvec.view(1, -1)
        rho = (X.abs() / d).reshape(-1)
        n = rho.numel()
        keep = int(round(n * density))
        if keep <= 0:
            return float("inf")
        if keep >= n:
            return 0.0
        return float(torch.sort(rho).values[n - keep - 1].item())   # a sort is far faster than kthvalue here
    X = np.asarray(X, dtype=np.float32)
    d = np.asarray(dvec, dtype=np.float32)
    d = d.reshape(-1, 1) if by_row else d.reshape(1, -1)
    rho = (np.abs(X) / d).reshape(-1)
    keep = int(round(rho.size * density))
    if keep <= 0:
        return float("inf")
    if keep >= rho.size:
        return 0.0
    kth = rho.size - keep                               # entries above index kth-1 are kept
    part = np.partition(rho, kth - 1)
    return float(np.float32(part[kth - 1]))
