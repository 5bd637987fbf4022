"""Blocked Householder QR whose matrix products run through the compensated quantized GEMM.

Sec. 4.2 of the paper takes a QR routine built on Householder reflections and substitutes the
quantized product for the multiplications that apply the orthogonal factor; it then reports
E_r = ||A - Q.R||_F / ||A||_F for the direct ("origin"), unreduced ("full") and sparse
("xigemm") variants.  The paper gives neither sizes nor block width nor which products exactly
were substituted; the reading taken here: a blocked factorization in compact-WY form whose
panels (block x block work, O(m nb^2)) stay in FP32 and whose four large products per panel,
plus the final Q.R, go through a pluggable `matmul`:

    W  = V^T . A2         the reflectors applied to the trailing matrix ...
    A2 = A2 - V . (T^T W) ... (I - V T V^T)^T A2
    Y  = Q2 . V           the same reflectors accumulated into the explicit Q ...
    Q2 = Q2 - (Y T) . V^T ... Q2 (I - V T V^T)

This module is host orchestration only (panel arithmetic in torch, any device); `LibraryMatmul`
is the product the experiment substitutes: one `srq_compensated_gemm` call per product.
"""
from __future__ import annotations

import math


def _panel(P):
    """Unblocked Householder factorization of the panel P (r x nb, r >= 1), in place: on return P
    holds R in its upper triangle.  Returns V (r x nb, unit lower trapezoid) and tau (nb)."""
    import torch
    r, nb = P.shape
    V = torch.zeros_like(P)
    tau = torch.zeros(nb, dtype=P.dtype, device=P.device)
    for c in range(min(r, nb)):
        x = P[c:, c]
        x0 = x[0].clone()
        norm = torch.linalg.vector_norm(x)
        if float(norm) == 0.0:                     # nothing to annihilate: H = I
            V[c, c] = 1.0
            continue
        beta = -norm if float(x0) >= 0.0 else norm
        v = x / (x0 - beta)
        v[0] = 1.0
        t = (beta - x0) / beta
        V[c:, c] = v
        tau[c] = t
        # the reflector applied to the rest of the panel, then its own column
        if c + 1 < nb:
            rest = P[c:, c + 1:]
            rest -= t * torch.outer(v, v @ rest)
        P[c, c] = beta
        P[c + 1:, c] = 0.0
    return V, tau


def _wy_t(V, tau):
    """Upper-triangular T with H_0 H_1 ... H_{nb-1} = I - V T V^T (forward, column-wise)."""
    import torch
    nb = V.shape[1]
    T = torch.zeros((nb, nb), dtype=V.dtype, device=V.device)
    G = V.T @ V
    for i in range(nb):
        T[i, i] = tau[i]
        if i:
            T[:i, i] = -tau[i] * (T[:i, :i] @ G[:i, i])
    return T


def householder_qr(A, matmul=None, block=64):
    """Q (m x m), R (m x n) of the float tensor A (m x n, m >= n) by blocked Householder
    reflections; every large product is `matmul(X, Y)` (default: torch.matmul).  With an exact
    matmul Q is orthogonal and Q.R = A to rounding; with a quantized matmul the errors of the
    products propagate through the trailing updates, which is what the experiment measures."""
    import torch
    if matmul is None:
        matmul = torch.matmul
    m, n = A.shape
    if m < n:
        raise ValueError("householder_qr expects m >= n")
    R = A.clone()
    Q = torch.eye(m, dtype=A.dtype, device=A.device)
    for j0 in range(0, n, block):
        jb = min(block, n - j0)
        V, tau = _panel(R[j0:, j0:j0 + jb])
        T = _wy_t(V, tau)
        if j0 + jb < n:
            A2 = R[j0:, j0 + jb:]
            W = matmul(V.T.contiguous(), A2.contiguous())
            A2 -= matmul(V, (T.T @ W).contiguous())
        Q2 = Q[:, j0:]
        Y = matmul(Q2.contiguous(), V)
        Q2 -= matmul((Y @ T).contiguous(), V.T.contiguous())
    return Q, R


class LibraryMatmul:
    """X @ Y through srq_compensated_gemm on a binding.Srq handle.

    mode "origin": theta = inf (direct quantization); "full": theta = 0 on the dense branch
    (unreduced residual compensation); "sparse": the reduced operands of the method, with either
    one fixed `theta` (the paper's single threshold) or, when `density` is given, theta_a and
    theta_b calibrated per call so that about that share of each operand is kept (harness-side
    calibration from the library's own first product, as in bench.py).
    `calls` keeps a dict per product when `record` is set (operands, theta_a, theta_b, the result,
    and the threshold vectors the library derived from its own means of |D_F|), so that a test can
    replay each one on the oracle."""

    def __init__(self, handle, mode="sparse", bits=8, theta=None, density=None, record=False):
        if mode not in ("origin", "full", "sparse"):
            raise ValueError(mode)
        if mode == "sparse" and (theta is None) == (density is None):
            raise ValueError("sparse mode takes exactly one of theta, density")
        self.h, self.mode, self.bits, self.theta, self.density = handle, mode, bits, theta, density
        self.record = record
        self.calls = []

    def thetas(self, X, Y):
        from . import binding as b
        from . import workloads as wl
        if self.mode == "origin":
            return math.inf, math.inf
        if self.mode == "full":
            return 0.0, 0.0
        if self.theta is not None:
            return float(self.theta), float(self.theta)
        Qx, sx, _ = self.h.quantize(X, b.AXIS_ROW, bits=self.bits)
        Qy, sy, _ = self.h.quantize(Y, b.AXIS_COL, bits=self.bits)
        _, _, drow, dcol = self.h.gemm_i8(Qx, sx, Qy, sy)
        ta = wl.theta_for_density(X, drow, 0, self.density) if bool((drow > 0).all()) else math.inf
        tb = wl.theta_for_density(Y, dcol, 1, self.density) if bool((dcol > 0).all()) else math.inf
        return ta, tb

    def __call__(self, X, Y):
        X, Y = X.contiguous(), Y.contiguous()
        ta, tb = self.thetas(X, Y)
        C, _, _ = self.h.compensated_gemm(X, Y, ta, tb, bits=self.bits,
                                          dense_fallback_density=0.0 if self.mode == "full" else 2.0)
        if self.record:
            im = self.h.intermediates(X.shape[0], Y.shape[1], X.shape[1])
            self.calls.append({"X": X.clone(), "Y": Y.clone(), "theta_a": ta, "theta_b": tb, "C": C.clone(),
                               "t_a": None if im["t_a"] is None else im["t_a"].clone(),
                               "t_b": None if im["t_b"] is None else im["t_b"].clone()})
        return C
