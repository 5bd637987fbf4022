"""Plain numpy oracle of the sparse-residual-compensated quantized GEMM.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Written from the paper
(Gu et al., "A method for accelerating low precision operations by sparse
matrix multiplication"), step by step in the order of its Algorithm 1, with no
blocking, fusion or reordering.  Every floating-point step is carried out on
``numpy.float32`` arrays, so each operation rounds once to IEEE binary32, which
is the precision the paper's "origin precision" T_F = FP32 fixes.  Integer
products are exact.

Pins (tests/test_oracle_*.py): the 1-D worked example of Sec. 2.3, every printed
intermediate of the 3x3 worked example of Sec. 3.1.2, exact integer brute force,
the theta = inf / theta = 0 bounds (Eq. gemm_r), the residual bound of
Eq. lambdaleq, a scale-free special case that reduces to an integer matmul, and
error monotonicity in theta.  Parity of alpha/beta and leading-dimension
handling is not fixed by anything the paper prints ("parity unpinned" beyond
their algebraic definition in Algorithm 1's last line).

Readings of the paper taken here (the paper is silent or inconsistent):
  * qmax = 2**(bits-1) - 1 (the prose form and the 1-D example; Eq. getlambda as
    printed would overflow the integer type).  The 3x3 example uses 64, so
    ``qmax`` can be overridden.
  * Rounding: round-to-nearest-even by default; truncation toward zero
    (what the worked examples do) on request.
  * Dequantization multiplies by s = fl(amax/qmax); lambda = fl(qmax/amax) is
    used only to quantize.
  * The sparse operand is the *reduced original* matrix A' (resp. B'), and it is
    multiplied by the dense quantized residual of the *other* operand
    (Sec. 3.1.1 last paragraphs, Algorithm 1 "Reduce"/"SPMM" lines).
  * Selection compares |x| with theta * mean|D_F| strictly (kept iff greater);
    ``signed_compare`` replays the printed example, which compares signed x.
  * A'_int = mask (.) A_int: the reduced operand keeps the codes and scale of
    the unreduced one (the example's printed codes agree).
  * The second correction term is RA . B' (the printed "B'*RA" is not
    dimensionally the product that the derivation sums).
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

F32 = np.float32

ROUND_NEAREST_EVEN = "nearest_even"
ROUND_TRUNC = "trunc"


def qmax_of_bits(bits: int) -> int:
    """Largest code magnitude of a symmetric N-bit integer (Sec. 2.3, the prose
    form lambda = (2^{N-1}-1)/a_max)."""
    if not (2 <= bits <= 8):
        raise ValueError("bits must be in 2..8")
    return (1 << (bits - 1)) - 1


# --------------------------------------------------------------------------
# Step 1-2 of Algorithm 1: Quant  (Eq. Quantization, Eq. getlambda, Sec. 3.2)
# --------------------------------------------------------------------------
def quantize_vectors(X, axis: str, qmax: int = 127, rounding: str = ROUND_NEAREST_EVEN):
    """Symmetric linear quantization with one scale per vector.

    axis = "row": one scale per row (matrix A and RA, Sec. 3.2);
    axis = "col": one scale per column (matrix B and RB);
    axis = "global": one scale for the whole matrix (Sec. 2.2 form, used by the
    3x3 example), returned broadcast as a length-1 vector.

    Returns (Q int8 same shape as X, s float32 vector, lam float32 vector) with
    lam = fl(qmax/amax), s = fl(amax/qmax), both 0 for an all-zero vector.
    """
    X = np.asarray(X, dtype=F32)
    if X.ndim != 2:
        raise ValueError("X must be 2-D")
    absX = np.abs(X)
    if axis == "row":
        amax = absX.max(axis=1) if X.shape[1] else np.zeros(X.shape[0], F32)
        shape = (-1, 1)
    elif axis == "col":
        amax = absX.max(axis=0) if X.shape[0] else np.zeros(X.shape[1], F32)
        shape = (1, -1)
    elif axis == "global":
        amax = np.array([absX.max() if X.size else 0.0], dtype=F32)
        shape = (1, 1)
    else:
        raise ValueError(axis)
    amax = amax.astype(F32)
    q = F32(qmax)
    nz = amax > 0
    lam = np.zeros_like(amax)
    s = np.zeros_like(amax)
    np.divide(q, amax, out=lam, where=nz)          # one rounding
    np.divide(amax, q, out=s, where=nz)            # one rounding
    y = X * lam.reshape(shape)                     # one rounding per element
    if rounding == ROUND_NEAREST_EVEN:
        r = np.rint(y)
    elif rounding == ROUND_TRUNC:
        r = np.trunc(y)
    else:
        raise ValueError(rounding)
    r = np.clip(r, -q, q)
    return r.astype(np.int8), s, lam


# --------------------------------------------------------------------------
# Step 2 of Algorithm 1: integer GEMM, exact
# --------------------------------------------------------------------------
def int_matmul(P, Q):
    """Exact integer product of two integer-valued matrices, returned as int64.

    Computed through float64 BLAS, which is exact here because every partial sum
    is an integer of magnitude <= K*128*128 < 2**53.
    """
    P = np.asarray(P)
    Q = np.asarray(Q)
    K = P.shape[1]
    if K * 128 * 128 >= 2 ** 53:
        raise ValueError("K too large for the exact float64 route")
    return np.rint(P.astype(np.float64) @ Q.astype(np.float64)).astype(np.int64)


def check_k_bound(K: int, qmax: int) -> None:
    """INT32 accumulators must not overflow: K*qmax^2 < 2^31."""
    if K * qmax * qmax >= 2 ** 31:
        raise OverflowError("K*qmax^2 would overflow an INT32 accumulator")


# --------------------------------------------------------------------------
# Step 3: Dequant of the product (Eq. quantized GEMM; Sec. 3.2 last sentence)
# --------------------------------------------------------------------------
def dequant_product(D_int, s_row, s_col):
    """D_F[i,j] = fl( fl(float(D_int[i,j])) * fl(s_row[i]*s_col[j]) )."""
    Df = np.asarray(D_int).astype(F32)             # int -> binary32, RNE
    sc = s_row.astype(F32).reshape(-1, 1) * s_col.astype(F32).reshape(1, -1)
    return Df * sc


# --------------------------------------------------------------------------
# Steps 4-6: residual matrices (Sec. 2.3, "A^Fp = A^Fp' + RA^Fp")
# --------------------------------------------------------------------------
def dequantize(Q, s, axis: str):
    """x_hat = fl(float(q) * s_v)  (Eq. Dequantization with s = 1/lambda)."""
    shape = {"row": (-1, 1), "col": (1, -1), "global": (1, 1)}[axis]
    return np.asarray(Q).astype(F32) * s.astype(F32).reshape(shape)


def residual(X, Q, s, axis: str):
    """R = fl(X - x_hat), element-wise, no fused multiply-add."""
    return np.asarray(X, dtype=F32) - dequantize(Q, s, axis)


# --------------------------------------------------------------------------
# Step 7: GetAvgVec  (Sec. 3.1.1 after Eq. avgQuan; Sec. 3.1.2 C_row, C_col)
# --------------------------------------------------------------------------
def abs_means(D_F):
    """D^row[i] = mean_j |D_F[i,j]|, D^col[j] = mean_i |D_F[i,j]|.

    Summed in float64, divided in float64, rounded once to float32.
    """
    a = np.abs(np.asarray(D_F, dtype=F32)).astype(np.float64)
    M, N = a.shape
    drow = (a.sum(axis=1) / N).astype(F32)
    dcol = (a.sum(axis=0) / M).astype(F32)
    return drow, dcol


# --------------------------------------------------------------------------
# Step 8: Reduce  (Eq. avgQuan)
# --------------------------------------------------------------------------
def thresholds(theta, dvec):
    """t_v = fl(theta * D_v)."""
    return F32(theta) * np.asarray(dvec, dtype=F32)


def select_mask(X, thresh, axis: str, signed_compare: bool = False):
    """Boolean mask of the entries of X that are kept in the reduced operand.

    axis = "row": thresh has one entry per row (operand A);
    axis = "col": one per column (operand B).  An entry is kept iff
    |x| > thresh_v; entries that do not exceed it are "reduced" (dropped).
    ``signed_compare`` uses x instead of |x| (replay of the printed example).
    """
    X = np.asarray(X, dtype=F32)
    t = np.asarray(thresh, dtype=F32).reshape((-1, 1) if axis == "row" else (1, -1))
    v = X if signed_compare else np.abs(X)
    return v > t


@dataclasses.dataclass
class Compressed:
    """CSR of an (n_vec x n_elem) matrix whose vectors are rows (operand A) or
    columns (operand B, i.e. CSC of B' = CSR of B'^T).  idx ascending in each
    vector.  Entries whose code is 0 but whose mask is true are stored."""
    ptr: np.ndarray   # int32 [n_vec+1]
    idx: np.ndarray   # int32 [nnz]
    val: np.ndarray   # int8  [nnz]
    n_vec: int
    n_elem: int

    @property
    def nnz(self) -> int:
        return int(self.ptr[-1])

    @property
    def density(self) -> float:
        tot = self.n_vec * self.n_elem
        return self.nnz / tot if tot else 0.0


def compress(mask, Q, axis: str) -> Compressed:
    """Compact the kept codes vector by vector (CSR for axis="row", CSC for
    axis="col")."""
    mask = np.asarray(mask, dtype=bool)
    Q = np.asarray(Q)
    if axis == "col":
        mask = mask.T
        Q = Q.T
    n_vec, n_elem = mask.shape
    counts = mask.sum(axis=1).astype(np.int64)
    ptr = np.zeros(n_vec + 1, dtype=np.int64)
    np.cumsum(counts, out=ptr[1:])
    if ptr[-1] >= 2 ** 31:
        raise OverflowError("nnz does not fit INT32 pointers")
    vi, ei = np.nonzero(mask)                       # row-major order: ascending idx per vector
    return Compressed(ptr.astype(np.int32), ei.astype(np.int32),
                      Q[vi, ei].astype(np.int8), n_vec, n_elem)


def decompress(c: Compressed, axis: str):
    """Dense int8 matrix of the reduced codes (zeros where dropped)."""
    out = np.zeros((c.n_vec, c.n_elem), dtype=np.int8)
    vec = np.repeat(np.arange(c.n_vec), np.diff(c.ptr.astype(np.int64)))
    out[vec, c.idx] = c.val
    return out.T.copy() if axis == "col" else out


# --------------------------------------------------------------------------
# Step 12: SpMM of the reduced operands with the residual codes
# --------------------------------------------------------------------------
def spmm_row_sparse(cA: Compressed, R_other):
    """DR1_int = A'_int . RB_int from the CSR of A', exact."""
    return int_matmul(decompress(cA, "row"), R_other)


def spmm_col_sparse(R_other, cB: Compressed):
    """DR2_int = RA_int . B'_int from the CSC of B', exact."""
    return int_matmul(R_other, decompress(cB, "col"))


# --------------------------------------------------------------------------
# Whole of Algorithm 1
# --------------------------------------------------------------------------
@dataclasses.dataclass
class Stages:
    qmax: int
    A_int: np.ndarray = None
    B_int: np.ndarray = None
    s_a: np.ndarray = None
    s_b: np.ndarray = None
    lam_a: np.ndarray = None
    lam_b: np.ndarray = None
    D_int: np.ndarray = None
    D_F: np.ndarray = None
    drow: np.ndarray = None
    dcol: np.ndarray = None
    RA: np.ndarray = None
    RB: np.ndarray = None
    RA_int: np.ndarray = None
    RB_int: np.ndarray = None
    s_ra: np.ndarray = None
    s_rb: np.ndarray = None
    t_a: np.ndarray = None
    t_b: np.ndarray = None
    csr_a: Compressed = None
    csc_b: Compressed = None
    dense_a: bool = False          # term 1 took the dense branch
    dense_b: bool = False          # term 2 took the dense branch
    DR1_int: np.ndarray = None
    DR2_int: np.ndarray = None
    C: np.ndarray = None


def quantized_product(A, B, bits=8, rounding=ROUND_NEAREST_EVEN, qmax=None,
                      scale_mode="vector") -> Stages:
    """Lines 1-3 of Algorithm 1: plain vector-wise quantized GEMM."""
    A = np.asarray(A, dtype=F32)
    B = np.asarray(B, dtype=F32)
    if A.shape[1] != B.shape[0]:
        raise ValueError("inner dimensions differ")
    qm = qmax_of_bits(bits) if qmax is None else int(qmax)
    check_k_bound(A.shape[1], qm)
    st = Stages(qmax=qm)
    ax_a, ax_b = ("row", "col") if scale_mode == "vector" else ("global", "global")
    st.A_int, st.s_a, st.lam_a = quantize_vectors(A, ax_a, qm, rounding)
    st.B_int, st.s_b, st.lam_b = quantize_vectors(B, ax_b, qm, rounding)
    if scale_mode != "vector":
        st.s_a = np.repeat(st.s_a, A.shape[0]); st.lam_a = np.repeat(st.lam_a, A.shape[0])
        st.s_b = np.repeat(st.s_b, B.shape[1]); st.lam_b = np.repeat(st.lam_b, B.shape[1])
    st.D_int = int_matmul(st.A_int, st.B_int)
    st.D_F = dequant_product(st.D_int, st.s_a, st.s_b)
    return st


def compensated_gemm(A, B, theta_a, theta_b=None, *, bits=8, rounding=ROUND_NEAREST_EVEN,
                     alpha=1.0, beta=0.0, C_in=None, dense_fallback_density=2.0,
                     qmax=None, scale_mode="vector", signed_compare=False,
                     thresh_a: Optional[np.ndarray] = None,
                     thresh_b: Optional[np.ndarray] = None) -> Stages:
    """Algorithm 1: D = alpha * (quantized A.B with sparse residual correction) + beta * C.

    theta_a / theta_b: the threshold of Eq. avgQuan for A and for B (the paper
    has a single theta; pass one value for both).  theta = +inf keeps nothing
    (plain quantized GEMM); theta = 0 keeps every non-zero entry.
    dense_fallback_density: Algorithm 1's limit "s".  A term whose reduced
    operand has density >= s is computed with the *unreduced* codes (the dense
    GEMM branch); values > 1 switch the branch off.
    thresh_a / thresh_b: if given, used instead of theta * D^row / theta * D^col
    (lets a test feed the same threshold vectors to two implementations).
    """
    if theta_b is None:
        theta_b = theta_a
    A = np.asarray(A, dtype=F32)
    B = np.asarray(B, dtype=F32)
    st = quantized_product(A, B, bits, rounding, qmax, scale_mode)
    qm = st.qmax
    M, K = A.shape
    N = B.shape[1]
    # residual matrices and their codes (lines 4-6)
    st.RA = residual(A, st.A_int, st.s_a, "row")
    st.RB = residual(B, st.B_int, st.s_b, "col")
    st.RA_int, st.s_ra, _ = quantize_vectors(st.RA, "row", qm, rounding)
    st.RB_int, st.s_rb, _ = quantize_vectors(st.RB, "col", qm, rounding)
    # average vectors and reduction (lines 7-10)
    st.drow, st.dcol = abs_means(st.D_F)
    st.t_a = thresholds(theta_a, st.drow) if thresh_a is None else np.asarray(thresh_a, F32)
    st.t_b = thresholds(theta_b, st.dcol) if thresh_b is None else np.asarray(thresh_b, F32)
    mask_a = select_mask(A, st.t_a, "row", signed_compare)
    mask_b = select_mask(B, st.t_b, "col", signed_compare)
    st.csr_a = compress(mask_a, st.A_int, "row")
    st.csc_b = compress(mask_b, st.B_int, "col")
    # residual products (lines 11-15), each term switching on its own density.  A threshold
    # factor of +inf means "no correction from this operand" (the plain quantized GEMM bound):
    # that term is dropped before the density switch is looked at, whatever the limit s is.
    skip_a = thresh_a is None and np.isinf(theta_a)
    skip_b = thresh_b is None and np.isinf(theta_b)
    st.dense_a = (not skip_a) and st.csr_a.density >= dense_fallback_density
    st.dense_b = (not skip_b) and st.csc_b.density >= dense_fallback_density
    if st.dense_a:
        st.DR1_int = int_matmul(st.A_int, st.RB_int)
    else:
        st.DR1_int = spmm_row_sparse(st.csr_a, st.RB_int)
    if st.dense_b:
        st.DR2_int = int_matmul(st.RA_int, st.B_int)
    else:
        st.DR2_int = spmm_col_sparse(st.RA_int, st.csc_b)
    # error compensation and the GEMM epilogue (lines 16-18)
    T1 = dequant_product(st.DR1_int, st.s_a, st.s_rb)
    T2 = dequant_product(st.DR2_int, st.s_ra, st.s_b)
    acc = (st.D_F + T1) + T2
    out = F32(alpha) * acc
    if beta != 0.0:
        if C_in is None:
            raise ValueError("beta != 0 needs C_in")
        out = out + F32(beta) * np.asarray(C_in, dtype=F32)
    st.C = out.astype(F32)
    return st


# --------------------------------------------------------------------------
# Error metrics (Sec. 3.1.2: E_r, E_delta)
# --------------------------------------------------------------------------
def error_abs(X_ref, X):
    """E_r = || X_ref - X ||_F, in float64."""
    d = np.asarray(X_ref, dtype=np.float64) - np.asarray(X, dtype=np.float64)
    return float(np.sqrt((d * d).sum()))


def error_rel(X_ref, X):
    """E_delta = E_r / || X_ref ||_F."""
    r = np.asarray(X_ref, dtype=np.float64)
    n = float(np.sqrt((r * r).sum()))
    return error_abs(X_ref, X) / n if n else 0.0
