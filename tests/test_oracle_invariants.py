"""Pins of the CPU oracle against what the definitions and the mathematics fix:
brute force on tiny inputs, closed forms, the theta = inf / theta = 0 bounds
(Eq. gemm_r), the residual bound (Eq. lambdaleq), the error decomposition of
Sec. 3.2, a scale-free special case, and monotonicity in theta (Sec. 5.2)."""

import numpy as np
import pytest

from oracle import srq_oracle as o
from paper_2403_06924_amd import workloads as wl

F32 = np.float32


# ---------------------------------------------------------------- integer products
def _brute_int_matmul(P, Q):
    M, K = P.shape
    N = Q.shape[1]
    out = [[0] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            acc = 0
            for k in range(K):
                acc += int(P[i, k]) * int(Q[k, j])
            out[i][j] = acc
    return np.array(out, dtype=np.int64)


@pytest.mark.parametrize("shape", [(7, 5, 9), (33, 17, 65), (1, 1, 1), (3, 40, 2)])
def test_int_matmul_brute_force(shape):
    M, N, K = shape
    rng = np.random.default_rng(sum(shape))
    P = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    Q = rng.integers(-127, 128, size=(K, N)).astype(np.int8)
    assert (o.int_matmul(P, Q) == _brute_int_matmul(P, Q)).all()


def test_int_matmul_worst_case_at_k_bound():
    K = (2 ** 31 - 1) // (127 * 127)                 # 133144, the largest K allowed
    o.check_k_bound(K, 127)
    with pytest.raises(OverflowError):
        o.check_k_bound(K + 1, 127)
    P = np.full((2, K), 127, dtype=np.int8)
    P[1] = -127
    Q = np.full((K, 2), 127, dtype=np.int8)
    Q[:, 1] = -127
    D = o.int_matmul(P, Q)
    v = K * 127 * 127
    assert D.tolist() == [[v, -v], [-v, v]] and v < 2 ** 31


# ---------------------------------------------------------------- quantization
def test_quantize_rounding_modes_and_ties():
    # amax = 127 makes lambda = s = 1, so codes are the rounded inputs themselves
    X = np.array([[127.0, 2.5, 3.5, -2.5, -0.5, 0.5, 1.5, -2.7, 2.7, 0.0]], dtype=F32)
    q, s, lam = o.quantize_vectors(X, "row", 127, o.ROUND_NEAREST_EVEN)
    assert lam[0] == 1 and s[0] == 1
    assert q.tolist() == [[127, 2, 4, -2, 0, 0, 2, -3, 3, 0]]
    q, _, _ = o.quantize_vectors(X, "row", 127, o.ROUND_TRUNC)
    assert q.tolist() == [[127, 2, 3, -2, 0, 0, 1, -2, 2, 0]]


def test_quantize_axes_are_independent_vectors():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((6, 11)).astype(F32)
    q, s, lam = o.quantize_vectors(X, "row")
    for i in range(6):
        qi, si, li = o.quantize_vectors(X[i:i + 1], "row")
        assert (qi[0] == q[i]).all() and si[0] == s[i] and li[0] == lam[i]
        assert s[i] == np.abs(X[i]).max() / F32(127)
        assert np.abs(q[i]).max() == 127
    qc, sc, lc = o.quantize_vectors(X, "col")
    qt, st_, lt = o.quantize_vectors(X.T.copy(), "row")
    assert (qc == qt.T).all() and (sc == st_).all() and (lc == lt).all()


def test_quantize_zero_vector_and_bits():
    X = np.zeros((2, 4), dtype=F32)
    X[1] = [1, -2, 3, -4]
    q, s, lam = o.quantize_vectors(X, "row", o.qmax_of_bits(4))
    assert s[0] == 0 and lam[0] == 0 and (q[0] == 0).all()
    assert o.qmax_of_bits(4) == 7 and np.abs(q[1]).max() == 7
    assert q[1].tolist() == [2, -4, 5, -7]           # 1.75 -> 2, 3.5 -> 4 (even), 5.25 -> 5


def test_residual_bound_eq_lambdaleq():
    """|r| <= s/2 for nearest rounding, |r| < s and sign(r) = sign(x) for
    truncation (the paper's bound |ra| <= 1/lambda), up to one float32 rounding."""
    A, _ = wl.make_inputs("C3", 64, 64, 512)
    for rounding, bound in ((o.ROUND_NEAREST_EVEN, 0.5), (o.ROUND_TRUNC, 1.0)):
        q, s, _ = o.quantize_vectors(A, "row", 127, rounding)
        r = o.residual(A, q, s, "row").astype(np.float64)
        lim = bound * s.astype(np.float64).reshape(-1, 1) * (1 + 1e-5)
        assert (np.abs(r) <= lim).all()
        if rounding == o.ROUND_TRUNC:
            big = np.abs(r) > 1e-6 * s.reshape(-1, 1)
            assert (np.sign(r[big]) == np.sign(A[big])).all()


# ---------------------------------------------------------------- product, means
def test_dequant_product_and_means_closed_form():
    D = np.array([[1, -2, 3], [-4, 5, -6]], dtype=np.int64)
    sa = np.array([0.5, 2.0], dtype=F32)
    sb = np.array([1.0, 0.25, 4.0], dtype=F32)
    DF = o.dequant_product(D, sa, sb)
    assert DF.tolist() == [[0.5, -0.25, 6.0], [-8.0, 2.5, -48.0]]
    drow, dcol = o.abs_means(DF)
    assert drow.tolist() == [F32(6.75 / 3), F32(58.5 / 3)]
    assert dcol.tolist() == [4.25, 1.375, 27.0]


def test_dequant_rounds_large_integers_to_float32_first():
    D = np.array([[2 ** 24 + 1]], dtype=np.int64)          # not representable in binary32
    out = o.dequant_product(D, np.array([1.0], F32), np.array([1.0], F32))
    assert out[0, 0] == F32(2 ** 24)


# ---------------------------------------------------------------- selection, CSR
def test_selection_is_strict_and_absolute():
    X = np.array([[1.0, -1.0, 0.5, -2.0, 0.0]], dtype=F32)
    m = o.select_mask(X, np.array([1.0], F32), "row")
    assert m.tolist() == [[False, False, False, True, False]]
    m = o.select_mask(X, np.array([0.0], F32), "row")
    assert m.tolist() == [[True, True, True, True, False]]
    m = o.select_mask(X, np.array([np.inf], F32), "row")
    assert not m.any()


def test_compress_layout_and_roundtrip():
    rng = np.random.default_rng(11)
    Q = rng.integers(-127, 128, size=(9, 13)).astype(np.int8)
    Q[2, 3] = 0
    mask = rng.random((9, 13)) < 0.3
    mask[2, 3] = True                                       # kept entry whose code is zero
    mask[5] = False                                         # empty row
    for axis in ("row", "col"):
        c = o.compress(mask, Q, axis)
        m2 = mask if axis == "row" else mask.T
        q2 = Q if axis == "row" else Q.T
        assert c.ptr[0] == 0 and c.nnz == mask.sum()
        for v in range(m2.shape[0]):
            idx = c.idx[c.ptr[v]:c.ptr[v + 1]]
            assert idx.tolist() == np.nonzero(m2[v])[0].tolist()      # ascending, complete
            assert (c.val[c.ptr[v]:c.ptr[v + 1]] == q2[v, idx]).all()
        assert (o.decompress(c, axis) == np.where(mask, Q, 0)).all()
    c = o.compress(mask, Q, "row")
    assert c.ptr[6] - c.ptr[5] == 0
    assert 3 in c.idx[c.ptr[2]:c.ptr[3]].tolist()


def test_spmm_against_loops_over_the_compressed_form():
    rng = np.random.default_rng(3)
    M, N, K = 6, 7, 10
    Aq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    Bq = rng.integers(-127, 128, size=(K, N)).astype(np.int8)
    RAq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    RBq = rng.integers(-127, 128, size=(K, N)).astype(np.int8)
    ca = o.compress(rng.random((M, K)) < 0.4, Aq, "row")
    cb = o.compress(rng.random((K, N)) < 0.4, Bq, "col")
    d1 = np.zeros((M, N), dtype=np.int64)
    for i in range(M):
        for p in range(ca.ptr[i], ca.ptr[i + 1]):
            for j in range(N):
                d1[i, j] += int(ca.val[p]) * int(RBq[ca.idx[p], j])
    d2 = np.zeros((M, N), dtype=np.int64)
    for j in range(N):
        for p in range(cb.ptr[j], cb.ptr[j + 1]):
            for i in range(M):
                d2[i, j] += int(RAq[i, cb.idx[p]]) * int(cb.val[p])
    assert (o.spmm_row_sparse(ca, RBq) == d1).all()
    assert (o.spmm_col_sparse(RAq, cb) == d2).all()


# ---------------------------------------------------------------- bounds of the method
@pytest.fixture(scope="module")
def small_case():
    A, B = wl.make_inputs("C3", 96, 80, 160)
    return A, B


def test_theta_inf_is_plain_vectorwise_int8(small_case):
    A, B = small_case
    st = o.compensated_gemm(A, B, np.inf)
    plain = o.quantized_product(A, B)
    assert st.csr_a.nnz == 0 and st.csc_b.nnz == 0
    assert not st.DR1_int.any() and not st.DR2_int.any()
    assert (st.C == plain.D_F).all()
    # and the plain product is what the definitions give, element by element
    i, j = 5, 7
    acc = sum(int(plain.A_int[i, k]) * int(plain.B_int[k, j]) for k in range(A.shape[1]))
    assert plain.D_int[i, j] == acc
    assert plain.D_F[i, j] == F32(acc) * (plain.s_a[i] * plain.s_b[j])


def test_theta_zero_is_dense_residual_compensation(small_case):
    A, B = small_case
    st = o.compensated_gemm(A, B, 0.0)
    assert st.csr_a.nnz == np.count_nonzero(A) and st.csc_b.nnz == np.count_nonzero(B)
    assert (st.DR1_int == _brute_int_matmul(st.A_int, st.RB_int)).all()
    assert (st.DR2_int == _brute_int_matmul(st.RA_int, st.B_int)).all()
    # first three terms of Eq. gemm_r, evaluated in float64 from the stage outputs
    sa, sb = st.s_a.astype(np.float64)[:, None], st.s_b.astype(np.float64)[None, :]
    sra, srb = st.s_ra.astype(np.float64)[:, None], st.s_rb.astype(np.float64)[None, :]
    ref = st.D_int * sa * sb + st.DR1_int * sa * srb + st.DR2_int * sra * sb
    assert o.error_rel(ref, st.C) < 5e-7
    # the dense branch of Algorithm 1 gives the same integers whatever theta is
    st2 = o.compensated_gemm(A, B, 3.0, dense_fallback_density=0.0)
    assert st2.dense_a and st2.dense_b
    assert (st2.DR1_int == st.DR1_int).all() and (st2.DR2_int == st.DR2_int).all()
    assert (st2.C == st.C).all()


def test_error_decomposition_sec_3_2(small_case):
    """A.B - C(theta=0) = RA.RB + A_hat.(RB - RB_hat) + (RA - RA_hat).B_hat,
    an exact identity in real arithmetic: checks every sign, scale pairing and
    operand order of the compensated sum."""
    A, B = small_case
    st = o.compensated_gemm(A, B, 0.0)
    f = np.float64
    Ah = st.A_int.astype(f) * st.s_a.astype(f)[:, None]
    Bh = st.B_int.astype(f) * st.s_b.astype(f)[None, :]
    RA, RB = A.astype(f) - Ah, B.astype(f) - Bh
    RAh = st.RA_int.astype(f) * st.s_ra.astype(f)[:, None]
    RBh = st.RB_int.astype(f) * st.s_rb.astype(f)[None, :]
    lhs = A.astype(f) @ B.astype(f) - st.C.astype(f)
    rhs = RA @ RB + Ah @ (RB - RBh) + (RA - RAh) @ Bh
    C64 = A.astype(f) @ B.astype(f)
    tol = 1e-6 * (np.abs(C64) + np.abs(C64).mean())           # float32 rounding of C only
    assert (np.abs(lhs - rhs) < tol).all()
    assert np.abs(rhs).max() > 50 * tol.mean()                # the identity is not vacuous
    # and the omitted part is far below the plain quantization error
    assert o.error_rel(C64, st.C) < 0.05 * o.error_rel(C64, st.D_F)


def test_scale_free_case_reduces_to_integer_matmul():
    """Integer inputs whose every row of A / column of B reaches +-127 have
    lambda = s = 1: codes equal the inputs, residuals vanish, and the whole path
    is the integer product."""
    rng = np.random.default_rng(9)
    M, N, K = 12, 10, 31
    Ai = rng.integers(-127, 128, size=(M, K))
    Bi = rng.integers(-127, 128, size=(K, N))
    Ai[:, 0] = 127
    Bi[0, :] = -127
    for theta in (0.0, 0.1, np.inf):
        st = o.compensated_gemm(Ai.astype(F32), Bi.astype(F32), theta)
        assert (st.s_a == 1).all() and (st.s_b == 1).all()
        assert (st.A_int == Ai).all() and (st.B_int == Bi).all()
        assert not st.RA.any() and not st.RB_int.any() and (st.s_rb == 0).all()
        assert (st.C == (Ai @ Bi).astype(F32)).all()


def test_alpha_beta_epilogue(small_case):
    A, B = small_case
    rng = np.random.default_rng(2)
    Cin = rng.standard_normal((A.shape[0], B.shape[1])).astype(F32)
    base = o.compensated_gemm(A, B, 0.5)
    st = o.compensated_gemm(A, B, 0.5, alpha=0.75, beta=-1.5, C_in=Cin)
    assert (st.C == F32(0.75) * base.C + F32(-1.5) * Cin).all()
    with pytest.raises(ValueError):
        o.compensated_gemm(A, B, 0.5, beta=1.0)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_error_non_increasing_as_theta_falls(name):
    A, B = wl.make_inputs(name, 128, 144, 256)
    C64 = A.astype(np.float64) @ B.astype(np.float64)
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    errs, dens = [], []
    for d in (0.0, 0.01, 0.05, 0.2, 0.5, 1.0):
        ta = wl.theta_for_density(A, drow, "row", d)
        tb = wl.theta_for_density(B, dcol, "col", d)
        st = o.compensated_gemm(A, B, ta, tb)
        errs.append(o.error_rel(C64, st.C))
        dens.append((st.csr_a.density, st.csc_b.density))
        assert abs(st.csr_a.density - d) < 2e-3 and abs(st.csc_b.density - d) < 2e-3
    assert errs[0] == o.error_rel(C64, plain.D_F)
    for hi, lo in zip(errs[:-1], errs[1:]):
        assert lo <= hi * 1.01
    assert errs[-1] < 0.2 * errs[0]


def test_dense_fallback_switch_is_per_term():
    A, B = wl.make_inputs("C4", 64, 96, 128)
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    ta = wl.theta_for_density(A, drow, "row", 0.30)
    tb = wl.theta_for_density(B, dcol, "col", 0.02)
    st = o.compensated_gemm(A, B, ta, tb, dense_fallback_density=0.1)
    assert st.dense_a and not st.dense_b
    assert (st.DR1_int == o.int_matmul(st.A_int, st.RB_int)).all()
    assert (st.DR2_int == o.spmm_col_sparse(st.RA_int, st.csc_b)).all()


def test_thresholds_override_feeds_selection():
    A, B = wl.make_inputs("C2", 40, 48, 64)
    st = o.compensated_gemm(A, B, 0.7)
    st2 = o.compensated_gemm(A, B, 123.0, thresh_a=st.t_a, thresh_b=st.t_b)
    assert (st2.csr_a.idx == st.csr_a.idx).all() and (st2.C == st.C).all()
    assert (st.t_a == F32(0.7) * st.drow).all()


def test_int4_path_has_larger_error_than_int8():
    A, B = wl.make_inputs("C2", 64, 64, 128)
    C64 = A.astype(np.float64) @ B.astype(np.float64)
    e8 = o.error_rel(C64, o.compensated_gemm(A, B, 0.0, bits=8).C)
    st4 = o.compensated_gemm(A, B, 0.0, bits=4)
    assert np.abs(st4.A_int).max() == 7 and np.abs(st4.RB_int).max() == 7
    assert e8 < o.error_rel(C64, st4.C) < o.error_rel(C64, o.quantized_product(A, B, bits=4).D_F)


def test_workload_recipes_are_seeded_and_shaped():
    for name in wl.WORKLOADS:
        A, B = wl.make_inputs(name, 32, 48, 64)
        A2, B2 = wl.make_inputs(name, 32, 48, 64)
        assert A.shape == (32, 64) and B.shape == (64, 48)
        assert A.dtype == np.float32 and (A == A2).all() and (B == B2).all()
    A, _ = wl.make_inputs("C4", 64, 8, 256)
    colmax = np.abs(A).max(axis=0)
    assert (colmax > 20).sum() == 16                           # the 16 outlier columns
    A, _ = wl.make_inputs("C5", 64, 8, 64)
    assert np.abs(A).min() >= 2.0 ** -10 and np.abs(A).max() < 2.0 ** 11


def test_infinite_threshold_drops_the_term_before_the_density_switch():
    """theta = +inf is the plain quantized product whatever the limit s of Algorithm 1's switch
    is: with s = 0 ("always dense") a term whose operand keeps nothing is still dropped, and the
    other term still takes the dense branch."""
    rng = np.random.default_rng(3)
    A = rng.standard_normal((20, 33)).astype(np.float32)
    B = rng.standard_normal((33, 17)).astype(np.float32)
    plain = o.quantized_product(A, B)
    both = o.compensated_gemm(A, B, np.inf, np.inf, dense_fallback_density=0.0)
    assert (both.C == plain.D_F).all() and not both.DR1_int.any() and not both.DR2_int.any()
    one = o.compensated_gemm(A, B, 0.5, np.inf, dense_fallback_density=0.0)
    assert one.dense_a and not one.dense_b and not one.DR2_int.any()
    assert (one.DR1_int == o.int_matmul(one.A_int, one.RB_int)).all()
    assert (one.C == (plain.D_F + o.dequant_product(one.DR1_int, one.s_a, one.s_rb))).all()
