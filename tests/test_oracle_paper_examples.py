"""Pins of the CPU oracle against the values the paper prints.

1-D example: Sec. 2.3.  3x3 example: Sec. 3.1.2 (one scale per matrix, code
range +-64, truncation, signed selection compare - all reproduced through the
oracle's replay switches).  The example's printed inputs are rounded to four
decimals, so intermediate values are pinned to 5e-5 and the two arg-max codes
(printed 64 / 63) to +-1; the corrected matrix, which the paper's own figures do
not reproduce exactly, is pinned structurally: the chosen reading lands within
8e-3 while each alternative reading misses by more than 5e-2.
"""
import numpy as np
import pytest

from oracle import srq_oracle as o

F32 = np.float32


def test_1d_example(golden_1d):
    g = golden_1d
    V = g["V"].astype(F32)
    q, s, lam = o.quantize_vectors(V, "row", qmax=o.qmax_of_bits(8), rounding=o.ROUND_TRUNC)
    assert o.qmax_of_bits(8) == 127
    assert lam[0] == F32(g["lambda"][0, 0])                      # 31.75 exactly
    assert int(q[0, 1]) == int(g["code_of_2p5"][0, 0])            # floor(79.375) = 79
    deq = o.dequantize(q, s, "row")
    assert abs(float(deq[0, 1]) - g["dequant_of_79"][0, 0]) < 5e-5
    r = o.residual(V, q, s, "row")
    np.testing.assert_allclose(r, g["residual"], atol=5e-5)
    # nearest-even rounding would give 79 as well here but 32 for 1*31.75
    q2, _, _ = o.quantize_vectors(V, "row", 127, o.ROUND_NEAREST_EVEN)
    assert q2.tolist() == [[32, 79, 127]]
    assert q.tolist() == [[31, 79, 127]]


def _example_inputs(g):
    A = g["A"].copy()
    A[1, 1] = g["max_A"][0, 0]          # the paper prints the unrounded maximum separately
    return A.astype(F32), g["B"].astype(F32)


def test_3x3_quantize_global(golden_3x3):
    g = golden_3x3
    A, B = _example_inputs(g)
    qa, sa, la = o.quantize_vectors(A, "global", 64, o.ROUND_TRUNC)
    qb, sb, lb = o.quantize_vectors(B, "global", 64, o.ROUND_TRUNC)
    assert abs(float(la[0]) - g["lambda_A"][0, 0]) < 5e-5
    assert abs(float(lb[0]) - g["lambda_B"][0, 0]) < 5e-5
    da = qa.astype(int) - g["A_int8"].astype(int)
    db = qb.astype(int) - g["B_int8"].astype(int)
    # every code equals the printed one except the two arg-max entries (+-1)
    assert np.abs(da).sum() <= 1 and (da != 0).sum() == (da[1, 1] != 0)
    assert np.abs(db).sum() <= 1 and (db != 0).sum() == (db[0, 0] != 0)
    # nearest-even rounding does not reproduce the printed codes (e.g. 4.93 -> 4)
    qa_rne, _, _ = o.quantize_vectors(A, "global", 64, o.ROUND_NEAREST_EVEN)
    assert (qa_rne.astype(int) != g["A_int8"].astype(int)).sum() >= 3


def test_3x3_product_dequant_and_means(golden_3x3):
    g = golden_3x3
    A, B = _example_inputs(g)
    _, sa, _ = o.quantize_vectors(A, "global", 64, o.ROUND_TRUNC)
    _, sb, _ = o.quantize_vectors(B, "global", 64, o.ROUND_TRUNC)
    Aq = g["A_int8"].astype(np.int8)
    Bq = g["B_int8"].astype(np.int8)
    D_int = o.int_matmul(Aq, Bq)
    D_F = o.dequant_product(D_int, np.repeat(sa, 3), np.repeat(sb, 3))
    np.testing.assert_allclose(D_F, g["C_quant"], atol=6e-5)
    drow, dcol = o.abs_means(D_F)
    np.testing.assert_allclose(drow, g["C_row"][0], atol=6e-5)
    np.testing.assert_allclose(dcol, g["C_col"][0], atol=6e-5)
    # a transposed operand or swapped mean axes would not pass
    assert np.abs(o.dequant_product(o.int_matmul(Bq, Aq), np.repeat(sa, 3),
                                    np.repeat(sb, 3)) - g["C_quant"]).max() > 1e-2
    assert np.abs(dcol - g["C_row"][0]).max() > 1e-2


def test_3x3_dequant_and_residuals(golden_3x3):
    g = golden_3x3
    A, B = _example_inputs(g)
    _, sa, _ = o.quantize_vectors(A, "global", 64, o.ROUND_TRUNC)
    _, sb, _ = o.quantize_vectors(B, "global", 64, o.ROUND_TRUNC)
    Aq = g["A_int8"].astype(np.int8)
    Bq = g["B_int8"].astype(np.int8)
    np.testing.assert_allclose(o.dequantize(Aq, sa, "global"), g["A_deq"], atol=6e-5)
    np.testing.assert_allclose(o.dequantize(Bq, sb, "global"), g["B_deq"], atol=6e-5)
    # residuals inherit the 4-decimal rounding of the printed inputs as well (2 x 5e-5)
    np.testing.assert_allclose(o.residual(A, Aq, sa, "global"), g["RA"], atol=1.1e-4)
    np.testing.assert_allclose(o.residual(B, Bq, sb, "global"), g["RB"], atol=1.1e-4)
    # a sign slip (x_hat - x) would be off by twice the residual
    assert np.abs(-o.residual(B, Bq, sb, "global") - g["RB"]).max() > 0.1


@pytest.mark.parametrize("theta", [0.2414, 0.30, 0.3538])
def test_3x3_selection_pattern(golden_3x3, theta):
    g = golden_3x3
    A, B = _example_inputs(g)
    drow = g["C_row"][0].astype(F32)
    dcol = g["C_col"][0].astype(F32)
    ma = o.select_mask(A, o.thresholds(theta, drow), "row", signed_compare=True)
    mb = o.select_mask(B, o.thresholds(theta, dcol), "col", signed_compare=True)
    assert (ma == (g["A_r"] != 0)).all()
    assert (mb == (g["B_r"] != 0)).all()
    ca = o.compress(ma, g["A_int8"].astype(np.int8), "row")
    cb = o.compress(mb, g["B_int8"].astype(np.int8), "col")
    assert (o.decompress(ca, "row") == g["A_r_int"]).all()
    assert (o.decompress(cb, "col") == g["B_r_int"]).all()
    assert ca.nnz == 4 and cb.nnz == 2
    # the |x| compare this build uses keeps the large negative entries as well
    ma_abs = o.select_mask(A, o.thresholds(theta, drow), "row")
    assert ma_abs.sum() > ma.sum() and (ma_abs | ma == ma_abs).all()


def test_3x3_selection_outside_theta_window(golden_3x3):
    g = golden_3x3
    A, _ = _example_inputs(g)
    drow = g["C_row"][0].astype(F32)
    for theta in (0.23, 0.36):
        ma = o.select_mask(A, o.thresholds(theta, drow), "row", signed_compare=True)
        assert not (ma == (g["A_r"] != 0)).all()


def test_3x3_corrected_product_structure(golden_3x3):
    """C' = C_q + A'.RB + RA.B' reproduces the printed corrected matrix; the
    alternatives (printed operand order B'.RA; sparsifying the residuals
    instead of the operands) do not."""
    g = golden_3x3
    A, B = _example_inputs(g)
    st = o.compensated_gemm(A, B, 0.30, qmax=64, rounding=o.ROUND_TRUNC,
                            scale_mode="global", signed_compare=True)
    P = g["C_quant_corrected"]
    # the driver's own codes differ from the printed ones at the two arg-max entries
    # (one quantum each), which the correction mostly absorbs
    assert np.abs(st.C.astype(np.float64) - P).max() < 2e-2
    # structure, from the printed codes and float residuals
    la, lb = 64 / g["max_A"][0, 0], 64 / g["max_B"][0, 0]
    Aq, Bq = g["A_int8"], g["B_int8"]
    ma, mb = g["A_r"] != 0, g["B_r"] != 0
    RA, RB = A - Aq / la, B - Bq / lb
    Cq = (Aq @ Bq) / (la * lb)
    good = Cq + (ma * Aq / la) @ RB + RA @ (mb * Bq / lb)
    swapped = Cq + (ma * Aq / la) @ RB + (mb * Bq / lb) @ RA
    sparse_resid = Cq + (ma * RA) @ (Bq / lb) + (Aq / la) @ (mb * RB)
    assert np.abs(good - P).max() < 8e-3
    assert np.abs(swapped - P).max() > 5e-2
    assert np.abs(sparse_resid - P).max() > 5e-2
    # the oracle's quantized-residual version of the same structure agrees with it
    RAq, sra, _ = o.quantize_vectors(RA.astype(F32), "global", 64, o.ROUND_TRUNC)
    RBq, srb, _ = o.quantize_vectors(RB.astype(F32), "global", 64, o.ROUND_TRUNC)
    t1 = o.int_matmul(ma * Aq, RBq) * (1 / la) * float(srb[0])
    t2 = o.int_matmul(RAq, mb * Bq) * float(sra[0]) * (1 / lb)
    assert np.abs(Cq + t1 + t2 - P).max() < 1.2e-2


def test_3x3_error_table(golden_3x3):
    g = golden_3x3
    A, B = _example_inputs(g)
    C64 = A.astype(np.float64) @ B.astype(np.float64)
    st = o.compensated_gemm(A, B, 0.30, qmax=64, rounding=o.ROUND_TRUNC,
                            scale_mode="global", signed_compare=True)
    e_direct = o.error_rel(C64, st.D_F)
    e_comp = o.error_rel(C64, st.C)
    assert abs(e_direct - g["E_delta_direct"][0, 0]) < 1e-3       # printed 0.035
    assert abs(e_comp - g["E_delta_residual"][0, 0]) < 2.5e-3     # printed 0.011
    # the printed matrices themselves give the printed relative errors
    assert abs(o.error_rel(g["C_fp32"], g["C_quant"]) - 0.035) < 1e-3
    assert abs(o.error_rel(g["C_fp32"], g["C_quant_corrected"]) - 0.011) < 1e-3
