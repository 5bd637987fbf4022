"""Parity at the full sizes of the seeded workloads, in the launch configuration bench.py
times (srq_compensated_gemm, SRQ_STRATEGY_AUTO, debug outputs off on the timed call).

C2 (2048^3) is compared element by element at every listed density and at both bounds.
C3 (8192^3, the headline workload), C4 (4096 x 14336 x 4096) and C5 (16384^3) are compared on
sampled rows and columns that the oracle computes one by one from the definitions: codes and
scales of every vector (cheap element-wise passes), and for the sampled vectors the INT32
products, the means, the compressed selection and the final FP32 output."""
import numpy as np
import pytest

from oracle import srq_oracle as o
from paper_2403_06924_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
F32 = np.float32
REL_TOL = 1e-5
MEAN_TOL = 1e-6


@pytest.fixture(scope="module")
def srq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2403_06924_amd import binding as b
    h = b.Srq(device=0)
    yield h
    h.close()


@pytest.fixture(scope="module")
def b():
    from paper_2403_06924_amd import binding
    return binding


def host(t):
    return t.detach().cpu().numpy()


def gpu_thetas(srq, b, Ad, Bd, density):
    """theta_a, theta_b for a target density, calibrated like bench.py does (harness only)."""
    Qa, sa, _ = srq.quantize(Ad, b.AXIS_ROW)
    Qb, sb, _ = srq.quantize(Bd, b.AXIS_COL)
    _, _, drow, dcol = srq.gemm_i8(Qa, sa, Qb, sb)

    return wl.theta_for_density(Ad, drow, 0, density), wl.theta_for_density(Bd, dcol, 1, density)


@pytest.mark.parametrize("density", [0.01, 0.05, 0.20])
def test_c2_full_every_density(srq, b, density):
    A, B = wl.make_inputs("C2")
    Ad, Bd = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    ta, tb = gpu_thetas(srq, b, Ad, Bd, density)
    stats = b.stats_tensor()
    C, _, dbg = srq.compensated_gemm(Ad, Bd, ta, tb, strategy=b.STRATEGY_AUTO, stats=stats, debug=True)
    torch.cuda.synchronize()
    M, K = A.shape
    N = B.shape[1]
    im = srq.intermediates(M, N, K)
    st = b.read_stats(stats)
    ref = o.compensated_gemm(A, B, ta, tb, thresh_a=host(im["t_a"]), thresh_b=host(im["t_b"]))
    assert (host(im["A_int"]) == ref.A_int).all() and (host(im["B_int"]) == ref.B_int.T).all()
    assert (host(im["s_a"]) == ref.s_a).all() and (host(im["s_rb"]) == ref.s_rb).all()
    assert (host(dbg["D_int"]) == ref.D_int).all()
    np.testing.assert_allclose(host(im["drow"]), ref.drow, rtol=MEAN_TOL)
    np.testing.assert_allclose(host(im["dcol"]), ref.dcol, rtol=MEAN_TOL)
    assert st["nnz_a"] == ref.csr_a.nnz and st["nnz_b"] == ref.csc_b.nnz
    assert abs(ref.csr_a.density - density) < 2e-3 and abs(ref.csc_b.density - density) < 2e-3
    for side, c in (("a", ref.csr_a), ("b", ref.csc_b)):
        assert (host(im[side + "_ptr"]) == c.ptr).all()
        assert (host(im[side + "_idx"]) == c.idx).all()
        assert (host(im[side + "_val"]) == c.val).all()
    assert (host(dbg["DR1_int"]) == ref.DR1_int).all() and (host(dbg["DR2_int"]) == ref.DR2_int).all()
    assert o.error_rel(ref.C, host(C)) <= REL_TOL
    # the timed configuration (no debug outputs) gives the same bits
    C2, _, _ = srq.compensated_gemm(Ad, Bd, ta, tb, strategy=b.STRATEGY_AUTO)
    torch.cuda.synchronize()
    assert torch.equal(C, C2)
    # error versus the exact product falls with the correction
    C64 = A.astype(np.float64) @ B.astype(np.float64)
    assert o.error_rel(C64, host(C)) < o.error_rel(C64, ref.D_F)


def test_c2_full_bounds(srq, b):
    A, B = wl.make_inputs("C2")
    Ad, Bd = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    inf = float("inf")
    C, _, _ = srq.compensated_gemm(Ad, Bd, inf, inf)
    plain = o.quantized_product(A, B)
    assert (host(C) == plain.D_F).all()                                   # theta = inf: plain INT8
    C0, _, dbg = srq.compensated_gemm(Ad, Bd, 0.0, 0.0, strategy=b.STRATEGY_AUTO, debug=True)
    torch.cuda.synchronize()
    ref0 = o.compensated_gemm(A, B, 0.0)
    assert (host(dbg["DR1_int"]) == ref0.DR1_int).all() and (host(dbg["DR2_int"]) == ref0.DR2_int).all()
    assert o.error_rel(ref0.C, host(C0)) <= REL_TOL                       # theta = 0: dense compensation
    Cd, _, _ = srq.compensated_gemm(Ad, Bd, 0.7, 0.7, dense_fallback_density=0.0)
    torch.cuda.synchronize()
    assert torch.equal(Cd, C0)                                            # the dense branch gives the same


def sampled_check(srq, b, name, density, nsample, seed, strategy=None, bit_identical=True):
    """Full-size parity on what the oracle can compute one by one: every element-wise stage and the
    compressed selection of every vector in full; the INT32 products, the means and the final FP32
    output C on `nsample` sampled rows and `nsample` sampled columns (C is NOT compared on the other
    rows and columns at these sizes: the oracle's three integer products of a whole 8192^3 or 16384^3
    problem do not fit a test's time)."""
    w = wl.WORKLOADS[name]
    M, N, K = w.M, w.N, w.K
    A, B = wl.make_inputs(name)
    Ad, Bd = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    ta, tb = gpu_thetas(srq, b, Ad, Bd, density)
    stats = b.stats_tensor()
    Cd, _, _ = srq.compensated_gemm(Ad, Bd, ta, tb, strategy=b.STRATEGY_AUTO if strategy is None else strategy,
                                    stats=stats, max_density=min(1.0, density * 1.25 + 0.01))
    torch.cuda.synchronize()
    st = b.read_stats(stats)
    im = srq.intermediates(M, N, K)
    # ---- element-wise stages in full
    A_int, s_a, lam_a = o.quantize_vectors(A, "row")
    assert (host(im["s_a"]) == s_a).all() and (host(im["lam_a"]) == lam_a).all()
    assert (host(im["A_int"]) == A_int).all()
    B_int, s_b, lam_b = o.quantize_vectors(B, "col")
    assert (host(im["s_b"]) == s_b).all() and (host(im["lam_b"]) == lam_b).all()
    assert (host(im["B_int"]) == B_int.T).all()
    RA_int, s_ra, _ = o.quantize_vectors(o.residual(A, A_int, s_a, "row"), "row")
    RB_int, s_rb, _ = o.quantize_vectors(o.residual(B, B_int, s_b, "col"), "col")
    assert (host(im["s_ra"]) == s_ra).all() and (host(im["s_rb"]) == s_rb).all()
    if im["RA_int"] is not None:
        assert (host(im["RA_int"]) == RA_int).all()
    if im["RB_int"] is not None:
        assert (host(im["RB_int"]) == RB_int.T).all()
    # ---- selection of every vector from the GPU's thresholds, compressed form bit for bit
    t_a, t_b = host(im["t_a"]), host(im["t_b"])
    mask_a = o.select_mask(A, t_a, "row")
    mask_b = o.select_mask(B, t_b, "col")
    ca, cb = o.compress(mask_a, A_int, "row"), o.compress(mask_b, B_int, "col")
    assert st["nnz_a"] == ca.nnz and st["nnz_b"] == cb.nnz
    assert abs(ca.density - density) < 3e-3 and abs(cb.density - density) < 3e-3
    assert (host(im["a_ptr"]) == ca.ptr).all() and (host(im["b_ptr"]) == cb.ptr).all()
    assert (host(im["a_idx"]) == ca.idx).all() and (host(im["a_val"]) == ca.val).all()
    assert (host(im["b_idx"]) == cb.idx).all() and (host(im["b_val"]) == cb.val).all()
    # ---- sampled rows and columns, straight from the definitions
    rng = np.random.default_rng(seed)
    rows = np.sort(rng.choice(M, size=nsample, replace=False))
    cols = np.sort(rng.choice(N, size=nsample, replace=False))
    Ap = np.where(mask_a, A_int, 0).astype(np.int8)
    Bp = np.where(mask_b, B_int, 0).astype(np.int8)
    D_rows = o.dequant_product(o.int_matmul(A_int[rows], B_int), s_a[rows], s_b)
    D_cols = o.dequant_product(o.int_matmul(A_int, B_int[:, cols]), s_a, s_b[cols])
    drow = (np.abs(D_rows).astype(np.float64).sum(axis=1) / N).astype(F32)
    dcol = (np.abs(D_cols).astype(np.float64).sum(axis=0) / M).astype(F32)
    np.testing.assert_allclose(host(im["drow"])[rows], drow, rtol=MEAN_TOL)
    np.testing.assert_allclose(host(im["dcol"])[cols], dcol, rtol=MEAN_TOL)
    np.testing.assert_allclose(t_a[rows], F32(ta) * drow, rtol=2 * MEAN_TOL)
    np.testing.assert_allclose(t_b[cols], F32(tb) * dcol, rtol=2 * MEAN_TOL)
    T1 = o.dequant_product(o.int_matmul(Ap[rows], RB_int), s_a[rows], s_rb)
    T2 = o.dequant_product(o.int_matmul(RA_int[rows], Bp), s_ra[rows], s_b)
    C_rows = (D_rows + T1) + T2
    got = host(Cd[torch.from_numpy(rows).cuda()])
    assert o.error_rel(C_rows, got) <= REL_TOL
    if bit_identical:
        assert (got == C_rows).mean() > 0.999        # in practice bit-identical
    T1c = o.dequant_product(o.int_matmul(Ap, RB_int[:, cols]), s_a, s_rb[cols])
    T2c = o.dequant_product(o.int_matmul(RA_int, Bp[:, cols]), s_ra, s_b[cols])
    C_cols = (D_cols + T1c) + T2c
    gotc = host(Cd[:, torch.from_numpy(cols).cuda()])
    assert o.error_rel(C_cols, gotc) <= REL_TOL
    return st


def test_c3_headline_sampled(srq, b):
    st = sampled_check(srq, b, "C3", 0.05, 192, seed=11)
    assert st["path_a"] in (1, 2) and st["path_b"] in (1, 2)


def test_c3_structured_2to4_sampled(srq, b):
    """Full size, the launch configuration `bench.py --strategy smfmac` times: the 2:4 execution of
    both correction terms against the oracle on sampled rows and columns (codes, scales, compressed
    selection of every vector in full, as for the other strategies)."""
    st = sampled_check(srq, b, "C3", 0.05, 192, seed=11, strategy=b.STRATEGY_CSR_SMFMAC)
    assert st["path_a"] == 4 and st["path_b"] == 4


def test_c4_rectangular_sampled(srq, b):
    sampled_check(srq, b, "C4", 0.02, 128, seed=12)


def test_c4_column_block_sampled(srq, b):
    """C4 with the column-block split (the 16 outlier columns of A form the dense strip of term 1;
    B has no such structure, its strip stays empty and is skipped on the device)."""
    st = sampled_check(srq, b, "C4", 0.02, 128, seed=12, strategy=b.STRATEGY_COLBLOCK, bit_identical=False)
    assert st["path_a"] == 5 and st["path_b"] == 5


@pytest.mark.parametrize("density", [0.05, 0.20, 0.50])
def test_c5_wide_range_sampled(srq, b, density):
    sampled_check(srq, b, "C5", density, 48, seed=13)


@pytest.mark.parametrize("shape", [(5888, 5888, 384), (2560, 13312, 640), (4096, 4096, 256), (4352, 4096, 128),
                                   (4224, 4096, 256), (4096, 4200, 128), (4300, 4500, 128)])
def test_persistent_gemm_uneven_tile_counts(srq, b, shape):
    """529 and 520 tiles of 256 x 256 on 256 compute units: workgroups of the persistent kernel
    get different numbers of tiles, and the load cursor runs ahead across tile boundaries.
    The last three shapes are no multiples of 256: the persistent kernel takes the block of whole
    tiles, the plain kernel the strips of rows and columns beside it, and the partial sums of
    |D_F| of the three launches interleave.
    First mode (with the means) and accumulate mode (through the expanded sparse operand),
    element by element."""
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    Qa = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    Qb = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    sa = rng.random(M).astype(F32) + F32(0.01)
    sb = rng.random(N).astype(F32) + F32(0.01)
    dQa, dQb, dsa, dsb = (torch.from_numpy(x).cuda() for x in (Qa, Qb, sa, sb))
    D_F, _, drow, dcol = srq.gemm_i8(dQa, dsa, dQb, dsb)
    ref_int = o.int_matmul(Qa, Qb.T)
    ref_F = o.dequant_product(ref_int, sa, sb)
    assert (host(D_F) == ref_F).all()
    r_row, r_col = o.abs_means(ref_F)
    np.testing.assert_allclose(host(drow), r_row, rtol=MEAN_TOL)
    np.testing.assert_allclose(host(dcol), r_col, rtol=MEAN_TOL)
    # accumulate mode: C += (sparse rows of Qa) . Qb^T with 3 % of the entries kept
    mask = rng.random((M, K)) < 0.03
    c = o.compress(mask, Qa, "row")
    C0 = rng.standard_normal((M, N)).astype(F32)
    Cd = torch.from_numpy(C0).cuda()
    srq.spmm_accumulate(0, b.STRATEGY_CSR_MFMA, M, N, K, torch.from_numpy(c.ptr).cuda(),
                        torch.from_numpy(c.idx).cuda(), torch.from_numpy(c.val).cuda(), dQb, dsa, dsb, Cd)
    ref_C = C0 + o.dequant_product(o.int_matmul(np.where(mask, Qa, 0), Qb.T), sa, sb)
    assert (host(Cd) == ref_C).all()


@pytest.mark.parametrize("shape", [(4352, 4096, 200), (4096, 5120, 129), (4224, 4200, 129)])
@pytest.mark.parametrize("variant", ["mfma", "auto_sparse", "dense_branch"])
def test_padded_inner_dimension_through_persistent_kernels(srq, b, shape, variant):
    """K that is no multiple of 64 with M, N multiples of 256: the code matrices are padded to a
    leading dimension of 256 with zero columns and the persistent kernels run on the padded K.
    The timed configuration (no debug outputs), every path, element by element, with alpha and beta
    (on the matrix-core paths both terms share one launch, which applies them after the second)."""
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    A = (rng.standard_normal((M, K)) * np.exp(rng.standard_normal((M, 1)))).astype(F32)
    B = (rng.standard_normal((K, N)) * np.exp(rng.standard_normal((1, N)))).astype(F32)
    strategy, s, density = {"mfma": (b.STRATEGY_CSR_MFMA, 2.0, 0.05), "auto_sparse": (b.STRATEGY_AUTO, 2.0, 0.004),
                            "dense_branch": (b.STRATEGY_CSR_MFMA, 0.01, 0.05)}[variant]
    drow, dcol = o.abs_means(o.quantized_product(A, B).D_F)
    ta = wl.theta_for_density(A, drow, "row", density)
    tb = wl.theta_for_density(B, dcol, "col", density)
    stats = b.stats_tensor()
    Cin = rng.standard_normal((M, N)).astype(F32)
    C, _, _ = srq.compensated_gemm(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), ta, tb, strategy=strategy,
                                   dense_fallback_density=s, stats=stats, alpha=0.5, beta=-0.75,
                                   C_in=torch.from_numpy(Cin).cuda())
    torch.cuda.synchronize()
    im = srq.intermediates(M, N, K)
    st = b.read_stats(stats)
    assert im["ld_codes"] == 256
    ref = o.compensated_gemm(A, B, ta, tb, alpha=0.5, beta=-0.75, C_in=Cin, dense_fallback_density=s,
                             thresh_a=host(im["t_a"]), thresh_b=host(im["t_b"]))
    assert st["path_a"] == st["path_b"] == {"mfma": 2, "auto_sparse": 1, "dense_branch": 3}[variant]
    assert (host(im["A_int"]) == ref.A_int).all() and (host(im["B_int"]) == ref.B_int.T).all()
    assert st["nnz_a"] == ref.csr_a.nnz and st["nnz_b"] == ref.csc_b.nnz
    if variant == "dense_branch":                        # counted, not compacted
        assert im["a_idx"] is None and im["b_val"] is None
        assert (host(im["a_ptr"]) == ref.csr_a.ptr).all() and (host(im["b_ptr"]) == ref.csc_b.ptr).all()
    else:
        assert (host(im["a_idx"]) == ref.csr_a.idx).all() and (host(im["b_val"]) == ref.csc_b.val).all()
    assert o.error_rel(ref.C, host(C)) <= REL_TOL
    assert (host(C) == ref.C).mean() > 0.999
