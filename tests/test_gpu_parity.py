"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element,
on the same seeded inputs.  Integer stages (codes, scales, compressed selection, INT32
products) must be bit-exact; the FP32 output within 1e-5 relative Frobenius error."""
import numpy as np
import pytest

from oracle import srq_oracle as o
from paper_2403_06924_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
F32 = np.float32
REL_TOL = 1e-5          # spec tolerance on the FP32 output
MEAN_TOL = 1e-6         # row/column means of |D_F|: summation order differs from the oracle


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


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def rel_fro(ref, x):
    return o.error_rel(ref, x)


ROUND = {0: o.ROUND_NEAREST_EVEN, 1: o.ROUND_TRUNC}


# ------------------------------------------------------------------ a1: quantize
@pytest.mark.parametrize("shape", [(256, 256), (257, 129), (1, 1), (64, 1000), (300, 77), (5, 3), (130, 64)])
@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("layout", [0, 1])
def test_quantize_bit_exact(srq, b, shape, axis, layout):
    rng = np.random.default_rng(shape[0] * 131 + shape[1])
    X = (rng.standard_normal(shape) * rng.choice([0.01, 1.0, 300.0], size=shape)).astype(F32)
    if shape[0] > 4:
        X[3, :] = 0                                          # an all-zero row
    if shape[1] > 2:
        X[:, 2] = 0                                          # an all-zero column
    for bits, rnd in ((8, 0), (8, 1), (4, 0), (3, 1)):
        Q, s, lam = srq.quantize(dev(X), axis, bits=bits, rounding=rnd, layout=layout)
        q_ref, s_ref, lam_ref = o.quantize_vectors(X, "row" if axis == 0 else "col",
                                                   o.qmax_of_bits(bits), ROUND[rnd])
        vm = q_ref if axis == 0 else q_ref.T
        expect = vm if layout == 0 else vm.T
        assert (host(s) == s_ref).all()
        assert (host(lam) == lam_ref).all()
        assert (host(Q) == expect).all()


def test_quantize_strided_input_and_ties(srq, b):
    rng = np.random.default_rng(1)
    big = rng.standard_normal((100, 200)).astype(F32)
    Xd = dev(big)[:, :150]                                   # ldx = 200 > cols = 150
    Q, s, lam = srq.quantize(Xd, 0)
    q_ref, s_ref, _ = o.quantize_vectors(big[:, :150], "row")
    assert (host(Q) == q_ref).all() and (host(s) == s_ref).all()
    # exact ties: amax = 127 makes lambda = 1
    X = np.array([[127.0, 2.5, 3.5, -2.5, -0.5, 0.5, 1.5, -2.7, 2.7, 0.0]], dtype=F32)
    Q, s, lam = srq.quantize(dev(X), 0)
    assert host(Q).tolist() == [[127, 2, 4, -2, 0, 0, 2, -3, 3, 0]]
    Q, _, _ = srq.quantize(dev(X), 0, rounding=1)
    assert host(Q).tolist() == [[127, 2, 3, -2, 0, 0, 1, -2, 2, 0]]


def test_quantize_empty(srq, b):
    X = torch.empty((0, 7), dtype=torch.float32, device="cuda")
    Q, s, lam = srq.quantize(X, 1)
    torch.cuda.synchronize()
    assert Q.shape == (7, 0) and (host(s) == 0).all() and (host(lam) == 0).all()


# ------------------------------------------------------------------ a2-a4: GEMM, dequant, means
@pytest.mark.parametrize("shape", [(128, 128, 64), (256, 256, 256), (257, 129, 511), (1, 1, 1),
                                   (130, 300, 96), (64, 640, 1000), (33, 17, 65)])
def test_gemm_i8_bit_exact(srq, b, shape):
    M, N, K = shape
    rng = np.random.default_rng(M + 7 * N + 13 * K)
    Qa = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    Qb = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    sa = rng.random(M).astype(F32) + F32(0.01)
    sb = rng.random(N).astype(F32) + F32(0.01)
    D_F, D_int, drow, dcol = srq.gemm_i8(dev(Qa), dev(sa), dev(Qb), dev(sb), want_int=True)
    ref_int = o.int_matmul(Qa, Qb.T)
    ref_F = o.dequant_product(ref_int, sa, sb)
    assert (host(D_int) == ref_int).all()
    assert (host(D_F) == ref_F).all()
    r_row, r_col = o.abs_means(ref_F)
    np.testing.assert_allclose(host(drow), r_row, rtol=MEAN_TOL)
    np.testing.assert_allclose(host(dcol), r_col, rtol=MEAN_TOL)


def test_gemm_i8_extreme_codes_and_unaligned_ld(srq, b):
    M, N, K = 96, 80, 1000
    Qa = np.full((M, K), 127, dtype=np.int8)
    Qb = np.full((N, K), -127, dtype=np.int8)
    Qb[::2] = 127
    big_a = np.zeros((M, K + 3), dtype=np.int8); big_a[:, :K] = Qa      # lda = K+3: unaligned rows
    big_b = np.zeros((N, K + 5), dtype=np.int8); big_b[:, :K] = Qb
    one_m, one_n = np.ones(M, F32), np.ones(N, F32)
    D_F, D_int, _, _ = srq.gemm_i8(dev(big_a)[:, :K], dev(one_m), dev(big_b)[:, :K], dev(one_n), want_int=True)
    ref = o.int_matmul(Qa, Qb.T)
    assert (host(D_int) == ref).all()
    assert (host(D_F) == ref.astype(F32)).all()


# ------------------------------------------------------------------ a5-a6: residual + selection
@pytest.mark.parametrize("shape", [(256, 256), (257, 129), (64, 1000), (300, 77), (1, 1), (700, 40)])
@pytest.mark.parametrize("axis", [0, 1])
def test_build_sparse_residual_bit_exact(srq, b, shape, axis):
    name = "row" if axis == 0 else "col"
    rng = np.random.default_rng(shape[0] + 3 * shape[1] + axis)
    X = rng.standard_normal(shape).astype(F32)
    X[rng.random(shape) < 0.01] *= 50
    nvec = shape[axis]
    for bits, rnd, r_layout in ((8, 0, 0), (8, 1, 1), (4, 0, 1)):
        qm = o.qmax_of_bits(bits)
        q_ref, s_ref, lam_ref = o.quantize_vectors(X, name, qm, ROUND[rnd])
        thresh = (np.abs(rng.standard_normal(nvec)) * 1.5).astype(F32)
        thresh[0] = np.inf if nvec > 1 else thresh[0]
        if nvec > 2:
            thresh[1] = 0.0
        out = srq.build_sparse_residual(dev(X), axis, dev(s_ref), dev(lam_ref), dev(thresh), bits=bits,
                                        rounding=rnd, r_layout=r_layout)
        R = o.residual(X, q_ref, s_ref, name)
        rq_ref, rs_ref, _ = o.quantize_vectors(R, name, qm, ROUND[rnd])
        vm = rq_ref if axis == 0 else rq_ref.T
        assert (host(out["rscale"]) == rs_ref).all()
        assert (host(out["Rq"]) == (vm if r_layout == 0 else vm.T)).all()
        c = o.compress(o.select_mask(X, thresh, name), q_ref, name)
        assert int(out["nnz"].item()) == c.nnz
        assert (host(out["ptr"]) == c.ptr).all()
        assert (host(out["idx"])[:c.nnz] == c.idx).all()
        assert (host(out["val"])[:c.nnz] == c.val).all()


def test_build_sparse_residual_capacity_truncates(srq, b):
    rng = np.random.default_rng(8)
    X = rng.standard_normal((64, 300)).astype(F32)
    q_ref, s_ref, lam_ref = o.quantize_vectors(X, "row")
    thresh = np.full(64, 0.5, F32)
    c = o.compress(o.select_mask(X, thresh, "row"), q_ref, "row")
    cap = c.nnz // 2
    out = srq.build_sparse_residual(dev(X), 0, dev(s_ref), dev(lam_ref), dev(thresh), capacity=cap,
                                    want_residual=False)
    assert int(out["nnz"].item()) == c.nnz > cap                 # the required size is reported
    assert (host(out["ptr"]) == c.ptr).all()
    assert (host(out["idx"])[:cap] == c.idx[:cap]).all()
    assert (host(out["val"])[:cap] == c.val[:cap]).all()


# ------------------------------------------------------------------ a7: sparse products
@pytest.mark.parametrize("shape", [(128, 128, 128), (257, 129, 511), (96, 300, 200), (5, 3, 9)])
@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("strategy", [1, 2])
def test_spmm_accumulate_bit_exact(srq, b, shape, side, strategy):
    M, N, K = shape
    rng = np.random.default_rng(M * 3 + N * 5 + K * 7 + side)
    nvec, nelem = (M, N) if side == 0 else (N, M)
    Qs = rng.integers(-127, 128, size=(nvec, K)).astype(np.int8)          # sparse operand, vector-major
    mask = rng.random((nvec, K)) < 0.1
    mask[0] = False
    c = o.compress(mask, Qs, "row")
    Rk = rng.integers(-127, 128, size=(K, nelem)).astype(np.int8)          # residual codes, k-major
    s_row = rng.random(M).astype(F32) + F32(0.1)
    s_col = rng.random(N).astype(F32) + F32(0.1)
    C0 = rng.standard_normal((M, N)).astype(F32)
    Cd = dev(C0)
    Rq = dev(Rk) if strategy == 1 else dev(Rk.T)
    DR = srq.spmm_accumulate(side, strategy, M, N, K, dev(c.ptr), dev(c.idx) if c.nnz else dev(np.zeros(1, np.int32)),
                             dev(c.val) if c.nnz else dev(np.zeros(1, np.int8)), Rq, dev(s_row), dev(s_col), Cd,
                             want_int=True)
    sparse = np.where(mask, Qs, 0)
    ref_int = o.int_matmul(sparse, Rk) if side == 0 else o.int_matmul(Rk.T, sparse.T)
    assert (host(DR) == ref_int).all()
    ref_C = C0 + o.dequant_product(ref_int, s_row, s_col)
    assert (host(Cd) == ref_C).all()


@pytest.mark.parametrize("shape", [(100, 520, 300), (264, 1032, 96), (2048, 1544, 640)])
@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("density", [0.3, 0.02])
@pytest.mark.parametrize("want_int", [False, True])
def test_spmm_tiled_kernel_bit_exact(srq, b, shape, side, density, want_int):
    """Aligned operands take the tiled vector-ALU kernel: several 64-pair batches per vector,
    pair counts that are not multiples of the unroll, empty vectors, a ragged block of vectors
    and a ragged last chunk of elements; with and without the INT32 side output (the two
    epilogue variants of side 0)."""
    M, N, K = shape
    rng = np.random.default_rng(M + 3 * N + 5 * K + side)
    nvec, nelem = (M, N) if side == 0 else (N, M)
    Qs = rng.integers(-127, 128, size=(nvec, K)).astype(np.int8)
    mask = rng.random((nvec, K)) < density
    mask[0] = False
    mask[nvec // 2] = False
    mask[nvec - 1] = True                                                  # a full vector
    c = o.compress(mask, Qs, "row")
    Rk = rng.integers(-127, 128, size=(K, nelem)).astype(np.int8)
    s_row = rng.random(M).astype(F32) + F32(0.1)
    s_col = rng.random(N).astype(F32) + F32(0.1)
    C0 = rng.standard_normal((M, N)).astype(F32)
    Cd = dev(C0)
    DR = srq.spmm_accumulate(side, 1, M, N, K, dev(c.ptr), dev(c.idx), dev(c.val), dev(Rk), dev(s_row),
                             dev(s_col), Cd, want_int=want_int)
    sparse = np.where(mask, Qs, 0)
    ref_int = o.int_matmul(sparse, Rk) if side == 0 else o.int_matmul(Rk.T, sparse.T)
    if want_int:
        assert (host(DR) == ref_int).all()
    ref_C = C0 + o.dequant_product(ref_int, s_row, s_col)
    assert (host(Cd) == ref_C).all()


# ------------------------------------------------------------------ whole path
def check_against_oracle(srq, b, A, B, theta_a, theta_b, *, bits=8, rnd=0, strategy=1, s=2.0,
                         alpha=1.0, beta=0.0, C_in=None, scale_mode="vector"):
    M, K = A.shape
    N = B.shape[1]
    stats = b.stats_tensor()
    Cd, _, dbg = srq.compensated_gemm(dev(A), dev(B), theta_a, theta_b, bits=bits, rounding=rnd,
                                      dense_fallback_density=s, strategy=strategy, alpha=alpha, beta=beta,
                                      C_in=None if C_in is None else dev(C_in), stats=stats, debug=True)
    torch.cuda.synchronize()
    im = srq.intermediates(M, N, K)
    st = b.read_stats(stats)
    comp = not (np.isinf(theta_a) and np.isinf(theta_b))
    # thresholds: compare the GPU's means with the oracle's, then feed the GPU's thresholds
    # to the oracle so that the selection can be compared bit for bit
    t_a = host(im["t_a"]) if comp else None
    t_b = host(im["t_b"]) if comp else None
    ref = o.compensated_gemm(A, B, theta_a, theta_b, bits=bits, rounding=ROUND[rnd], alpha=alpha, beta=beta,
                             C_in=C_in, dense_fallback_density=s, scale_mode=scale_mode,
                             thresh_a=t_a if comp and not np.isinf(theta_a) else None,
                             thresh_b=t_b if comp and not np.isinf(theta_b) else None)
    assert (host(im["A_int"]) == ref.A_int).all()
    assert (host(im["B_int"]) == ref.B_int.T).all()
    assert (host(im["s_a"]) == ref.s_a).all() and (host(im["s_b"]) == ref.s_b).all()
    assert (host(im["lam_a"]) == ref.lam_a).all() and (host(im["lam_b"]) == ref.lam_b).all()
    assert (host(dbg["D_int"]) == ref.D_int).all()
    assert (host(dbg["D_F"]) == ref.D_F).all()
    if comp:
        np.testing.assert_allclose(host(im["drow"]), ref.drow, rtol=MEAN_TOL)
        np.testing.assert_allclose(host(im["dcol"]), ref.dcol, rtol=MEAN_TOL)
        pure = o.compensated_gemm(A, B, theta_a, theta_b, bits=bits, rounding=ROUND[rnd], scale_mode=scale_mode)
        np.testing.assert_allclose(t_a, pure.t_a, rtol=2 * MEAN_TOL)
        np.testing.assert_allclose(t_b, pure.t_b, rtol=2 * MEAN_TOL)
        assert (host(im["s_ra"]) == ref.s_ra).all() and (host(im["s_rb"]) == ref.s_rb).all()
        if not np.isinf(theta_a):
            assert st["nnz_a"] == ref.csr_a.nnz
            assert (host(im["a_ptr"]) == ref.csr_a.ptr).all()
            if st["path_a"] != 3:                                # the dense branch counts, it does not compact
                assert (host(im["a_idx"]) == ref.csr_a.idx).all()
                assert (host(im["a_val"]) == ref.csr_a.val).all()
            assert st["path_a"] == (3 if ref.dense_a else st["path_a"]) and st["path_a"] in (1, 2, 3, 5)
            assert (host(dbg["DR1_int"]) == ref.DR1_int).all()
        if not np.isinf(theta_b):
            assert st["nnz_b"] == ref.csc_b.nnz
            assert (host(im["b_ptr"]) == ref.csc_b.ptr).all()
            if st["path_b"] != 3:
                assert (host(im["b_idx"]) == ref.csc_b.idx).all()
                assert (host(im["b_val"]) == ref.csc_b.val).all()
            assert (host(dbg["DR2_int"]) == ref.DR2_int).all()
        for key, mat in (("RA_int", ref.RA_int), ("RB_int", ref.RB_int.T), ("RA_em", ref.RA_int.T),
                         ("RB_em", ref.RB_int)):
            if im[key] is not None:
                assert (host(im[key]) == mat).all(), key
    err = rel_fro(ref.C, host(Cd))
    assert err <= REL_TOL, err
    return ref, host(Cd), st


@pytest.mark.parametrize("strategy", [1, 2])
def test_config_c1_full(srq, b, strategy):
    """C1: 256^3 uniform[-1,1), seed 0, about 5 % of each operand kept."""
    A, B = wl.make_inputs("C1")
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    ta = wl.theta_for_density(A, drow, "row", 0.05)
    tb = wl.theta_for_density(B, dcol, "col", 0.05)
    ref, C, st = check_against_oracle(srq, b, A, B, ta, tb, strategy=strategy)
    assert abs(ref.csr_a.density - 0.05) < 5e-3 and abs(ref.csc_b.density - 0.05) < 5e-3
    assert (C == ref.C).all()                                   # in fact bit-exact
    C64 = A.astype(np.float64) @ B.astype(np.float64)
    assert rel_fro(C64, C) < rel_fro(C64, ref.D_F)


@pytest.mark.parametrize("name,shape", [("C2", (384, 320, 512)), ("C3", (257, 129, 511)),
                                        ("C4", (200, 330, 260)), ("C5", (130, 70, 1000))])
@pytest.mark.parametrize("strategy", [0, 1, 2])
def test_ragged_shapes_all_strategies(srq, b, name, shape, strategy):
    A, B = wl.make_inputs(name, *shape)
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    ta = wl.theta_for_density(A, drow, "row", 0.05)
    tb = wl.theta_for_density(B, dcol, "col", 0.05)
    check_against_oracle(srq, b, A, B, ta, tb, strategy=strategy)


@pytest.mark.parametrize("shape", [(300, 200, 2048), (257, 129, 1531), (64, 96, 4100), (132, 260, 640)])
@pytest.mark.parametrize("density", [1e-3, 2e-4])
def test_very_sparse_operands_auto(srq, b, shape, density):
    """Well under one kept entry per 512 elements, host-synchronising mode: the compaction takes the
    variant that leaves the codes of empty 256-element chunks unread (ragged tails included)."""
    A, B = wl.make_inputs("C2", *shape)
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    ta = wl.theta_for_density(A, drow, "row", density)
    tb = wl.theta_for_density(B, dcol, "col", density)
    ref, _, st = check_against_oracle(srq, b, A, B, ta, tb, strategy=0)
    assert 0 < ref.csr_a.nnz * 512 < A.size and 0 < ref.csc_b.nnz * 512 < B.size
    assert st["path_a"] == 1 and st["path_b"] == 1


def test_auto_repeated_calls_reuse_the_previous_choice(srq, b):
    """With SRQ_STRATEGY_AUTO the layouts written ahead of the host's decision follow the previous
    call's choice (selection passes that also write residual codes); every call in a sequence that
    moves between the vector-ALU and the matrix-core regime must still match the oracle."""
    A, B = wl.make_inputs("C2", 256, 192, 512)
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    for density in (1e-3, 1e-3, 0.2, 0.2, 1e-3, 1e-3):
        ta = wl.theta_for_density(A, drow, "row", density)
        tb = wl.theta_for_density(B, dcol, "col", density)
        _, _, st = check_against_oracle(srq, b, A, B, ta, tb, strategy=0)
        assert st["path_a"] == st["path_b"] == (1 if density < 0.005 else 2)


@pytest.mark.parametrize("shape", [(256, 256, 256), (512, 768, 384), (768, 512, 200), (256, 512, 1000), (256, 256, 9000)])
@pytest.mark.parametrize("density", [0.05, 0.3])
def test_structured_2to4_execution(srq, b, shape, density):
    """SRQ_STRATEGY_CSR_SMFMAC: the compaction pass writes the reduced operand as two operands of
    2:4 form for the sparse matrix-core instruction (first two / third and fourth non-zero code of
    every group of four k; the second is multiplied only where it holds anything).  Selection and
    compressed arrays are the same as on every path (bit-exact); both parts feed the same INT32
    accumulators, so C is bit-identical to the plain matrix-core execution (and within the
    spec tolerance of the oracle, in practice identical).  Densities of 5 % and 30 %: the
    second operand is nearly empty resp. needed almost everywhere."""
    M, N, K = shape
    A, B = wl.make_inputs("C2", M, N, K)
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    ta = wl.theta_for_density(A, drow, "row", density)
    tb = wl.theta_for_density(B, dcol, "col", density)
    stats = b.stats_tensor()
    C24, _, _ = srq.compensated_gemm(dev(A), dev(B), ta, tb, strategy=b.STRATEGY_CSR_SMFMAC, stats=stats)
    torch.cuda.synchronize()
    st = b.read_stats(stats)
    im = srq.intermediates(M, N, K)
    t_a, t_b = host(im["t_a"]), host(im["t_b"])
    a_ptr, a_idx, a_val = host(im["a_ptr"]), host(im["a_idx"]), host(im["a_val"])
    b_ptr, b_idx, b_val = host(im["b_ptr"]), host(im["b_idx"]), host(im["b_val"])
    C24 = host(C24)
    ref = o.compensated_gemm(A, B, ta, tb, thresh_a=t_a, thresh_b=t_b)
    assert st["path_a"] == 4 and st["path_b"] == 4
    assert st["nnz_a"] == ref.csr_a.nnz and st["nnz_b"] == ref.csc_b.nnz
    assert (a_ptr == ref.csr_a.ptr).all() and (a_idx == ref.csr_a.idx).all() and (a_val == ref.csr_a.val).all()
    assert (b_ptr == ref.csc_b.ptr).all() and (b_idx == ref.csc_b.idx).all() and (b_val == ref.csc_b.val).all()
    assert rel_fro(ref.C, C24) <= REL_TOL
    C2, _, _ = srq.compensated_gemm(dev(A), dev(B), ta, tb, strategy=b.STRATEGY_CSR_MFMA)
    assert (host(C2) == C24).all()
    # with alpha and beta the scaling is applied once, after the second term
    Cin = np.random.default_rng(5).standard_normal((M, N)).astype(np.float32)
    Cab, _, _ = srq.compensated_gemm(dev(A), dev(B), ta, tb, strategy=b.STRATEGY_CSR_SMFMAC, alpha=0.5, beta=-1.5,
                                     C_in=dev(Cin))
    refab = o.compensated_gemm(A, B, ta, tb, thresh_a=t_a, thresh_b=t_b, alpha=0.5, beta=-1.5, C_in=Cin)
    assert rel_fro(refab.C, host(Cab)) <= REL_TOL
    # one term alone on the sparse matrix cores (the other operand is not reduced): the unpaired
    # launches, rows of C resp. columns of C
    inf = float("inf")
    for tha, thb in ((ta, inf), (inf, tb)):
        C1, _, _ = srq.compensated_gemm(dev(A), dev(B), tha, thb, strategy=b.STRATEGY_CSR_SMFMAC, stats=stats)
        C1m, _, _ = srq.compensated_gemm(dev(A), dev(B), tha, thb, strategy=b.STRATEGY_CSR_MFMA)
        torch.cuda.synchronize()
        st1 = b.read_stats(stats)
        assert (st1["path_a"], st1["path_b"]) == ((4, 0) if np.isinf(thb) else (0, 4))
        assert torch.equal(C1, C1m)


@pytest.mark.parametrize("shape", [(256, 384, 512), (192, 200, 300), (512, 1024, 4096), (130, 257, 129)])
def test_column_block_execution(srq, b, shape):
    """SRQ_STRATEGY_COLBLOCK on an operand with whole outlier columns (the C4 recipe: 16 columns of
    A times 50) and, on the other side, an operand whose first rows are large (whole k-columns of
    the transposed B): the indices kept in at least 90 % of the vectors run as a dense strip on the
    matrix cores, the rest of the CSR on the vector ALUs.  Every stage against the oracle with the
    raw INT32 sums of the two parts added up (bit-exact), then the timed configuration without
    debug outputs against the oracle and against the plain vector-ALU execution."""
    M, N, K = shape
    A, B = wl.make_inputs("C4", M, N, K)
    B = B.copy()
    B[:5, :] *= np.float32(40.0)                                 # five k kept in (nearly) every column of B
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    da = min(0.9, 16.0 / K + 0.02)
    ta = wl.theta_for_density(A, drow, "row", da)
    tb = wl.theta_for_density(B, dcol, "col", 5.0 / K + 0.02)
    ref, C, st = check_against_oracle(srq, b, A, B, ta, tb, strategy=b.STRATEGY_COLBLOCK)
    assert st["path_a"] == 5 and st["path_b"] == (5 if N % 4 == 0 else 1)   # (unaligned B: no keep-mask, plain CSR)
    # the structure is there: some k are kept in at least 90 % of the vectors of either operand
    mask_a = o.select_mask(A, host(srq.intermediates(M, N, K)["t_a"]), "row")
    mask_b = o.select_mask(B, host(srq.intermediates(M, N, K)["t_b"]), "col")
    assert (mask_a.mean(axis=0) >= 0.9).sum() >= 1 and (mask_b.mean(axis=1) >= 0.9).sum() >= 1
    Cin = np.random.default_rng(6).standard_normal((M, N)).astype(np.float32)
    for alpha, beta, cin in ((1.0, 0.0, None), (0.5, -1.5, Cin)):
        Ct, _, _ = srq.compensated_gemm(dev(A), dev(B), ta, tb, strategy=b.STRATEGY_COLBLOCK, alpha=alpha, beta=beta,
                                        C_in=None if cin is None else dev(cin))
        Cv, _, _ = srq.compensated_gemm(dev(A), dev(B), ta, tb, strategy=b.STRATEGY_CSR_VALU, alpha=alpha, beta=beta,
                                        C_in=None if cin is None else dev(cin))
        im = srq.intermediates(M, N, K)
        refab = o.compensated_gemm(A, B, ta, tb, thresh_a=host(im["t_a"]), thresh_b=host(im["t_b"]), alpha=alpha,
                                   beta=beta, C_in=cin)
        assert rel_fro(refab.C, host(Ct)) <= REL_TOL
        assert rel_fro(host(Cv), host(Ct)) <= 1e-6
    # an operand without such structure: the strip is empty and its product is skipped on the device
    A2, B2 = wl.make_inputs("C2", M, N, K)
    check_against_oracle(srq, b, A2, B2, 0.9, 0.9, strategy=b.STRATEGY_COLBLOCK)
    C2, _, _ = srq.compensated_gemm(dev(A2), dev(B2), 0.9, 0.9, strategy=b.STRATEGY_COLBLOCK)
    Cv2, _, _ = srq.compensated_gemm(dev(A2), dev(B2), 0.9, 0.9, strategy=b.STRATEGY_CSR_VALU)
    assert torch.equal(C2, Cv2)


def test_bounds_theta_inf_and_zero(srq, b):
    A, B = wl.make_inputs("C2", 200, 136, 300)
    inf = float("inf")
    ref, C, st = check_against_oracle(srq, b, A, B, inf, inf)
    assert (C == ref.D_F).all() and st["path_a"] == 0 and st["path_b"] == 0
    for strategy in (1, 2):
        ref0, C0, st0 = check_against_oracle(srq, b, A, B, 0.0, 0.0, strategy=strategy)
        assert st0["nnz_a"] == np.count_nonzero(A) and st0["nnz_b"] == np.count_nonzero(B)
    # one-sided compensation
    check_against_oracle(srq, b, A, B, 0.8, inf, strategy=1)
    check_against_oracle(srq, b, A, B, inf, 0.8, strategy=2)


def test_dense_fallback_branch(srq, b):
    A, B = wl.make_inputs("C4", 192, 256, 384)
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    ta = wl.theta_for_density(A, drow, "row", 0.30)
    tb = wl.theta_for_density(B, dcol, "col", 0.02)
    ref, C, st = check_against_oracle(srq, b, A, B, ta, tb, strategy=1, s=0.1)
    assert ref.dense_a and not ref.dense_b
    assert st["path_a"] == 3 and st["path_b"] == 1


def test_alpha_beta_bits_and_truncation(srq, b):
    A, B = wl.make_inputs("C3", 160, 200, 256)
    rng = np.random.default_rng(4)
    Cin = rng.standard_normal((160, 200)).astype(F32)
    check_against_oracle(srq, b, A, B, 0.9, 0.7, alpha=0.75, beta=-1.5, C_in=Cin, strategy=1)
    check_against_oracle(srq, b, A, B, 0.9, 0.7, alpha=2.0, beta=0.0, strategy=2)
    check_against_oracle(srq, b, A, B, float("inf"), float("inf"), alpha=0.5, beta=2.0, C_in=Cin)
    check_against_oracle(srq, b, A, B, 0.9, 0.7, bits=4, strategy=1)
    check_against_oracle(srq, b, A, B, 0.9, 0.7, rnd=1, strategy=2)


def test_capacity_status_in_synchronising_mode(srq, b):
    A, B = wl.make_inputs("C2", 128, 128, 256)
    srq.ws = None                                              # force a workspace sized for 1 % density
    srq.check = False
    try:
        # the density switch (at 90 %: not reached by the half that is kept) is the synchronising mode
        plain = o.quantized_product(A, B)
        drow, dcol = o.abs_means(plain.D_F)
        ta = wl.theta_for_density(A, drow, "row", 0.5)
        tb = wl.theta_for_density(B, dcol, "col", 0.5)
        srq.compensated_gemm(dev(A), dev(B), ta, tb, strategy=0, max_density=0.01, dense_fallback_density=0.9)
        assert srq.last_status == b.CAPACITY
    finally:
        srq.check = True
        srq.ws = None


@pytest.mark.parametrize("strategy", [0, 1, 2, 3])
@pytest.mark.parametrize("shape", [(128, 128, 256), (2048, 2048, 256)])
def test_overflow_in_non_synchronising_modes(srq, b, strategy, shape):
    """A fixed strategy cannot read the counts on the host.  With a workspace sized for 1 % and a
    selection that keeps everything, every execution must leave C = D_F (no correction from
    truncated arrays), say so in the statistics, and still report the true counts; the same call
    with enough room then gives the oracle's result (the guard does not trip by mistake).
    The larger shape takes the persistent matrix-core kernels."""
    M, N, K = shape
    A, B = wl.make_inputs("C2", M, N, K)
    plain = o.quantized_product(A, B)
    srq.ws = None                                              # force a workspace sized for 1 % density
    try:
        stats = b.stats_tensor()
        C, _, _ = srq.compensated_gemm(dev(A), dev(B), 0.0, 0.0, strategy=strategy, max_density=0.01,
                                       stats=stats, alpha=0.5)
        torch.cuda.synchronize()
        assert srq.last_status == b.OK
        st = b.read_stats(stats)
        assert st["overflow"] == 3
        assert st["nnz_a"] == int((A != 0).sum()) and st["nnz_b"] == int((B != 0).sum())
        assert (host(C) == plain.D_F).all()                    # uncorrected, alpha not applied
    finally:
        srq.ws = None
    stats = b.stats_tensor()
    C, _, _ = srq.compensated_gemm(dev(A), dev(B), 0.0, 0.0, strategy=strategy, stats=stats, alpha=0.5)
    torch.cuda.synchronize()
    assert b.read_stats(stats)["overflow"] == 0
    ref = o.compensated_gemm(A, B, 0.0, alpha=0.5)
    assert o.error_rel(ref.C, host(C)) <= REL_TOL


def test_auto_on_small_aligned_problems_is_the_matrix_core_execution(srq, b):
    """Where the small-tile kernel runs the products (M, N multiples of 128 below 256 big tiles) the
    matrix cores win at any density: SRQ_STRATEGY_AUTO takes them without deciding anything."""
    A, B = wl.make_inputs("C2", 256, 384, 512)
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    for density in (0.003, 0.05):
        ta = wl.theta_for_density(A, drow, "row", density)
        tb = wl.theta_for_density(B, dcol, "col", density)
        _, _, st = check_against_oracle(srq, b, A, B, ta, tb, strategy=0)
        assert (st["path_a"], st["path_b"]) == (2, 2)


@pytest.mark.parametrize("shape", [(4096, 4096, 128), (2368, 2048, 256), (130, 257, 129)])
@pytest.mark.parametrize("da,db,want", [(0.003, 0.05, (1, 2)), (0.05, 0.003, (2, 1)), (0.003, 0.003, (1, 1)),
                                        (0.05, 0.05, (2, 2))])
def test_auto_decides_on_the_device(srq, b, shape, da, db, want):
    """SRQ_STRATEGY_AUTO without the density switch never reads anything back: the executions are
    chosen by a kernel from the counts, per term, and every stage matches the oracle whichever
    combination comes out and whatever the caller's hint said (right, wrong or none).  The largest
    shape takes the persistent kernels (one paired launch for whichever terms go to the matrix
    cores), the others the plain kernel."""
    M, N, K = shape
    A, B = wl.make_inputs("C2", M, N, K)
    plain = o.quantized_product(A, B)
    drow, dcol = o.abs_means(plain.D_F)
    ta = wl.theta_for_density(A, drow, "row", da)
    tb = wl.theta_for_density(B, dcol, "col", db)
    outs = []
    try:
        for hint in ((0, 0), want, (3 - want[0], 3 - want[1])):
            srq.set_auto_hint(*hint)
            ref, C, st = check_against_oracle(srq, b, A, B, ta, tb, strategy=0)
            assert (st["path_a"], st["path_b"]) == want
            Ct, _, _ = srq.compensated_gemm(dev(A), dev(B), ta, tb, strategy=0, alpha=0.5)   # the timed configuration
            outs.append(host(Ct))
            assert rel_fro(np.float32(0.5) * ref.C, outs[-1]) <= REL_TOL
    finally:
        srq.set_auto_hint(0, 0)
    assert (outs[0] == outs[1]).all() and (outs[0] == outs[2]).all()
    # one term only
    inf = float("inf")
    ref, C, st = check_against_oracle(srq, b, A, B, ta, inf, strategy=0)
    assert (st["path_a"], st["path_b"]) == (want[0], 0)
    ref, C, st = check_against_oracle(srq, b, A, B, inf, tb, strategy=0)
    assert (st["path_a"], st["path_b"]) == (0, want[1])


def test_stage_timers_sum_over_calls(srq, b):
    """srq_profile_read returns the stage times summed over the calls since the previous read,
    without the library waiting between those calls."""
    A, B = wl.make_inputs("C2", 256, 256, 256)
    Ad, Bd = dev(A), dev(B)
    srq.profile_enable(True)
    try:
        for _ in range(3):                                                  # (the first calls are cold)
            srq.compensated_gemm(Ad, Bd, 0.5, 0.5, strategy=b.STRATEGY_CSR_MFMA)
        srq.profile_read()
        singles = []
        for _ in range(3):
            srq.compensated_gemm(Ad, Bd, 0.5, 0.5, strategy=b.STRATEGY_CSR_MFMA)
            singles.append(srq.profile_read())
        one = {k: min(s[k] for s in singles) for k in singles[0]}          # (a single call can be an outlier)
        assert one["quantize"] > 0 and one["gemm"] > 0 and one["select"] > 0 and one["term1"] > 0
        for _ in range(5):
            srq.compensated_gemm(Ad, Bd, 0.5, 0.5, strategy=b.STRATEGY_CSR_MFMA)
        five = srq.profile_read()
        assert all(five[k] > 2.0 * one[k] for k in ("quantize", "gemm", "select")), (one, five)
        assert all(v == 0.0 for v in srq.profile_read().values())          # nothing since the last read
        for _ in range(70):                                                 # more than the ring holds
            srq.compensated_gemm(Ad, Bd, 0.5, 0.5, strategy=b.STRATEGY_CSR_MFMA)
        many = srq.profile_read()
        assert 0 < many["gemm"] < 64 * 4.0 * max(one["gemm"], five["gemm"] / 5)
    finally:
        srq.profile_enable(False)


def test_stage_timers_products_only(srq, b):
    """SRQ_PROFILE_PRODUCTS times the three products and nothing else (fewer event records in
    the call); the result of the call is the same with the timers at either level or off."""
    A, B = wl.make_inputs("C2", 256, 256, 256)
    Ad, Bd = dev(A), dev(B)
    C0, _, _ = srq.compensated_gemm(Ad, Bd, 0.5, 0.5, strategy=b.STRATEGY_CSR_MFMA)
    srq.profile_enable(True, products_only=True)
    try:
        for _ in range(3):
            C1, _, _ = srq.compensated_gemm(Ad, Bd, 0.5, 0.5, strategy=b.STRATEGY_CSR_MFMA)
        ms = srq.profile_read()
        assert ms["gemm"] > 0 and ms["term1"] > 0
        assert all(ms[k] == 0.0 for k in ("quantize", "select", "residual", "term1_prep", "term2_prep"))
        assert (host(C1) == host(C0)).all()
        srq.profile_enable(True)                                            # back to every stage
        C2, _, _ = srq.compensated_gemm(Ad, Bd, 0.5, 0.5, strategy=b.STRATEGY_CSR_MFMA)
        ms = srq.profile_read()
        assert ms["quantize"] > 0 and ms["select"] > 0 and ms["gemm"] > 0
        assert (host(C2) == host(C0)).all()
    finally:
        srq.profile_enable(False)


def test_run_twice_is_deterministic(srq, b):
    A, B = wl.make_inputs("C3", 300, 260, 512)
    Ad, Bd = dev(A), dev(B)
    outs = []
    for _ in range(2):
        C, _, _ = srq.compensated_gemm(Ad, Bd, 0.8, 0.8, strategy=0)
        torch.cuda.synchronize()
        im = srq.intermediates(300, 260, 512)
        outs.append((host(C).copy(), host(im["a_idx"]).copy(), host(im["t_b"]).copy()))
    for x, y in zip(*outs):
        assert x.tobytes() == y.tobytes()


# ------------------------------------------------------------------ the paper's precision-test inputs
@pytest.mark.parametrize("kind", ["uniform", "normal", "exponential", "poisson", "chisquare"])
@pytest.mark.parametrize("bits", [8, 4])
def test_paper_distributions_1024(srq, b, kind, bits):
    """The five non-negative distributions of the precision test (Sec. 4.1.1) at 1024^2, INT8
    and INT4 codes: every stage against the oracle at a density of about 20 %, and the
    direct and unreduced variants' outputs."""
    n = 1024
    A = wl.paper_distribution(kind, (n, n), 21)
    B = wl.paper_distribution(kind, (n, n), 22)
    plain = o.quantized_product(A, B, bits=bits)
    drow, dcol = o.abs_means(plain.D_F)
    ta = wl.theta_for_density(A, drow, "row", 0.2)
    tb = wl.theta_for_density(B, dcol, "col", 0.2)
    check_against_oracle(srq, b, A, B, ta, tb, bits=bits, strategy=0)
    inf = float("inf")
    C, _, _ = srq.compensated_gemm(dev(A), dev(B), inf, inf, bits=bits)
    assert (host(C) == plain.D_F).all()
    C0, _, _ = srq.compensated_gemm(dev(A), dev(B), 0.0, 0.0, bits=bits, dense_fallback_density=0.0)
    ref0 = o.compensated_gemm(A, B, 0.0, bits=bits)
    assert o.error_rel(ref0.C, host(C0)) <= 1e-5


# ------------------------------------------------------------------ matrix-wide first-level scale
@pytest.mark.parametrize("shape", [(256, 256, 256), (257, 129, 511)])
@pytest.mark.parametrize("bits", [8, 4])
def test_global_scale_mode(srq, b, shape, bits):
    """One scale for the whole of A and one for the whole of B (Sec. 2.3, Eq. getlambda; the
    setting of the worked 3x3 example), residual codes still per vector: every stage against
    the oracle's global mode, and the handle returns to vector-wise scales afterwards."""
    M, N, K = shape
    rng = np.random.default_rng(M + N + K + bits)
    A = (rng.standard_normal((M, K)) * np.exp(rng.standard_normal((M, 1)))).astype(F32)
    B = (rng.standard_normal((K, N)) * np.exp(rng.standard_normal((1, N)))).astype(F32)
    srq.set_scale_mode(b.SCALE_GLOBAL)
    try:
        ref, C, st = check_against_oracle(srq, b, A, B, 0.05, 0.05, bits=bits, strategy=0, scale_mode="global")
        assert len(np.unique(ref.s_a)) == 1 and len(np.unique(ref.s_b)) == 1
        ref0, _, _ = check_against_oracle(srq, b, A, B, 0.0, 0.0, bits=bits, strategy=2, s=0.0, scale_mode="global")
    finally:
        srq.set_scale_mode(b.SCALE_VECTOR)
    refv, _, _ = check_against_oracle(srq, b, A, B, 0.05, 0.05, bits=bits, strategy=0)
    assert len(np.unique(refv.s_a)) > 1


# ------------------------------------------------------------------ degenerate inputs
def test_degenerate_shapes_and_vectors(srq, b):
    """Empty dimensions, K = 0, a 1x1x1 problem, all-zero operands and zero vectors
    (amax = 0 gives scale 0, lambda 0 and zero codes)."""
    rng = np.random.default_rng(5)
    # M = 0 / N = 0: nothing to write, status OK
    for M, N, K in ((0, 8, 8), (8, 0, 8)):
        C, _, _ = srq.compensated_gemm(dev(np.zeros((M, K), F32)), dev(np.zeros((K, N), F32)), 0.5, 0.5)
        assert tuple(C.shape) == (M, N)
    # K = 0: the product is empty, C = alpha * 0 + beta * C_in
    Cin = rng.standard_normal((6, 7)).astype(F32)
    C, _, _ = srq.compensated_gemm(dev(np.zeros((6, 0), F32)), dev(np.zeros((0, 7), F32)), 0.5, 0.5,
                                   alpha=2.0, beta=0.5, C_in=dev(Cin))
    assert (host(C) == F32(0.5) * Cin).all()
    # 1 x 1 x 1
    A = np.array([[0.75]], F32); B = np.array([[-1.5]], F32)
    check_against_oracle(srq, b, A, B, 0.0, 0.0, strategy=1)
    check_against_oracle(srq, b, A, B, 0.0, 0.0, strategy=2)
    # all-zero A: every scale of A is 0, C = 0
    A = np.zeros((40, 72), F32); B = rng.standard_normal((72, 24)).astype(F32)
    ref, C, _ = check_against_oracle(srq, b, A, B, 0.3, 0.3, strategy=0)
    assert (ref.s_a == 0).all() and (C == 0).all()
    # zero rows of A, zero columns of B, one zero column of A and row of B
    A = rng.standard_normal((130, 200)).astype(F32); B = rng.standard_normal((200, 70)).astype(F32)
    A[3] = 0; A[129] = 0; A[:, 17] = 0; B[:, 0] = 0; B[:, 69] = 0; B[50] = 0
    for strategy in (1, 2):
        ref, C, _ = check_against_oracle(srq, b, A, B, 0.4, 0.4, strategy=strategy)
        assert ref.s_a[3] == 0 and ref.s_b[0] == 0 and (C[3] == 0).all() and (C[:, 69] == 0).all()


def test_inner_dimension_at_the_int32_bound(srq, b):
    """K = 133144 is the largest inner dimension whose worst-case sum K * 127^2 stays below
    2^31; operands of constant maximum magnitude reach it.  One more is refused."""
    K = 133144
    M, N = 2, 3
    A = np.full((M, K), 3.0, F32); A[1] = -3.0
    B = np.full((K, N), 2.0, F32); B[:, 2] = -2.0
    C, _, dbg = srq.compensated_gemm(dev(A), dev(B), float("inf"), float("inf"), debug=True)
    D = host(dbg["D_int"]).astype(np.int64)
    assert (np.abs(D) == K * 127 * 127).all() and K * 127 * 127 < 2 ** 31
    ref = o.compensated_gemm(A, B, np.inf)
    assert (host(C) == ref.C).all()
    with pytest.raises(b.SrqError) as ei:
        srq.compensated_gemm(dev(np.zeros((M, K + 1), F32)), dev(np.zeros((K + 1, N), F32)), 0.5, 0.5)
    assert ei.value.status == b.K_OVERFLOW


# ------------------------------------------------------------------ the QR experiment's operands
@pytest.mark.parametrize("kind", ["chisquare", "uniform", "normal", "exponential"])
def test_qr_factors_product(srq, b, kind):
    """Sec. 4.2 multiplies the Householder factors Q (orthogonal) and R (upper triangular, so
    half of every column is zero) with the compensated product: every stage against the
    oracle, all three strategies, and the error against the factored matrix falls from the
    direct quantization to the sparse compensation to the unreduced one."""
    n = 384
    X, Q, R = wl.qr_factors(kind, n, 31)
    plain = o.quantized_product(Q, R)
    drow, dcol = o.abs_means(plain.D_F)
    ta = wl.theta_for_density(Q, drow, "row", 0.3)
    tb = wl.theta_for_density(R, dcol, "col", 0.3)
    for strategy in (0, 1, 2):
        ref, C, st = check_against_oracle(srq, b, Q, R, ta, tb, strategy=strategy)
    full = o.compensated_gemm(Q, R, 0.0)
    X64 = X.astype(np.float64)
    e_origin, e_sparse, e_full = (o.error_rel(X64, plain.D_F), o.error_rel(X64, ref.C), o.error_rel(X64, full.C))
    assert e_origin > e_sparse > e_full


# ------------------------------------------------------------------ leading dimensions
@pytest.mark.parametrize("pad", [(0, 0, 0, 0), (16, 32, 64, 4), (3, 5, 7, 1)])
@pytest.mark.parametrize("strategy", [1, 2])
def test_leading_dimensions(srq, b, pad, strategy):
    """A, B, C and C_in as windows of wider allocations: aligned paddings keep the streaming
    kernels, odd ones fall to the generic kernels; the result is the same bits either way and
    nothing outside the window of C is touched."""
    M, N, K = 192, 320, 256
    rng = np.random.default_rng(17)
    A = rng.standard_normal((M, K)).astype(F32); B = rng.standard_normal((K, N)).astype(F32)
    Cin = rng.standard_normal((M, N)).astype(F32)
    pa, pb, pc, pi = pad
    Abig = torch.full((M, K + pa), 7.0, device="cuda"); Abig[:, :K] = dev(A)
    Bbig = torch.full((K, N + pb), 7.0, device="cuda"); Bbig[:, :N] = dev(B)
    Cbig = torch.full((M, N + pc), -5.0, device="cuda")
    Ibig = torch.full((M, N + pi), 9.0, device="cuda"); Ibig[:, :N] = dev(Cin)
    theta = 2.0 / (0.8 * K ** 0.5)
    srq.compensated_gemm(Abig[:, :K], Bbig[:, :N], theta, theta, strategy=strategy, alpha=0.5, beta=2.0,
                         C_in=Ibig[:, :N], out=Cbig[:, :N])
    torch.cuda.synchronize()
    C0, _, _ = srq.compensated_gemm(dev(A), dev(B), theta, theta, strategy=strategy, alpha=0.5, beta=2.0,
                                    C_in=dev(Cin))
    assert torch.equal(Cbig[:, :N], C0)
    if pc:
        assert (Cbig[:, N:] == -5.0).all()
    ref = o.compensated_gemm(A, B, theta, theta, alpha=0.5, beta=2.0, C_in=Cin)
    assert rel_fro(ref.C, host(C0)) <= REL_TOL


# ------------------------------------------------------------------ randomized configurations
@pytest.mark.parametrize("seed", [101, 102, 103])
def test_randomized_configurations(srq, b, seed):
    """Seeded sweep over shapes (ragged, aligned, skinny), densities including both bounds,
    code widths, roundings, strategies, the density switch and alpha / beta: every stage
    against the oracle for each drawn case."""
    rng = np.random.default_rng(seed)
    for it in range(20):
        kind = rng.integers(0, 4)
        if kind == 0:
            M, N, K = (int(x) for x in rng.integers(1, 500, size=3))
        elif kind == 1:
            M, N, K = (int(x) * 64 for x in rng.integers(1, 9, size=3))
        elif kind == 2:
            M, N, K = int(rng.integers(1, 60)) * 8, int(rng.integers(1, 60)) * 4, int(rng.integers(1, 40)) * 16
        else:
            M, N, K = int(rng.integers(1, 8)), int(rng.integers(200, 900)), int(rng.integers(1, 1200))
            if rng.random() < 0.5:
                M, N = N, M
        A = (rng.standard_normal((M, K)) * np.exp(rng.standard_normal((M, 1)))).astype(F32)
        B = (rng.standard_normal((K, N)) * np.exp(rng.standard_normal((1, N)))).astype(F32)
        if rng.random() < 0.3:
            A[rng.random((M, K)) < 0.02] *= 40
        if rng.random() < 0.3:
            B[:, rng.integers(0, N)] = 0
        drow, dcol = o.abs_means(o.quantized_product(A, B).D_F)
        da, db = (float(rng.choice([0.0, 0.01, 0.05, 0.3, 1.0])) for _ in range(2))
        ta = wl.theta_for_density(A, drow, "row", da) if (drow > 0).all() else 0.5
        tb = wl.theta_for_density(B, dcol, "col", db) if (dcol > 0).all() else 0.5
        bits = int(rng.choice([8, 8, 8, 4, 6]))
        rnd = int(rng.integers(0, 2))
        strategy = int(rng.integers(0, 3))
        s = float(rng.choice([2.0, 2.0, 0.2, 0.0]))
        alpha, beta = (1.0, 0.0) if rng.random() < 0.5 else (float(rng.normal()), float(rng.normal()))
        Cin = rng.standard_normal((M, N)).astype(F32) if beta != 0.0 else None
        try:
            check_against_oracle(srq, b, A, B, ta, tb, bits=bits, rnd=rnd, strategy=strategy, s=s,
                                 alpha=alpha, beta=beta, C_in=Cin)
        except AssertionError as e:
            raise AssertionError("case %d of seed %d: M=%d N=%d K=%d densities %.2f/%.2f bits=%d rounding=%d "
                                 "strategy=%d s=%.1f alpha=%.3f beta=%.3f: %s"
                                 % (it, seed, M, N, K, da, db, bits, rnd, strategy, s, alpha, beta, e)) from e
