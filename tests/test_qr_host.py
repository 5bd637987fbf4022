"""Host logic of the blocked Householder QR driver (Sec. 4.2's application), no GPU: with an exact
product it must be a QR factorization; with the oracle's compensated product plugged in, the
error of Q.R against the matrix orders as the paper's table does (origin > sparse > full)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import srq_oracle as o
from paper_2403_06924_amd import qr
from paper_2403_06924_amd import workloads as wl


@pytest.mark.parametrize("shape,block", [((96, 96), 32), ((130, 70), 16), ((64, 64), 64), ((50, 50), 7)])
def test_exact_product_gives_a_qr_factorization(shape, block):
    rng = np.random.default_rng(shape[0] + block)
    A = torch.from_numpy(rng.standard_normal(shape))            # float64
    Q, R = qr.householder_qr(A, block=block)
    m, n = shape
    assert float((Q.T @ Q - torch.eye(m, dtype=A.dtype)).abs().max()) < 1e-12
    assert float(torch.tril(R, -1).abs().max()) == 0.0
    assert float((Q @ R - A).abs().max()) < 1e-12
    # same factorization as the library routine up to the signs of the reflectors
    Rn = np.linalg.qr(A.numpy(), mode="r")
    np.testing.assert_allclose(np.abs(R[:n].numpy()), np.abs(Rn), atol=1e-10)


def test_rank_deficient_and_zero_columns():
    A = torch.zeros((40, 24), dtype=torch.float64)
    A[:, 3] = 1.0
    A[5:, 7] = torch.arange(35, dtype=torch.float64)
    Q, R = qr.householder_qr(A, block=8)
    assert float((Q @ R - A).abs().max()) < 1e-12
    assert float((Q.T @ Q - torch.eye(40, dtype=A.dtype)).abs().max()) < 1e-12


def _oracle_matmul(theta, s=2.0):
    def mm(X, Y):
        ref = o.compensated_gemm(X.numpy(), Y.numpy(), theta, theta, dense_fallback_density=s)
        return torch.from_numpy(ref.C)
    return mm


def test_oracle_products_order_the_errors_as_the_paper_does():
    n = 128
    X = torch.from_numpy(wl.paper_distribution("normal", (n, n), 5))
    X64 = X.double()
    errs = {}
    for name, theta, s in (("origin", float("inf"), 2.0), ("sparse", 0.05, 2.0), ("full", 0.0, 0.0)):
        mm = _oracle_matmul(theta, s)
        Q, R = qr.householder_qr(X, mm, block=32)
        errs[name] = float(torch.linalg.norm(X64 - mm(Q, R).double()) / torch.linalg.norm(X64))
    assert errs["origin"] > errs["sparse"] > errs["full"]
    assert errs["full"] < 0.2 * errs["origin"]
