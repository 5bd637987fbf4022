"""A call with the density switch off enqueues kernels only (no allocation, no read-back, no
memset node; SRQ_STRATEGY_AUTO decides on the device), so a caller may record it into a HIP graph.  The
graph is replayed several times with new operand contents and eager work in between, and
every replay is compared with the eager call on the same operands."""
import numpy as np
import pytest

from paper_2403_06924_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def srq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2403_06924_amd import binding as b
    h = b.Srq(device=0)
    yield h
    h.close()


@pytest.mark.parametrize("strategy_name", ["mfma", "valu", "smfmac", "auto", "dense"])
@pytest.mark.parametrize("shape", [(256, 256, 256), (1024, 768, 512)])
def test_fixed_strategy_call_replays_from_a_graph(srq, strategy_name, shape):
    from paper_2403_06924_amd import binding as b
    strategy = {"mfma": b.STRATEGY_CSR_MFMA, "valu": b.STRATEGY_CSR_VALU, "smfmac": b.STRATEGY_CSR_SMFMAC,
                "auto": b.STRATEGY_AUTO, "dense": b.STRATEGY_AUTO}[strategy_name]
    # "dense": every term on the dense branch of Algorithm 1 line 11 (limit 0), which needs no count on the host
    kw = dict(strategy=strategy, max_density=1.0, dense_fallback_density=0.0 if strategy_name == "dense" else 2.0)
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    def draw():
        A = rng.standard_normal((M, K)).astype(np.float32)
        B = rng.standard_normal((K, N)).astype(np.float32)
        return torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    theta = 2.0 / (0.8 * K ** 0.5)                       # a few percent of each operand
    Ad, Bd = draw()
    Cg = torch.empty((M, N), dtype=torch.float32, device="cuda")
    stats = b.stats_tensor()
    srq.ensure_workspace(b.workspace_bytes(M, N, K, 1.0))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                        # warm-up on the capture stream
        srq.compensated_gemm(Ad, Bd, theta, theta, out=Cg, stats=stats, **kw)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        srq.compensated_gemm(Ad, Bd, theta, theta, out=Cg, stats=stats, **kw)
    for _ in range(3):
        A2, B2 = draw()
        Ad.copy_(A2); Bd.copy_(B2)
        Cg.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = Cg.clone()
        st_graph = b.read_stats(stats)
        Ce = torch.empty_like(Cg)
        stats_e = b.stats_tensor()
        srq.compensated_gemm(A2, B2, theta, theta, out=Ce, stats=stats_e, **kw)
        torch.cuda.synchronize()
        st_eager = b.read_stats(stats_e)
        assert st_graph["nnz_a"] == st_eager["nnz_a"] > 0 and st_graph["nnz_b"] == st_eager["nnz_b"] > 0
        assert torch.equal(got, Ce)
