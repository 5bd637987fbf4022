"""srq_gemm_i8_static_scratch (the entry point for callers that cannot allocate or hand over a
workspace) against srq_gemm_i8 on the same operands, through the C ABI: bit for bit, two calls in
a row, the second on a smaller problem (the shared static array keeps the first call's contents),
with no workspace attached to the handle; and the refusal of a problem beyond the array's size."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _operands(M, N, K, seed):
    rng = np.random.default_rng(seed)
    Qa = torch.from_numpy(rng.integers(-127, 128, size=(M, K)).astype(np.int8)).cuda()
    Qb = torch.from_numpy(rng.integers(-127, 128, size=(N, K)).astype(np.int8)).cuda()
    sa = torch.from_numpy((rng.random(M) + 0.01).astype(np.float32)).cuda()
    sb = torch.from_numpy((rng.random(N) + 0.01).astype(np.float32)).cuda()
    return Qa, sa, Qb, sb


def test_static_scratch_matches_workspace_entry_point():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2403_06924_amd import binding as b
    ref_h = b.Srq(device=0)                      # srq_gemm_i8 with a workspace
    h = b.Srq(device=0)                          # never gets a workspace
    assert b.load().srq_static_scratch_bytes() == 8 << 20
    try:
        # first a problem that takes the persistent kernel (one partial per 128 columns / rows),
        # then smaller ones on the generic kernel (ragged 256- and 128-tiles)
        for shape, seed in (((4096, 4352, 256), 1), ((1000, 777, 200), 2), ((130, 64, 64), 3)):
            M, N, K = shape
            Qa, sa, Qb, sb = _operands(M, N, K, seed)
            want_F, _, want_row, want_col = ref_h.gemm_i8(Qa, sa, Qb, sb)
            outs = (torch.empty((M, N), dtype=torch.float32, device="cuda"),
                    torch.empty(M, dtype=torch.float32, device="cuda"),
                    torch.empty(N, dtype=torch.float32, device="cuda"))
            got_F, _, got_row, got_col = h.gemm_i8(Qa, sa, Qb, sb, static_scratch=True, out=outs)
            torch.cuda.synchronize()
            assert h.ws is None
            assert torch.equal(got_F, want_F), shape
            assert torch.equal(got_row, want_row) and torch.equal(got_col, want_col), shape
        # beyond the array: refused before any launch
        h.check = False
        M = N = 16384
        fake = torch.empty(16, dtype=torch.int8, device="cuda")
        f32 = torch.empty(16, dtype=torch.float32, device="cuda")
        st = h.lib.srq_gemm_i8_static_scratch(h.h, M, N, 64, fake.data_ptr(), 64, f32.data_ptr(), fake.data_ptr(), 64,
                                              f32.data_ptr(), f32.data_ptr(), None, N, f32.data_ptr(),
                                              f32.data_ptr(), None)
        assert st == b.WORKSPACE
    finally:
        h.close()
        ref_h.close()
