"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol include/srq.h declares, sizes workspaces, and rejects bad arguments before
launching anything (a handle created with device = -1 validates and then returns
SRQ_STATUS_NO_DEVICE)."""
import ctypes as C
import os
import re

import pytest

from paper_2403_06924_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(b.LIB_PATH):
        from paper_2403_06924_amd import build
        build.build(verbose=False)
    return b.load()


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "srq.h")).read()
    declared = set(re.findall(r"\b(srq_[a-z0-9_]+)\s*\(", text))
    assert declared == set(b.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    assert b.status_string(b.OK) == "ok"
    assert "workspace" in b.status_string(b.WORKSPACE)
    assert b.status_string(99) == "unknown status"


def test_workspace_sizes_grow_with_problem_and_density(lib):
    small = b.workspace_bytes(256, 256, 256, 0.05)
    big = b.workspace_bytes(2048, 2048, 2048, 0.05)
    dense = b.workspace_bytes(2048, 2048, 2048, 1.0)
    assert 0 < small < big < dense
    assert dense - big >= int(0.95 * 2 * 2048 * 2048 * 5 * 0.99)
    assert b.stage_workspace_bytes(256, 256, 256) <= small
    out = C.c_size_t()
    assert lib.srq_workspace_bytes(-1, 2, 2, 0.5, C.byref(out)) == b.INVALID_ARG
    assert lib.srq_workspace_bytes(2, 2, 2, 1.5, C.byref(out)) == b.INVALID_ARG
    assert lib.srq_workspace_bytes(2, 2, 2, 0.5, None) == b.INVALID_ARG


@pytest.fixture()
def dry(lib):
    h = b.Srq(device=None, check=False)
    yield h
    h.close()


FAKE = C.c_void_p(0x1000)        # never dereferenced: no launch happens without a device


def _quantize(h, **kw):
    a = dict(X=FAKE, rows=8, cols=8, ldx=8, axis=b.AXIS_ROW, bits=8, rnd=b.ROUND_NEAREST_EVEN,
             layout=b.LAYOUT_VECTOR_MAJOR, Q=FAKE, ldq=8, scale=FAKE, lam=FAKE)
    a.update(kw)
    return h.lib.srq_quantize(h.h, a["X"], a["rows"], a["cols"], a["ldx"], a["axis"], a["bits"], a["rnd"],
                              a["layout"], a["Q"], a["ldq"], a["scale"], a["lam"], None)


def test_quantize_validation(dry):
    assert _quantize(dry) == b.NO_DEVICE                       # valid arguments, no device
    assert _quantize(dry, bits=1) == b.UNSUPPORTED
    assert _quantize(dry, bits=9) == b.UNSUPPORTED
    assert _quantize(dry, bits=4) == b.NO_DEVICE
    assert _quantize(dry, rows=-1) == b.INVALID_ARG
    assert _quantize(dry, ldx=7) == b.INVALID_ARG
    assert _quantize(dry, ldq=7) == b.INVALID_ARG
    assert _quantize(dry, axis=2) == b.INVALID_ARG
    assert _quantize(dry, rnd=5) == b.INVALID_ARG
    assert _quantize(dry, layout=3) == b.INVALID_ARG
    assert _quantize(dry, X=None) == b.INVALID_ARG
    assert _quantize(dry, Q=None) == b.INVALID_ARG
    assert _quantize(dry, scale=None) == b.INVALID_ARG
    assert _quantize(dry, lam=None) == b.WORKSPACE             # lambda scratch needs a workspace
    assert _quantize(dry, rows=0) == b.NO_DEVICE               # empty input is a valid no-op
    # column vectors, element-major: ld counts vectors
    assert _quantize(dry, rows=4, cols=8, axis=b.AXIS_COL, layout=b.LAYOUT_ELEMENT_MAJOR, ldq=8) == b.NO_DEVICE
    assert _quantize(dry, rows=4, cols=8, axis=b.AXIS_COL, layout=b.LAYOUT_VECTOR_MAJOR, ldq=4) == b.NO_DEVICE
    assert _quantize(dry, rows=4, cols=8, axis=b.AXIS_COL, layout=b.LAYOUT_VECTOR_MAJOR, ldq=3) == b.INVALID_ARG
    assert dry.lib.srq_quantize(None, FAKE, 8, 8, 8, 0, 8, 0, 0, FAKE, 8, FAKE, FAKE, None) == b.INVALID_ARG


def _cg(h, **kw):
    a = dict(M=64, N=64, K=64, A=FAKE, lda=64, B=FAKE, ldb=64, ta=1.0, tb=1.0, bits=8, rnd=0, s=2.0,
             strat=b.STRATEGY_CSR_VALU, alpha=1.0, beta=0.0, Cin=None, ldcin=0, Cc=FAKE, ldc=64)
    a.update(kw)
    return h.lib.srq_compensated_gemm(h.h, a["M"], a["N"], a["K"], a["A"], a["lda"], a["B"], a["ldb"],
                                      a["ta"], a["tb"], a["bits"], a["rnd"], a["s"], a["strat"], a["alpha"],
                                      a["beta"], a["Cin"], a["ldcin"], a["Cc"], a["ldc"], None, None, None)


def test_compensated_gemm_validation(dry):
    assert _cg(dry) == b.WORKSPACE                              # nothing attached yet
    nbytes = b.workspace_bytes(64, 64, 64, 1.0)
    assert dry.lib.srq_set_workspace(dry.h, C.c_void_p(0x10000), nbytes) == b.OK
    assert dry.lib.srq_set_workspace(dry.h, C.c_void_p(0x10001), nbytes) == b.INVALID_ARG   # alignment
    assert _cg(dry) == b.NO_DEVICE
    assert _cg(dry, bits=16) == b.UNSUPPORTED
    assert _cg(dry, M=-1) == b.INVALID_ARG
    assert _cg(dry, lda=63) == b.INVALID_ARG
    assert _cg(dry, ldb=63) == b.INVALID_ARG
    assert _cg(dry, ldc=63) == b.INVALID_ARG
    assert _cg(dry, A=None) == b.INVALID_ARG
    assert _cg(dry, Cc=None) == b.INVALID_ARG
    assert _cg(dry, ta=-0.5) == b.INVALID_ARG
    assert _cg(dry, ta=float("nan")) == b.INVALID_ARG
    assert _cg(dry, strat=7) == b.INVALID_ARG
    assert _cg(dry, strat=b.STRATEGY_CSR_SMFMAC) == b.NO_DEVICE
    assert _cg(dry, beta=1.0) == b.INVALID_ARG                  # beta needs Cin
    assert _cg(dry, beta=1.0, Cin=FAKE, ldcin=64) == b.NO_DEVICE
    assert _cg(dry, ta=float("inf"), tb=float("inf")) == b.NO_DEVICE
    # a reduced operand of 2^31 or more elements could wrap the INT32 row pointers
    assert _cg(dry, M=65536, K=32768, lda=32768) == b.UNSUPPORTED
    assert _cg(dry, M=65536, K=32768, lda=32768, ta=float("inf")) != b.UNSUPPORTED
    # K bound: 133144 is the largest K for 8 bits; 4-bit codes allow far more
    big = 133145
    assert _cg(dry, K=big, lda=big) == b.K_OVERFLOW
    assert _cg(dry, K=big, lda=big, bits=4) == b.WORKSPACE      # passes the bound, workspace too small
    # a workspace sized for a smaller problem is rejected
    assert dry.lib.srq_set_workspace(dry.h, C.c_void_p(0x10000), b.workspace_bytes(32, 32, 32, 1.0)) == b.OK
    assert _cg(dry) == b.WORKSPACE
    # fixed part fits but there is no room for any compressed entry
    tiny = b.workspace_bytes(64, 64, 64, 0.0)
    assert dry.lib.srq_set_workspace(dry.h, C.c_void_p(0x10000), tiny) == b.OK
    assert _cg(dry) == b.NO_DEVICE


def test_staged_entry_points_validation(dry):
    lib, h = dry.lib, dry.h
    assert lib.srq_set_workspace(h, C.c_void_p(0x10000), b.stage_workspace_bytes(64, 64, 64)) == b.OK
    g = lambda **kw: lib.srq_gemm_i8(h, kw.get("M", 64), 64, kw.get("K", 64), kw.get("Qa", FAKE),
                                     kw.get("lda", 64), FAKE, FAKE, 64, FAKE, kw.get("D", FAKE), None,
                                     kw.get("ldd", 64), kw.get("drow", FAKE), kw.get("dcol", FAKE), None)
    assert g() == b.NO_DEVICE
    assert g(lda=32) == b.INVALID_ARG
    assert g(Qa=None) == b.INVALID_ARG
    assert g(D=None) == b.INVALID_ARG
    assert g(ldd=8) == b.INVALID_ARG
    assert g(drow=None) == b.INVALID_ARG                       # means come as a pair
    assert g(drow=None, dcol=None) == b.NO_DEVICE
    assert g(K=200000, lda=200000) == b.K_OVERFLOW
    # the variant on the library's static scratch array: same validation, no workspace needed, and a
    # problem whose partial sums exceed the array is refused before the device is even looked at
    lib.srq_set_workspace(h, None, 0)
    gs = lambda **kw: lib.srq_gemm_i8_static_scratch(h, kw.get("M", 64), kw.get("N", 64), 64, FAKE, 64, FAKE, FAKE,
                                                     64, FAKE, kw.get("D", FAKE), None, kw.get("N", 64),
                                                     kw.get("drow", FAKE), kw.get("dcol", FAKE), None)
    assert g() == b.WORKSPACE and gs() == b.NO_DEVICE
    assert gs(D=None) == b.INVALID_ARG
    assert lib.srq_static_scratch_bytes() == 8 << 20
    assert gs(M=8192, N=8192) == b.NO_DEVICE                   # exactly fills the array
    assert gs(M=8192, N=8192 + 128) == b.WORKSPACE
    assert gs(M=1 << 20, N=1 << 20, drow=None, dcol=None) == b.NO_DEVICE   # no means, no scratch
    assert lib.srq_set_workspace(h, C.c_void_p(0x10000), b.stage_workspace_bytes(64, 64, 64)) == b.OK
    sp = lambda **kw: lib.srq_spmm_accumulate(h, kw.get("side", 0), kw.get("strat", b.STRATEGY_CSR_VALU), 64, 64,
                                              64, kw.get("ptr", FAKE), FAKE, FAKE, FAKE, kw.get("ldr", 64), FAKE,
                                              FAKE, FAKE, None, 64, None)
    assert sp() == b.NO_DEVICE
    assert sp(strat=b.STRATEGY_AUTO) == b.INVALID_ARG
    assert sp(strat=b.STRATEGY_CSR_SMFMAC) == b.INVALID_ARG   # whole-path call only
    assert sp(side=3) == b.INVALID_ARG
    assert sp(ptr=None) == b.INVALID_ARG
    assert sp(ldr=8) == b.INVALID_ARG
    assert sp(strat=b.STRATEGY_CSR_MFMA) == b.NO_DEVICE
    bs = lambda **kw: lib.srq_build_sparse_residual(
        h, FAKE, 64, 64, 64, kw.get("axis", 0), FAKE, kw.get("lam", FAKE), kw.get("thresh", FAKE), 8, 0,
        kw.get("Rq", FAKE), 64, 0, kw.get("rscale", FAKE), kw.get("ptr", FAKE), FAKE, FAKE,
        kw.get("cap", 100), FAKE, None)
    assert bs() == b.NO_DEVICE
    assert bs(lam=None) == b.INVALID_ARG
    assert bs(thresh=None) == b.INVALID_ARG
    assert bs(rscale=None) == b.INVALID_ARG                    # Rq without rscale
    assert bs(Rq=None, rscale=None) == b.NO_DEVICE             # selection only
    assert bs(cap=-1) == b.INVALID_ARG
    assert bs(cap=2 ** 31) == b.INVALID_ARG
    assert lib.srq_set_scale_mode(h, b.SCALE_GLOBAL) == b.OK
    assert lib.srq_set_scale_mode(h, 7) == b.INVALID_ARG
    assert lib.srq_set_scale_mode(None, b.SCALE_VECTOR) == b.INVALID_ARG
    assert lib.srq_set_scale_mode(h, b.SCALE_VECTOR) == b.OK


def test_missing_library_fails_loudly(monkeypatch, lib):
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", os.path.join(ROOT, "does_not_exist", "libsrq.so"))
    with pytest.raises(RuntimeError, match="not built"):
        b.load()


def test_handle_settings_validation(dry):
    """Host-side setters: argument checks without a device (nothing is launched by any of them)."""
    lib, h = dry.lib, dry.h
    assert lib.srq_set_auto_hint(h, 0, 0) == b.OK
    assert lib.srq_set_auto_hint(h, 1, 2) == b.OK
    assert lib.srq_set_auto_hint(h, 3, 0) == b.INVALID_ARG        # only 0 (none), 1 (vector ALUs), 2 (matrix cores)
    assert lib.srq_set_auto_hint(h, 0, -1) == b.INVALID_ARG
    assert lib.srq_set_auto_hint(None, 0, 0) == b.INVALID_ARG
    assert lib.srq_set_scale_mode(h, b.SCALE_GLOBAL) == b.OK
    assert lib.srq_set_scale_mode(h, 7) == b.INVALID_ARG
    assert lib.srq_set_scale_mode(h, b.SCALE_VECTOR) == b.OK
    ms = (C.c_float * len(b.STAGES))(*([1.0] * len(b.STAGES)))
    assert lib.srq_profile_read(h, ms) == b.OK and all(x == 0.0 for x in ms)   # nothing recorded: zeros
    assert lib.srq_profile_read(h, None) == b.INVALID_ARG
    assert lib.srq_profile_enable(h, 1) == b.NO_DEVICE            # events need a device
    assert lib.srq_profile_enable(h, b.PROFILE_PRODUCTS) == b.NO_DEVICE
    assert lib.srq_profile_enable(h, 0) == b.OK

