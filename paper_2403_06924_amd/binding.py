"""ctypes binding of libsrq.so (declared in include/srq.h).

Argument marshalling only: every step of the compensated GEMM runs in the HIP
kernels of the library.  PyTorch is used for device memory (tensors are passed
as raw device pointers) and for the current HIP stream.  There is no CPU
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsrq.so")

# enums of include/srq.h
OK, INVALID_ARG, UNSUPPORTED, K_OVERFLOW, CAPACITY, WORKSPACE, HIP_ERROR, NO_DEVICE = range(8)
AXIS_ROW, AXIS_COL = 0, 1
LAYOUT_VECTOR_MAJOR, LAYOUT_ELEMENT_MAJOR = 0, 1
ROUND_NEAREST_EVEN, ROUND_TRUNC = 0, 1
STRATEGY_AUTO, STRATEGY_CSR_VALU, STRATEGY_CSR_MFMA, STRATEGY_CSR_SMFMAC, STRATEGY_COLBLOCK = 0, 1, 2, 3, 4
SCALE_VECTOR, SCALE_GLOBAL = 0, 1
PROFILE_ALL, PROFILE_PRODUCTS = 1, 2

EXPORTS = [
    "srq_create", "srq_destroy", "srq_workspace_bytes", "srq_set_workspace",
    "srq_stage_workspace_bytes", "srq_last_hip_error", "srq_status_string", "srq_quantize",
    "srq_build_sparse_residual", "srq_gemm_i8", "srq_spmm_accumulate", "srq_compensated_gemm",
    "srq_get_intermediates", "srq_profile_enable", "srq_profile_read", "srq_set_scale_mode",
    "srq_gemm_i8_static_scratch", "srq_static_scratch_bytes", "srq_set_auto_hint",
]
STAGES = ["quantize", "gemm", "select", "residual", "term1_prep", "term1", "term2_prep", "term2"]


class Stats(C.Structure):
    _fields_ = [("nnz_a", C.c_int64), ("nnz_b", C.c_int64), ("path_a", C.c_int32), ("path_b", C.c_int32),
                ("overflow", C.c_int32), ("reserved", C.c_int32)]


class Debug(C.Structure):
    _fields_ = [("D_int", C.c_void_p), ("D_F", C.c_void_p), ("DR1_int", C.c_void_p), ("DR2_int", C.c_void_p)]


class Intermediates(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "A_int", "B_int", "RA_int", "RB_int", "RA_em", "RB_em",
        "s_a", "lam_a", "s_ra", "s_b", "lam_b", "s_rb",
        "drow", "dcol", "t_a", "t_b",
        "a_ptr", "a_idx", "a_val", "b_ptr", "b_idx", "b_val")] + [
        ("capacity_a", C.c_int64), ("capacity_b", C.c_int64), ("ld_codes", C.c_int64)]


class SrqError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: status %d (%s)" % (what, status, status_string(status)))


_lib = None


def load():
    """Load libsrq.so and declare its signatures; raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libsrq.so is not built (%s missing): run `python -m paper_2403_06924_amd.build` "
            "or __graft_entry__.build(); there is no fallback path" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    i64, vp, f32, i32, sz = C.c_int64, C.c_void_p, C.c_float, C.c_int, C.c_size_t
    lib.srq_create.argtypes = [C.POINTER(vp), i32]
    lib.srq_destroy.argtypes = [vp]
    lib.srq_workspace_bytes.argtypes = [i64, i64, i64, C.c_double, C.POINTER(sz)]
    lib.srq_stage_workspace_bytes.argtypes = [i64, i64, i64, C.POINTER(sz)]
    lib.srq_set_workspace.argtypes = [vp, vp, sz]
    lib.srq_last_hip_error.argtypes = [vp]
    lib.srq_status_string.argtypes = [i32]
    lib.srq_status_string.restype = C.c_char_p
    lib.srq_quantize.argtypes = [vp, vp, i64, i64, i64, i32, i32, i32, i32, vp, i64, vp, vp, vp]
    lib.srq_build_sparse_residual.argtypes = [vp, vp, i64, i64, i64, i32, vp, vp, vp, i32, i32, vp, i64, i32,
                                              vp, vp, vp, vp, i64, vp, vp]
    lib.srq_gemm_i8.argtypes = [vp, i64, i64, i64, vp, i64, vp, vp, i64, vp, vp, vp, i64, vp, vp, vp]
    lib.srq_gemm_i8_static_scratch.argtypes = lib.srq_gemm_i8.argtypes
    lib.srq_static_scratch_bytes.argtypes = []
    lib.srq_spmm_accumulate.argtypes = [vp, i32, i32, i64, i64, i64, vp, vp, vp, vp, i64, vp, vp, vp, vp, i64, vp]
    lib.srq_compensated_gemm.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, f32, f32, i32, i32, f32, i32,
                                         f32, f32, vp, i64, vp, i64, vp, C.POINTER(Debug), vp]
    lib.srq_get_intermediates.argtypes = [vp, C.POINTER(Intermediates)]
    lib.srq_profile_enable.argtypes = [vp, i32]
    lib.srq_set_scale_mode.argtypes = [vp, i32]
    lib.srq_set_auto_hint.argtypes = [vp, i32, i32]
    lib.srq_profile_read.argtypes = [vp, C.POINTER(f32)]
    for name in EXPORTS:
        if name not in ("srq_status_string", "srq_static_scratch_bytes"):
            getattr(lib, name).restype = i32
    lib.srq_static_scratch_bytes.restype = sz
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().srq_status_string(int(status)).decode()


def workspace_bytes(M, N, K, max_density=1.0) -> int:
    out = C.c_size_t(0)
    st = load().srq_workspace_bytes(M, N, K, float(max_density), C.byref(out))
    if st:
        raise SrqError(st, "srq_workspace_bytes")
    return out.value


def stage_workspace_bytes(M, N, K) -> int:
    out = C.c_size_t(0)
    st = load().srq_stage_workspace_bytes(M, N, K, C.byref(out))
    if st:
        raise SrqError(st, "srq_stage_workspace_bytes")
    return out.value


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Srq:
    """A library handle plus its workspace.  ``device=None`` gives a handle
    without a device (argument validation only)."""

    def __init__(self, device=0, check=True):
        self.lib = load()
        self.h = C.c_void_p()
        st = self.lib.srq_create(C.byref(self.h), -1 if device is None else int(device))
        if st:
            raise SrqError(st, "srq_create")
        self.device = device
        self.ws = None
        self.check = check

    def close(self):
        if self.h:
            self.lib.srq_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers --------------------------------------------------------------------
    def _ret(self, st, what):
        if st and self.check:
            extra = ""
            if st == HIP_ERROR:
                extra = " hipError=%d" % self.lib.srq_last_hip_error(self.h)
            raise SrqError(st, what + extra)
        return st

    def _stream(self):
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def ensure_workspace(self, nbytes: int):
        """Attach a torch-allocated workspace of at least nbytes."""
        import torch
        if self.ws is None or self.ws.numel() < nbytes:
            self.ws = None
            self.ws = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device="cuda:%d" % self.device)
            off = (-self.ws.data_ptr()) % 256
            self._ws_off = off
            st = self.lib.srq_set_workspace(self.h, C.c_void_p(self.ws.data_ptr() + off), int(nbytes))
            self._ret(st, "srq_set_workspace")
        return self.ws

    def _view(self, ptr, count, dtype):
        """Tensor view of `count` elements of the workspace starting at device pointer ptr."""
        import torch
        if not ptr or count == 0:
            return None
        off = ptr - self.ws.data_ptr()
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        return self.ws[off:off + nbytes].view(dtype)

    def set_scale_mode(self, mode):
        """srq_set_scale_mode: SCALE_VECTOR (default) or SCALE_GLOBAL for later compensated_gemm calls."""
        self._ret(self.lib.srq_set_scale_mode(self.h, int(mode)), "srq_set_scale_mode")

    def set_auto_hint(self, path_a, path_b):
        """srq_set_auto_hint: the executions (1 vector ALUs, 2 matrix cores, 0 none) the caller expects
        STRATEGY_AUTO to pick for term 1 / term 2 in the following calls."""
        self._ret(self.lib.srq_set_auto_hint(self.h, int(path_a), int(path_b)), "srq_set_auto_hint")

    def profile_enable(self, on=True, products_only=False):
        """Stage timers on (every stage, or only the three products: fewer event records in the
        call) or off."""
        level = 0 if not on else (PROFILE_PRODUCTS if products_only else PROFILE_ALL)
        self._ret(self.lib.srq_profile_enable(self.h, level), "srq_profile_enable")

    def profile_read(self):
        """Milliseconds per stage, summed over the compensated_gemm calls since the previous read
        (at most the last 64); waits for their events."""
        ms = (C.c_float * len(STAGES))()
        self._ret(self.lib.srq_profile_read(self.h, ms), "srq_profile_read")
        return dict(zip(STAGES, [float(x) for x in ms]))

    # -- entry points -----------------------------------------------------------------
    def quantize(self, X, axis, bits=8, rounding=ROUND_NEAREST_EVEN, layout=LAYOUT_VECTOR_MAJOR):
        """srq_quantize on a 2-D float32 CUDA tensor (any row stride).  Returns (Q, scale, lambda)."""
        import torch
        rows, cols = X.shape
        nvec, veclen = (rows, cols) if axis == AXIS_ROW else (cols, rows)
        shape = (nvec, veclen) if layout == LAYOUT_VECTOR_MAJOR else (veclen, nvec)
        Q = torch.empty(shape, dtype=torch.int8, device=X.device)
        scale = torch.empty(nvec, dtype=torch.float32, device=X.device)
        lam = torch.empty(nvec, dtype=torch.float32, device=X.device)
        st = self.lib.srq_quantize(self.h, _ptr(X), rows, cols, X.stride(0) if rows else cols, axis, bits,
                                   rounding, layout, _ptr(Q), shape[1], _ptr(scale), _ptr(lam), self._stream())
        self._ret(st, "srq_quantize")
        return Q, scale, lam

    def build_sparse_residual(self, X, axis, scale, lam, thresh, bits=8, rounding=ROUND_NEAREST_EVEN,
                              r_layout=LAYOUT_VECTOR_MAJOR, capacity=None, want_residual=True,
                              want_selection=True):
        """srq_build_sparse_residual.  Returns dict(Rq, rscale, ptr, idx, val, nnz)."""
        import torch
        rows, cols = X.shape
        nvec, veclen = (rows, cols) if axis == AXIS_ROW else (cols, rows)
        self.ensure_workspace(stage_workspace_bytes(max(rows, 1), max(cols, 1), max(rows, cols, 1)))
        dev = X.device
        out = {}
        Rq = rscale = ptr = idx = val = nnz = None
        shape = (nvec, veclen) if r_layout == LAYOUT_VECTOR_MAJOR else (veclen, nvec)
        if want_residual:
            Rq = torch.empty(shape, dtype=torch.int8, device=dev)
            rscale = torch.empty(nvec, dtype=torch.float32, device=dev)
        if want_selection:
            if capacity is None:
                capacity = rows * cols
            ptr = torch.empty(nvec + 1, dtype=torch.int32, device=dev)
            idx = torch.empty(max(capacity, 1), dtype=torch.int32, device=dev)
            val = torch.empty(max(capacity, 1), dtype=torch.int8, device=dev)
            nnz = torch.zeros(1, dtype=torch.int64, device=dev)
        st = self.lib.srq_build_sparse_residual(
            self.h, _ptr(X), rows, cols, X.stride(0) if rows else cols, axis, _ptr(scale), _ptr(lam),
            _ptr(thresh), bits, rounding, _ptr(Rq), shape[1], r_layout, _ptr(rscale), _ptr(ptr), _ptr(idx),
            _ptr(val), capacity or 0, _ptr(nnz), self._stream())
        self._ret(st, "srq_build_sparse_residual")
        out.update(Rq=Rq, rscale=rscale, ptr=ptr, idx=idx, val=val, nnz=nnz)
        return out

    def gemm_i8(self, Qa, sa, Qb, sb, want_int=False, want_means=True, static_scratch=False, out=None):
        """srq_gemm_i8 on vector-major code matrices Qa[M,K], Qb[N,K]; with static_scratch=True
        srq_gemm_i8_static_scratch (no workspace is attached or used; `out` = (D_F, drow, dcol)
        lets the caller pass every output, so that the call itself allocates nothing)."""
        import torch
        M, K = Qa.shape
        N = Qb.shape[0]
        dev = Qa.device
        if not static_scratch:
            self.ensure_workspace(stage_workspace_bytes(max(M, 1), max(N, 1), max(K, 1)))
        D_int = torch.empty((M, N), dtype=torch.int32, device=dev) if want_int else None
        if out is not None:
            D_F, drow, dcol = out
        else:
            D_F = torch.empty((M, N), dtype=torch.float32, device=dev)
            drow = torch.empty(M, dtype=torch.float32, device=dev) if want_means else None
            dcol = torch.empty(N, dtype=torch.float32, device=dev) if want_means else None
        fn = self.lib.srq_gemm_i8_static_scratch if static_scratch else self.lib.srq_gemm_i8
        st = fn(self.h, M, N, K, _ptr(Qa), Qa.stride(0) if M else K, _ptr(sa), _ptr(Qb),
                Qb.stride(0) if N else K, _ptr(sb), _ptr(D_F), _ptr(D_int), N, _ptr(drow),
                _ptr(dcol), self._stream())
        self._ret(st, "srq_gemm_i8_static_scratch" if static_scratch else "srq_gemm_i8")
        self.last_status = st
        return D_F, D_int, drow, dcol

    def spmm_accumulate(self, side, strategy, M, N, K, ptr, idx, val, Rq, s_row, s_col, C_out, want_int=False):
        import torch
        self.ensure_workspace(stage_workspace_bytes(max(M, 1), max(N, 1), max(K, 1)))
        DR = torch.empty((M, N), dtype=torch.int32, device=C_out.device) if want_int else None
        st = self.lib.srq_spmm_accumulate(self.h, side, strategy, M, N, K, _ptr(ptr), _ptr(idx), _ptr(val),
                                          _ptr(Rq), Rq.stride(0), _ptr(s_row), _ptr(s_col), _ptr(C_out),
                                          _ptr(DR), C_out.stride(0), self._stream())
        self._ret(st, "srq_spmm_accumulate")
        return DR

    def compensated_gemm(self, A, B, theta_a, theta_b=None, bits=8, rounding=ROUND_NEAREST_EVEN,
                         dense_fallback_density=2.0, strategy=STRATEGY_AUTO, alpha=1.0, beta=0.0,
                         C_in=None, out=None, stats=None, debug=False, max_density=1.0):
        """srq_compensated_gemm.  Returns (C, stats tensor or None, debug dict or None)."""
        import torch
        if theta_b is None:
            theta_b = theta_a
        M, K = A.shape
        N = B.shape[1]
        dev = A.device
        self.ensure_workspace(workspace_bytes(M, N, K, max_density))
        Cout = out if out is not None else torch.empty((M, N), dtype=torch.float32, device=dev)
        dbg_struct, dbg = None, None
        if debug:
            dbg = {k: torch.zeros((M, N), dtype=torch.int32 if k != "D_F" else torch.float32, device=dev)
                   for k in ("D_int", "D_F", "DR1_int", "DR2_int")}
            dbg_struct = Debug(*[C.c_void_p(dbg[k].data_ptr()) for k in ("D_int", "D_F", "DR1_int", "DR2_int")])
        st = self.lib.srq_compensated_gemm(
            self.h, M, N, K, _ptr(A), A.stride(0) if M else K, _ptr(B), B.stride(0) if K else N,
            float(theta_a), float(theta_b), bits, rounding, float(dense_fallback_density), strategy,
            float(alpha), float(beta), _ptr(C_in), C_in.stride(0) if C_in is not None else 0, _ptr(Cout),
            Cout.stride(0) if M else N, _ptr(stats), C.byref(dbg_struct) if dbg_struct else None,
            self._stream())
        self._ret(st, "srq_compensated_gemm")
        self.last_status = st
        return Cout, stats, dbg

    def intermediates(self, M, N, K):
        """Tensor views (into the workspace) of the last compensated_gemm call's intermediates."""
        import torch
        im = Intermediates()
        self._ret(self.lib.srq_get_intermediates(self.h, C.byref(im)), "srq_get_intermediates")
        out = {}

        def mat(name, r, c, ld):
            v = self._view(getattr(im, name), r * ld, torch.int8)
            out[name] = None if v is None else v.view(r, ld)[:, :c]

        ldc = int(im.ld_codes) if im.ld_codes else K
        mat("A_int", M, K, ldc); mat("B_int", N, K, ldc); mat("RA_int", M, K, ldc); mat("RB_int", N, K, ldc)
        mat("RA_em", K, M, M); mat("RB_em", K, N, N)
        out["ld_codes"] = ldc
        for name, n in (("s_a", M), ("lam_a", M), ("s_ra", M), ("drow", M), ("t_a", M),
                        ("s_b", N), ("lam_b", N), ("s_rb", N), ("dcol", N), ("t_b", N)):
            out[name] = self._view(getattr(im, name), n, torch.float32)
        for side, n, cap in (("a", M, im.capacity_a), ("b", N, im.capacity_b)):
            ptr = self._view(getattr(im, side + "_ptr"), n + 1, torch.int32)
            out[side + "_ptr"] = ptr
            if ptr is not None:
                nnz = min(int(ptr[-1].item()), cap)
                out[side + "_idx"] = self._view(getattr(im, side + "_idx"), nnz, torch.int32) if nnz else \
                    torch.empty(0, dtype=torch.int32, device=ptr.device)
                out[side + "_val"] = self._view(getattr(im, side + "_val"), nnz, torch.int8) if nnz else \
                    torch.empty(0, dtype=torch.int8, device=ptr.device)
        out["capacity_a"], out["capacity_b"] = im.capacity_a, im.capacity_b
        return out


def stats_tensor(device="cuda:0"):
    """Device buffer laid out as srq_stats_t: int64 nnz_a, nnz_b, then int32 path_a, path_b,
    overflow, reserved."""
    import torch
    return torch.zeros(C.sizeof(Stats) // 8, dtype=torch.int64, device=device)


def read_stats(t):
    """Decode a stats tensor written by srq_compensated_gemm (synchronises)."""
    host = t.cpu()
    words = host[2:4].view(dtype=__import__("torch").int32)
    return {"nnz_a": int(host[0]), "nnz_b": int(host[1]), "path_a": int(words[0]), "path_b": int(words[1]),
            "overflow": int(words[2])}
