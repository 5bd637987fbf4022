"""Precision sweep on the GPU: the paper's five input distributions at 1024^2, INT8 and INT4
(Sec. 4.1.1, caption of the precision figure), with the direct quantization ("origin",
theta = inf), the compensation with unreduced operands ("full", theta = 0) and the sparse
compensation over a sweep of densities; "full, global scale" is the unreduced compensation under
one matrix-wide first-level scale per operand (Sec. 2.3), the setting of the paper's "Full" curve.

    python -m paper_2403_06924_amd.precision_sweep [--size 1024] [--seed 7]

Prints one markdown table per bit width.  The error is E_delta = ||C64 - C||_F / ||C64||_F
against an FP64 product (Sec. 3.2's metric).  The sweep is over the density of A' and B'
rather than over the paper's Th axis: the printed selection rule (Eq. avgQuan) compares an
entry with theta times the mean |D_F| of its row, which grows with K, so the theta that
gives a certain density is workload dependent; the harness calibrates it per operand from
the quantile of |x| / mean|D_F| and reports it.  The column "Th(2*mean)" gives, for
orientation, the same threshold expressed as a multiple of twice the mean |x| of the
vector, the scale on which the densities quoted in Sec. 4.1.4 (0.2 at Th = 0.8 for
uniform(0,1); 0.3 at about 0.6 for exponential, normal and Poisson, at about 0.5 for
chi-square) come out.
"""
import argparse

import numpy as np

from . import workloads as wl

KINDS = ("uniform", "normal", "exponential", "poisson", "chisquare")
DENSITIES = (0.01, 0.05, 0.10, 0.20, 0.30, 0.50)


def rel_err(torch, C64, C):
    return float(torch.linalg.norm(C64 - C.double()) / torch.linalg.norm(C64))


def sweep(size, seed, bits_list=(8, 4), kinds=KINDS, densities=DENSITIES, out=print):
    import torch
    from . import binding as b
    if not torch.cuda.is_available():
        raise RuntimeError("precision_sweep needs a GPU")
    h = b.Srq(device=0)
    rows = []
    for bits in bits_list:
        out("\n### INT%d, %d x %d x %d, seed %d\n" % (bits, size, size, size, seed))
        out("| distribution | origin | full | full, global scale | " + " | ".join("d=%.2f" % d for d in densities) + " |")
        out("|---|---|---|---|" + "---|" * len(densities))
        for kind in kinds:
            A = torch.from_numpy(wl.paper_distribution(kind, (size, size), seed)).cuda()
            B = torch.from_numpy(wl.paper_distribution(kind, (size, size), seed + 1)).cuda()
            C64 = A.double() @ B.double()
            inf = float("inf")
            C, _, _ = h.compensated_gemm(A, B, inf, inf, bits=bits)
            e_origin = rel_err(torch, C64, C)
            C, _, _ = h.compensated_gemm(A, B, 0.0, 0.0, bits=bits, dense_fallback_density=0.0)
            e_full = rel_err(torch, C64, C)
            h.set_scale_mode(b.SCALE_GLOBAL)        # the matrix-wide scale of the paper's earlier method
            C, _, _ = h.compensated_gemm(A, B, 0.0, 0.0, bits=bits, dense_fallback_density=0.0)
            e_full_global = rel_err(torch, C64, C)
            h.set_scale_mode(b.SCALE_VECTOR)
            Qa, sa, _ = h.quantize(A, b.AXIS_ROW, bits=bits)
            Qb, sb, _ = h.quantize(B, b.AXIS_COL, bits=bits)
            _, _, drow, dcol = h.gemm_i8(Qa, sa, Qb, sb)
            cells = []
            for d in densities:
                ta, tb = wl.theta_for_density(A, drow, 0, d), wl.theta_for_density(B, dcol, 1, d)
                stats = b.stats_tensor()
                C, _, _ = h.compensated_gemm(A, B, ta, tb, bits=bits, stats=stats)
                torch.cuda.synchronize()
                st = b.read_stats(stats)
                e = rel_err(torch, C64, C)
                th2 = float((ta * drow / (2.0 * A.abs().mean(dim=1))).mean())
                rows.append({"bits": bits, "kind": kind, "target_density": d,
                             "density_a": st["nnz_a"] / (size * size), "density_b": st["nnz_b"] / (size * size),
                             "theta_a": ta, "theta_b": tb, "th_2mean": th2, "err": e,
                             "err_origin": e_origin, "err_full": e_full, "err_full_global": e_full_global})
                cells.append("%.2e (Th %.2f)" % (e, th2))
            out("| %s | %.2e | %.2e | %.2e | %s |" % (kind, e_origin, e_full, e_full_global, " | ".join(cells)))
    h.close()
    return rows


def qr_driver_table(size, seed, bits_list=(8, 4), kinds=("chisquare", "uniform", "normal", "exponential"),
                    densities=(0.05, 0.2, 0.5), block=64, out=print):
    """The QR experiment of Sec. 4.2 in the form of its table: a blocked Householder QR
    (qr.householder_qr) whose trailing updates, accumulation of Q and final Q.R all run through
    srq_compensated_gemm, E = ||X - Q.R||_F / ||X||_F per distribution, bit width and method
    (origin = direct quantization, full = unreduced compensation, sparse at the given densities)."""
    import torch
    from . import binding as b
    from . import qr
    h = b.Srq(device=0)
    rows = []
    out("\n### Householder QR (block %d) with every large product through the library, %d x %d, seed %d: "
        "E = ||X - Q.R||_F / ||X||_F\n" % (block, size, size, seed))
    out("| distribution | bits | FP32 | origin | full | " + " | ".join("d=%.2f" % d for d in densities) + " |")
    out("|---|---|---|---|---|" + "---|" * len(densities))
    for kind in kinds:
        X = torch.from_numpy(wl.paper_distribution(kind, (size, size), seed)).cuda()
        X64 = X.double()
        Q, R = qr.householder_qr(X, block=block)
        e_fp32 = rel_err(torch, X64, Q @ R)
        for bits in bits_list:
            cells = []
            for mm in ([qr.LibraryMatmul(h, "origin", bits), qr.LibraryMatmul(h, "full", bits)] +
                       [qr.LibraryMatmul(h, "sparse", bits, density=d) for d in densities]):
                Q, R = qr.householder_qr(X, mm, block=block)
                cells.append(rel_err(torch, X64, mm(Q, R)))
            rows.append((kind, bits, e_fp32, cells))
            out("| %s | %d | %.2e | %s |" % (kind, bits, e_fp32, " | ".join("%.2e" % c for c in cells)))
    h.close()
    return rows


def qr_table(size, seed, bits_list=(8, 4), kinds=("chisquare", "uniform", "normal", "exponential"),
             densities=(0.05, 0.2, 0.5), out=print):
    """The last product of the QR experiment alone: Q.R of finished (numpy) Householder factors by
    the quantized products against the factored matrix."""
    import torch
    from . import binding as b
    h = b.Srq(device=0)
    rows = []
    out("\n### Q.R of a Householder factorization, %d x %d, seed %d: E = ||X - Q.R||_F / ||X||_F\n" % (size, size, seed))
    out("| distribution | bits | FP32 | origin | full | " + " | ".join("d=%.2f" % d for d in densities) + " |")
    out("|---|---|---|---|---|" + "---|" * len(densities))
    for kind in kinds:
        X, Qh, Rh = wl.qr_factors(kind, size, seed)
        X64 = torch.from_numpy(X).cuda().double()
        Q, R = torch.from_numpy(Qh).cuda(), torch.from_numpy(Rh).cuda()
        e_fp32 = rel_err(torch, X64, Q @ R)
        for bits in bits_list:
            inf = float("inf")
            C, _, _ = h.compensated_gemm(Q, R, inf, inf, bits=bits)
            e_origin = rel_err(torch, X64, C)
            C, _, _ = h.compensated_gemm(Q, R, 0.0, 0.0, bits=bits, dense_fallback_density=0.0)
            e_full = rel_err(torch, X64, C)
            Qa, sa, _ = h.quantize(Q, b.AXIS_ROW, bits=bits)
            Qb, sb, _ = h.quantize(R, b.AXIS_COL, bits=bits)
            _, _, drow, dcol = h.gemm_i8(Qa, sa, Qb, sb)
            cells = []
            for d in densities:
                ta, tb = wl.theta_for_density(Q, drow, 0, d), wl.theta_for_density(R, dcol, 1, d)
                C, _, _ = h.compensated_gemm(Q, R, ta, tb, bits=bits)
                cells.append(rel_err(torch, X64, C))
            rows.append((kind, bits, e_fp32, e_origin, e_full, cells))
            out("| %s | %d | %.2e | %.2e | %.2e | %s |" % (kind, bits, e_fp32, e_origin, e_full,
                                                          " | ".join("%.2e" % c for c in cells)))
    h.close()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--size", type=int, default=1024)
    ap.add_argument("--seed", type=int, default=7)
    ap.add_argument("--qr", action="store_true",
                    help="also run the QR experiment of Sec. 4.2 (blocked Householder QR through the library)")
    ap.add_argument("--qr-factors", action="store_true", help="also multiply finished QR factors (last product only)")
    ap.add_argument("--only-qr", action="store_true", help="skip the precision sweep")
    args = ap.parse_args()
    if not args.only_qr:
        sweep(args.size, args.seed)
    if args.qr or args.only_qr:
        qr_driver_table(args.size, args.seed)
    if args.qr_factors:
        qr_table(args.size, args.seed)


if __name__ == "__main__":
    main()
