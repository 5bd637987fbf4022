"""Speed table on the GPU in the form of the paper's Sec. 4.1.3 (TOPS of the algorithm at
different densities, with "Full" and "Origin" beside it): square uniform(0,1) operands, as
in the paper's speed test, effective TOPS = 2 n^3 / t of one srq_compensated_gemm call
(FP32 operands in HBM to FP32 result in HBM, every stage of Algorithm 1 inside t).

    python -m paper_2403_06924_amd.speed_table [--sizes 1024 4096 8192 16384] [--graph]

"Origin" is theta = inf (plain vector-wise INT8), "Full" is theta = 0 on the dense branch
(both corrections with unreduced operands).  The densities are reached by calibrating
theta per operand (quantile of |x| / mean|D_F|, outside the timed region); the strategy is
SRQ_STRATEGY_AUTO, so low densities run on the vector ALUs and high ones on the matrix cores.
"""
import argparse
import time

from . import workloads as wl

DENSITIES = (0.2, 0.05, 0.01, 0.001, 0.0001)


def timed(torch, fn, reps, graph=False):
    fn()
    torch.cuda.synchronize()
    if graph:
        # the call recorded once, replayed `reps` times: no launch gaps between its kernels
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            fn()
        g.replay()
        torch.cuda.synchronize()
        fn = g.replay
    t = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t) / reps


def table(sizes, densities=DENSITIES, seed=11, out=print, graph=False):
    import torch
    from . import binding as b
    if not torch.cuda.is_available():
        raise RuntimeError("speed_table needs a GPU")
    h = b.Srq(device=0)
    out("| size | " + " | ".join("d=%g" % d for d in densities) + " | Full | Origin |")
    out("|---|" + "---|" * (len(densities) + 2))
    rows = []
    for n in sizes:
        A = torch.from_numpy(wl.paper_distribution("uniform", (n, n), seed)).cuda()
        B = torch.from_numpy(wl.paper_distribution("uniform", (n, n), seed + 1)).cuda()
        C = torch.empty((n, n), dtype=torch.float32, device="cuda")
        reps = 3 if n > 8192 else 10
        ops = 2.0 * n ** 3
        Qa, sa, _ = h.quantize(A, b.AXIS_ROW)
        Qb, sb, _ = h.quantize(B, b.AXIS_COL)
        _, _, drow, dcol = h.gemm_i8(Qa, sa, Qb, sb)
        del Qa, Qb
        cells = []
        for d in densities:
            ta, tb = wl.theta_for_density(A, drow, 0, d), wl.theta_for_density(B, dcol, 1, d)
            md = min(1.0, 1.3 * d + 0.01)
            t = timed(torch, lambda: h.compensated_gemm(A, B, ta, tb, out=C, max_density=md), reps, graph)
            cells.append(ops / t / 1e12)
        inf = float("inf")
        t_full = timed(torch, lambda: h.compensated_gemm(A, B, 0.0, 0.0, dense_fallback_density=0.0, out=C), reps,
                       graph)
        t_origin = timed(torch, lambda: h.compensated_gemm(A, B, inf, inf, out=C), reps, graph)
        rows.append((n, cells, ops / t_full / 1e12, ops / t_origin / 1e12))
        out("| %d | %s | %.1f | %.1f |" % (n, " | ".join("%.1f" % c for c in cells), rows[-1][2], rows[-1][3]))
        del A, B, C
    h.close()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sizes", type=int, nargs="+", default=[1024, 4096, 8192, 16384])
    ap.add_argument("--graph", action="store_true",
                    help="time replays of each call recorded into a HIP graph instead of eager calls")
    args = ap.parse_args()
    table(args.sizes, graph=args.graph)


if __name__ == "__main__":
    main()
