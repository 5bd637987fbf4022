#!/usr/bin/env python3
"""Throughput of the sparse-residual-compensated INT8 GEMM on one MI355X.

One step = one srq_compensated_gemm call: FP32 A, B resident in HBM -> FP32 C in HBM, every
step of Algorithm 1 (quantize, INT8 GEMM, dequantize, means, residual codes, threshold-select
and compaction, sparse correction products, epilogue).  Prints ONE JSON line:
effective TOPS = 2MNK / t, the roofline of the dominant kernel from HIP events recorded on
the launch stream inside the timed region, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0       # MI355X dense INT8 MFMA peak, 5.0 POP/s
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E, 8 TB/s
# plain vector ALU integer multiply-add: 256 CU x 4 SIMD x 16 lanes x 2.4 GHz x 2 ops
PEAK_VALU_INT_TOPS = 256 * 4 * 16 * 2.4e9 * 2 / 1e12


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (the chip's clocks settle over the first tens of milliseconds of load: ten warm-up calls)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C3", help="C1..C5 (default C3: 8192^3 with outliers)")
    ap.add_argument("--density", type=float, default=None, help="target density of A' and B'")
    ap.add_argument("--strategy", default="auto", choices=["auto", "valu", "mfma", "smfmac", "colblock"])
    ap.add_argument("--dense-fallback", type=float, default=2.0, help="Algorithm 1's limit s (>1: off)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-accuracy", action="store_true")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the timing of the plain (theta=inf) and unreduced (theta=0) variants")
    ap.add_argument("--stage", default=None, choices=["quantize", "build_sparse_residual", "gemm"],
                    help="time one staged entry point on the workload's operands instead of the whole path "
                         "(prints its own JSON line: achieved GB/s against the HBM peak; gemm: srq_gemm_i8 without "
                         "the means, TOP/s against the INT8 matrix-core peak)")
    ap.add_argument("--operands", default="workload", choices=["workload", "random", "zeros"],
                    help="--stage gemm only: the workload's own codes, uniformly random codes or all-zero codes "
                         "(the chip's clock under load depends on how much the operands toggle)")
    ap.add_argument("--compare-library", action="store_true",
                    help="--stage gemm only: also time the vendor library's INT8 GEMM (torch._int_mm, INT32 out, no "
                         "scaling) on the same codes, in alternating blocks of launches, and report it beside "
                         "the kernel's own figure as `library_int_mm` (a reference point, not part of the path)")
    ap.add_argument("--eager", "--no-graph", dest="eager", action="store_true",
                    help="skip the graph replay that is otherwise measured after the timed region and reported "
                         "beside it as `graph_replay`")
    ap.add_argument("--time-all-stages", action="store_true",
                    help="record the library's events around every stage inside the timed region (0.04 ms per "
                         "call at C3) instead of around the three products only, with the other stages timed "
                         "over further calls after the region")
    ap.add_argument("--report", default=None, help="also write the full report to this JSON file")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device copy (reference point for the FETCH_SIZE / "
                         "WRITE_SIZE counters) and exit")
    return ap.parse_args()


def recorded_traffic(workload):
    """HBM bytes per first-product launch from the committed rocprofv3 counter summary of this
    workload (FETCH_SIZE and WRITE_SIZE runs, scaled by a plain copy) and where the figure comes
    from; (None, None) when no summary exists.  bench.py cannot run the profiler on itself, so the
    figure is recorded, not measured in this run: `traffic_source` in the JSON line says so."""
    rel = os.path.join("profiles", "bench_%s_hbm_traffic.md" % workload)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), rel)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("TRAFFIC_BYTES_PER_GEMM_LAUNCH"):
                    return int(line.split("=")[1]), rel + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE; recorded, not measured in this run)"
    except OSError:
        pass
    return None, None


def cpu_baseline(name, A, B, theta_a, theta_b):
    """The oracle as it stands, on a bounded sample: the first rows of A against all of B."""
    import numpy as np
    from oracle import srq_oracle as o
    M, K = A.shape
    N = B.shape[1]
    budget = 3.3e12                                   # about 10-30 s of oracle work on 16 cores
    per_row = 3.0 * 2.0 * N * K
    ms = int(max(64, min(M, budget // per_row)))
    As = np.ascontiguousarray(A[:ms])
    t0 = time.perf_counter()
    o.compensated_gemm(As, B, theta_a, theta_b)
    dt = time.perf_counter() - t0
    try:
        import threadpoolctl
        cores = max(int(i.get("num_threads", 1)) for i in threadpoolctl.threadpool_info()) \
            if threadpoolctl.threadpool_info() else os.cpu_count()
    except Exception:
        cores = os.cpu_count()
    return {"value": 2.0 * ms * N * K / dt / 1e12, "unit": "TOPS", "cores": int(cores), "kind": "oracle",
            "sample": "rows 0..%d of A against all of B (M=%d, N=%d, K=%d), full Algorithm 1, %.1f s"
                      % (ms - 1, ms, N, K, dt)}


def stage_bench(args, b, torch, h, w, Ad, Bd, sa, sb, drow, dcol, theta_a, theta_b):
    """srq_quantize or srq_build_sparse_residual on both operands of the workload (A by rows, B by
    columns), HIP-event timed on the launch stream; algorithmic bytes: quantize reads 4 B and writes
    1 B per element; build_sparse_residual reads each element for the residual codes (4 B in, 1 B
    out), once more for the selection (4 B) and writes 5 B per kept entry and 4 B per vector."""
    M, N, K = w.M, w.N, w.K
    Qa, sa, lam_a = h.quantize(Ad, b.AXIS_ROW)
    Qb, sb, lam_b = h.quantize(Bd, b.AXIS_COL)
    t_a = (drow * theta_a).contiguous()
    t_b = (dcol * theta_b).contiguous()
    nnz = [0, 0]
    if args.stage == "gemm":
        if args.operands == "random":
            Qa = torch.randint(-127, 128, (M, K), dtype=torch.int8, device="cuda")
            Qb = torch.randint(-127, 128, (N, K), dtype=torch.int8, device="cuda")
        elif args.operands == "zeros":
            Qa.zero_()
            Qb.zero_()
        out = (torch.empty((M, N), dtype=torch.float32, device="cuda"), None, None)
        for _ in range(args.warmup):
            h.gemm_i8(Qa, sa, Qb, sb, want_means=False, out=out)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            h.gemm_i8(Qa, sa, Qb, sb, want_means=False, out=out)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        tops = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        line = {"metric": "TOP/s of srq_gemm_i8 (first product, no means), %s codes" % args.operands,
                "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                "ms_per_step": ms, "higher_is_better": True, "dtype": "int8", "data": "synthetic",
                "config": {"workload": "%s: M=%d N=%d K=%d" % (w.name, M, N, K), "operands": args.operands},
                "roofline": {"bound": "mfma", "achieved": tops, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                             "frac": tops / PEAK_INT8_TOPS}}
        if args.compare_library:
            # the clock under sustained matrix-core load settles over tens of launches and differs from
            # box to box, so the two are timed in alternating blocks inside one warm sequence
            Ci = torch.empty((M, N), dtype=torch.int32, device="cuda")
            QbT = Qb.t()                              # the library takes B as K x N; this view is column-major
            try:
                torch._int_mm(Qa, QbT, out=Ci)
            except Exception as ex:                   # no INT8 GEMM in this torch build / for this shape
                line["library_int_mm"] = {"value": None, "note": "torch._int_mm failed: %r" % (ex,)}
                print(json.dumps(line))
                return
            blocks, per = 6, max(1, args.steps // 6)
            t_own, t_lib = [], []
            for blk in range(blocks + 1):
                for fn, acc in ((lambda: h.gemm_i8(Qa, sa, Qb, sb, want_means=False, out=out), t_own),
                                (lambda: torch._int_mm(Qa, QbT, out=Ci), t_lib)):
                    e0.record()
                    for _ in range(per):
                        fn()
                    e1.record()
                    torch.cuda.synchronize()
                    if blk:                           # the first pair of blocks warms both up
                        acc.append(e0.elapsed_time(e1) / per)
            mo, ml = sum(t_own) / len(t_own), sum(t_lib) / len(t_lib)
            line["library_int_mm"] = {"ms_per_launch": ml, "value": 2.0 * M * N * K / (ml * 1e-3) / 1e12, "unit": "TOPS",
                                      "own_ms_per_launch_alternating": mo, "own_over_library_time": mo / ml,
                                      "note": "torch._int_mm (INT32 output, no scales) on the same codes; blocks of %d "
                                              "launches, alternating, %d blocks each" % (per, blocks)}
        print(json.dumps(line))
        return

    def run():
        if args.stage == "quantize":
            h.quantize(Ad, b.AXIS_ROW)
            h.quantize(Bd, b.AXIS_COL)
        else:
            ra = h.build_sparse_residual(Ad, b.AXIS_ROW, sa, lam_a, t_a, capacity=int(M * K * 0.08))
            rb = h.build_sparse_residual(Bd, b.AXIS_COL, sb, lam_b, t_b, capacity=int(N * K * 0.08))
            nnz[0], nnz[1] = ra["nnz"], rb["nnz"]

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    elems = float(M * K + K * N)
    if args.stage == "quantize":
        nbytes = 5.0 * elems + 8.0 * (M + N)
        kept = None
    else:
        kept = int(nnz[0].item()) + int(nnz[1].item())
        nbytes = 9.0 * elems + 5.0 * kept + 4.0 * (M + N + 2)
    print(json.dumps({"metric": "achieved HBM GB/s of srq_%s (A by rows + B by columns)" % args.stage,
                      "value": nbytes / (ms * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "dtype": "int8",
                      "data": "synthetic", "config": {"workload": "%s: M=%d N=%d K=%d" % (w.name, M, N, K)},
                      "roofline": {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                                   "unit": "GB/s", "frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                   "algorithmic_bytes": nbytes, "kept_entries": kept,
                                   "note": "includes the binding's output allocations (torch caching allocator)"}}))


def main():
    args = parse()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build measures one GPU only (the path is a single-device "
                         "kernel pipeline; sharding would split C by row blocks, one handle per GPU); "
                         "run with --gpus 1\n")
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2403_06924_amd import binding as b
    from paper_2403_06924_amd import workloads as wl

    if not os.path.exists(b.LIB_PATH):
        from paper_2403_06924_amd import build
        build.build()
    if not torch.cuda.is_available():
        sys.stderr.write("bench.py needs a GPU\n")
        sys.exit(3)
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": 1 << 30, "copies": 5}))
        return
    w = wl.WORKLOADS[args.workload]
    density = args.density if args.density is not None else w.densities[0 if len(w.densities) == 1 else 1]
    M, N, K = w.M, w.N, w.K
    A, B = wl.make_inputs(w.name)
    Ad, Bd = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    h = b.Srq(device=0)

    # threshold factors for the requested density, from the GPU's own first product
    Qa, sa, _ = h.quantize(Ad, b.AXIS_ROW)
    Qb, sb, _ = h.quantize(Bd, b.AXIS_COL)
    _, _, drow, dcol = h.gemm_i8(Qa, sa, Qb, sb)
    theta_a = wl.theta_for_density(Ad, drow, 0, density)
    theta_b = wl.theta_for_density(Bd, dcol, 1, density)
    if args.stage:
        stage_bench(args, b, torch, h, w, Ad, Bd, sa, sb, drow, dcol, theta_a, theta_b)
        h.close()
        return
    del Qa, Qb
    torch.cuda.empty_cache()

    strategy = {"auto": b.STRATEGY_AUTO, "valu": b.STRATEGY_CSR_VALU, "mfma": b.STRATEGY_CSR_MFMA,
                "smfmac": b.STRATEGY_CSR_SMFMAC, "colblock": b.STRATEGY_COLBLOCK}[args.strategy]
    stats = b.stats_tensor()
    Cd = torch.empty((M, N), dtype=torch.float32, device="cuda")
    max_density = min(1.0, density * 1.25 + 0.01)

    def step():
        h.compensated_gemm(Ad, Bd, theta_a, theta_b, strategy=strategy,
                           dense_fallback_density=args.dense_fallback, out=Cd, stats=stats,
                           max_density=max_density)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Inside the timed region the library times the three products only (the launches of the
    # roofline below): every event record costs a call about 3 us, because the kernel after it
    # cannot start under the tail of the kernel before it.  The other stages are timed over a few
    # further calls after the region.
    product_stages = ("gemm", "term1", "term2")
    h.profile_enable(True, products_only=not args.time_all_stages)
    stage_ms = {k: 0.0 for k in b.STAGES}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
        if (i + 1) % 64 == 0 or i + 1 == args.steps:    # the library keeps the events of 64 calls
            for k, v in h.profile_read().items():       # waits for the events of the steps so far
                stage_ms[k] += v
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    stage_ms = {k: v / args.steps for k, v in stage_ms.items()}
    extra = 0 if args.time_all_stages else min(args.steps, 20)
    if extra:
        h.profile_enable(True)
        for _ in range(extra):
            step()
        for k, v in h.profile_read().items():
            if k not in product_stages:
                stage_ms[k] = v / extra
    h.profile_enable(False)
    graph_replay = None
    recordable = args.dense_fallback > 1.0 or args.dense_fallback <= 0.0
    if recordable and not args.eager:
        # Beside the timed region: the same K steps recorded once into a HIP graph (kernels only: a call
        # allocates nothing and reads nothing back) and replayed, so that no launch gap separates the
        # kernels of a step.  Reported as `graph_replay`; the headline stays the eager region above,
        # whose stage events are live (event records inside a replayed graph cannot be read back).
        gs = max(d for d in range(1, min(args.steps, 64) + 1) if args.steps % d == 0)
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(gs):
                    step()
            for _ in range(max(1, args.warmup // gs)):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps // gs):
                graph.replay()
            torch.cuda.synchronize()
            g_ms = (time.perf_counter() - t0) / args.steps * 1e3
            graph_replay = {"ms_per_step": g_ms, "value": 2.0 * M * N * K / (g_ms * 1e-3) / 1e12, "unit": "TOPS",
                            "note": "%d steps recorded once into a HIP graph, replayed %d time(s), after the "
                                    "timed region" % (gs, args.steps // gs)}
        except RuntimeError as e:
            sys.stderr.write("bench.py: graph replay not available (%s)\n" % (e,))
    st = b.read_stats(stats)
    ops = 2.0 * M * N * K
    value = ops / (ms_per_step * 1e-3) / 1e12

    # ---- roofline.  Two kinds of launches of the matrix-core kernel make up a step:
    #  * the first product (a2 + a3 + a4): a dense contraction, 2MNK integer operations, against
    #    the dense INT8 matrix-core peak.  This is the `roofline` entry proper.
    #  * the correction launch(es) (a7 + a8).  The method's own work there is
    #    2 (nnz_A N + nnz_B M) operations (the sparse products of Algorithm 1 line 12); what the
    #    chosen execution actually issues is reported next to it: on the dense matrix-core kernel
    #    (paths 2, 3) every term issues a full 2MNK, of which the zero-filled part multiplies zeros;
    #    on the 2:4 kernel (path 4) a term issues half of that; on the vector ALUs (path 1) only the
    #    method's own operations are issued.
    # Times are HIP events recorded by the library on the launch stream around each stage, inside
    # the timed region (srq_profile_enable).
    gemm_ms = stage_ms["gemm"]
    ach = ops / (gemm_ms * 1e-3) / 1e12
    traffic, traffic_src = recorded_traffic(args.workload)
    roof = {"kernel": "gemm_i8_persistent_kernel, first product (a2+a3+a4)", "bound": "mfma", "achieved": ach,
            "peak": PEAK_INT8_TOPS, "unit": "TOP/s", "frac": ach / PEAK_INT8_TOPS, "launch_ms": gemm_ms,
            "ops_per_launch": ops, "traffic": traffic, "traffic_source": traffic_src,
            # context, not the roofline: what a register-resident loop of the same instruction
            # sustained on this chip with random operand bytes (it reaches 4950 on zeros)
            "mfma_sustained_random_operands": 3440.0}
    own_ops = 2.0 * (st["nnz_a"] * N + st["nnz_b"] * M)
    corr_ms = sum(stage_ms[k] for k in ("term1_prep", "term1", "term2_prep", "term2"))
    issued, units = 0.0, set()
    for path, own in ((st["path_a"], 2.0 * st["nnz_a"] * N), (st["path_b"], 2.0 * st["nnz_b"] * M)):
        if path in (2, 3):
            issued += ops
            units.add("mfma")
        elif path == 4:
            issued += ops / 2
            units.add("smfmac")
        elif path == 1:
            issued += own
            units.add("valu")
        elif path == 5:                      # dense strip of one K-tile on the matrix cores + CSR remainder
            issued += own + 2.0 * M * N * 128
            units.update(("mfma", "valu"))
    corr = None
    if corr_ms > 0:
        on_valu = units == {"valu"}
        peak = PEAK_VALU_INT_TOPS if on_valu else PEAK_INT8_TOPS
        corr = {"stages": "a7+a8 (both correction terms" + (", one paired launch)" if stage_ms["term2"] == 0
                                                            and st["path_b"] else ")"),
                "executed_on": sorted(units), "launch_ms": corr_ms,
                "own_work_ops": own_ops, "own_work_achieved": own_ops / (corr_ms * 1e-3) / 1e12,
                "peak": peak, "unit": "TOP/s",
                "own_work_frac": own_ops / (corr_ms * 1e-3) / 1e12 / peak,
                "issued_ops": issued, "issued_frac": issued / (corr_ms * 1e-3) / 1e12 / peak,
                "zero_fraction_of_sparse_operands": 1.0 - (st["nnz_a"] + st["nnz_b"]) / float(M * K + N * K)}
    roof["corrections"] = corr
    # the products of a whole step on their own work: first product + the method's sparse products
    prod_ms = gemm_ms + corr_ms
    roof["products_own_work"] = {"ops": ops + own_ops, "ms": prod_ms,
                                 "frac_of_int8_mfma_peak": (ops + own_ops) / (prod_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS}

    accuracy = None
    if not args.no_accuracy:
        C64 = Ad.double() @ Bd.double()
        nrm = torch.linalg.norm(C64)
        e_comp = float(torch.linalg.norm(C64 - Cd.double()) / nrm)
        inf = float("inf")
        h.compensated_gemm(Ad, Bd, inf, inf, out=Cd)
        e_plain = float(torch.linalg.norm(C64 - Cd.double()) / nrm)
        h.compensated_gemm(Ad, Bd, 0.0, 0.0, strategy=b.STRATEGY_CSR_MFMA, dense_fallback_density=0.0, out=Cd)
        e_dense = float(torch.linalg.norm(C64 - Cd.double()) / nrm)
        accuracy = {"rel_err_vs_fp64_plain_int8": e_plain, "rel_err_vs_fp64_compensated": e_comp,
                    "rel_err_vs_fp64_dense_residual": e_dense}
        del C64

    # the paper's reference columns on the same inputs: plain vector-wise INT8 (theta = inf,
    # "origin") and compensation with the unreduced operands (theta = 0, "full"); and the part
    # of a step that remains when both operands arrive quantized (everything but a1 and a5)
    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / reps * 1e3
    variants = None
    if not args.no_variants:
        inf = float("inf")
        ms_plain = timed(lambda: h.compensated_gemm(Ad, Bd, inf, inf, out=Cd))
        ms_full = timed(lambda: h.compensated_gemm(Ad, Bd, 0.0, 0.0, dense_fallback_density=0.0, out=Cd))
        variants = {"plain_int8_ms": ms_plain, "plain_int8_tops": ops / (ms_plain * 1e-3) / 1e12,
                    "dense_compensated_ms": ms_full, "dense_compensated_tops": ops / (ms_full * 1e-3) / 1e12,
                    "prequantized_ms": sum(v for k, v in stage_ms.items() if k not in ("quantize", "residual"))}

    # the streaming stages against the HBM peak, on their algorithmic bytes: a1 + a5 read each
    # FP32 element once and write its code and its residual code; a6 reads each FP32 element
    # once more and writes 5 bytes per kept entry plus one pointer per vector
    PEAK_HBM_GBS = 8000.0
    q_bytes = 6.0 * (M * K + K * N) + 16.0 * (M + N)
    s_bytes = 4.0 * (M * K + K * N) + 5.0 * (st["nnz_a"] + st["nnz_b"]) + 4.0 * (M + N + 2)
    q_ms = stage_ms["quantize"] + stage_ms["residual"]
    stage_rooflines = {
        "quantize+residual": {"bound": "hbm", "algorithmic_bytes": q_bytes,
                              "achieved": q_bytes / (q_ms * 1e-3) / 1e9 if q_ms > 0 else None,
                              "peak": PEAK_HBM_GBS, "unit": "GB/s"},
        "select": {"bound": "hbm", "algorithmic_bytes": s_bytes,
                   "achieved": s_bytes / (stage_ms["select"] * 1e-3) / 1e9 if stage_ms["select"] > 0 else None,
                   "peak": PEAK_HBM_GBS, "unit": "GB/s"},
    }
    for r in stage_rooflines.values():
        r["frac"] = r["achieved"] / r["peak"] if r["achieved"] else None

    out = {
        "metric": "effective TOPS (2MNK/s) of compensated INT8 GEMM", "value": value, "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "%s: M=%d N=%d K=%d, %s, seed %d" % (w.name, M, N, K, w.recipe, w.seed),
                   "target_density": density, "theta_a": theta_a, "theta_b": theta_b,
                   "strategy": args.strategy, "dense_fallback_density": args.dense_fallback,
                   "bits": 8, "rounding": "nearest_even",
                   "launch": "eager"},
        "frac_of_int8_mfma_peak": value / PEAK_INT8_TOPS,
        "density_a": st["nnz_a"] / (M * K), "density_b": st["nnz_b"] / (N * K),
        "path_a": st["path_a"], "path_b": st["path_b"],
        "stage_ms": stage_ms,
        "stage_ms_source": "HIP events around every stage inside the timed region" if args.time_all_stages else
                           "gemm, term1, term2: HIP events around the launches inside the timed region; the other "
                           "stages: the same events over %d further calls after it" % min(args.steps, 20),
        "graph_replay": graph_replay,
        "variants": variants,
        "roofline": roof,
        "stage_rooflines": stage_rooflines,
        "accuracy": accuracy,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w.name, A, B, theta_a, theta_b)
    line = json.dumps(out)
    if args.report:
        os.makedirs(os.path.dirname(os.path.abspath(args.report)), exist_ok=True)
        with open(args.report, "w") as f:
            f.write(json.dumps(out, indent=1) + "\n")
    print(line)
    h.close()


if __name__ == "__main__":
    main()
