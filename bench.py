#!/usr/bin/env python3
"""Benchmark of the Triangle Block SYRK on one MI355X.

One step = one call of tbs_syrk_lower on the benchmark workload (N = 4096, M = 4096, fp64,
C <- C - A A^T on the lower triangle), inputs resident in HBM.  Prints one JSON line with the
whole-job throughput (N(N+1)M flops per step), the roofline figures of the SYRK kernel (HIP events
around every launch on the launch stream) and the CPU oracle timed on the host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--square] [--no-cpu]
"""
import argparse
import json
import sys
import time

import numpy as np

PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3}       # MI355X dense matrix peaks, TFLOP/s
# HBM bytes per launch from rocprofv3 counter runs (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel
# of known size); filled in from the summaries under profiles/ for the workloads measured there.
MEASURED_TRAFFIC_BYTES = {
    # profiles/tbs_syrk_persistent_kernel_f64_n4096_m4096.md: 1.884e9 read + 8.35e7 written (the reading
    # varies by about 5 % from run to run)
    ("syrk_n4096_m4096_f64", False): 1.968e9,
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the clock of the chip rises for some tens of milliseconds after load sets in (the first
    # launches after an idle phase run at about 2.1 GHz, later ones faster), so the warm-up is long enough
    # for the timed launches to see the steady state; a launch of the default workload takes 1.1 ms
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="syrk_n4096_m4096_f64")
    ap.add_argument("--shape", default=None, help="N,M,dtype: a SYRK shape outside the configuration list "
                    "(C <- C - A A^T, A iid N(0,1)/sqrt(M)), for kernel studies")
    ap.add_argument("--square", action="store_true", help="time the square-block baseline instead")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--copy-bytes", type=int, default=0,
                    help="instead of the benchmark: run a plain device copy of this many bytes --steps "
                         "times (reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2202_10217_amd import binding as tb
    from paper_2202_10217_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    tb.load()                                    # fails loudly when the HIP library is missing

    if args.copy_bytes > 0:
        src = torch.ones(args.copy_bytes // 8, dtype=torch.float64, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": src.numel() * 8, "launches": args.steps}))
        return 0

    if args.shape:
        n_, m_, dt_ = args.shape.split(",")
        dt_ = np.float64 if dt_ in ("f64", "float64") else np.float32
        args.workload = f"syrk_n{n_}_m{m_}_{'f64' if dt_ == np.float64 else 'f32'}_custom"
        op, alpha, beta = "syrk", -1.0, 1.0
        A = inputs.normal_matrix(int(n_), int(m_), 7, 1.0 / np.sqrt(int(m_)), dt_)
        C0 = inputs.symmetric_uniform(int(n_), 8, dtype=dt_)
    else:
        op, A, C0, alpha, beta = inputs.make_config(args.workload)
    if op == "potrf":
        # Large Block Cholesky of the configuration's SPD matrix: one step = one factorisation of a
        # fresh copy (the copy is made outside the timed events)
        N = C0.shape[0]
        dS = torch.from_numpy(C0).cuda()
        dW = torch.empty_like(dS)
        ws = torch.empty(tb.tbs_potrf_lower_workspace(tb.TBS_F64, N), dtype=torch.uint8, device="cuda")
        times = []
        for s in range(args.warmup + args.steps):
            dW.copy_(dS)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            info = tb.tbs_potrf_lower(dW, workspace=ws, want_info=False)
            e1.record()
            torch.cuda.synchronize()
            if s >= args.warmup:
                times.append(e0.elapsed_time(e1))
        ms = float(np.mean(times))
        flops = float(N) ** 3 / 3.0
        print(json.dumps({"metric": "Cholesky fp64 TFLOP/s (N^3/3 flops)", "value": round(flops / ms / 1e9, 3),
                          "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
                          "vs_baseline": None, "dtype": "f64", "data": "synthetic",
                          "config": {"workload": args.workload, "N": N},
                          "roofline": {"bound": "mfma", "achieved": round(flops / ms / 1e9, 3), "peak": 78.6,
                                       "unit": "TFLOP/s", "frac": round(flops / ms / 1e9 / 78.6, 4),
                                       "traffic": None}}))
        return 0
    N, M = A.shape
    dname = "f64" if A.dtype == np.float64 else "f32"
    dA = torch.from_numpy(A).cuda()
    dC = torch.from_numpy(C0).cuda()
    flops = float(N) * float(N + 1) * float(M)
    # the library's workspace (parts of blocks that are cut along the contraction dimension), allocated
    # once, outside the timed region, as a caller in a loop would
    code = tb.TBS_F64 if dname == "f64" else tb.TBS_F32
    ws_bytes = 0 if args.square else tb.tbs_syrk_lower_workspace(code, N, M)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda") if ws_bytes > 0 else False
    if args.square:
        def fn(a, c, al, be):
            return tb.tbs_syrk_lower_square(a, c, al, be)
    else:
        def fn(a, c, al, be):
            return tb.tbs_syrk_lower(a, c, al, be, workspace=ws)

    for _ in range(args.warmup):
        fn(dA, dC, alpha, beta)
    torch.cuda.synchronize()

    # the timed region: exactly K steps, wall clock, bracketed by synchronisation; each launch is
    # also bracketed by events on the launch stream (torch's current stream is the one passed down)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        starts[s].record()
        fn(dA, dC, alpha, beta)
        ends[s].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kern_ms = float(np.mean([a.elapsed_time(b) for a, b in zip(starts, ends)]))

    value = flops / (ms_per_step * 1e-3) / 1e12
    achieved = flops / (kern_ms * 1e-3) / 1e12
    info = tb.tbs_syrk_lower_query(tb.TBS_F64 if dname == "f64" else tb.TBS_F32, N, M, args.square)
    es = 8 if dname == "f64" else 4
    out = {
        "metric": "SYRK fp64 TFLOP/s (N^2 M flops)" if dname == "f64" else "SYRK fp32 TFLOP/s (N^2 M flops)",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dname,
        "data": "synthetic",
        "config": {"workload": args.workload, "N": N, "M": M, "alpha": alpha, "beta": beta,
                   "schedule": "square-blocks" if args.square else "triangle-blocks",
                   "k": info["k"], "b": info["b"], "c": info["c"], "l": info["l"],
                   "workgroups": info["n_items"]},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 3), "peak": PEAK_TFLOPS[dname],
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_TFLOPS[dname], 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, args.square)),
                     "kernel": "tbs_syrk_persistent_kernel", "kernel_ms": round(kern_ms, 4),
                     "flops_per_launch": flops},
        "io_model": {"S_C_elems": info["S_C_elems"], "S_res_elems": info["S_res_elems"],
                     "A_bytes_plan": info["A_elems"] * es, "C_bytes_read": info["C_elems"] * es * (beta != 0),
                     "C_bytes_written": info["C_elems"] * es,
                     "tbs_bound_bytes": info["tbs_bound_elems"] * es,
                     "tiled_tbs_lead_bytes": info["tiled_lead_elems"] * es,
                     "square_equal_area_bytes": info["square_elems"] * es},
    }

    if not args.no_cpu:
        import oracle
        # the oracle as it stands (plain loops, OpenMP over rows), on a bounded sample of the same
        # workload: the first n rows of A and the leading n x n block of C, all M columns
        n = min(N, 4096)
        As = np.ascontiguousarray(A[:n]).astype(np.float64)
        Cs = np.ascontiguousarray(C0[:n, :n]).astype(np.float64)
        # repeated until about ten seconds of CPU work have been timed (at least once)
        reps, dt = 0, 0.0
        while reps == 0 or (dt < 10.0 and reps < 50):
            Cw = Cs.copy()
            t0 = time.perf_counter()
            oracle.syrk_lower(As, Cw, alpha, beta, extended=False)
            dt += time.perf_counter() - t0
            reps += 1
        out["cpu_baseline"] = {"value": round(reps * float(n) * (n + 1) * M / dt / 1e12, 5), "unit": "TFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"rows 0..{n - 1} of the workload (n={n}, M={M}), {reps} repetition(s), "
                                         f"{dt:.2f} s in all"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
