#!/usr/bin/env python3
"""Benchmark of the Triangle Block SYRK and Large Block Cholesky on one MI355X.

One step = one call of tbs_syrk_lower on the benchmark workload (N = 4096, M = 4096, fp64,
C <- C - A A^T on the lower triangle), inputs resident in HBM.  Prints ONE JSON line:
  - the whole-job throughput of that workload (N^2 M flops per step) over exactly --steps steps after
    --warmup warm-up steps, wall clock between two synchronisations;
  - `roofline`: the SYRK kernel's own time (HIP events around every launch on the launch stream) against
    the published MFMA peak, and the HBM traffic per launch read from the committed rocprofv3 summary;
  - `workloads`: the other configurations (N = M = 256; N = 16384, M = 512; Cholesky N = 16384; fp32
    N = 32768, M = 8192) and the square-block baseline at the benchmark shape, each timed the same way
    with a few steps;
  - `cpu_baseline`: the CPU oracle timed on the host cores.
Before anything is timed the chip is brought to its steady clock by untimed launches of the same kernel
(`preheat_ms`; after an idle phase the first launches run at about 2.1 instead of 2.4 GHz).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--square] [--no-cpu] [--only]
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3}       # MI355X dense matrix peaks (published, 2.4 GHz), TFLOP/s
PREHEAT_MS = 150.0                              # untimed launches before a measurement, at least this long
HEADLINE = "syrk_n4096_m4096_f64"
# steps / warm-ups of the side workloads (the headline takes --steps / --warmup)
SIDE = [("syrk_n256_m256_f64", 200, 20), ("syrk_n16384_m512_f64", 20, 5), ("potrf_n16384_f64", 5, 2),
        ("syrk_n32768_m8192_f32", 5, 2)]


def profile_traffic(workload, square):
    """HBM bytes per launch of the SYRK kernel from the committed rocprofv3 summary of this workload
    (FETCH_SIZE and WRITE_SIZE, scaled by a copy of known size): (bytes or None, file name)."""
    dt = "f64" if workload.endswith("f64") else "f32"
    shape = re.search(r"n\d+_m\d+", workload)
    if not shape:
        return None, None
    name = f"tbs_syrk_kernel_{dt}_{shape.group(0)}.md"
    path = os.path.join(ROOT, "profiles", name)
    key = "traffic_bytes_per_launch_square" if square else "traffic_bytes_per_launch"
    try:
        m = re.search(r"^" + key + r"\s*=\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    except OSError:
        return None, "profiles/" + name
    return (float(m.group(1)) if m else None), "profiles/" + name


class Syrk:
    """One SYRK workload resident on the device."""

    def __init__(self, tb, torch, name, A, C0, alpha, beta, square=False):
        self.tb, self.torch, self.name, self.alpha, self.beta, self.square = tb, torch, name, alpha, beta, square
        self.N, self.M = A.shape
        self.dname = "f64" if A.dtype == np.float64 else "f32"
        self.code = tb.TBS_F64 if self.dname == "f64" else tb.TBS_F32
        self.dA = torch.from_numpy(A).cuda()
        self.dC = torch.from_numpy(C0).cuda()
        # the library's workspace (parts of blocks that are cut along the contraction dimension),
        # allocated once, outside the timed region, as a caller in a loop would
        need = 0 if square else tb.tbs_syrk_lower_workspace(self.code, self.N, self.M)
        self.ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need > 0 else False
        self.flops = float(self.N) * float(self.N) * float(self.M)

    def step(self):
        if self.square:
            self.tb.tbs_syrk_lower_square(self.dA, self.dC, self.alpha, self.beta)
        else:
            self.tb.tbs_syrk_lower(self.dA, self.dC, self.alpha, self.beta, workspace=self.ws)


class Potrf:
    """Large Block Cholesky of the configuration's SPD matrix: one step = one factorisation of a fresh
    copy (the copy is made before the step's first event)."""

    def __init__(self, tb, torch, name, S0):
        self.tb, self.torch, self.name = tb, torch, name
        self.N = S0.shape[0]
        self.dname = "f64"
        self.dS = torch.from_numpy(S0).cuda()
        self.dW = torch.empty_like(self.dS)
        self.ws = torch.empty(tb.tbs_potrf_lower_workspace(tb.TBS_F64, self.N), dtype=torch.uint8, device="cuda")
        self.flops = float(self.N) ** 3 / 3.0

    def prepare(self):
        self.dW.copy_(self.dS)

    def step(self):
        self.tb.tbs_potrf_lower(self.dW, workspace=self.ws, want_info=False)


def measure(torch, w, steps, warmup, preheat_ms=PREHEAT_MS):
    """(wall ms per step, mean event ms per step, untimed preheat ms): preheat, warm-up, then exactly
    `steps` steps between two synchronisations, every step also bracketed by events on its stream."""
    prepare = getattr(w, "prepare", None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < preheat_ms:
        for _ in range(4):
            if prepare:
                prepare()
            w.step()
        torch.cuda.synchronize()
    heat = (time.perf_counter() - t0) * 1e3
    for _ in range(warmup):
        if prepare:
            prepare()
        w.step()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        if prepare:
            prepare()
        starts[s].record()
        w.step()
        ends[s].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ev = float(np.mean([a.elapsed_time(b) for a, b in zip(starts, ends)]))
    return (t1 - t0) * 1e3 / steps, ev, heat


def side_entry(w, wall_ms, ev_ms, steps, warmup, with_copy=False):
    # a step of the Cholesky workload includes the copy that restores the input: its rate comes from the
    # events around the factorisation alone
    ms = ev_ms if with_copy else wall_ms
    tf = w.flops / (ms * 1e-3) / 1e12
    out = {"tflops": round(tf, 3), "ms_per_step": round(ms, 4), "kernel_ms": round(ev_ms, 4), "steps": steps,
           "warmup": warmup, "dtype": w.dname, "peak": PEAK_TFLOPS[w.dname],
           "frac": round(w.flops / (ev_ms * 1e-3) / 1e12 / PEAK_TFLOPS[w.dname], 4)}
    if isinstance(w, Syrk):                                 # HBM bytes per launch, where a summary is committed
        out["traffic"], out["traffic_source"] = profile_traffic(w.name, w.square)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--shape", default=None, help="N,M,dtype: a SYRK shape outside the configuration list "
                    "(C <- C - A A^T, A iid N(0,1)/sqrt(M)), for kernel studies")
    ap.add_argument("--square", action="store_true", help="time the square-block baseline instead")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--only", action="store_true", help="skip the side workloads (profiling runs)")
    ap.add_argument("--preheat-ms", type=float, default=PREHEAT_MS)
    ap.add_argument("--device-inputs", action="store_true",
                    help="fill the matrices on the device with torch's generator instead of the seeded host "
                         "generator (same shapes and distributions; for profiler runs, where only the access "
                         "pattern matters and the host generator's time would be paid under the profiler)")
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

    def make(name, square=False):
        if args.device_inputs:
            op, N, M, dtype, alpha, beta, seed = inputs.CONFIGS[name]
            tdt = torch.float64 if dtype == np.float64 else torch.float32
            gen = torch.Generator(device="cuda").manual_seed(seed)
            if op == "potrf":
                w = Potrf.__new__(Potrf)
                S = torch.rand((N, N), dtype=tdt, device="cuda", generator=gen) * 2 - 1
                S = torch.tril(S, -1)
                S = S + S.T
                S.diagonal().fill_(float(N))
                w.tb, w.torch, w.name, w.N, w.dname, w.dS = tb, torch, name, N, "f64", S
                w.dW = torch.empty_like(S)
                w.ws = torch.empty(tb.tbs_potrf_lower_workspace(tb.TBS_F64, N), dtype=torch.uint8, device="cuda")
                w.flops = float(N) ** 3 / 3.0
                return w
            w = Syrk(tb, torch, name, np.zeros((1, 1), dtype=dtype), np.zeros((1, 1), dtype=dtype), alpha, beta, square)
            w.N, w.M = N, M
            w.dA = torch.randn((N, M), dtype=tdt, device="cuda", generator=gen) / (1.0 if N == M == 4096 else np.sqrt(M))
            w.dC = torch.zeros((N, N), dtype=tdt, device="cuda") if beta == 0.0 else \
                torch.rand((N, N), dtype=tdt, device="cuda", generator=gen) * 2 - 1
            need = 0 if square else tb.tbs_syrk_lower_workspace(w.code, N, M)
            w.ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need > 0 else False
            w.flops = float(N) * float(N) * float(M)
            return w
        op, A, C0, alpha, beta = inputs.make_config(name)
        return Potrf(tb, torch, name, C0) if op == "potrf" else Syrk(tb, torch, name, A, C0, alpha, beta, square)

    if args.shape:
        n_, m_, dt_ = args.shape.split(",")
        dt_ = np.float64 if dt_ in ("f64", "float64") else np.float32
        args.workload = f"syrk_n{n_}_m{m_}_{'f64' if dt_ == np.float64 else 'f32'}_custom"
        A = inputs.normal_matrix(int(n_), int(m_), 7, 1.0 / np.sqrt(int(m_)), dt_)
        C0 = inputs.symmetric_uniform(int(n_), 8, dtype=dt_)
        w = Syrk(tb, torch, args.workload, A, C0, -1.0, 1.0, args.square)
    else:
        w = make(args.workload, args.square)
        A = None
    is_potrf = isinstance(w, Potrf)
    wall_ms, kern_ms, heat = measure(torch, w, args.steps, args.warmup, args.preheat_ms)
    ms_per_step = kern_ms if is_potrf else wall_ms
    value = w.flops / (ms_per_step * 1e-3) / 1e12
    achieved = w.flops / (kern_ms * 1e-3) / 1e12
    peak = PEAK_TFLOPS[w.dname]
    out = {
        "metric": ("Cholesky fp64 TFLOP/s (N^3/3 flops)" if is_potrf else
                   f"SYRK {'fp64' if w.dname == 'f64' else 'fp32'} TFLOP/s (N^2 M flops)"),
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dname,
        "data": "synthetic (device generator)" if args.device_inputs else "synthetic",
        "preheat_ms": round(heat, 1),
    }
    if is_potrf:
        out["config"] = {"workload": args.workload, "N": w.N}
        out["roofline"] = {"bound": "mfma", "achieved": round(achieved, 3), "peak": peak, "peak_source": "published",
                           "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": None,
                           "kernel": "tbs_potrf_lower (all kernels of one factorisation)",
                           "kernel_ms": round(kern_ms, 4), "flops_per_launch": w.flops}
    else:
        info = tb.tbs_syrk_lower_query(w.code, w.N, w.M, args.square)
        es = 8 if w.dname == "f64" else 4
        traffic, source = profile_traffic(args.workload, args.square)
        out["config"] = {"workload": args.workload, "N": w.N, "M": w.M, "alpha": w.alpha, "beta": w.beta,
                         "schedule": "square-blocks" if args.square else
                                     ("triangle-blocks-of-eight-tiles" if info["S_C_elems"] == 8 * 64 * 64
                                      else "triangle-blocks"),
                         "k": info["k"], "b": info["b"], "c": info["c"], "l": info["l"],
                         "workgroups": info["n_items"]}
        out["roofline"] = {"bound": "mfma", "achieved": round(achieved, 3), "peak": peak, "peak_source": "published",
                           "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                           "traffic": traffic, "traffic_source": source,
                           "kernel": "tbs_syrk_kernel (persistent form)", "kernel_ms": round(kern_ms, 4),
                           "flops_per_launch": w.flops}
        out["io_model"] = {"S_C_elems": info["S_C_elems"], "S_res_elems": info["S_res_elems"],
                           "A_bytes_plan": info["A_elems"] * es, "C_bytes_read": info["C_elems"] * es * (w.beta != 0),
                           "C_bytes_written": info["C_elems"] * es,
                           "tbs_bound_bytes": info["tbs_bound_elems"] * es,
                           "tiled_tbs_lead_bytes": info["tiled_lead_elems"] * es,
                           "square_equal_area_bytes": info["square_elems"] * es,
                           "plan_over_bound": round(info["A_elems"] / info["tbs_bound_elems"], 4)}

    if not args.only and not args.shape and args.workload == HEADLINE and not args.square:
        # the other configurations and the square-block baseline, a few steps each
        side = {}
        sq = make(HEADLINE, square=True)
        wl, ev, _ = measure(torch, sq, 20, 5, args.preheat_ms)
        side[HEADLINE + "_square_blocks"] = side_entry(sq, wl, ev, 20, 5)
        del sq
        del w
        for name, steps, warm in SIDE:
            torch.cuda.empty_cache()
            sw = make(name)
            wl, ev, _ = measure(torch, sw, steps, warm, args.preheat_ms)
            side[name] = side_entry(sw, wl, ev, steps, warm, with_copy=isinstance(sw, Potrf))
            del sw
        out["workloads"] = side

    if not args.no_cpu and not is_potrf:
        import oracle
        # the oracle as it stands (plain loops, OpenMP over rows), on a bounded sample of the same
        # workload: the first n rows of A and the leading n x n block of C, all M columns
        if A is None:
            _, A, C0, alpha, beta = inputs.make_config(args.workload)
        else:
            alpha, beta = -1.0, 1.0
        N, M = A.shape
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
        out["cpu_baseline"] = {"value": round(reps * float(n) * n * M / dt / 1e12, 5), "unit": "TFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"rows 0..{n - 1} of the workload (n={n}, M={M}), {reps} repetition(s), "
                                         f"{dt:.2f} s in all"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
