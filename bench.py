"""Benchmark of the DEER hot path on one MI355X.

A step is one deer_eval(): the whole Newton solve (every iteration: f + Jacobian at all positions,
the blocked scan, the convergence test) over one batch of synthetic input that is already resident
in HBM.  The workload is the benchmark's configs[1]: GRU, d=4, n=8, T=10,000, B=16, fp32.

Prints one JSON line: whole-job throughput in sequence-steps/s, the roofline fraction of the dominant
kernel (the scan; duration from HIP events on the library's stream) and the CPU oracle's throughput on
the host cores as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def scan_algorithmic_bytes_per_step(n, esz=4):
    # read J (n*n) and the right-hand side (n), write y (n), read the previous iterate (n) for the
    # fused convergence maximum
    return esz * (n * n + 3 * n)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration (1-based), default 2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--scan-stream", type=str, default="",
                    help="n,B,T: time deer_linrec_solve alone on a random stream of that shape and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB a few times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2309_12252_amd import deer, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "calibrate_copy_bytes_written": src.numel() * 4,
                          "launches": 5}))
        return
    if args.scan_stream:
        n, B, T = [int(v) for v in args.scan_stream.split(",")]
        A, b, y0 = inputs.scan_inputs(1, B, T, n)
        cfg = deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, B, T, n, d=1)
        sctx = deer.DeerContext(cfg, device=dev)
        dA, db, dy0 = [torch.from_numpy(a).to(dev) for a in (A, b, y0)]
        out = torch.empty((B, T, n), dtype=torch.float32, device=dev)
        for _ in range(3):
            sctx.linrec_solve(dA, db, dy0, out=out)
        sctx.set_profiling(True)
        for _ in range(args.steps):
            sctx.linrec_solve(dA, db, dy0, out=out)
        prof = sctx.profile()
        ms = prof["scan_ms"] / max(1, prof["scan_launches"])
        nbytes = 4 * (n * n + 2 * n) * B * T   # J, b in; y out (no previous iterate in this entry point)
        print(json.dumps({"scan_stream": {"n": n, "B": B, "T": T}, "avg_launch_ms": ms, "algorithmic_bytes": nbytes,
                          "achieved_GBs": nbytes / (ms * 1e-3) / 1e9, "frac_of_8TBs": nbytes / (ms * 1e-3) / 8e12,
                          "algorithmic_flops": (2 * n ** 3 + 4 * n * n) * B * T,
                          "achieved_TFLOPs": (2 * n ** 3 + 4 * n * n) * B * T / (ms * 1e-3) / 1e12}))
        sctx.close()
        return
    w = inputs.config(args.config)
    ctx = deer.context_for(w, device=dev)
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
    th, x, y0 = t(w.theta), t(w.x), t(w.y0)
    y = torch.empty((w.B, w.T, w.n), dtype=torch.float32, device=dev)

    def step():
        return ctx.eval(th, x, y0, tol=w.tol, max_iter=w.max_iter, out=y)

    for _ in range(args.warmup):
        _, iters, err, conv, _ = step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        _, iters, err, conv, _ = step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    S = w.B * w.T
    value = S * args.steps / elapsed

    # per-kernel durations: the same steps again with HIP events around every launch
    ctx.set_profiling(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = ctx.profile()
    ctx.set_profiling(False)
    scan_ms = prof["scan_ms"] / max(1, prof["scan_launches"])
    scan_T = w.T - 1 if w.cell == inputs.CELL_MLP_ODE else w.T
    alg_bytes = scan_algorithmic_bytes_per_step(w.n) * w.B * scan_T
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "scan_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(w.name)
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "kernel": "affine scan (n=%d)" % w.n, "avg_launch_us": round(1e3 * scan_ms, 2),
                "algorithmic_bytes_per_launch": alg_bytes}

    out = {"metric": "DEER sequence-steps/s (B*T/s), forward eval to convergence", "value": value,
           "unit": "sequence-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": w.name, "cell": "gru" if w.cell == inputs.CELL_GRU else "mlp_ode", "B": w.B,
                      "T": w.T, "n": w.n, "d": w.d, "tol": w.tol, "max_iter": w.max_iter,
                      "newton_iterations": iters, "converged": bool(conv)},
           "kernels_ms_per_launch": {
               "funceval": prof["funceval_ms"] / max(1, prof["funceval_launches"]),
               "discretise": prof["discretise_ms"] / max(1, prof["discretise_launches"]),
               "scan": scan_ms},
           "roofline": roofline}

    if not args.no_cpu_baseline:
        import oracle
        threads = max(1, min(w.B, oracle.max_threads(), 16))
        if w.cell == inputs.CELL_GRU:
            cell = oracle.make_cell(oracle.CELL_GRU, w.n, w.d)
            run = lambda: oracle.deer_eval(cell, w.theta, w.x, w.y0, tol=w.tol, max_iter=w.max_iter, nthreads=threads)
        else:
            cell = oracle.make_cell(oracle.CELL_MLP, w.n, 0, w.mlp_width, w.mlp_hidden_layers)
            run = lambda: oracle.ode_deer_eval(cell, w.theta, w.y0, w.T, w.t0, w.t1, tol=w.tol,
                                               max_iter=w.max_iter, nthreads=threads)
        times = []
        t_start = time.perf_counter()
        while len(times) < 3 or (time.perf_counter() - t_start < 10.0 and len(times) < 40):
            a = time.perf_counter()
            run()
            times.append(time.perf_counter() - a)
        med = float(np.median(times))
        out["cpu_baseline"] = {"value": S / med, "unit": "sequence-steps/s", "cores": threads, "kind": "oracle",
                               "sample": "the full workload (same DEER solve in fp64), median of %d runs" % len(times)}
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
