"""Benchmark of the DEER hot path on one MI355X.

A step is one deer_eval(): the whole Newton solve (every iteration: f + Jacobian at all positions,
the blocked scan, the convergence test) over one batch of synthetic input that is already resident
in HBM.  The default workload is the second benchmark configuration: GRU, d=4, n=8, T=10,000, B=16, fp32.

Prints one JSON line: whole-job throughput in sequence-steps/s, the roofline entry of the kernel that
takes most of the step (duration from HIP events on the library's stream) and the CPU oracle's
throughput on the host cores as a reported baseline.
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


VALU_F32_PEAK_TFLOPS = 157.3   # published fp32 vector peak (256 CUs x 128 lanes x 2 (packed) x 2 (fma) x 2.4 GHz)
MFMA_F32_PEAK_TFLOPS = 157.3   # published dense fp32 matrix peak


def scan_bytes_per_position(n, esz=4):
    # read J (n*n) and the right-hand side (n), write y (n), read the previous iterate (n) for the
    # fused convergence maximum
    return esz * (n * n + 3 * n)


def scan_flops_per_position(n):
    # composition of the pair into the running product (2 n^3 + 2 n^2) and the second walk (2 n^2)
    return 2 * n ** 3 + 4 * n * n


def fused_flops_per_position(n, d):
    # GRU gates 2*3n(n+d), Jacobian rows 2*4n^2 (three scaled rows + diagonal), right-hand side 2n^2,
    # about 30 n elementwise operations, and the scan's own work
    return 6 * n * (n + d) + 8 * n * n + 2 * n * n + 30 * n + scan_flops_per_position(n)


def mlp_flops_per_point(n, width):
    # f: 2(wn + w^2 + nw); J y for the right-hand side: the same chain again; J = W3 D2 W2 D1 W1: 2 w^2 n + 2 n w n
    # plus the two diagonal scalings (2 w n each)
    chain = 2 * (width * n + width * width + n * width)
    return 2 * chain + 2 * width * width * n + 2 * n * width * n + 4 * width * n


def dominant_roofline(kind, ms, w, newton_iterations=0.0):
    """Roofline entry of the kernel that takes most of a step (durations from HIP events)."""
    from paper_2309_12252_amd import inputs
    ode = w.cell == inputs.CELL_MLP_ODE
    positions = w.B * ((w.T - 1) if (ode and kind != "funceval") else w.T)
    sec = ms * 1e-3
    if kind == "newton":
        # the whole solve in one launch: the per-iteration work of the fused step times the iterations it ran;
        # HBM sees the inputs and the guess once and the result once
        fl = fused_flops_per_position(w.n, w.d) * positions * newton_iterations
        a = fl / sec / 1e12
        return {"bound": "alu", "achieved": round(a, 2), "peak": VALU_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(a / VALU_F32_PEAK_TFLOPS, 4), "traffic": None,
                "kernel": "GRU Newton solve in one launch (n=%d, %g iterations)" % (w.n, newton_iterations),
                "avg_launch_us": round(1e3 * ms, 2), "algorithmic_flops_per_launch": fl,
                "hbm_bytes_per_launch": 4 * (w.n + w.d) * positions}
    if kind == "fused" and w.n >= 16:
        # the GRU step with the cell inside the MFMA scan: the matrix products dominate the arithmetic
        fl = fused_flops_per_position(w.n, w.d) * positions
        a = fl / sec / 1e12
        return {"bound": "mfma", "achieved": round(a, 2), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(a / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None,
                "kernel": "GRU cell + MFMA affine scan in one launch (n=%d)" % w.n, "avg_launch_us": round(1e3 * ms, 2),
                "algorithmic_flops_per_launch": fl, "hbm_bytes_per_launch": 4 * (2 * w.n + w.d) * positions}
    if kind == "fused":
        fl = fused_flops_per_position(w.n, w.d) * positions
        a = fl / sec / 1e12
        return {"bound": "alu", "achieved": round(a, 2), "peak": VALU_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(a / VALU_F32_PEAK_TFLOPS, 4), "traffic": None,
                "kernel": "GRU cell + affine scan in one launch (n=%d)" % w.n, "avg_launch_us": round(1e3 * ms, 2),
                "algorithmic_flops_per_launch": fl,
                "hbm_bytes_per_launch": 4 * (2 * w.n + w.d) * positions}
    if kind == "scan" and w.n >= 16:
        fl = scan_flops_per_position(w.n) * positions
        a = fl / sec / 1e12
        return {"bound": "mfma", "achieved": round(a, 2), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(a / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None, "kernel": "affine scan (n=%d)" % w.n,
                "avg_launch_us": round(1e3 * ms, 2), "algorithmic_flops_per_launch": fl,
                "hbm_bytes_per_launch": scan_bytes_per_position(w.n) * positions}
    if kind == "funceval" and ode and w.n == 8:
        fl = mlp_flops_per_point(w.n, w.mlp_width) * positions
        a = fl / sec / 1e12
        return {"bound": "mfma", "achieved": round(a, 2), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(a / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None, "kernel": "MLP field + Jacobian",
                "avg_launch_us": round(1e3 * ms, 2), "algorithmic_flops_per_launch": fl}
    if kind == "scan":
        nbytes = scan_bytes_per_position(w.n) * positions
    elif kind == "discretise":
        nbytes = 4 * (2 * w.n * w.n + 3 * w.n) * positions    # G, z, y in; Gbar, residual out
    else:
        nbytes = 4 * (w.n * w.n + 2 * w.n + w.d) * positions   # GRU cell: y, x in; J, rhs out
    a = nbytes / sec / 1e9
    return {"bound": "hbm", "achieved": round(a, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(a / HBM_PEAK_GBS, 4), "traffic": None, "kernel": "%s (n=%d)" % (kind, w.n),
            "avg_launch_us": round(1e3 * ms, 2), "algorithmic_bytes_per_launch": nbytes}


def scan_stream(torch, deer, dev, n, B, T, steps):
    """deer_linrec_solve alone on a random stream [B, T, n, n] (fp32): duration from HIP events, algorithmic
    bytes and flop rates against the MI355X peaks."""
    # the recipe of inputs.scan_inputs (random matrices scaled to spectral norm 0.9), drawn on the device:
    # a multi-GB stream takes the host generator most of a minute
    torch.manual_seed(1)
    dA = torch.randn(B, T, n, n, device=dev)
    # spectral norms by 12 power iterations (the batched SVD behind matrix_norm does not take millions
    # of matrices); an estimate from below, so the scaled norms are 0.9 or slightly more.  In chunks of
    # 2^22 matrices: one batched product over tens of millions of them has faulted in the library.
    flat = dA.view(B * T, n, n)
    for lo in range(0, B * T, 1 << 22):
        a = flat[lo:lo + (1 << 22)]
        v = torch.randn(a.shape[0], n, 1, device=dev)
        for _ in range(12):
            v = a.transpose(-1, -2) @ (a @ v)
            v /= torch.linalg.vector_norm(v, dim=-2, keepdim=True)
        a *= 0.9 / torch.linalg.vector_norm(a @ v, dim=-2, keepdim=True)
        del v
    db, dy0 = torch.randn(B, T, n, device=dev), torch.randn(B, n, device=dev)
    cfg = deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, B, T, n, d=1)
    sctx = deer.DeerContext(cfg, device=dev)
    out = torch.empty((B, T, n), dtype=torch.float32, device=dev)
    for _ in range(3):
        sctx.linrec_solve(dA, db, dy0, out=out)
    sctx.set_profiling(True)
    for _ in range(steps):
        sctx.linrec_solve(dA, db, dy0, out=out)
    prof = sctx.profile()
    sctx.close()
    ms = prof["scan_ms"] / max(1, prof["scan_launches"])
    nbytes = 4 * (n * n + 2 * n) * B * T   # J, b in; y out (no previous iterate in this entry point)
    flops = scan_flops_per_position(n) * B * T
    return {"scan_stream": {"n": n, "B": B, "T": T}, "avg_launch_ms": ms, "algorithmic_bytes": nbytes,
            "achieved_GBs": nbytes / (ms * 1e-3) / 1e9, "frac_of_8TBs": nbytes / (ms * 1e-3) / 8e12,
            "algorithmic_flops": flops, "achieved_TFLOPs": flops / (ms * 1e-3) / 1e12,
            "frac_of_mfma_f32_peak": flops / (ms * 1e-3) / 1e12 / MFMA_F32_PEAK_TFLOPS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration (1-based), default 2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-scan-kernels", action="store_true",
                    help="skip the stand-alone measurements of the scan kernels on chip-filling streams")
    ap.add_argument("--scan-stream", type=str, default="",
                    help="n,B,T: time deer_linrec_solve alone on a random stream of that shape and exit")
    ap.add_argument("--grad", action="store_true",
                    help="time deer_grad (Jacobians at the solution, transposed reverse scan, VJP + parameter "
                         "reduction; for the ODE cell: field Jacobians, discretisation, reverse scan with one refinement, "
                         "dual discretisation, MLP VJP) on the chosen configuration and exit")
    ap.add_argument("--train", action="store_true",
                    help="time one training step per step: deer_eval to convergence, then deer_grad at that trajectory")
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
        print(json.dumps(scan_stream(torch, deer, dev, n, B, T, args.steps)))
        return
    w = inputs.config(args.config)
    ctx = deer.context_for(w, device=dev)
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
    th, x, y0 = t(w.theta), t(w.x), t(w.y0)
    y = torch.empty((w.B, w.T, w.n), dtype=torch.float32, device=dev)

    def step():
        return ctx.eval(th, x, y0, tol=w.tol, max_iter=w.max_iter, out=y)

    if args.train:
        torch.manual_seed(2)
        g = torch.randn_like(y) / (w.B * w.T)
        gx = None if w.cell != inputs.CELL_GRU else x

        def train_step():
            yy, iters, err, conv, _ = step()
            ctx.grad(th, gx, y0, yy, g)
            return iters, conv

        for _ in range(args.warmup):
            train_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            iters, conv = train_step()
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / args.steps
        print(json.dumps({"deer_train_step": w.name, "ms_per_step": ms, "sequence_steps_per_s": w.B * w.T / (ms * 1e-3),
                          "newton_iterations": int(iters), "converged": bool(conv),
                          "what": "deer_eval to convergence + deer_grad of a random cotangent at that trajectory"}))
        ctx.close()
        return
    if args.grad:
        y, iters, err, conv, _ = step()
        torch.manual_seed(2)
        g = torch.randn_like(y) / (w.B * w.T)
        for _ in range(args.warmup):
            ctx.grad(th, x, y0, y, g)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ctx.grad(th, x, y0, y, g)
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / args.steps
        ctx.set_profiling(True)
        for _ in range(args.steps):
            ctx.grad(th, x, y0, y, g)
        torch.cuda.synchronize()
        prof = ctx.profile()
        keys = ("funceval", "fused", "scan", "vjp") if w.cell == inputs.CELL_GRU else ("funceval", "discretise", "scan", "vjp")
        keys = tuple(k for k in keys if prof[k + "_launches"] > 0)   # "fused": the reverse scan with the cell inside (n = 16, 32)
        per = {k: prof[k + "_ms"] / max(1, prof[k + "_launches"]) for k in keys}
        per_call = {k: prof[k + "_ms"] / args.steps for k in keys}
        S = w.B * w.T
        jbytes = 4 * w.n * w.n * S
        line = {"deer_grad": w.name, "ms_per_call": ms, "sequence_steps_per_s": S / (ms * 1e-3),
                "kernels_ms_per_launch": per, "kernels_ms_per_call": per_call}
        if "scan" in per:
            line["reverse_scan_GBs"] = 4 * (w.n * w.n + 2 * w.n) * S / (per["scan"] * 1e-3) / 1e9
        if "funceval" in per:
            line["funceval_write_GBs"] = (jbytes + 4 * w.n * S) / (per["funceval"] * 1e-3) / 1e9
        print(json.dumps(line))
        ctx.close()
        return

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
    per_launch = {k: prof[k + "_ms"] / max(1, prof[k + "_launches"])
                  for k in ("funceval", "discretise", "scan", "fused", "newton")}
    totals = {k: prof[k + "_ms"] for k in per_launch}
    dominant = max(totals, key=totals.get)
    its = prof["newton_iterations"] / max(1, prof["newton_launches"])   # iterations inside a one-launch solve
    roofline = dominant_roofline(dominant, per_launch[dominant], w, its)
    tpath = os.path.join(ROOT, "profiles", "kernel_traffic.json")
    if os.path.exists(tpath):
        # HBM bytes per launch from the committed rocprofv3 counter runs (FETCH_SIZE + WRITE_SIZE, calibrated)
        tr = json.load(open(tpath)).get(w.name, {}).get(dominant)
        if tr:
            roofline["traffic"] = tr["total_bytes"]
            roofline["traffic_fetched"] = tr["fetched_bytes"]
            roofline["traffic_written"] = tr["written_bytes"]

    out = {"metric": "DEER sequence-steps/s (B*T/s), forward eval to convergence", "value": value,
           "unit": "sequence-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": w.name, "cell": "gru" if w.cell == inputs.CELL_GRU else "mlp_ode", "B": w.B,
                      "T": w.T, "n": w.n, "d": w.d, "tol": w.tol, "max_iter": w.max_iter,
                      "newton_iterations": iters, "converged": bool(conv)},
           "kernels_ms_per_launch": per_launch,
           "roofline": roofline}

    if not args.no_scan_kernels:
        # the scan kernels on their own, on streams that fill the chip: the HBM fraction of the n <= 8 kernel
        # and the MFMA fraction of the n = 32 kernel (HIP events, 10 launches each)
        ctx.close()
        ctx = None
        torch.cuda.empty_cache()
        s8 = scan_stream(torch, deer, dev, 8, 16, 400000, 10)
        torch.cuda.empty_cache()
        s32 = scan_stream(torch, deer, dev, 32, 16, 100000, 10)
        torch.cuda.empty_cache()
        s4 = scan_stream(torch, deer, dev, 4, 16, 800000, 10)
        torch.cuda.empty_cache()
        out["scan_kernels"] = {
            "n4_B16_T800k": {"bound": "hbm", "achieved": round(s4["achieved_GBs"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": round(s4["frac_of_8TBs"], 4), "avg_launch_us": round(1e3 * s4["avg_launch_ms"], 1)},
            "n8_B16_T400k": {"bound": "hbm", "achieved": round(s8["achieved_GBs"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": round(s8["frac_of_8TBs"], 4), "avg_launch_us": round(1e3 * s8["avg_launch_ms"], 1)},
            "n32_B16_T100k": {"bound": "mfma", "achieved": round(s32["achieved_TFLOPs"], 2), "peak": MFMA_F32_PEAK_TFLOPS,
                              "unit": "TFLOP/s", "frac": round(s32["frac_of_mfma_f32_peak"], 4),
                              "hbm_GBs": round(s32["achieved_GBs"], 1), "avg_launch_us": round(1e3 * s32["avg_launch_ms"], 1)}}

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
        if w.cell == inputs.CELL_GRU:
            # for context: the oracle's plain sequential evaluation of the same recurrence (what DEER replaces)
            seq = []
            for _ in range(5):
                a = time.perf_counter()
                oracle.seq_eval(cell, w.theta, w.x, w.y0, nthreads=threads)
                seq.append(time.perf_counter() - a)
            out["cpu_baseline"]["sequential_value"] = S / float(np.median(seq))
    if ctx is not None:
        ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
