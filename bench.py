"""Benchmark of the DEER hot path on one MI355X.

A step is one deer_eval(): the whole Newton solve (every iteration: f + Jacobian at all positions,
the blocked scan, the convergence test) over one batch of synthetic input that is already resident
in HBM.  The default workload is the largest single-GPU benchmark configuration, the third one:
GRU, d=8, n=32, T=100,000, B=16, fp32 (1.6 M sequence positions per solve).

Prints one JSON line: whole-job throughput in sequence-steps/s, the roofline entry of the kernel that
takes most of the step (duration from HIP events on the library's stream), the same figures for the
other configurations and for deer_grad ("configs"), the scan kernels alone on chip-filling streams
("scan_kernels"), and the CPU oracle's throughput on the host cores as a reported baseline.
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


def mlp_flops_per_point(n, width, nhid=2):
    # f: 2(wn + (nhid-1) w^2 + nw); J y for the right-hand side: the same chain again; J = W_out D W ... D W_1:
    # (nhid-1) products of w x w with w x n, one of n x w with w x n, plus the diagonal scalings (2 w n each)
    chain = 2 * (width * n + (nhid - 1) * width * width + n * width)
    return 2 * chain + (nhid - 1) * 2 * width * width * n + 2 * n * width * n + nhid * 2 * width * n


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
        fl = mlp_flops_per_point(w.n, w.mlp_width, w.mlp_hidden_layers) * positions
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
    # Entries i.i.d. N(0, (0.45 / sqrt(n))^2), drawn on the device (a multi-GB stream takes the host generator
    # most of a minute): the spectral norm of such a matrix concentrates at 2 sigma sqrt(n) = 0.9, the scale of
    # inputs.scan_inputs, and products contract (growth rate sigma sqrt(n) < 1 per factor), without any
    # per-matrix normalisation (no batched products or decompositions in the generator).
    torch.manual_seed(1)
    dA = torch.randn(B, T, n, n, device=dev)
    dA *= 0.45 / float(np.sqrt(n))
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


class Bench:
    """One configuration resident on the device: context, inputs and the timed calls."""

    def __init__(self, torch, deer, inputs, dev, k):
        self.torch, self.inputs = torch, inputs
        self.w = w = inputs.config(k) if isinstance(k, int) else k   # a benchmark configuration or any workload
        self.ctx = deer.context_for(w, device=dev)
        t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
        self.th, self.x, self.y0 = t(w.theta), t(w.x), t(w.y0)
        self.y = torch.empty(self.ctx._shapes()[0], dtype=torch.float32, device=dev)
        torch.manual_seed(2)
        self.g = torch.randn_like(self.y) / (w.B * w.T)
        self.S = w.B * w.T * max(1, w.heads)   # sequence positions (of every head)

    def step(self):
        w = self.w
        return self.ctx.eval(self.th, self.x, self.y0, tol=w.tol, max_iter=w.max_iter, out=self.y)

    def grad(self):
        gx = self.x if self.w.cell != self.inputs.CELL_MLP_ODE else None
        return self.ctx.grad(self.th, gx, self.y0, self.y, self.g)

    def _timed(self, fn, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            r = fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            r = fn()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, r

    def _profiled(self, fn, steps):
        self.ctx.set_profiling(True)
        for _ in range(steps):
            fn()
        self.torch.cuda.synchronize()
        prof = self.ctx.profile()
        self.ctx.set_profiling(False)
        return prof

    def time_eval(self, steps, warmup):
        """Exactly `steps` timed solves after `warmup` untimed ones; then the same steps again with HIP events
        around every launch for the per-kernel durations."""
        elapsed, (_, iters, err, conv, _) = self._timed(self.step, steps, warmup)
        prof = self._profiled(self.step, steps)
        per_launch = {k: prof[k + "_ms"] / max(1, prof[k + "_launches"])
                      for k in ("funceval", "discretise", "scan", "fused", "newton")}
        totals = {k: prof[k + "_ms"] for k in per_launch}
        dominant = max(totals, key=totals.get)
        its = prof["newton_iterations"] / max(1, prof["newton_launches"])   # iterations inside a one-launch solve
        roofline = None if self.w.extra.get("no_roofline") else dominant_roofline(dominant, per_launch[dominant], self.w, its)
        return {"elapsed": elapsed, "ms_per_step": 1e3 * elapsed / steps, "value": self.S * steps / elapsed,
                "iters": int(iters), "converged": bool(conv), "per_launch": per_launch, "dominant": dominant,
                "roofline": roofline}

    def time_grad(self, steps, warmup):
        """deer_grad of a random cotangent at the trajectory of the last solve (self.y)."""
        elapsed, _ = self._timed(self.grad, steps, warmup)
        prof = self._profiled(self.grad, steps)
        keys = ("funceval", "fused", "discretise", "scan", "vjp")
        per_call = {k: round(prof[k + "_ms"] / steps, 5) for k in keys if prof[k + "_launches"] > 0}
        ms = 1e3 * elapsed / steps
        return {"ms_per_call": ms, "sequence_steps_per_s": self.S / (ms * 1e-3), "kernels_ms_per_call": per_call}

    def time_train(self, steps, warmup):
        def train_step():
            r = self.step()
            self.grad()
            return r
        elapsed, (_, iters, _, conv, _) = self._timed(train_step, steps, warmup)
        ms = 1e3 * elapsed / steps
        return {"ms_per_step": ms, "sequence_steps_per_s": self.S / (ms * 1e-3), "newton_iterations": int(iters),
                "converged": bool(conv)}

    def close(self):
        self.ctx.close()
        self.ctx = None


def attach_traffic(roofline, workload_name, dominant):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter runs (FETCH_SIZE and
    WRITE_SIZE, each scaled by the same counter's reading for a plain device copy).  They are not measured in this
    run: the source file and what it says about its own run travel with the number."""
    tpath = os.path.join(ROOT, "profiles", "kernel_traffic.json")
    if not os.path.exists(tpath):
        return
    table = json.load(open(tpath))
    tr = table.get(workload_name, {}).get(dominant)
    if tr:
        roofline["traffic"] = tr["total_bytes"]
        roofline["traffic_fetched"] = tr["fetched_bytes"]
        roofline["traffic_written"] = tr["written_bytes"]
        roofline["traffic_source"] = "profiles/kernel_traffic.json (separate rocprofv3 --pmc runs; %s)" % table.get(
            "_measured", "date not recorded")


def cpu_baseline(w, inputs):
    """The oracle's DEER solve of the same workload on the host cores (OpenMP over the batch): once on the full
    workload with every thread it can use, once single-threaded on a bounded sample (one sequence, a quarter of
    the length: the cost is linear in B*T), plus the oracle's plain sequential evaluation for context."""
    import oracle
    S = w.B * w.T
    threads = max(1, min(w.B, oracle.max_threads(), 16))
    if w.cell == inputs.CELL_GRU:
        cell = oracle.make_cell(oracle.CELL_GRU, w.n, w.d)
        run = lambda th: oracle.deer_eval(cell, w.theta, w.x, w.y0, tol=w.tol, max_iter=w.max_iter, nthreads=th)
        T1 = max(1, w.T // 4)
        run1 = lambda: oracle.deer_eval(cell, w.theta, w.x[:1, :T1], w.y0[:1], tol=w.tol, max_iter=w.max_iter, nthreads=1)
    else:
        cell = oracle.make_cell(oracle.CELL_MLP, w.n, 0, w.mlp_width, w.mlp_hidden_layers, w.mlp_activation)
        run = lambda th: oracle.ode_deer_eval(cell, w.theta, w.y0, w.T, w.t0, w.t1, tol=w.tol, max_iter=w.max_iter,
                                              nthreads=th)
        T1 = max(2, w.T // 4)
        run1 = lambda: oracle.ode_deer_eval(cell, w.theta, w.y0[:1], T1, w.t0, w.t0 + (w.t1 - w.t0) * (T1 - 1) / (w.T - 1),
                                            tol=w.tol, max_iter=w.max_iter, nthreads=1)
    times = []
    t_start = time.perf_counter()
    while len(times) < 1 or (time.perf_counter() - t_start < 12.0 and len(times) < 20):
        a = time.perf_counter()
        run(threads)
        times.append(time.perf_counter() - a)
    med = float(np.median(times))
    a = time.perf_counter()
    run1()
    t1 = time.perf_counter() - a
    try:
        affinity = len(os.sched_getaffinity(0))
    except AttributeError:
        affinity = os.cpu_count()
    out = {"value": S / med, "unit": "sequence-steps/s", "cores": threads, "kind": "oracle",
           "sample": "the full workload (the same DEER solve in fp64, OpenMP over the batch), median of %d run(s) "
                     "of %.1f s" % (len(times), med),
           "nproc": os.cpu_count(), "cpus_in_affinity_mask": affinity, "omp_max_threads": oracle.max_threads(),
           "single_thread_value": T1 / t1,
           "single_thread_sample": "one sequence, first %d of %d positions, one thread, %.1f s" % (T1, w.T, t1)}
    if w.cell == inputs.CELL_GRU:
        # for context: the oracle's plain sequential evaluation of the same recurrence (what DEER replaces)
        a = time.perf_counter()
        oracle.seq_eval(cell, w.theta, w.x, w.y0, nthreads=threads)
        out["sequential_value"] = S / (time.perf_counter() - a)
        a = time.perf_counter()
        oracle.seq_eval(cell, w.theta, w.x[:1], w.y0[:1], nthreads=1)
        out["sequential_single_thread_value"] = w.T / (time.perf_counter() - a)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3,
                    help="benchmark configuration of the headline (1-based), default 3: the largest single-GPU one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-scan-kernels", action="store_true",
                    help="skip the stand-alone measurements of the scan kernels on chip-filling streams")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the other configurations and the deer_grad / training-step timings")
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

    bench = Bench(torch, deer, inputs, dev, args.config)
    w = bench.w
    if args.train:
        r = bench.time_train(args.steps, args.warmup)
        r.update({"deer_train_step": w.name,
                  "what": "deer_eval to convergence + deer_grad of a random cotangent at that trajectory"})
        print(json.dumps(r))
        bench.close()
        return
    if args.grad:
        bench.step()
        r = bench.time_grad(args.steps, args.warmup)
        r["deer_grad"] = w.name
        print(json.dumps(r))
        bench.close()
        return

    head = bench.time_eval(args.steps, args.warmup)
    roofline = head["roofline"]
    attach_traffic(roofline, w.name, head["dominant"])
    out = {"metric": "DEER sequence-steps/s (B*T/s), forward eval to convergence", "value": head["value"],
           "unit": "sequence-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": w.name, "cell": "gru" if w.cell == inputs.CELL_GRU else "mlp_ode", "B": w.B,
                      "T": w.T, "n": w.n, "d": w.d, "tol": w.tol, "max_iter": w.max_iter,
                      "newton_iterations": head["iters"], "converged": head["converged"]},
           "kernels_ms_per_launch": head["per_launch"],
           "roofline": roofline}

    if not args.no_configs:
        # every other configuration, deer_grad at each, and the training step of the fourth one: fewer repetitions
        # (the headline's region above is the one the contract times)
        configs = {}
        ksteps = max(3, min(args.steps, 10))
        for k in (1, 2, 3, 4, 5):
            if k == args.config:
                b = bench
                entry = {}
            else:
                b = Bench(torch, deer, inputs, dev, k)
                r = b.time_eval(ksteps, 2)
                attach_traffic(r["roofline"], b.w.name, r["dominant"])
                entry = {"ms_per_eval": round(r["ms_per_step"], 5), "sequence_steps_per_s": r["value"],
                         "newton_iterations": r["iters"], "converged": r["converged"],
                         "kernels_ms_per_launch": {kk: round(v, 5) for kk, v in r["per_launch"].items() if v > 0},
                         "dominant_kernel": r["roofline"]}
            if k != 1:
                b.step()
                entry["deer_grad"] = b.time_grad(ksteps, 2)
            if k == 4:
                entry["train_step"] = b.time_train(ksteps, 2)
            configs[b.w.name] = entry
            if b is not bench:
                b.close()
                del b
                torch.cuda.empty_cache()
        # shapes of the paper's other experiments that the library also runs (random weights stand in for trained
        # ones): the two-body network's field (App. B.2), the multi-head GRU with strides (App. B.4), an LSTM (Sec. 3.4), the LEM cell
        extras = [inputs.mlp_ode_workload("two_body_shape_mlp_n8_w64_L5_softplus_T10k_B16", 4242, B=16, T=10000, n=8, width=64,
                                          nhid=5, t0=0.0, t1=10.0, act=inputs.ACT_SOFTPLUS),
                  inputs.mh_gru_workload("multihead_gru_32x8_strides8_T1024_B64", 4321, B=64, T=1024, n=8, d=8, H=32, K=8),
                  inputs.lstm_workload("lstm_u8_d4_T50k_B16", 88, B=16, T=50000, units=8, d=4),
                  # the LEM cell on the length and channels of the series the paper trains it on (App. B.3 shapes)
                  inputs.lem_workload("lem_u16_d6_T17984_B32", 89, B=32, T=17984, units=16, d=6, dt=1.0),
                  # the largest state size of the paper's speed table (Table 4: n = 64, 10k steps, batch 16)
                  inputs.gru_workload("gru_n64_T10k_B16", 6464, B=16, T=10000, n=64, d=8)]
        for wx in extras:
            wx.extra["no_roofline"] = True
            b = Bench(torch, deer, inputs, dev, wx)
            r = b.time_eval(ksteps, 2)
            entry = {"ms_per_eval": round(r["ms_per_step"], 5), "sequence_steps_per_s": r["value"],
                     "newton_iterations": r["iters"], "converged": r["converged"],
                     "kernels_ms_per_launch": {kk: round(v, 5) for kk, v in r["per_launch"].items() if v > 0}}
            b.step()
            entry["deer_grad"] = b.time_grad(ksteps, 2)
            configs[wx.name] = entry
            b.close()
            del b
            torch.cuda.empty_cache()
        out["configs"] = configs
    bench.close()
    del bench
    torch.cuda.empty_cache()

    if not args.no_scan_kernels:
        # the scan kernels on their own, on streams that fill the chip: the HBM fraction of the n <= 8 kernels
        # and the MFMA fraction of the n = 16 and n = 32 kernels (HIP events, 10 launches each)
        sk = {}
        for n, B, T, label in ((2, 16, 2000000, "n2_B16_T2M"), (4, 16, 800000, "n4_B16_T800k"),
                               (8, 16, 400000, "n8_B16_T400k"), (16, 16, 100000, "n16_B16_T100k"),
                               (32, 16, 100000, "n32_B16_T100k")):
            s = scan_stream(torch, deer, dev, n, B, T, 10)
            torch.cuda.empty_cache()
            if n <= 8:
                sk[label] = {"bound": "hbm", "achieved": round(s["achieved_GBs"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": round(s["frac_of_8TBs"], 4), "avg_launch_us": round(1e3 * s["avg_launch_ms"], 1)}
            else:
                sk[label] = {"bound": "mfma", "achieved": round(s["achieved_TFLOPs"], 2), "peak": MFMA_F32_PEAK_TFLOPS,
                             "unit": "TFLOP/s", "frac": round(s["frac_of_mfma_f32_peak"], 4),
                             "hbm_GBs": round(s["achieved_GBs"], 1), "hbm_frac": round(s["frac_of_8TBs"], 4),
                             "avg_launch_us": round(1e3 * s["avg_launch_ms"], 1)}
        out["scan_kernels"] = sk

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, inputs)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
