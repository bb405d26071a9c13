"""GPU parity of deer_grad (reverse scan + GRU VJP + parameter reduction) against the oracle."""
import numpy as np
import pytest

import oracle
from paper_2309_12252_amd import deer, inputs
from helpers import DEV, TOL_ABS, dev, grad_errors, host, oracle_cell

pytestmark = pytest.mark.gpu


def check_grad(w, g, dtype):
    cell = oracle_cell(w)
    y = oracle.seq_eval(cell, w.theta, w.x, w.y0, nthreads=8)
    dth_o, dx_o, dy0_o = oracle.gru_grad(w.n, w.d, w.theta, w.x, w.y0, y, g)
    ctx = deer.context_for(w, dtype=dtype, device=DEV)
    try:
        dth, dx, dy0 = ctx.grad(dev(w.theta, dtype), dev(w.x, dtype), dev(w.y0, dtype), dev(y, dtype), dev(g, dtype))
        dth2, _, _ = ctx.grad(dev(w.theta, dtype), dev(w.x, dtype), dev(w.y0, dtype), dev(y, dtype), dev(g, dtype),
                              want_dx=False, want_dy0=False)
    finally:
        ctx.close()
    # plain max-abs against the oracle, the same bar as for the trajectory
    assert grad_errors(w.name, "dL/dtheta", host(dth), dth_o) <= TOL_ABS[dtype]
    assert grad_errors(w.name, "dL/dx", host(dx), dx_o) <= TOL_ABS[dtype]
    assert grad_errors(w.name, "dL/dy0", host(dy0), dy0_o) <= TOL_ABS[dtype]
    assert np.array_equal(host(dth), host(dth2))   # the reduction order is fixed: run-to-run identical


@pytest.mark.parametrize("n,d", [(1, 1), (2, 2), (4, 3), (8, 4), (16, 6), (32, 8), (2, 7), (4, 16), (8, 12), (32, 16)])
@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
def test_small_shapes(n, d, dtype):
    for k, (B, T) in enumerate([(1, 1), (2, 9), (3, 700), (2, 3001)]):
        w = inputs.gru_workload("g_n%d_T%d" % (n, T), 70 * n + k, B=B, T=T, n=n, d=d)
        w.y0 = np.random.default_rng(k).standard_normal((B, n)).astype(np.float32)
        g = np.random.default_rng(k + 1).standard_normal((B, T, n)) / np.sqrt(T)
        check_grad(w, g.astype(np.float32).astype(np.float64), dtype)


@pytest.mark.parametrize("knob", ["DEER_VJP_MFMA", "DEER_GRAD_FUSED"])
@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
@pytest.mark.parametrize("n,d", [(2, 2), (8, 4), (16, 6), (32, 16)])
def test_separate_kernels_stay_selectable(n, d, dtype, knob, monkeypatch):
    # by default the transposed Jacobians are computed inside the reverse scan (n <= 8; fp32 n = 16, 32) and the
    # fp32 VJP at n = 16, 32 runs on the matrix cores; the Jacobian kernel + plain reverse scan and the vector-ALU
    # VJP are the same computation in separate kernels
    monkeypatch.setenv(knob, "0")
    for k, (B, T) in enumerate([(2, 9), (3, 700), (1, 1)]):
        w = inputs.gru_workload("g_n%d_T%d" % (n, T), 70 * n + k, B=B, T=T, n=n, d=d)
        g = np.random.default_rng(k + 1).standard_normal((B, T, n)) / np.sqrt(T)
        check_grad(w, g.astype(np.float32).astype(np.float64), dtype)


def test_config4_training_step_gradients():
    # mean-pooled linear readout to 5 classes + cross-entropy on random labels; the loss lives here
    w = inputs.config(4)
    cell = oracle_cell(w)
    y = oracle.seq_eval(cell, w.theta, w.x, w.y0, nthreads=8)
    Wo, bo, labels = w.extra["W_o"].astype(np.float64), w.extra["b_o"].astype(np.float64), w.extra["labels"]
    logits = y.mean(axis=1) @ Wo.T + bo
    p = np.exp(logits - logits.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    p[np.arange(w.B), labels] -= 1.0
    g_b = (p @ Wo) / (w.B * w.T)                       # dL/dy_{b,i}, the same for every i
    g = np.broadcast_to(g_b[:, None, :], y.shape).astype(np.float32).astype(np.float64)
    check_grad(w, g, deer.DEER_F32)


def test_gradient_at_the_deer_trajectory():
    # eval then grad on the GPU, against oracle eval then oracle grad
    w = inputs.gru_workload("chain", 11, B=4, T=2500, n=8, d=4)
    g = (np.random.default_rng(3).standard_normal((w.B, w.T, w.n)) / 50).astype(np.float32).astype(np.float64)
    yo, _, _, _ = oracle.deer_eval(oracle_cell(w), w.theta, w.x, w.y0, tol=w.tol, max_iter=w.max_iter, nthreads=4)
    dth_o, dx_o, dy0_o = oracle.gru_grad(w.n, w.d, w.theta, w.x, w.y0, yo, g)
    ctx = deer.context_for(w, device=DEV)
    try:
        th, x, y0 = dev(w.theta, 0), dev(w.x, 0), dev(w.y0, 0)
        y, it, err, conv, st = ctx.eval(th, x, y0, tol=w.tol, max_iter=w.max_iter)
        dth, dx, dy0 = ctx.grad(th, x, y0, y, dev(g, 0))
    finally:
        ctx.close()
    assert conv
    assert grad_errors(w.name, "dL/dtheta", host(dth), dth_o) <= 1e-4
    assert grad_errors(w.name, "dL/dx", host(dx), dx_o) <= 1e-4 and grad_errors(w.name, "dL/dy0", host(dy0), dy0_o) <= 1e-4


@pytest.mark.parametrize("k", [2, 3])
def test_gradient_at_full_benchmark_sizes(k):
    # cfg 2 (n = 8, T = 10,000, B = 16) and cfg 3 (n = 32, T = 100,000, B = 16) in the launch configuration the bench
    # times: hundreds to thousands of tiles per sequence in the reverse scan with the cell inside
    w = inputs.config(k)
    print("gradient at %s" % w.name, flush=True)
    g = np.random.default_rng(5).standard_normal((w.B, w.T, w.n)) / np.sqrt(w.T)
    check_grad(w, g.astype(np.float32).astype(np.float64), deer.DEER_F32)
