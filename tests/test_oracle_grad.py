"""Pins of the oracle's backward derivative (dual operator + VJP of f) against autograd through a
sequential loop of the library GRU cell, and against finite differences.  CPU only."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_12252_amd import inputs
from test_oracle_cells import torch_gru_cell


def torch_bptt(w, g):
    tc = torch_gru_cell(w.n, w.d, w.theta)
    x = torch.tensor(w.x, dtype=torch.float64, requires_grad=True)
    y0 = torch.tensor(w.y0, dtype=torch.float64, requires_grad=True)
    h, ys = y0, []
    for i in range(w.T):
        h = tc(x[:, i], h)
        ys.append(h)
    y = torch.stack(ys, dim=1)
    (y * torch.tensor(g)).sum().backward()
    n = w.n
    dtheta = np.concatenate([tc.weight_ih.grad.numpy().ravel(), tc.weight_hh.grad.numpy().ravel(),
                             tc.bias_ih.grad.numpy(), tc.bias_hh.grad.numpy()[2 * n:]])
    return y.detach().numpy(), dtheta, x.grad.numpy(), y0.grad.numpy()


@pytest.mark.parametrize("n,d,T,B", [(2, 2, 50, 2), (4, 3, 120, 3), (16, 6, 64, 2), (1, 1, 30, 1)])
def test_grad_matches_autograd_bptt(n, d, T, B):
    w = inputs.gru_workload("t", 3 * n + T, B=B, T=T, n=n, d=d)
    w.y0 = np.random.default_rng(1).standard_normal((B, n)).astype(np.float32)
    g = np.random.default_rng(2).standard_normal((B, T, n))
    y, dth_t, dx_t, dy0_t = torch_bptt(w, g)
    dth, dx, dy0 = oracle.gru_grad(n, d, w.theta, w.x, w.y0, y, g)
    np.testing.assert_allclose(dth, dth_t, atol=1e-11)
    np.testing.assert_allclose(dx, dx_t, atol=1e-12)
    np.testing.assert_allclose(dy0, dy0_t, atol=1e-12)


def test_grad_matches_finite_differences_of_the_sequential_loss():
    n, d, T, B = 3, 2, 8, 2
    w = inputs.gru_workload("t", 42, B=B, T=T, n=n, d=d)
    rng = np.random.default_rng(0)
    w.y0 = rng.standard_normal((B, n)).astype(np.float32)
    g = rng.standard_normal((B, T, n))
    cell = oracle.make_cell(oracle.CELL_GRU, n, d)
    theta = w.theta.astype(np.float64)

    def loss(th, x, y0):
        return float((oracle.seq_eval(cell, th, x, y0) * g).sum())

    y = oracle.seq_eval(cell, theta, w.x, w.y0)
    dth, dx, dy0 = oracle.gru_grad(n, d, theta, w.x, w.y0, y, g)
    eps = 1e-6
    x64, y064 = w.x.astype(np.float64), w.y0.astype(np.float64)
    for k in range(theta.size):
        e = np.zeros_like(theta); e[k] = eps
        fd = (loss(theta + e, x64, y064) - loss(theta - e, x64, y064)) / (2 * eps)
        assert abs(fd - dth[k]) < 1e-7, (k, fd, dth[k])
    for idx in [(0, 0, 0), (1, 3, 1), (0, 7, 1)]:
        e = np.zeros_like(x64); e[idx] = eps
        fd = (loss(theta, x64 + e, y064) - loss(theta, x64 - e, y064)) / (2 * eps)
        assert abs(fd - dx[idx]) < 1e-7
    for idx in [(0, 0), (1, 2)]:
        e = np.zeros_like(y064); e[idx] = eps
        fd = (loss(theta, x64, y064 + e) - loss(theta, x64, y064 - e)) / (2 * eps)
        assert abs(fd - dy0[idx]) < 1e-7


def test_grad_uses_exactly_one_linear_solve_and_the_given_trajectory():
    # Sec. 3.1.1: the gradient needs one application of the (dual) inverse operator; it is taken at
    # whatever trajectory is handed in, so the DEER result and the sequential result give the same
    # gradient up to their own difference
    w = inputs.gru_workload("t", 6, B=2, T=200, n=4, d=2)
    cell = oracle.make_cell(oracle.CELL_GRU, w.n, w.d)
    g = np.random.default_rng(3).standard_normal((w.B, w.T, w.n))
    ys = oracle.seq_eval(cell, w.theta, w.x, w.y0)
    yd, _, _, _ = oracle.deer_eval(cell, w.theta, w.x, w.y0, tol=1e-7, max_iter=100)
    a = oracle.gru_grad(w.n, w.d, w.theta, w.x, w.y0, ys, g)
    b = oracle.gru_grad(w.n, w.d, w.theta, w.x, w.y0, yd, g)
    for u, v in zip(a, b):
        np.testing.assert_allclose(u, v, atol=1e-9)
