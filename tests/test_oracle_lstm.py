"""Pins of the oracle's LSTM cell (Sec. 3.4 names LSTM as an instance of the recurrence): f against the library
cell, the Jacobian against autograd and finite differences, the vector-Jacobian product against autograd, DEER
against the sequential evaluation, the backward derivative against autograd through time.  CPU only."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_12252_amd import inputs


def torch_lstm_cell(u, d, theta):
    th = torch.tensor(np.asarray(theta, dtype=np.float64))
    cell = torch.nn.LSTMCell(d, u, dtype=torch.float64)
    o = 0
    W = th[o:o + 4 * u * d].reshape(4 * u, d); o += 4 * u * d
    U = th[o:o + 4 * u * u].reshape(4 * u, u); o += 4 * u * u
    b = th[o:o + 4 * u]
    with torch.no_grad():
        cell.weight_ih.copy_(W)
        cell.weight_hh.copy_(U)
        cell.bias_ih.copy_(b)
        cell.bias_hh.zero_()
    return cell


def step(tc, x, y, u):
    h, c = tc(x[None], (y[None, :u], y[None, u:]))
    return torch.cat([h[0], c[0]])


@pytest.mark.parametrize("u,d", [(1, 1), (2, 3), (4, 4), (8, 6), (16, 8)])
def test_lstm_f_jacobian_and_vjp_match_the_library_cell(u, d):
    rng = np.random.default_rng(100 * u + d)
    theta = rng.standard_normal(inputs.lstm_theta_count(u, d)) / np.sqrt(u)
    cell = oracle.make_cell(oracle.CELL_LSTM, 2 * u, d)
    assert oracle.theta_count(cell) == theta.size
    tc = torch_lstm_cell(u, d, theta)
    for _ in range(3):
        y, x, lam = rng.standard_normal(2 * u), rng.standard_normal(d), rng.standard_normal(2 * u)
        yt = torch.tensor(y, requires_grad=True)
        xt = torch.tensor(x, requires_grad=True)
        out = step(tc, xt, yt, u)
        np.testing.assert_allclose(oracle.cell_f(cell, theta, y, x), out.detach().numpy(), rtol=0, atol=1e-14)
        Jt = torch.autograd.functional.jacobian(lambda yy: step(tc, torch.tensor(x), yy, u), torch.tensor(y)).numpy()
        J = oracle.cell_jac(cell, theta, y, x)
        np.testing.assert_allclose(J, Jt, rtol=0, atol=1e-13)
        eps = 1e-6
        for j in range(2 * u):
            e = np.zeros(2 * u); e[j] = eps
            fd = (oracle.cell_f(cell, theta, y + e, x) - oracle.cell_f(cell, theta, y - e, x)) / (2 * eps)
            np.testing.assert_allclose(J[:, j], fd, rtol=0, atol=1e-8)
        for p in tc.parameters():
            p.grad = None
        (out * torch.tensor(lam)).sum().backward()
        dth, dx, dy = oracle.cell_vjp(cell, theta, y, x, lam)
        np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-13)
        np.testing.assert_allclose(dy, yt.grad.numpy(), atol=1e-13)
        np.testing.assert_allclose(dy, J.T @ lam, atol=1e-13)
        want = np.concatenate([tc.weight_ih.grad.numpy().ravel(), tc.weight_hh.grad.numpy().ravel(), tc.bias_ih.grad.numpy()])
        np.testing.assert_allclose(dth, want, atol=1e-13)


def test_deer_reaches_the_sequential_solution_and_its_gradient_matches_autograd():
    u, d, B, T = 3, 2, 2, 60
    w = inputs.lstm_workload("lstm", 5, B=B, T=T, units=u, d=d)
    cell = oracle.make_cell(oracle.CELL_LSTM, 2 * u, d)
    rng = np.random.default_rng(1)
    y0 = rng.standard_normal((B, 2 * u)) * 0.5
    ys = oracle.seq_eval(cell, w.theta, w.x, y0)
    yd, it, err, hist = oracle.deer_eval(cell, w.theta, w.x, y0, tol=1e-11, max_iter=60)
    assert it < 60
    np.testing.assert_allclose(yd, ys, rtol=0, atol=1e-11)
    # sequential result against the library cell run step by step, and the gradient of L = sum g . y against BPTT
    tc = torch_lstm_cell(u, d, w.theta)
    g = rng.standard_normal((B, T, 2 * u))
    xt = torch.tensor(w.x.astype(np.float64), requires_grad=True)
    y0t = torch.tensor(y0, requires_grad=True)
    loss = 0.0
    for b in range(B):
        y = y0t[b]
        for i in range(T):
            y = step(tc, xt[b, i], y, u)
            np.testing.assert_allclose(ys[b, i], y.detach().numpy(), rtol=0, atol=1e-12)
            loss = loss + (y * torch.tensor(g[b, i])).sum()
    loss.backward()
    dth, dx, dy0 = oracle.rnn_grad(cell, w.theta, w.x, y0, ys, g)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dy0, y0t.grad.numpy(), atol=1e-11)
    want = np.concatenate([tc.weight_ih.grad.numpy().ravel(), tc.weight_hh.grad.numpy().ravel(), tc.bias_ih.grad.numpy()])
    np.testing.assert_allclose(dth, want, atol=1e-10)


def test_generic_backward_derivative_is_the_gru_one_for_the_gru():
    w = inputs.gru_workload("g", 8, B=2, T=50, n=4, d=3)
    cell = oracle.make_cell(oracle.CELL_GRU, 4, 3)
    y = oracle.seq_eval(cell, w.theta, w.x, w.y0)
    g = np.random.default_rng(0).standard_normal(y.shape)
    a = oracle.gru_grad(4, 3, w.theta, w.x, w.y0, y, g)
    b = oracle.rnn_grad(cell, w.theta, w.x, w.y0, y, g)
    for u_, v_ in zip(a, b):
        np.testing.assert_allclose(u_, v_, rtol=0, atol=1e-13)
