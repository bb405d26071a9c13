"""Pins of the oracle's LEM cell (the cell of the paper's last experiment; the equations are those of the cited
publication, the paper prints none).  No library implements the cell, so its definition is checked only against a
second, vectorised statement of the same equations and against its limits (PARITY UNPINNED for the definition); the
Jacobian is pinned to finite differences and autograd, the vector-Jacobian product to autograd, DEER to the sequential
evaluation and the backward derivative to autograd through time.  CPU only."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_12252_amd import inputs


def split(theta, u, d):
    th = torch.as_tensor(theta, dtype=torch.float64)
    o = 0
    W = th[o:o + 4 * u * d].reshape(4, u, d); o += 4 * u * d
    U = th[o:o + 4 * u * u].reshape(4, u, u); o += 4 * u * u
    b = th[o:o + 4 * u].reshape(4, u)
    return W, U, b


def lem_step(theta, u, d, dt, s, x):
    W, U, b = split(theta, u, d)
    y, z = s[:u], s[u:]
    s1 = dt * torch.sigmoid(W[0] @ x + U[0] @ y + b[0])
    s2 = dt * torch.sigmoid(W[1] @ x + U[1] @ y + b[1])
    zn = (1 - s1) * z + s1 * torch.tanh(W[2] @ x + U[2] @ y + b[2])
    yn = (1 - s2) * y + s2 * torch.tanh(W[3] @ x + U[3] @ zn + b[3])
    return torch.cat([yn, zn])


@pytest.mark.parametrize("u,d,dt", [(1, 1, 1.0), (2, 3, 0.5), (4, 4, 1.0), (8, 6, 0.25), (16, 8, 1.0)])
def test_lem_f_jacobian_and_vjp(u, d, dt):
    rng = np.random.default_rng(100 * u + d)
    theta = rng.standard_normal(inputs.lstm_theta_count(u, d)) / np.sqrt(u)
    cell = oracle.make_cell(oracle.CELL_LEM, 2 * u, d, dt=dt)
    assert oracle.theta_count(cell) == theta.size
    for _ in range(3):
        s, x, lam = rng.standard_normal(2 * u), rng.standard_normal(d), rng.standard_normal(2 * u)
        tht = torch.tensor(theta, requires_grad=True)
        st = torch.tensor(s, requires_grad=True)
        xt = torch.tensor(x, requires_grad=True)
        out = lem_step(tht, u, d, dt, st, xt)
        np.testing.assert_allclose(oracle.cell_f(cell, theta, s, x), out.detach().numpy(), rtol=0, atol=1e-14)
        J = oracle.cell_jac(cell, theta, s, x)
        Jt = torch.autograd.functional.jacobian(lambda ss: lem_step(torch.tensor(theta), u, d, dt, ss, torch.tensor(x)),
                                                torch.tensor(s)).numpy()
        np.testing.assert_allclose(J, Jt, rtol=0, atol=1e-13)
        eps = 1e-6
        for j in range(2 * u):
            e = np.zeros(2 * u); e[j] = eps
            fd = (oracle.cell_f(cell, theta, s + e, x) - oracle.cell_f(cell, theta, s - e, x)) / (2 * eps)
            np.testing.assert_allclose(J[:, j], fd, rtol=0, atol=1e-8)
        (out * torch.tensor(lam)).sum().backward()
        dth, dx, ds = oracle.cell_vjp(cell, theta, s, x, lam)
        np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-13)
        np.testing.assert_allclose(ds, st.grad.numpy(), atol=1e-13)
        np.testing.assert_allclose(ds, J.T @ lam, atol=1e-13)
        np.testing.assert_allclose(dth, tht.grad.numpy(), atol=1e-13)
        # finite differences of the parameters (independent of autograd and of the second statement's derivative)
        for q in rng.choice(theta.size, size=min(12, theta.size), replace=False):
            e = np.zeros(theta.size); e[q] = eps
            fd = (oracle.cell_f(cell, theta + e, s, x) - oracle.cell_f(cell, theta - e, s, x)) / (2 * eps)
            assert abs(fd @ lam - dth[q]) <= 1e-8


def test_limits_of_the_cell():
    u, d = 3, 2
    rng = np.random.default_rng(3)
    theta = rng.standard_normal(inputs.lstm_theta_count(u, d))
    W, U, b = [t.numpy().copy() for t in split(theta, u, d)]
    s, x = rng.standard_normal(2 * u), rng.standard_normal(d)
    # closed time gates (pre-activations -> -inf): the state does not move
    b0 = b.copy(); b0[0] = -800.0; b0[1] = -800.0
    W0 = W.copy(); W0[0] = 0; W0[1] = 0
    U0 = U.copy(); U0[0] = 0; U0[1] = 0
    th0 = np.concatenate([W0.ravel(), U0.ravel(), b0.ravel()])
    cell = oracle.make_cell(oracle.CELL_LEM, 2 * u, d, dt=1.0)
    np.testing.assert_allclose(oracle.cell_f(cell, th0, s, x), s, rtol=0, atol=1e-300)
    # fully open gates with dt = 1: the state is replaced, z' = tanh(W_z x + U_z y + b_z), y' = tanh(W_y x + U_y z' + b_y)
    b1 = b.copy(); b1[0] = 800.0; b1[1] = 800.0
    th1 = np.concatenate([W0.ravel(), U0.ravel(), b1.ravel()])
    zn = np.tanh(W[2] @ x + U[2] @ s[:u] + b[2])
    yn = np.tanh(W[3] @ x + U[3] @ zn + b[3])
    np.testing.assert_allclose(oracle.cell_f(cell, th1, s, x), np.concatenate([yn, zn]), rtol=0, atol=1e-15)
    # the step scales the time gates: with open gates and dt = 0.25 the update is a quarter of the way
    cell4 = oracle.make_cell(oracle.CELL_LEM, 2 * u, d, dt=0.25)
    zq = 0.75 * s[u:] + 0.25 * zn
    yq = 0.75 * s[:u] + 0.25 * np.tanh(W[3] @ x + U[3] @ zq + b[3])
    np.testing.assert_allclose(oracle.cell_f(cell4, th1, s, x), np.concatenate([yq, zq]), rtol=0, atol=1e-15)


def test_deer_reaches_the_sequential_solution_and_its_gradient_matches_autograd():
    u, d, B, T, dt = 3, 2, 2, 60, 0.5
    w = inputs.lem_workload("lem", 5, B=B, T=T, units=u, d=d, dt=dt)
    cell = oracle.make_cell(oracle.CELL_LEM, 2 * u, d, dt=dt)
    rng = np.random.default_rng(1)
    y0 = rng.standard_normal((B, 2 * u)) * 0.5
    ys = oracle.seq_eval(cell, w.theta, w.x, y0)
    yd, it, err, hist = oracle.deer_eval(cell, w.theta, w.x, y0, tol=1e-11, max_iter=60)
    assert it < 60
    np.testing.assert_allclose(yd, ys, rtol=0, atol=1e-11)
    g = rng.standard_normal((B, T, 2 * u))
    tht = torch.tensor(w.theta.astype(np.float64), requires_grad=True)
    xt = torch.tensor(w.x.astype(np.float64), requires_grad=True)
    y0t = torch.tensor(y0, requires_grad=True)
    loss = 0.0
    for b in range(B):
        y = y0t[b]
        for i in range(T):
            y = lem_step(tht, u, d, dt, y, xt[b, i])
            np.testing.assert_allclose(ys[b, i], y.detach().numpy(), rtol=0, atol=1e-12)
            loss = loss + (y * torch.tensor(g[b, i])).sum()
    loss.backward()
    dth, dx, dy0 = oracle.rnn_grad(cell, w.theta, w.x, y0, ys, g)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dy0, y0t.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dth, tht.grad.numpy(), atol=1e-10)
