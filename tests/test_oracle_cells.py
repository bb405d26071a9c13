"""Pins of the oracle's cell functions (f, Jacobian, VJP) against PyTorch's own GRU cell and
autograd in fp64, and against finite differences.  CPU only."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_12252_amd import inputs


def torch_gru_cell(n, d, theta):
    """torch.nn.GRUCell carrying the oracle's flat theta (gate order r|z|candidate; the hidden
    biases of r and z are zero, the candidate's hidden bias is b_hc)."""
    th = torch.tensor(np.asarray(theta, dtype=np.float64))
    cell = torch.nn.GRUCell(d, n, dtype=torch.float64)
    o = 0
    W = th[o:o + 3 * n * d].reshape(3 * n, d); o += 3 * n * d
    U = th[o:o + 3 * n * n].reshape(3 * n, n); o += 3 * n * n
    b = th[o:o + 3 * n]; o += 3 * n
    bhc = th[o:o + n]
    with torch.no_grad():
        cell.weight_ih.copy_(W)
        cell.weight_hh.copy_(U)
        cell.bias_ih.copy_(b)
        cell.bias_hh.zero_()
        cell.bias_hh[2 * n:].copy_(bhc)
    return cell


def torch_mlp(n, width, nhid, theta, act=torch.tanh):
    th = torch.tensor(np.asarray(theta, dtype=np.float64))
    mats = []
    o, nin = 0, n
    for _ in range(nhid):
        W = th[o:o + width * nin].reshape(width, nin); o += width * nin
        b = th[o:o + width]; o += width
        mats.append((W, b))
        nin = width
    Wo = th[o:o + n * nin].reshape(n, nin); o += n * nin
    bo = th[o:o + n]

    def f(y):
        a = y
        for W, b in mats:
            a = act(W @ a + b)
        return Wo @ a + bo
    return f


@pytest.mark.parametrize("n,d", [(1, 1), (2, 2), (3, 5), (8, 4), (16, 6), (32, 8)])
def test_gru_f_matches_library_cell(n, d):
    rng = np.random.default_rng(n * 100 + d)
    theta = rng.standard_normal(inputs.gru_theta_count(n, d)) / np.sqrt(n)
    cell = oracle.make_cell(oracle.CELL_GRU, n, d)
    assert oracle.theta_count(cell) == theta.size
    tc = torch_gru_cell(n, d, theta)
    for _ in range(5):
        h, x = rng.standard_normal(n), rng.standard_normal(d)
        want = tc(torch.tensor(x)[None], torch.tensor(h)[None])[0].detach().numpy()
        got = oracle.cell_f(cell, theta, h, x)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)


@pytest.mark.parametrize("n,d", [(1, 1), (2, 2), (3, 5), (8, 4), (16, 6)])
def test_gru_jacobian_matches_autograd_and_fd(n, d):
    rng = np.random.default_rng(7 * n + d)
    theta = rng.standard_normal(inputs.gru_theta_count(n, d)) / np.sqrt(n)
    cell = oracle.make_cell(oracle.CELL_GRU, n, d)
    tc = torch_gru_cell(n, d, theta)
    h, x = rng.standard_normal(n), rng.standard_normal(d)
    J = oracle.cell_jac(cell, theta, h, x)
    Jt = torch.autograd.functional.jacobian(lambda hh: tc(torch.tensor(x)[None], hh[None])[0],
                                            torch.tensor(h)).numpy()
    np.testing.assert_allclose(J, Jt, rtol=0, atol=1e-13)
    eps = 1e-6
    Jfd = np.empty((n, n))
    for j in range(n):
        e = np.zeros(n); e[j] = eps
        Jfd[:, j] = (oracle.cell_f(cell, theta, h + e, x) - oracle.cell_f(cell, theta, h - e, x)) / (2 * eps)
    np.testing.assert_allclose(J, Jfd, rtol=0, atol=1e-8)


@pytest.mark.parametrize("n,d", [(1, 1), (2, 3), (8, 4), (16, 6)])
def test_gru_vjp_matches_autograd(n, d):
    rng = np.random.default_rng(11 * n + d)
    theta = rng.standard_normal(inputs.gru_theta_count(n, d)) / np.sqrt(n)
    tc = torch_gru_cell(n, d, theta)
    h, x, lam = rng.standard_normal(n), rng.standard_normal(d), rng.standard_normal(n)
    ht = torch.tensor(h, requires_grad=True)
    xt = torch.tensor(x, requires_grad=True)
    out = tc(xt[None], ht[None])[0]
    (out * torch.tensor(lam)).sum().backward()
    dtheta, dx, dh = oracle.gru_vjp(n, d, theta, h, x, lam)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dh, ht.grad.numpy(), atol=1e-13)
    o = 0
    np.testing.assert_allclose(dtheta[o:o + 3 * n * d], tc.weight_ih.grad.numpy().ravel(), atol=1e-13); o += 3 * n * d
    np.testing.assert_allclose(dtheta[o:o + 3 * n * n], tc.weight_hh.grad.numpy().ravel(), atol=1e-13); o += 3 * n * n
    np.testing.assert_allclose(dtheta[o:o + 3 * n], tc.bias_ih.grad.numpy(), atol=1e-13); o += 3 * n
    np.testing.assert_allclose(dtheta[o:o + n], tc.bias_hh.grad.numpy()[2 * n:], atol=1e-13)
    # dh must be J^T lam
    cell = oracle.make_cell(oracle.CELL_GRU, n, d)
    np.testing.assert_allclose(dh, oracle.cell_jac(cell, theta, h, x).T @ lam, atol=1e-13)


def test_gru_vjp_accumulates_into_dtheta():
    n, d = 3, 2
    rng = np.random.default_rng(5)
    theta = rng.standard_normal(inputs.gru_theta_count(n, d))
    h, x, lam = rng.standard_normal(n), rng.standard_normal(d), rng.standard_normal(n)
    a, _, _ = oracle.gru_vjp(n, d, theta, h, x, lam)
    b, _, _ = oracle.gru_vjp(n, d, theta, h, x, 2 * lam)
    np.testing.assert_allclose(b, 2 * a, atol=1e-14)


@pytest.mark.parametrize("n,width,nhid", [(8, 32, 2), (3, 5, 1), (4, 7, 3), (2, 0, 0)])
def test_mlp_f_and_jacobian_match_autograd(n, width, nhid):
    rng = np.random.default_rng(n + width + nhid)
    theta = rng.standard_normal(inputs.mlp_theta_count(n, width, nhid)) / np.sqrt(max(width, 1))
    cell = oracle.make_cell(oracle.CELL_MLP, n, 0, width, nhid)
    assert oracle.theta_count(cell) == theta.size
    f = torch_mlp(n, width, nhid, theta)
    y = rng.standard_normal(n)
    np.testing.assert_allclose(oracle.cell_f(cell, theta, y), f(torch.tensor(y)).numpy(), atol=1e-14)
    Jt = torch.autograd.functional.jacobian(f, torch.tensor(y)).numpy()
    np.testing.assert_allclose(oracle.cell_jac(cell, theta, y), Jt, atol=1e-13)


@pytest.mark.parametrize("n,width,nhid", [(8, 64, 5), (8, 16, 1), (4, 12, 3), (2, 8, 4)])
@pytest.mark.parametrize("act", [oracle.ACT_TANH, oracle.ACT_SOFTPLUS])
def test_mlp_of_any_depth_and_activation_matches_autograd(n, width, nhid, act):
    # the general field (App. B.2 uses six linear layers with softplus): f, Jacobian and the vector-Jacobian
    # product of every parameter block against the library's own softplus / tanh and autograd
    rng = np.random.default_rng(10 * n + width + nhid + act)
    theta = rng.standard_normal(inputs.mlp_theta_count(n, width, nhid)) / np.sqrt(width)
    cell = oracle.make_cell(oracle.CELL_MLP, n, 0, width, nhid, act)
    fun = torch.tanh if act == oracle.ACT_TANH else torch.nn.functional.softplus
    tht = torch.tensor(theta, requires_grad=True)

    def f_of(th, y):
        o, nin, a = 0, n, y
        for _ in range(nhid):
            W = th[o:o + width * nin].reshape(width, nin); o += width * nin
            b = th[o:o + width]; o += width
            a = fun(W @ a + b)
            nin = width
        Wo = th[o:o + n * nin].reshape(n, nin); o += n * nin
        return Wo @ a + th[o:o + n]

    y = rng.standard_normal(n) * 3.0        # softplus is exercised on both of its branches
    yt = torch.tensor(y, requires_grad=True)
    out = f_of(tht, yt)
    np.testing.assert_allclose(oracle.cell_f(cell, theta, y), out.detach().numpy(), atol=1e-13)
    Jt = torch.autograd.functional.jacobian(lambda yy: f_of(tht.detach(), yy), torch.tensor(y)).numpy()
    np.testing.assert_allclose(oracle.cell_jac(cell, theta, y), Jt, atol=1e-12)
    w = rng.standard_normal(n)
    (out * torch.tensor(w)).sum().backward()
    dth, dy = oracle.mlp_vjp(cell, theta, y, w)
    np.testing.assert_allclose(dth, tht.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dy, yt.grad.numpy(), atol=1e-12)


def test_softplus_limits():
    # log(1 + e^a) must not overflow and must approach a (large a) and e^a (very negative a)
    cell = oracle.make_cell(oracle.CELL_MLP, 1, 0, 1, 1, oracle.ACT_SOFTPLUS)
    theta = np.array([1.0, 0.0, 1.0, 0.0])     # f(y) = softplus(y)
    for a, want in [(800.0, 800.0), (-800.0, 0.0), (0.0, np.log(2.0)), (40.0, 40.0), (-40.0, np.exp(-40.0))]:
        got = oracle.cell_f(cell, theta, np.array([a]))[0]
        assert np.isfinite(got) and abs(got - want) <= 1e-15 * max(1.0, abs(want)) + 1e-30
    assert abs(oracle.cell_jac(cell, theta, np.array([0.0]))[0, 0] - 0.5) < 1e-15


def test_affine_cell():
    n, d = 3, 2
    rng = np.random.default_rng(3)
    A, Bm, c = rng.standard_normal((n, n)), rng.standard_normal((n, d)), rng.standard_normal(n)
    theta = np.concatenate([A.ravel(), Bm.ravel(), c])
    cell = oracle.make_cell(oracle.CELL_AFFINE, n, d)
    h, x = rng.standard_normal(n), rng.standard_normal(d)
    np.testing.assert_allclose(oracle.cell_f(cell, theta, h, x), A @ h + Bm @ x + c, atol=1e-14)
    np.testing.assert_allclose(oracle.cell_jac(cell, theta, h, x), A, atol=0)
