"""GPU parity of deer_eval and deer_grad for the LEM cell (the cell of the paper's last experiment) against the
oracle's DEER and backward derivative, element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_12252_amd import deer, inputs
from helpers import DEV, TOL_ABS, dev, grad_errors, host

pytestmark = pytest.mark.gpu


def run(w, dtype):
    tol = w.tol if dtype == deer.DEER_F32 else 1e-9
    u, d = w.n, w.d
    cell = oracle.make_cell(oracle.CELL_LEM, 2 * u, d, dt=w.t1)
    yo, ito, _, _ = oracle.deer_eval(cell, w.theta, w.x, w.y0, tol=tol, max_iter=w.max_iter, nthreads=8)
    ctx = deer.context_for(w, dtype=dtype, device=DEV)
    try:
        th, x, y0 = dev(w.theta, dtype), dev(w.x, dtype), dev(w.y0, dtype)
        y, it, err, conv, st = ctx.eval(th, x, y0, tol=tol, max_iter=w.max_iter)
        torch.cuda.synchronize()
        assert st == deer.DEER_OK and conv and abs(it - ito) <= 1, (w.name, it, ito)
        e = np.abs(host(y) - yo).max()
        assert e <= TOL_ABS[dtype], (w.name, dtype, e)
        ys = oracle.seq_eval(cell, w.theta, w.x, w.y0, nthreads=8)
        g = (np.random.default_rng(1).standard_normal(ys.shape) / np.sqrt(w.T)).astype(np.float32).astype(np.float64)
        dth_o, dx_o, dy0_o = oracle.rnn_grad(cell, w.theta, w.x, w.y0, ys, g)
        dth, dx, dy0 = ctx.grad(th, x, y0, dev(ys, dtype), dev(g, dtype))
        dth2, _, _ = ctx.grad(th, x, y0, dev(ys, dtype), dev(g, dtype), want_dx=False, want_dy0=False)
        assert grad_errors(w.name, "dL/dtheta", host(dth), dth_o) <= TOL_ABS[dtype]
        assert grad_errors(w.name, "dL/dx", host(dx), dx_o) <= TOL_ABS[dtype]
        assert grad_errors(w.name, "dL/dy0", host(dy0), dy0_o) <= TOL_ABS[dtype]
        assert np.array_equal(host(dth), host(dth2))
    finally:
        ctx.close()


@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
@pytest.mark.parametrize("u,d,dt", [(1, 1, 1.0), (2, 2, 0.5), (3, 5, 1.0), (4, 4, 0.25), (5, 8, 1.0), (8, 6, 0.5), (12, 3, 1.0),
                                    (16, 8, 1.0)])
def test_lem_shapes(u, d, dt, dtype):
    for k, (B, T) in enumerate([(1, 1), (2, 9), (3, 700), (2, 3001)]):
        w = inputs.lem_workload("lem_u%d_d%d_T%d" % (u, d, T), 30 * u + d + k, B=B, T=T, units=u, d=d, dt=dt)
        w.y0 = (np.random.default_rng(k).standard_normal((B, 2 * u)) * 0.5).astype(np.float32)
        run(w, dtype)


def test_lem_long_sequences():
    # the length of the series the paper trains this cell on (App. B.3: 17,984 samples, 6 channels)
    w = inputs.lem_workload("lem_u16_T17984", 89, B=8, T=17984, units=16, d=6, dt=1.0)
    run(w, deer.DEER_F32)


def test_lem_step_must_be_positive():
    with pytest.raises(deer.DeerError) as e:
        deer.workspace_bytes(deer.make_config(deer.DEER_CELL_LEM, deer.DEER_F32, 1, 10, 4, d=2, t1=0.0))
    assert e.value.status == deer.DEER_ERR_UNSUPPORTED
