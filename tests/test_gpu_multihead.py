"""GPU parity of the multi-head GRU with strides (Sec. 4.4, App. B.4): deer_eval and deer_grad against the oracle's
own DEER and backward derivative for the same strided recurrence, element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_12252_amd import deer, inputs
from helpers import DEV, TOL_ABS, dev, grad_errors, host

pytestmark = pytest.mark.gpu


def run(w, dtype, check_grad=True):
    tol = w.tol if dtype == deer.DEER_F32 else 1e-9
    n, d, H, K = w.n, w.d, w.heads, w.stride_levels
    yo, ito, _, _ = oracle.mh_deer_eval(n, d, H, K, w.theta, w.x, w.y0, tol=tol, max_iter=w.max_iter, nthreads=8)
    ctx = deer.context_for(w, dtype=dtype, device=DEV)
    try:
        th, x, y0 = dev(w.theta, dtype), dev(w.x, dtype), dev(w.y0, dtype)
        y, it, err, conv, st = ctx.eval(th, x, y0, tol=tol, max_iter=w.max_iter)
        torch.cuda.synchronize()
        assert st == deer.DEER_OK and conv and abs(it - ito) <= 1, (w.name, it, ito)
        e = np.abs(host(y) - yo).max()
        assert e <= TOL_ABS[dtype], (w.name, dtype, e)
        if not check_grad:
            return
        # backward at the sequential trajectory (deer_grad takes any trajectory, Sec. 3.1.1)
        ys = oracle.mh_seq_eval(n, d, H, K, w.theta, w.x, w.y0, nthreads=8)
        g = (np.random.default_rng(1).standard_normal(ys.shape) / np.sqrt(w.T)).astype(np.float32).astype(np.float64)
        dth_o, dx_o, dy0_o = oracle.mh_gru_grad(n, d, H, K, w.theta, w.x, w.y0, ys, g)
        dth, dx, dy0 = ctx.grad(th, x, y0, dev(ys, dtype), dev(g, dtype))
        dth2, _, _ = ctx.grad(th, x, y0, dev(ys, dtype), dev(g, dtype), want_dx=False, want_dy0=False)
        assert grad_errors(w.name, "dL/dtheta", host(dth).reshape(H, -1), dth_o) <= TOL_ABS[dtype]
        assert grad_errors(w.name, "dL/dx", host(dx), dx_o) <= TOL_ABS[dtype]
        assert grad_errors(w.name, "dL/dy0", host(dy0), dy0_o) <= TOL_ABS[dtype]
        assert np.array_equal(host(dth), host(dth2))
    finally:
        ctx.close()


@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
@pytest.mark.parametrize("n,d,H,K,B,T", [(8, 4, 4, 3, 2, 300), (4, 3, 5, 2, 3, 77), (2, 2, 3, 3, 2, 1000), (8, 8, 8, 8, 1, 700),
                                         (8, 5, 2, 1, 2, 600), (4, 1, 1, 4, 2, 129), (8, 4, 6, 4, 2, 5), (8, 4, 3, 2, 1, 1)])
def test_small_multihead_shapes(n, d, H, K, B, T, dtype):
    _small(n, d, H, K, B, T, dtype)


# short recurrences share a tile (two, four or eight of them on a half, a quarter or an eighth of its wavefronts):
# fewer steps than the largest stride, recurrence counts that leave a remainder, every state size
@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
@pytest.mark.parametrize("n,d,H,K,B,T", [(8, 4, 8, 8, 2, 100), (8, 8, 8, 8, 2, 1030), (2, 2, 8, 8, 2, 333), (4, 3, 8, 7, 3, 50),
                                         (8, 4, 8, 8, 1, 131), (4, 2, 16, 6, 2, 2050), (8, 3, 5, 8, 2, 515)])
def test_short_recurrences_that_share_tiles(n, d, H, K, B, T, dtype):
    _small(n, d, H, K, B, T, dtype)


def _small(n, d, H, K, B, T, dtype):
    w = inputs.mh_gru_workload("mh_n%d_H%d_K%d_T%d" % (n, H, K, T), 40 * n + H + K, B=B, T=T, n=n, d=d, H=H, K=K)
    w.y0 = np.random.default_rng(3).standard_normal((B, H, n)).astype(np.float32)
    run(w, dtype)


@pytest.mark.parametrize("L", ["1", "2", "4"])
def test_tile_shapes(L, monkeypatch):
    # positions per lane group of the fused step; sequences of every stride level end inside, at and past a tile edge
    monkeypatch.setenv("DEER_FUSED_L", L)
    tile = 8 * 8 * int(L)
    for k, T in enumerate([tile, 2 * tile + 3, 4 * tile - 1]):
        w = inputs.mh_gru_workload("mh_L%s_T%d" % (L, T), 800 + k, B=2, T=T, n=8, d=4, H=4, K=4)
        run(w, deer.DEER_F32)


def test_the_papers_multihead_shape():
    # 32 heads of 8 channels, strides 2^0 .. 2^7 dealt out to the heads in turn, sequences of 1,024 steps
    # (App. B.4: images read as sequences of 1,024 pixels)
    w = inputs.mh_gru_workload("mh_32x8_T1024", 4321, B=4, T=1024, n=8, d=8, H=32, K=8)
    run(w, deer.DEER_F32)


def test_warm_start_and_iteration_cap():
    w = inputs.mh_gru_workload("mh_ctl", 9, B=2, T=500, n=8, d=4, H=4, K=3)
    n, d, H, K = w.n, w.d, w.heads, w.stride_levels
    yo, _, _, _ = oracle.mh_deer_eval(n, d, H, K, w.theta, w.x, w.y0, tol=1e-10, max_iter=50)
    y2, it2, err2, _ = oracle.mh_deer_eval(n, d, H, K, w.theta, w.x, w.y0, tol=1e-4, max_iter=2)
    ctx = deer.context_for(w, device=DEV)
    try:
        th, x, y0 = dev(w.theta, 0), dev(w.x, 0), dev(w.y0, 0)
        y, it, err, conv, st = ctx.eval(th, x, y0, tol=1e-4, max_iter=2)
        assert it == 2 and not conv and np.abs(host(y) - y2).max() <= 1e-4 and abs(err - err2) <= 1e-4
        y, it, err, conv, st = ctx.eval(th, x, y0, y_guess=dev(yo, 0), tol=1e-4, max_iter=50)
        assert it == 1 and conv and np.abs(host(y) - yo).max() <= 1e-5
    finally:
        ctx.close()
