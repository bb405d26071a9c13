"""GPU parity on seeded random shapes: forward solve and backward pass of both cells against the oracle.

The fixed lists of the other files pick the shapes around the tile boundaries by hand; this one draws state size,
input width, batch, length and precision at random (fixed seeds), so that kernel variants meet shapes nobody chose."""
import numpy as np
import pytest

import oracle
from paper_2309_12252_amd import deer, inputs
from helpers import DEV, TOL_ABS, dev, host, oracle_cell, oracle_eval, gpu_eval

pytestmark = pytest.mark.gpu

LENGTHS = [1, 2, 3, 17, 63, 64, 65, 95, 96, 97, 127, 129, 511, 513, 1000, 2049, 4097]


def abs_err(got, want):
    return np.abs(got - want).max()


@pytest.mark.parametrize("seed", range(10))
def test_gru_random_shapes(seed):
    rng = np.random.default_rng(4000 + seed)
    for it in range(8):
        n = int(rng.choice([1, 2, 4, 8, 16, 32]))
        d = int(rng.integers(1, 17))
        B = int(rng.integers(1, 6))
        T = int(rng.choice(LENGTHS + [int(rng.integers(1, 6000))]))
        dtype = int(rng.choice([deer.DEER_F32, deer.DEER_F64]))
        case = (seed, it, n, d, B, T, dtype)
        print("gru case", case, flush=True)
        w = inputs.gru_workload("rand", 5000 + 10 * seed + it, B=B, T=T, n=n, d=d)
        w.y0 = rng.standard_normal((B, n)).astype(np.float32)
        w.tol = 1e-4 if dtype == deer.DEER_F32 else 1e-9
        # forward: Newton iterations to convergence
        yo, ito, _, _ = oracle_eval(w)
        yg, itg, _, conv, st = gpu_eval(w, dtype=dtype)
        assert st == deer.DEER_OK and conv, case
        assert abs(itg - ito) <= 1, (case, itg, ito)
        assert np.abs(yg - yo).max() <= TOL_ABS[dtype], (case, np.abs(yg - yo).max())
        # backward at the sequential trajectory
        g = (rng.standard_normal((B, T, n)) / np.sqrt(T)).astype(np.float32).astype(np.float64)
        y = oracle.seq_eval(oracle_cell(w), w.theta, w.x, w.y0, nthreads=8)
        dth_o, dx_o, dy0_o = oracle.gru_grad(w.n, w.d, w.theta, w.x, w.y0, y, g)
        ctx = deer.context_for(w, dtype=dtype, device=DEV)
        try:
            dth, dx, dy0 = ctx.grad(dev(w.theta, dtype), dev(w.x, dtype), dev(w.y0, dtype), dev(y, dtype), dev(g, dtype))
        finally:
            ctx.close()
        for got, want in ((dth, dth_o), (dx, dx_o), (dy0, dy0_o)):
            assert abs_err(host(got), want) <= TOL_ABS[dtype], (case, abs_err(host(got), want))


@pytest.mark.parametrize("seed", range(5))
def test_ode_random_shapes(seed):
    rng = np.random.default_rng(4100 + seed)
    for it in range(6):
        n, width = [(2, 16), (4, 32), (8, 16), (8, 32), (8, 64), (4, 16)][int(rng.integers(0, 6))]
        B = int(rng.integers(1, 5))
        T = int(rng.choice([2, 3, 16, 17, 33, 100, 1025, 3000, int(rng.integers(2, 8000))]))
        t1 = float(rng.choice([0.1, 1.0, 2.0, 4.0]))
        dtype = int(rng.choice([deer.DEER_F32, deer.DEER_F64]))
        case = (seed, it, n, width, B, T, t1, dtype)
        print("ode case", case, flush=True)
        w = inputs.mlp_ode_workload("rand_ode", 5100 + 10 * seed + it, B=B, T=T, n=n, width=width, nhid=2, t0=0.0, t1=t1,
                                    tol=1e-4 if dtype == deer.DEER_F32 else 1e-9)
        yo, ito, _, _ = oracle_eval(w)
        yg, itg, _, conv, st = gpu_eval(w, dtype=dtype)
        assert st == deer.DEER_OK and conv, case
        assert abs(itg - ito) <= 1, (case, itg, ito)
        assert np.abs(yg - yo).max() <= TOL_ABS[dtype], (case, np.abs(yg - yo).max())
        # backward at the oracle's converged trajectory
        g = (rng.standard_normal((B, T, n)) / np.sqrt(T)).astype(np.float32).astype(np.float64)
        yt = oracle_eval(w, tol=1e-9)[0].astype(np.float32).astype(np.float64)   # what the device sees in either precision
        dth_o, dy0_o = oracle.ode_grad(oracle_cell(w), w.theta, yt, g, w.t0, w.t1)
        ctx = deer.context_for(w, dtype=dtype, device=DEV)
        try:
            dth, _, dy0 = ctx.grad(dev(w.theta, dtype), None, None, dev(yt, dtype), dev(g, dtype))
        finally:
            ctx.close()
        assert abs_err(host(dth), dth_o) <= TOL_ABS[dtype], (case, abs_err(host(dth), dth_o))
        assert abs_err(host(dy0), dy0_o) <= TOL_ABS[dtype], (case, abs_err(host(dy0), dy0_o))
