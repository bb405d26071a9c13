"""GPU parity on the GRU shapes outside the kernels' own menu: state sizes that are not a power of two (run embedded
in the next size with kernels, e.g. the 24 channels of the long-series classifier, App. B.3) and input sizes up to 32
(the 32 hidden / 32 input channels of the output comparison, Sec. 4.1, Fig. 3).  Forward solve and backward pass."""
import numpy as np
import pytest

import oracle
from paper_2309_12252_amd import deer, inputs
from helpers import DEV, TOL_ABS, dev, gpu_eval, grad_errors, host, oracle_cell, oracle_eval

pytestmark = pytest.mark.gpu


def forward_and_backward(w, dtype):
    tol = 1e-4 if dtype == deer.DEER_F32 else 1e-9
    yo, ito, _, _ = oracle_eval(w, tol=tol)
    yg, itg, _, conv, st = gpu_eval(w, dtype=dtype, tol=tol)
    assert st == deer.DEER_OK and conv and abs(itg - ito) <= 1, (w.name, itg, ito)
    assert np.abs(yg - yo).max() <= TOL_ABS[dtype], (w.name, np.abs(yg - yo).max())
    ys = oracle.seq_eval(oracle_cell(w), w.theta, w.x, w.y0, nthreads=8)
    g = (np.random.default_rng(2).standard_normal(ys.shape) / np.sqrt(w.T)).astype(np.float32).astype(np.float64)
    dth_o, dx_o, dy0_o = oracle.gru_grad(w.n, w.d, w.theta, w.x, w.y0, ys, g)
    ctx = deer.context_for(w, dtype=dtype, device=DEV)
    try:
        dth, dx, dy0 = ctx.grad(dev(w.theta, dtype), dev(w.x, dtype), dev(w.y0, dtype), dev(ys, dtype), dev(g, dtype))
    finally:
        ctx.close()
    assert grad_errors(w.name, "dL/dtheta", host(dth), dth_o) <= TOL_ABS[dtype]
    assert grad_errors(w.name, "dL/dx", host(dx), dx_o) <= TOL_ABS[dtype]
    assert grad_errors(w.name, "dL/dy0", host(dy0), dy0_o) <= TOL_ABS[dtype]


@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
@pytest.mark.parametrize("n,d", [(32, 32), (24, 6), (3, 5), (5, 2), (7, 9), (12, 20), (17, 3), (31, 16), (8, 24), (2, 32), (6, 8)])
def test_state_and_input_sizes_outside_the_menu(n, d, dtype):
    for k, (B, T) in enumerate([(2, 9), (3, 700), (2, 2100)]):
        w = inputs.gru_workload("shape_n%d_d%d_T%d" % (n, d, T), 60 * n + d + k, B=B, T=T, n=n, d=d)
        w.y0 = np.random.default_rng(k).standard_normal((B, n)).astype(np.float32)
        forward_and_backward(w, dtype)


@pytest.mark.parametrize("n,d", [(64, 8), (40, 3), (64, 32)])
def test_state_sizes_up_to_64(n, d):
    # Sec. 4.1, Table 4 lists n = 64; these sizes run in fp32 only (cell kernel, matrix-core scan, vector-ALU VJP)
    for k, (B, T) in enumerate([(2, 9), (3, 700), (2, 2100)]):
        w = inputs.gru_workload("shape_n%d_d%d_T%d" % (n, d, T), 60 * n + d + k, B=B, T=T, n=n, d=d)
        w.y0 = np.random.default_rng(k).standard_normal((B, n)).astype(np.float32)
        forward_and_backward(w, deer.DEER_F32)


def test_output_comparison_shape():
    # Sec. 4.1, Fig. 3: an untrained GRU with 32 hidden and 32 input channels on 10,000 steps, DEER against the
    # sequential evaluation (here: the oracle's sequential fp64 evaluation)
    w = inputs.gru_workload("fig3_shape", 3232, B=1, T=10000, n=32, d=32)
    yg, it, err, conv, st = gpu_eval(w)
    ys = oracle.seq_eval(oracle_cell(w), w.theta, w.x, w.y0)
    assert st == deer.DEER_OK and conv
    assert np.abs(yg - ys).max() <= 1e-4


def test_long_series_classifier_shape():
    # App. B.3: GRU cells with 24 hidden channels on series of 17,984 samples
    w = inputs.gru_workload("eigenworms_cell_shape", 2424, B=4, T=17984, n=24, d=6)
    forward_and_backward(w, deer.DEER_F32)
