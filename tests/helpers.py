"""Shared helpers of the GPU parity tests (marshalling only)."""
import numpy as np
import torch

import oracle
from paper_2309_12252_amd import deer, inputs

TOL_ABS = {deer.DEER_F32: 1e-4, deer.DEER_F64: 1e-9}   # parity bars: max-abs vs the fp64 oracle
NP_DTYPE = {deer.DEER_F32: np.float32, deer.DEER_F64: np.float64}
DEV = "cuda:0"


def dev(a, dtype):
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=NP_DTYPE[dtype]))).to(DEV)


def host(t):
    return t.detach().cpu().numpy().astype(np.float64)


def oracle_cell(w):
    if w.cell == inputs.CELL_GRU:
        return oracle.make_cell(oracle.CELL_GRU, w.n, w.d)
    return oracle.make_cell(oracle.CELL_MLP, w.n, 0, w.mlp_width, w.mlp_hidden_layers, w.mlp_activation)


def oracle_eval(w, tol=None, max_iter=None, guess=None, nthreads=8):
    tol = w.tol if tol is None else tol
    max_iter = w.max_iter if max_iter is None else max_iter
    if w.cell == inputs.CELL_GRU:
        return oracle.deer_eval(oracle_cell(w), w.theta, w.x, w.y0, guess=guess, tol=tol, max_iter=max_iter,
                                nthreads=nthreads)
    return oracle.ode_deer_eval(oracle_cell(w), w.theta, w.y0, w.T, w.t0, w.t1, guess=guess, tol=tol,
                                max_iter=max_iter, nthreads=nthreads)


def gpu_eval(w, dtype=deer.DEER_F32, tol=None, max_iter=None, guess=None, allow_nonfinite=False):
    tol = w.tol if tol is None else tol
    max_iter = w.max_iter if max_iter is None else max_iter
    ctx = deer.context_for(w, dtype=dtype, device=DEV)
    try:
        y, it, err, conv, st = ctx.eval(dev(w.theta, dtype), dev(w.x, dtype), dev(w.y0, dtype),
                                        y_guess=dev(guess, dtype), tol=tol, max_iter=max_iter,
                                        allow_nonfinite=allow_nonfinite)
        torch.cuda.synchronize()
        return host(y), it, err, conv, st
    finally:
        ctx.close()


def dual_serial(A, b):
    """Oracle for the dual operator on one sequence: y_T = b_T, y_i = b_i + A_{i+1}^T y_{i+1},
    obtained from the oracle's serial solver on the reversed, transposed sequence."""
    T, n = b.shape
    Ar = np.zeros_like(A, dtype=np.float64)
    for k in range(1, T):
        Ar[k] = np.asarray(A[T - k], dtype=np.float64).T
    br = np.asarray(b[::-1], dtype=np.float64)
    yr = oracle.linrec_serial(Ar, br, np.zeros(n))
    return yr[::-1]


def grad_errors(name, what, got, want):
    """max-abs error of a gradient array against the oracle's, printed with the scale of the oracle's values
    (pytest -s or a failing test shows the line); returns the max-abs error."""
    err = float(np.abs(got - want).max())
    scale = float(np.abs(want).max())
    print("%s: max|%s - oracle| = %.3e  (max|oracle| = %.3e)" % (name, what, err, scale), flush=True)
    return err
