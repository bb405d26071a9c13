"""ctypes front end of the CPU fp64 oracle (``deer_oracle.c``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu_baseline leg use it; the product path never does.  Nothing here touches
the HIP library, and the HIP path imports nothing from here.

All arrays are converted to C-contiguous float64 before the call, so fp32
inputs are up-cast exactly.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "deer_oracle.c")
_LIB = os.path.join(_HERE, "libdeer_oracle.so")

CELL_GRU, CELL_MLP, CELL_AFFINE, CELL_LSTM, CELL_LEM = 0, 1, 2, 3, 4


class _Cell(ctypes.Structure):
    _fields_ = [("cell", ctypes.c_int), ("n", ctypes.c_int), ("d", ctypes.c_int),
                ("width", ctypes.c_int), ("nhid", ctypes.c_int), ("act", ctypes.c_int), ("dt", ctypes.c_double)]


def build(force=False):
    """Compile the oracle with gcc (plain -O2, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_theta_count.restype = ctypes.c_long
        _lib.oracle_deer_eval.restype = ctypes.c_int
        _lib.oracle_ode_deer_eval.restype = ctypes.c_int
        _lib.oracle_mh_deer_eval.restype = ctypes.c_int
        _lib.oracle_max_threads.restype = ctypes.c_int
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


ACT_TANH, ACT_SOFTPLUS = 0, 1


def make_cell(cell, n, d=0, width=0, nhid=0, act=ACT_TANH, dt=1.0):
    """n is the state size (LSTM, LEM: twice the units); dt is the LEM cell's step."""
    return _Cell(int(cell), int(n), int(d), int(width), int(nhid), int(act), float(dt))


def theta_count(cell):
    return int(lib().oracle_theta_count(ctypes.byref(cell)))


def max_threads():
    return int(lib().oracle_max_threads())


def cell_f(cell, theta, h, x=None):
    theta, h = _f64(theta), _f64(h)
    x = _f64(x) if x is not None else None
    out = np.empty(cell.n)
    lib().oracle_cell_f(ctypes.byref(cell), _p(theta), _p(h), _p(x), _p(out))
    return out


def cell_jac(cell, theta, h, x=None):
    theta, h = _f64(theta), _f64(h)
    x = _f64(x) if x is not None else None
    J = np.empty((cell.n, cell.n))
    lib().oracle_cell_jac(ctypes.byref(cell), _p(theta), _p(h), _p(x), _p(J))
    return J


def gru_vjp(n, d, theta, h, x, lam):
    theta, h, x, lam = _f64(theta), _f64(h), _f64(x), _f64(lam)
    dtheta = np.zeros(theta.size)
    dx = np.empty(d)
    dh = np.empty(n)
    lib().oracle_gru_vjp(n, d, _p(theta), _p(h), _p(x), _p(lam), _p(dtheta), _p(dx), _p(dh))
    return dtheta, dx, dh


def cell_vjp(cell, theta, h, x, lam):
    """GRU / LSTM: (dtheta, dx, dh) for an output cotangent lam (cell.n is the state size)."""
    theta, h, x, lam = _f64(theta), _f64(h), _f64(x), _f64(lam)
    dtheta = np.zeros(theta.size)
    dx = np.empty(cell.d)
    dh = np.empty(cell.n)
    lib().oracle_cell_vjp(ctypes.byref(cell), _p(theta), _p(h), _p(x), _p(lam), _p(dtheta), _p(dx), _p(dh))
    return dtheta, dx, dh


def rnn_grad(cell, theta, x, y0, y, g):
    """Backward derivative for a recurrent cell (GRU, LSTM).  Returns (dtheta, dx [B,T,d], dy0 [B,n])."""
    theta, x, y0, y, g = _f64(theta), _f64(x), _f64(y0), _f64(y), _f64(g)
    B, T, _ = x.shape
    dtheta = np.empty(theta.size)
    dx = np.empty((B, T, cell.d))
    dy0 = np.empty((B, cell.n))
    lib().oracle_rnn_grad(ctypes.byref(cell), _p(theta), ctypes.c_long(B), ctypes.c_long(T), _p(x), _p(y0), _p(y), _p(g),
                          _p(dtheta), _p(dx), _p(dy0))
    return dtheta, dx, dy0


def affine_combine(Gi, zi, Gj, zj):
    """(Gi|zi) earlier, (Gj|zj) later -> (Gj Gi | Gj zi + zj)."""
    Gi, zi, Gj, zj = _f64(Gi), _f64(zi), _f64(Gj), _f64(zj)
    n = zi.size
    Go, zo = np.empty((n, n)), np.empty(n)
    lib().oracle_affine_combine(n, _p(Gi), _p(zi), _p(Gj), _p(zj), _p(Go), _p(zo))
    return Go, zo


def linrec_serial(Gbar, zbar, y0):
    """y_i = Gbar_i y_{i-1} + zbar_i for one sequence; Gbar [T,n,n], zbar [T,n]."""
    Gbar, zbar, y0 = _f64(Gbar), _f64(zbar), _f64(y0)
    T, n = zbar.shape
    y = np.empty((T, n))
    lib().oracle_linrec_serial(n, ctypes.c_long(T), _p(Gbar), _p(zbar), _p(y0), _p(y))
    return y


def affine_scan(Gbar, zbar, y0):
    Gbar, zbar, y0 = _f64(Gbar), _f64(zbar), _f64(y0)
    T, n = zbar.shape
    y = np.empty((T, n))
    lib().oracle_affine_scan(n, ctypes.c_long(T), _p(Gbar), _p(zbar), _p(y0), _p(y))
    return y


def seq_eval(cell, theta, x, y0, T=None, nthreads=1):
    """Sequential evaluation.  x [B,T,d] (None for cells without input: pass T), y0 [B,n]."""
    theta, y0 = _f64(theta), _f64(y0)
    B = y0.shape[0]
    if x is not None:
        x = _f64(x)
        T = x.shape[1]
    y = np.empty((B, T, cell.n))
    lib().oracle_seq_eval(ctypes.byref(cell), _p(theta), ctypes.c_long(B), ctypes.c_long(T), _p(x),
                          _p(y0), _p(y), int(nthreads))
    return y


def deer_eval(cell, theta, x, y0, guess=None, tol=1e-7, max_iter=100, T=None, nthreads=1):
    """DEER for an RNN.  Returns (y [B,T,n], iterations, final err, err history)."""
    theta, y0 = _f64(theta), _f64(y0)
    B = y0.shape[0]
    if x is not None:
        x = _f64(x)
        T = x.shape[1]
    guess = _f64(guess) if guess is not None else None
    y = np.empty((B, T, cell.n))
    err = ctypes.c_double(0.0)
    hist = np.full(max_iter, np.nan)
    it = lib().oracle_deer_eval(ctypes.byref(cell), _p(theta), ctypes.c_long(B), ctypes.c_long(T), _p(x),
                                _p(y0), _p(guess), ctypes.c_double(tol), int(max_iter), _p(y),
                                ctypes.byref(err), _p(hist), int(nthreads))
    return y, int(it), float(err.value), hist[:it]


def gru_grad(n, d, theta, x, y0, y, g):
    """Backward derivative for the GRU recurrence.  Returns (dtheta, dx [B,T,d], dy0 [B,n])."""
    theta, x, y0, y, g = _f64(theta), _f64(x), _f64(y0), _f64(y), _f64(g)
    B, T, _ = x.shape
    dtheta = np.empty(theta.size)
    dx = np.empty((B, T, d))
    dy0 = np.empty((B, n))
    lib().oracle_gru_grad(n, d, _p(theta), ctypes.c_long(B), ctypes.c_long(T), _p(x), _p(y0), _p(y), _p(g),
                          _p(dtheta), _p(dx), _p(dy0))
    return dtheta, dx, dy0


def mh_seq_eval(n, d, H, K, theta, x, y0, nthreads=1):
    """Multi-head strided GRU, sequential.  theta [H, P], x [B,T,H,d], y0 [B,H,n] -> y [B,T,H,n]."""
    theta, x, y0 = _f64(theta), _f64(x), _f64(y0)
    B, T = x.shape[0], x.shape[1]
    y = np.empty((B, T, H, n))
    lib().oracle_mh_seq_eval(n, d, H, K, _p(theta), ctypes.c_long(B), ctypes.c_long(T), _p(x), _p(y0), _p(y), int(nthreads))
    return y


def mh_deer_eval(n, d, H, K, theta, x, y0, guess=None, tol=1e-7, max_iter=100, nthreads=1):
    """DEER for the multi-head strided GRU.  Returns (y [B,T,H,n], iterations, final err, err history)."""
    theta, x, y0 = _f64(theta), _f64(x), _f64(y0)
    B, T = x.shape[0], x.shape[1]
    guess = _f64(guess) if guess is not None else None
    y = np.empty((B, T, H, n))
    err = ctypes.c_double(0.0)
    hist = np.full(max_iter, np.nan)
    it = lib().oracle_mh_deer_eval(n, d, H, K, _p(theta), ctypes.c_long(B), ctypes.c_long(T), _p(x), _p(y0), _p(guess),
                                   ctypes.c_double(tol), int(max_iter), _p(y), ctypes.byref(err), _p(hist), int(nthreads))
    return y, int(it), float(err.value), hist[:it]


def mh_gru_grad(n, d, H, K, theta, x, y0, y, g):
    """Backward derivative of the multi-head strided GRU.  Returns (dtheta [H,P], dx [B,T,H,d], dy0 [B,H,n])."""
    theta, x, y0, y, g = _f64(theta), _f64(x), _f64(y0), _f64(y), _f64(g)
    B, T = x.shape[0], x.shape[1]
    dtheta = np.empty(theta.size).reshape(H, -1)
    dx = np.empty((B, T, H, d))
    dy0 = np.empty((B, H, n))
    lib().oracle_mh_gru_grad(n, d, H, K, _p(theta), ctypes.c_long(B), ctypes.c_long(T), _p(x), _p(y0), _p(y), _p(g),
                             _p(dtheta), _p(dx), _p(dy0))
    return dtheta, dx, dy0


def mlp_vjp(cell, theta, y, w):
    """VJP of the MLP field at one point.  Returns (dtheta, dy)."""
    theta, y, w = _f64(theta), _f64(y), _f64(w)
    dth, dy = np.zeros(theta.size), np.empty(cell.n)
    lib().oracle_mlp_vjp(ctypes.byref(cell), _p(theta), _p(y), _p(w), _p(dth), _p(dy))
    return dth, dy


def ode_grad(cell, theta, y, g, t0, t1):
    """Backward derivative for the ODE form.  y, g: [B,T,n].  Returns (dtheta, dy0 [B,n])."""
    theta, y, g = _f64(theta), _f64(y), _f64(g)
    B, T, n = y.shape
    dth, dy0 = np.empty(theta.size), np.empty((B, n))
    lib().oracle_ode_grad(ctypes.byref(cell), _p(theta), ctypes.c_long(B), ctypes.c_long(T), ctypes.c_double(t0),
                          ctypes.c_double(t1), _p(y), _p(g), _p(dth), _p(dy0))
    return dth, dy0


def expm_phi1(A):
    A = _f64(A)
    n = A.shape[0]
    E, P = np.empty((n, n)), np.empty((n, n))
    lib().oracle_expm_phi1(n, _p(A), _p(E), _p(P))
    return E, P


def ode_discretise(G0, z0, G1, z1, dt):
    G0, z0, G1, z1 = _f64(G0), _f64(z0), _f64(G1), _f64(z1)
    n = z0.size
    Gbar, zbar = np.empty((n, n)), np.empty(n)
    lib().oracle_ode_discretise(n, _p(G0), _p(z0), _p(G1), _p(z1), ctypes.c_double(dt), _p(Gbar), _p(zbar))
    return Gbar, zbar


def ode_deer_eval(cell, theta, y0, T, t0, t1, guess=None, tol=1e-7, max_iter=100, nthreads=1):
    """DEER for dy/dt = f(y) on a uniform grid.  Returns (y [B,T,n], iterations, err, err history)."""
    theta, y0 = _f64(theta), _f64(y0)
    B = y0.shape[0]
    guess = _f64(guess) if guess is not None else None
    y = np.empty((B, T, cell.n))
    err = ctypes.c_double(0.0)
    hist = np.full(max_iter, np.nan)
    it = lib().oracle_ode_deer_eval(ctypes.byref(cell), _p(theta), ctypes.c_long(B), ctypes.c_long(T),
                                    ctypes.c_double(t0), ctypes.c_double(t1), _p(y0), _p(guess),
                                    ctypes.c_double(tol), int(max_iter), _p(y), ctypes.byref(err),
                                    _p(hist), int(nthreads))
    return y, int(it), float(err.value), hist[:it]
