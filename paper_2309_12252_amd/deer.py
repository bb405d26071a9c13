"""Thin ctypes binding of the C-ABI HIP library (include/deer.h).

Argument marshalling only: every step of the path runs in the library's kernels.
PyTorch supplies device memory and the stream.  Loading fails loudly when the
library has not been built (``python -m paper_2309_12252_amd.build``); there is no
CPU fallback.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdeer_hip.so")

DEER_OK, DEER_ERR_INVALID_ARG, DEER_ERR_UNSUPPORTED, DEER_ERR_WORKSPACE, DEER_ERR_HIP, DEER_ERR_NONFINITE = range(6)
DEER_CELL_GRU, DEER_CELL_MLP_ODE, DEER_CELL_LSTM, DEER_CELL_LEM = 0, 1, 2, 3
DEER_F32, DEER_F64 = 0, 1

EXPORTS = ["deer_theta_count", "deer_workspace_bytes", "deer_create", "deer_eval", "deer_grad",
           "deer_linrec_solve", "deer_linrec_solve_static", "deer_set_profiling", "deer_get_profile", "deer_last_error", "deer_destroy"]


class DeerConfig(ctypes.Structure):
    _fields_ = [("cell", ctypes.c_int32), ("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("T", ctypes.c_int32),
                ("n", ctypes.c_int32), ("d", ctypes.c_int32), ("mlp_width", ctypes.c_int32),
                ("mlp_hidden_layers", ctypes.c_int32), ("t0", ctypes.c_double), ("t1", ctypes.c_double),
                ("mlp_activation", ctypes.c_int32), ("heads", ctypes.c_int32), ("stride_levels", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class DeerProfile(ctypes.Structure):
    _fields_ = [("funceval_ms", ctypes.c_double), ("funceval_launches", ctypes.c_int64),
                ("discretise_ms", ctypes.c_double), ("discretise_launches", ctypes.c_int64),
                ("scan_ms", ctypes.c_double), ("scan_launches", ctypes.c_int64),
                ("vjp_ms", ctypes.c_double), ("vjp_launches", ctypes.c_int64),
                ("fused_ms", ctypes.c_double), ("fused_launches", ctypes.c_int64),
                ("newton_ms", ctypes.c_double), ("newton_launches", ctypes.c_int64),
                ("newton_iterations", ctypes.c_int64)]


class DeerError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("deer status %d: %s" % (status, message))
        self.status = status


_lib = None


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: build it with `python -m paper_2309_12252_amd.build` "
                           "(there is no fallback path)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_double
    cfgp = ctypes.POINTER(DeerConfig)
    lib.deer_theta_count.restype = ctypes.c_size_t
    lib.deer_theta_count.argtypes = [cfgp]
    lib.deer_workspace_bytes.restype = ctypes.c_int
    lib.deer_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t)]
    lib.deer_create.restype = ctypes.c_int
    lib.deer_create.argtypes = [cfgp, vp, ctypes.c_size_t, vp, ctypes.POINTER(vp)]
    lib.deer_eval.restype = ctypes.c_int
    lib.deer_eval.argtypes = [vp, vp, vp, vp, vp, dbl, i32, vp, ctypes.POINTER(i32), ctypes.POINTER(dbl),
                              ctypes.POINTER(i32)]
    lib.deer_grad.restype = ctypes.c_int
    lib.deer_grad.argtypes = [vp] * 9
    lib.deer_linrec_solve.restype = ctypes.c_int
    lib.deer_linrec_solve.argtypes = [vp, vp, vp, vp, vp, i32]
    lib.deer_linrec_solve_static.restype = ctypes.c_int
    lib.deer_linrec_solve_static.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, i32, vp, vp]
    lib.deer_set_profiling.restype = ctypes.c_int
    lib.deer_set_profiling.argtypes = [vp, i32]
    lib.deer_get_profile.restype = ctypes.c_int
    lib.deer_get_profile.argtypes = [vp, ctypes.POINTER(DeerProfile)]
    lib.deer_last_error.restype = ctypes.c_char_p
    lib.deer_last_error.argtypes = [vp]
    lib.deer_destroy.restype = None
    lib.deer_destroy.argtypes = [vp]
    _lib = lib
    return lib


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


DEER_ACT_TANH, DEER_ACT_SOFTPLUS = 0, 1


def make_config(cell, dtype, B, T, n, d=0, mlp_width=0, mlp_hidden_layers=0, t0=0.0, t1=0.0, mlp_activation=0,
                heads=0, stride_levels=0):
    return DeerConfig(int(cell), int(dtype), int(B), int(T), int(n), int(d), int(mlp_width),
                      int(mlp_hidden_layers), float(t0), float(t1), int(mlp_activation), int(heads), int(stride_levels), 0)


def theta_count(cfg):
    return int(load_library().deer_theta_count(ctypes.byref(cfg)))


def workspace_bytes(cfg):
    lib = load_library()
    out = ctypes.c_size_t(0)
    st = lib.deer_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out))
    if st != DEER_OK:
        raise DeerError(st, lib.deer_last_error(None).decode())
    return int(out.value)


class DeerContext:
    """One deer_ctx plus the torch tensor that backs its workspace."""

    def __init__(self, cfg, device="cuda:0", stream=None):
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        self.torch_dtype = torch.float32 if cfg.dtype == DEER_F32 else torch.float64
        nbytes = workspace_bytes(cfg)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        handle = ctypes.c_void_p(None)
        st = self.lib.deer_create(ctypes.byref(cfg), ctypes.c_void_p(self._ws_ptr), nbytes,
                                  ctypes.c_void_p(self.stream.cuda_stream), ctypes.byref(handle))
        if st != DEER_OK:
            raise DeerError(st, self.lib.deer_last_error(None).decode())
        self.handle = handle

    def _check(self, st, allow=()):
        if st != DEER_OK and st not in allow:
            raise DeerError(st, self.lib.deer_last_error(self.handle).decode())
        return st

    def _tensor(self, t, shape=None):
        if t is None:
            return None
        assert t.is_cuda and t.dtype == self.torch_dtype and t.is_contiguous(), "need a contiguous device tensor"
        if shape is not None:
            assert tuple(t.shape) == tuple(shape), (tuple(t.shape), tuple(shape))
        return t

    def _shapes(self):
        """(trajectory, inputs, initial state) shapes: with heads, arrays carry a head axis in front of the channels"""
        c = self.cfg
        if c.cell == DEER_CELL_GRU and (c.heads > 1 or c.stride_levels > 1):
            H = max(1, c.heads)
            return (c.B, c.T, H, c.n), (c.B, c.T, H, c.d), (c.B, H, c.n)
        if c.cell in (DEER_CELL_LSTM, DEER_CELL_LEM):   # n units, state (h | c) or (y | z)
            return (c.B, c.T, 2 * c.n), (c.B, c.T, c.d), (c.B, 2 * c.n)
        return (c.B, c.T, c.n), (c.B, c.T, c.d), (c.B, c.n)

    def eval(self, theta, x, y0, y_guess=None, tol=1e-4, max_iter=100, out=None, allow_nonfinite=False):
        """deer_eval.  Returns (y, iters, final_err, converged, status)."""
        c = self.cfg
        ys, xs, y0s = self._shapes()
        y = out if out is not None else torch.empty(ys, dtype=self.torch_dtype, device=self.device)
        assert theta.numel() == theta_count(c)
        self._tensor(theta)
        if c.cell != DEER_CELL_MLP_ODE:
            self._tensor(x, xs)
        self._tensor(y0, y0s)
        self._tensor(y_guess, ys)
        self._tensor(y, ys)
        iters, conv, err = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_double(0.0)
        st = self.lib.deer_eval(self.handle, _ptr(theta), _ptr(x), _ptr(y0), _ptr(y_guess), float(tol),
                                int(max_iter), _ptr(y), ctypes.byref(iters), ctypes.byref(err), ctypes.byref(conv))
        self._check(st, allow=(DEER_ERR_NONFINITE,) if allow_nonfinite else ())
        return y, int(iters.value), float(err.value), bool(conv.value), st

    def grad(self, theta, x, y0, y, dLdy, want_dx=True, want_dy0=True):
        """deer_grad.  Returns (dL/dtheta, dL/dx or None, dL/dy0 or None)."""
        c = self.cfg
        ode = c.cell == DEER_CELL_MLP_ODE   # autonomous field: no inputs, hence no dL/dx; x and y0 may be None
        for t in (theta, x, y0, y, dLdy):
            self._tensor(t)
        ys, xs, y0s = self._shapes()
        dtheta = torch.empty(theta_count(c), dtype=self.torch_dtype, device=self.device)
        dx = torch.empty(xs, dtype=self.torch_dtype, device=self.device) if (want_dx and not ode) else None
        dy0 = torch.empty(y0s, dtype=self.torch_dtype, device=self.device) if want_dy0 else None
        st = self.lib.deer_grad(self.handle, _ptr(theta), _ptr(x), _ptr(y0), _ptr(y), _ptr(dLdy), _ptr(dx),
                                _ptr(dtheta), _ptr(dy0))
        self._check(st)
        return dtheta, dx, dy0

    def linrec_solve(self, A, b, y0=None, reverse=False, out=None):
        c = self.cfg
        self._tensor(A, (c.B, c.T, c.n, c.n))
        self._tensor(b, (c.B, c.T, c.n))
        self._tensor(y0, (c.B, c.n))
        y = out if out is not None else torch.empty((c.B, c.T, c.n), dtype=self.torch_dtype, device=self.device)
        st = self.lib.deer_linrec_solve(self.handle, _ptr(A), _ptr(b), _ptr(y0), _ptr(y), 1 if reverse else 0)
        self._check(st)
        return y

    def set_profiling(self, on):
        self._check(self.lib.deer_set_profiling(self.handle, 1 if on else 0))

    def profile(self):
        p = DeerProfile()
        self._check(self.lib.deer_get_profile(self.handle, ctypes.byref(p)))
        return {k: getattr(p, k) for k, _ in DeerProfile._fields_}

    def close(self):
        if getattr(self, "handle", None):
            self.lib.deer_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def linrec_solve_static(A, b, y0=None, reverse=False, out=None, status=None, stream=None):
    """deer_linrec_solve_static: the scan alone without a context or workspace (nothing is allocated by the
    library).  A [B,T,n,n], b [B,T,n], y0 [B,n] or None; `out` and the int32 device tensor `status` are the
    caller's.  Asynchronous on `stream` (default: torch's current stream).  Returns out."""
    lib = load_library()
    assert A.is_cuda and A.is_contiguous() and b.is_contiguous() and A.dtype == b.dtype
    B, T, n, _ = A.shape
    assert tuple(b.shape) == (B, T, n) and (y0 is None or tuple(y0.shape) == (B, n))
    dtype = DEER_F32 if A.dtype == torch.float32 else DEER_F64
    y = out if out is not None else torch.empty((B, T, n), dtype=A.dtype, device=A.device)
    stream = stream if stream is not None else torch.cuda.current_stream(A.device)
    st = lib.deer_linrec_solve_static(dtype, B, T, n, _ptr(A), _ptr(b), _ptr(y0), _ptr(y), 1 if reverse else 0,
                                      ctypes.c_void_p(stream.cuda_stream), _ptr(status))
    if st != DEER_OK:
        raise DeerError(st, lib.deer_last_error(None).decode())
    return y


def context_for(workload, dtype=DEER_F32, device="cuda:0"):
    """Context for an ``inputs.Workload``."""
    cfg = make_config(workload.cell, dtype, workload.B, workload.T, workload.n, workload.d, workload.mlp_width,
                      workload.mlp_hidden_layers, workload.t0, workload.t1, workload.mlp_activation,
                      workload.heads, workload.stride_levels)
    return DeerContext(cfg, device=device)
