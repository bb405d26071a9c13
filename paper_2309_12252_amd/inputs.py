"""Seeded synthetic inputs for the DEER workloads.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic.  Both the GPU tests/benchmark and the CPU oracle's tests
take their inputs from here so that the two sides see bit-identical fp32
values (the oracle up-casts them to fp64).

Every draw comes from ``numpy.random.default_rng(seed)`` (PCG64) in fp64 and is
rounded once to fp32.  Draw order: theta, x, y0, then anything workload specific.
"""
from dataclasses import dataclass, field

import numpy as np

CELL_GRU = 0
CELL_MLP_ODE = 1
CELL_LSTM = 2
CELL_LEM = 3


@dataclass
class Workload:
    name: str
    cell: int
    B: int
    T: int
    n: int
    d: int = 0
    mlp_width: int = 0
    mlp_hidden_layers: int = 0
    mlp_activation: int = 0    # 0 tanh, 1 softplus
    t0: float = 0.0
    t1: float = 0.0
    tol: float = 1e-4
    max_iter: int = 50
    heads: int = 1             # GRU: heads (each a GRU of its own on its own input slice)
    stride_levels: int = 1     # GRU multi-head: head h looks back 2^(h mod stride_levels) steps
    theta: np.ndarray = None   # flat fp32
    x: np.ndarray = None       # [B,T,d] fp32 or None
    y0: np.ndarray = None      # [B,n] fp32
    extra: dict = field(default_factory=dict)


def gru_theta_count(n, d):
    return 3 * n * d + 3 * n * n + 3 * n + n


def mlp_theta_count(n, width, nhid):
    if nhid == 0:
        return n * n + n
    return (width * n + width) + (nhid - 1) * (width * width + width) + (n * width + n)


def _normal(rng, shape, std):
    return (rng.standard_normal(shape) * std).astype(np.float32)


def gru_workload(name, seed, B, T, n, d, tol=1e-4, max_iter=50, x_kind="normal", theta_std=None):
    """GRU cell with every weight and bias ~ N(0, 1/n); x i.i.d. N(0,1) or sinusoids + noise; y0 = 0."""
    rng = np.random.default_rng(seed)
    std = (1.0 / np.sqrt(n)) if theta_std is None else theta_std
    theta = _normal(rng, gru_theta_count(n, d), std)
    if x_kind == "normal":
        x = _normal(rng, (B, T, d), 1.0)
    elif x_kind == "sinusoid":
        # sum of 3 sinusoids, frequency U[1e-4, 1e-2] cycles/step, phase U[0, 2pi), plus N(0, 0.1^2)
        freq = rng.uniform(1e-4, 1e-2, size=(B, 1, d, 3))
        phase = rng.uniform(0.0, 2.0 * np.pi, size=(B, 1, d, 3))
        t = np.arange(T, dtype=np.float64).reshape(1, T, 1, 1)
        x = np.sin(2.0 * np.pi * freq * t + phase).sum(axis=-1)
        x = (x + 0.1 * rng.standard_normal((B, T, d))).astype(np.float32)
    else:
        raise ValueError(x_kind)
    y0 = np.zeros((B, n), dtype=np.float32)
    return Workload(name=name, cell=CELL_GRU, B=B, T=T, n=n, d=d, tol=tol, max_iter=max_iter,
                    theta=theta, x=x, y0=y0)


ACT_TANH, ACT_SOFTPLUS = 0, 1


def lstm_theta_count(u, d):
    return 4 * u * d + 4 * u * u + 4 * u


def lstm_workload(name, seed, B, T, units, d, tol=1e-4, max_iter=50):
    """LSTM cell with `units` units (state (h | c) of 2 units entries; Workload.n holds the units): weights and biases
    ~ N(0, 1/units), x ~ N(0,1), y0 = 0."""
    rng = np.random.default_rng(seed)
    theta = _normal(rng, lstm_theta_count(units, d), 1.0 / np.sqrt(units))
    x = _normal(rng, (B, T, d), 1.0)
    y0 = np.zeros((B, 2 * units), dtype=np.float32)
    return Workload(name=name, cell=CELL_LSTM, B=B, T=T, n=units, d=d, tol=tol, max_iter=max_iter, theta=theta, x=x, y0=y0)


def lem_workload(name, seed, B, T, units, d, dt=1.0, tol=1e-4, max_iter=50):
    """LEM cell with `units` units (state (y | z) of 2 units entries; Workload.n holds the units, Workload.t1 the
    cell's step dt): weights and biases ~ N(0, 1/units), x ~ N(0,1), y0 = 0."""
    rng = np.random.default_rng(seed)
    theta = _normal(rng, lstm_theta_count(units, d), 1.0 / np.sqrt(units))
    x = _normal(rng, (B, T, d), 1.0)
    y0 = np.zeros((B, 2 * units), dtype=np.float32)
    return Workload(name=name, cell=CELL_LEM, B=B, T=T, n=units, d=d, t1=float(dt), tol=tol, max_iter=max_iter, theta=theta,
                    x=x, y0=y0)


def mh_gru_workload(name, seed, B, T, n, d, H, K, tol=1e-4, max_iter=50):
    """Multi-head GRU with strides: H heads of n channels, head h with its own parameters (~ N(0, 1/n)), its own
    d input channels (x [B,T,H,d] ~ N(0,1)) and stride 2^(h mod K); y0 [B,H,n] = 0."""
    rng = np.random.default_rng(seed)
    theta = _normal(rng, (H, gru_theta_count(n, d)), 1.0 / np.sqrt(n))
    x = _normal(rng, (B, T, H, d), 1.0)
    y0 = np.zeros((B, H, n), dtype=np.float32)
    return Workload(name=name, cell=CELL_GRU, B=B, T=T, n=n, d=d, heads=H, stride_levels=K, tol=tol, max_iter=max_iter,
                    theta=theta, x=x, y0=y0)


def mlp_ode_workload(name, seed, B, T, n, width, nhid, t0, t1, tol=1e-4, max_iter=50, act=ACT_TANH):
    """dy/dt = MLP(y): weights and biases ~ N(0, 1/width); y0 ~ N(0,1); uniform grid of T points."""
    rng = np.random.default_rng(seed)
    theta = _normal(rng, mlp_theta_count(n, width, nhid), 1.0 / np.sqrt(width))
    y0 = _normal(rng, (B, n), 1.0)
    return Workload(name=name, cell=CELL_MLP_ODE, B=B, T=T, n=n, mlp_width=width, mlp_hidden_layers=nhid,
                    mlp_activation=act, t0=t0, t1=t1, tol=tol, max_iter=max_iter, theta=theta, y0=y0)


def config(k, rep=0, T=None, B=None):
    """The k-th benchmark configuration (1-based), seed 1000*k + rep.  T and B can be
    overridden to get a reduced copy of the same recipe for quick tests."""
    seed = 1000 * k + rep
    if k == 1:
        return gru_workload("cfg1_gru_n2_T1k_B1", seed, B or 1, T or 1000, 2, 2, tol=1e-6, max_iter=50)
    if k == 2:
        return gru_workload("cfg2_gru_n8_T10k_B16", seed, B or 16, T or 10000, 8, 4)
    if k == 3:
        return gru_workload("cfg3_gru_n32_T100k_B16", seed, B or 16, T or 100000, 32, 8, x_kind="sinusoid")
    if k == 4:
        w = gru_workload("cfg4_gru_n16_T17984_B32_train", seed, B or 32, T or 17984, 16, 6)
        rng = np.random.default_rng(seed + 500000)
        w.extra["W_o"] = _normal(rng, (5, 16), 0.25)     # N(0, 1/16)
        w.extra["b_o"] = _normal(rng, (5,), 0.25)
        w.extra["labels"] = rng.integers(0, 5, size=w.B)
        return w
    if k == 5:
        return mlp_ode_workload("cfg5_mlpode_n8_T100k_B8", seed, B or 8, T or 100000, 8, 32, 2, 0.0, 10.0)
    raise ValueError(k)


def scan_inputs(seed, B, T, n, dtype=np.float32, contraction=0.9):
    """Random affine pairs for scan-only tests: A = contraction * (random matrix scaled to unit
    spectral norm), b ~ N(0,1), y0 ~ N(0,1).  Products of the A stay bounded."""
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((B, T, n, n))
    A *= contraction / np.linalg.norm(A, ord=2, axis=(-2, -1), keepdims=True)
    b = rng.standard_normal((B, T, n))
    y0 = rng.standard_normal((B, n))
    return A.astype(dtype), b.astype(dtype), y0.astype(dtype)
