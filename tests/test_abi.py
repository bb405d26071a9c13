"""Host-side checks of the C-ABI library: it loads, exports every symbol the header declares, and its
argument validation works without a GPU.  No compute calls."""
import ctypes
import os
import re

import pytest

from paper_2309_12252_amd import deer

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "deer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(deer_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = deer.load_library()
    names = declared_symbols()
    assert set(names) == set(deer.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_theta_count_and_validation_on_host():
    gru = deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, 16, 10000, 8, d=4)
    assert deer.theta_count(gru) == 3 * 8 * 4 + 3 * 8 * 8 + 4 * 8
    mlp = deer.make_config(deer.DEER_CELL_MLP_ODE, deer.DEER_F32, 8, 100000, 8, mlp_width=32,
                           mlp_hidden_layers=2, t0=0.0, t1=10.0)
    assert deer.theta_count(mlp) == 32 * 8 + 32 + 32 * 32 + 32 + 8 * 32 + 8
    assert deer.workspace_bytes(mlp) > 2 * 8 * 100000 * 8 * 8 * 4 - 8 * 64 * 4
    with pytest.raises(deer.DeerError) as e:
        deer.workspace_bytes(deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, 1, 10, 65, d=2))
    assert e.value.status == deer.DEER_ERR_UNSUPPORTED
    with pytest.raises(deer.DeerError) as e:   # state sizes above 32 run in fp32 only
        deer.workspace_bytes(deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F64, 1, 10, 64, d=2))
    assert e.value.status == deer.DEER_ERR_UNSUPPORTED
    assert deer.workspace_bytes(deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, 1, 10, 64, d=2)) > 0
    with pytest.raises(deer.DeerError) as e:
        deer.workspace_bytes(deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, 0, 10, 4, d=2))
    assert e.value.status == deer.DEER_ERR_INVALID_ARG
    with pytest.raises(deer.DeerError) as e:
        deer.workspace_bytes(deer.make_config(deer.DEER_CELL_MLP_ODE, deer.DEER_F32, 1, 10, 8, mlp_width=32,
                                              mlp_hidden_layers=6, t0=0.0, t1=1.0))
    assert e.value.status == deer.DEER_ERR_UNSUPPORTED
    # the two-body network's shape (App. B.2): five hidden layers of width 64, softplus
    hnn = deer.make_config(deer.DEER_CELL_MLP_ODE, deer.DEER_F32, 4, 10000, 8, mlp_width=64, mlp_hidden_layers=5,
                           t0=0.0, t1=10.0, mlp_activation=deer.DEER_ACT_SOFTPLUS)
    assert deer.theta_count(hnn) == 64 * 8 + 64 + 4 * (64 * 64 + 64) + 8 * 64 + 8
    assert deer.workspace_bytes(hnn) > 0


def test_workspace_follows_the_plan(monkeypatch):
    # Sec. 3.5: the Jacobian stream is O(n^2 T) memory.  It is part of the workspace only where two kernels
    # exchange it; with the cell inside the scans the third benchmark configuration (6.55 GB of Jacobians, a
    # shape the paper's 16 GB device could not run: Table 4) needs well under 1 GB.
    for var in ("DEER_FUSED", "DEER_GRAD_FUSED"):
        monkeypatch.delenv(var, raising=False)
    cfg2 = deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, 16, 10000, 8, d=4)
    cfg3 = deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, 16, 100000, 32, d=8)
    jac2, jac3 = 16 * 10000 * 8 * 8 * 4, 16 * 100000 * 32 * 32 * 4
    assert deer.workspace_bytes(cfg2) < jac2
    assert deer.workspace_bytes(cfg3) < (1 << 30) < jac3
    # fp64 at n = 32 runs the cell kernel and the plain scan: the stream is there
    cfg3_64 = deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F64, 16, 100000, 32, d=8)
    assert deer.workspace_bytes(cfg3_64) > 2 * jac3
    # and so it is when a knob asks for the separate kernels in either direction
    for var in ("DEER_FUSED", "DEER_GRAD_FUSED"):
        monkeypatch.setenv(var, "0")
        assert deer.workspace_bytes(cfg2) > jac2 and deer.workspace_bytes(cfg3) > jac3
        monkeypatch.delenv(var)


def test_create_rejects_bad_arguments_without_touching_the_gpu():
    lib = deer.load_library()
    cfg = deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, 1, 10, 4, d=2)
    handle = ctypes.c_void_p(None)
    st = lib.deer_create(ctypes.byref(cfg), None, 1 << 20, None, ctypes.byref(handle))
    assert st == deer.DEER_ERR_WORKSPACE and not handle.value
    st = lib.deer_create(ctypes.byref(cfg), ctypes.c_void_p(256), 16, None, ctypes.byref(handle))
    assert st == deer.DEER_ERR_WORKSPACE and not handle.value
    assert b"workspace" in lib.deer_last_error(None)
    assert lib.deer_eval(None, None, None, None, None, 1e-4, 1, None, None, None, None) == deer.DEER_ERR_INVALID_ARG
