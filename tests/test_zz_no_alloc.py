"""deer_linrec_solve_static (the scan without a workspace: its scratch is a static device array inside the
library) against deer_linrec_solve on the same inputs, called through the C ABI twice in a row, the second time
on a smaller input, so that whatever the first call left in the array must not leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2309_12252_amd import deer, inputs
from helpers import DEV, TOL_ABS, dev, host

pytestmark = pytest.mark.gpu


def existing(A, b, y0, dtype, reverse):
    B, T, n, _ = A.shape
    ctx = deer.DeerContext(deer.make_config(deer.DEER_CELL_GRU, dtype, B, T, n, d=1), device=DEV)
    try:
        y = ctx.linrec_solve(A, b, y0, reverse=reverse)
        torch.cuda.synchronize()
        return host(y)
    finally:
        ctx.close()


@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
@pytest.mark.parametrize("n", [2, 8, 32])
@pytest.mark.parametrize("reverse", [False, True])
def test_two_calls_in_a_row_second_one_smaller(n, dtype, reverse):
    lib = deer.load_library()
    shapes = [(3, 9000 if n < 32 else 2100), (2, 1300 if n < 32 else 333)]   # several tiles and a ragged tail, then fewer
    status = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    for k, (B, T) in enumerate(shapes):
        A, b, y0 = inputs.scan_inputs(600 + 10 * n + k, B, T, n)
        dA, db, dy0 = dev(A, dtype), dev(b, dtype), dev(y0, dtype)
        out = torch.full((B, T, n), float("nan"), dtype=dA.dtype, device=DEV)
        stream = torch.cuda.current_stream()
        st = lib.deer_linrec_solve_static(dtype, B, T, n, ctypes.c_void_p(dA.data_ptr()), ctypes.c_void_p(db.data_ptr()),
                                          ctypes.c_void_p(dy0.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                          1 if reverse else 0, ctypes.c_void_p(stream.cuda_stream),
                                          ctypes.c_void_p(status.data_ptr()))
        assert st == deer.DEER_OK, lib.deer_last_error(None)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        want = existing(dA, db, dy0, dtype, reverse)
        got = host(out)
        assert np.isfinite(got).all()
        assert np.abs(got - want).max() <= TOL_ABS[dtype], (n, dtype, reverse, B, T, np.abs(got - want).max())


def test_shapes_beyond_the_static_scratch_are_rejected():
    lib = deer.load_library()
    x = torch.zeros(16, dtype=torch.float32, device=DEV)
    p = ctypes.c_void_p(x.data_ptr())
    # n = 32: 1,600,000 positions publish 217 MB of words, the array holds 64 MiB; nothing is enqueued or touched
    st = lib.deer_linrec_solve_static(deer.DEER_F32, 16, 100000, 32, p, p, p, p, 0, None, None)
    assert st == deer.DEER_ERR_WORKSPACE and b"static scratch" in lib.deer_last_error(None)
    assert lib.deer_linrec_solve_static(deer.DEER_F32, 1, 10, 5, p, p, p, p, 0, None, None) == deer.DEER_ERR_UNSUPPORTED
    assert lib.deer_linrec_solve_static(deer.DEER_F32, 1, 10, 4, None, p, p, p, 0, None, None) == deer.DEER_ERR_INVALID_ARG
