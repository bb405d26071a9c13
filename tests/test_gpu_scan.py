"""GPU parity of the inverse linear operator (blocked associative scan) against the oracle's serial
solver, element by element, on random contractive affine pairs."""
import numpy as np
import pytest

import oracle
from paper_2309_12252_amd import deer, inputs
from helpers import DEV, TOL_ABS, NP_DTYPE, dev, host, dual_serial

pytestmark = pytest.mark.gpu

# lengths span empty-ish, one lane, one wavefront, tile edges and several tiles with a ragged tail
SHAPES = [(1, 1), (1, 2), (1, 63), (2, 64), (1, 65), (3, 511), (1, 512), (2, 513), (3, 1537), (1, 6000)]


def run_case(n, B, T, dtype, reverse, seed):
    A, b, y0 = inputs.scan_inputs(seed, B, T, n, dtype=NP_DTYPE[dtype])
    cfg = deer.make_config(deer.DEER_CELL_GRU, dtype, B, T, n, d=1)
    ctx = deer.DeerContext(cfg, device=DEV)
    try:
        y = host(ctx.linrec_solve(dev(A, dtype), dev(b, dtype), None if reverse else dev(y0, dtype),
                                  reverse=reverse))
    finally:
        ctx.close()
    for s in range(B):
        want = dual_serial(A[s], b[s]) if reverse else oracle.linrec_serial(A[s], b[s], y0[s])
        err = np.abs(y[s] - want).max()
        assert err <= TOL_ABS[dtype], (n, B, T, dtype, reverse, s, err)


@pytest.mark.parametrize("n", [1, 2, 4, 8, 16, 32])
@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
def test_forward_scan_matches_serial_solve(n, dtype):
    for k, (B, T) in enumerate(SHAPES):
        run_case(n, B, T, dtype, False, 100 * n + k)


@pytest.mark.parametrize("n", [1, 2, 4, 8, 16, 32])
@pytest.mark.parametrize("dtype", [deer.DEER_F32, deer.DEER_F64])
def test_dual_scan_matches_serial_solve(n, dtype):
    for k, (B, T) in enumerate(SHAPES):
        run_case(n, B, T, dtype, True, 200 * n + k)


@pytest.mark.parametrize("reverse", [False, True])
def test_scan_of_64_by_64_matrices(reverse):
    # the largest state size of the paper's speed table (Sec. 4.1, Table 4); fp32 only
    for k, (B, T) in enumerate(SHAPES + [(2, 3000)]):
        run_case(64, B, T, deer.DEER_F32, reverse, 6400 + k)


@pytest.mark.parametrize("n,B,T", [(8, 2, 50000), (2, 1, 300000), (16, 2, 20000), (32, 1, 10000)])
def test_many_tiles_per_sequence(n, B, T):
    # long chains of tiles: exercises the look-back window and the carry chain
    run_case(n, B, T, deer.DEER_F32, False, 7 * n)
    run_case(n, B, T, deer.DEER_F32, True, 9 * n)


@pytest.mark.parametrize("n,L", [(2, 8), (2, 16), (2, 32), (4, 8), (4, 16), (4, 24), (8, 16)])
def test_tile_shapes_of_the_small_state_scan(n, L, monkeypatch):
    # positions per lane group through the knob; for n = 2 and 4 the longer runs take the loads that are staged
    # through LDS (tiles inside the sequence) next to the lane-per-row loads of the ragged last tile, and an odd
    # batch index puts a sequence at an address that is not a multiple of 16 bytes
    monkeypatch.setenv("DEER_SCAN_L", str(L))
    tile = 8 * (64 // n) * L
    for k, (B, T) in enumerate([(3, 2 * tile + 77), (2, tile), (1, 5 * tile - 1)]):
        run_case(n, B, T, deer.DEER_F32, False, 300 * n + L + k)
        run_case(n, B, T, deer.DEER_F32, True, 400 * n + L + k)


def test_identity_matrices_give_a_prefix_sum():
    n, B, T = 4, 2, 3000
    rng = np.random.default_rng(0)
    A = np.broadcast_to(np.eye(n, dtype=np.float64), (B, T, n, n)).copy()
    b = rng.integers(-3, 4, size=(B, T, n)).astype(np.float64)   # integers: sums are exact in fp32
    y0 = rng.integers(-3, 4, size=(B, n)).astype(np.float64)
    ctx = deer.DeerContext(deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, B, T, n, d=1), device=DEV)
    try:
        y = host(ctx.linrec_solve(dev(A, deer.DEER_F32), dev(b, deer.DEER_F32), dev(y0, deer.DEER_F32)))
    finally:
        ctx.close()
    assert np.array_equal(y, y0[:, None, :] + np.cumsum(b, axis=1))


def test_repeated_calls_on_one_context_agree():
    # flags and tickets from an earlier launch must not leak into the next one
    n, B, T = 8, 3, 5000
    A, b, y0 = inputs.scan_inputs(5, B, T, n)
    ctx = deer.DeerContext(deer.make_config(deer.DEER_CELL_GRU, deer.DEER_F32, B, T, n, d=1), device=DEV)
    try:
        dA, db, dy0 = dev(A, 0), dev(b, 0), dev(y0, 0)
        first = host(ctx.linrec_solve(dA, db, dy0))
        for _ in range(5):
            assert np.array_equal(host(ctx.linrec_solve(dA, db, dy0)), first)
        back = host(ctx.linrec_solve(dA, db, None, reverse=True))
        assert np.array_equal(host(ctx.linrec_solve(dA, db, dy0)), first)
        assert np.array_equal(host(ctx.linrec_solve(dA, db, None, reverse=True)), back)
    finally:
        ctx.close()
