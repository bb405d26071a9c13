"""Pins of the oracle's affine-pair operator and linear-recurrence solvers.  CPU only."""
import numpy as np
import pytest

import oracle
from paper_2309_12252_amd import inputs


def rand_pairs(seed, T, n):
    A, b, y0 = inputs.scan_inputs(seed, 1, T, n, dtype=np.float64)
    return A[0], b[0], y0[0]


@pytest.mark.parametrize("n", [1, 2, 3, 8])
def test_combine_is_function_composition(n):
    # the pair (G|z) stands for the map y -> G y + z; combining earlier with later must give
    # the map "later after earlier" (Sec. 3.3 eq. 10)
    A, b, y0 = rand_pairs(n, 2, n)
    G, z = oracle.affine_combine(A[0], b[0], A[1], b[1])
    np.testing.assert_allclose(G @ y0 + z, A[1] @ (A[0] @ y0 + b[0]) + b[1], atol=1e-14)
    np.testing.assert_allclose(G, A[1] @ A[0], atol=1e-15)


@pytest.mark.parametrize("n", [1, 2, 4])
def test_combine_is_associative_not_commutative(n):
    A, b, _ = rand_pairs(10 + n, 3, n)
    c = [(A[i], b[i]) for i in range(3)]
    left = oracle.affine_combine(*oracle.affine_combine(*c[0], *c[1]), *c[2])
    right = oracle.affine_combine(*c[0], *oracle.affine_combine(*c[1], *c[2]))
    np.testing.assert_allclose(left[0], right[0], atol=1e-14)
    np.testing.assert_allclose(left[1], right[1], atol=1e-14)
    if n > 1:
        swapped = oracle.affine_combine(*c[1], *c[0])
        assert np.abs(swapped[0] - oracle.affine_combine(*c[0], *c[1])[0]).max() > 1e-3


@pytest.mark.parametrize("n,T", [(1, 1), (1, 50), (2, 33), (4, 100), (8, 64), (16, 20)])
def test_scan_and_serial_agree_with_brute_force(n, T):
    A, b, y0 = rand_pairs(100 * n + T, T, n)
    ys = oracle.linrec_serial(A, b, y0)
    ya = oracle.affine_scan(A, b, y0)
    # brute force: y_i = sum_{j<=i} (A_i ... A_{j+1}) b_j + (A_i ... A_1) y0 with numpy products
    want = np.empty((T, n))
    for i in range(T):
        acc = np.zeros(n)
        for j in range(i + 1):
            P = np.eye(n)
            for k in range(j + 1, i + 1):
                P = A[k] @ P
            acc += P @ b[j]
        P = np.eye(n)
        for k in range(i + 1):
            P = A[k] @ P
        want[i] = acc + P @ y0
    np.testing.assert_allclose(ys, want, atol=1e-12)
    np.testing.assert_allclose(ya, want, atol=1e-12)


def test_tree_shaped_reduction_matches_serial():
    # any parenthesisation of the operator gives the same total map
    n, T = 3, 37
    A, b, y0 = rand_pairs(5, T, n)
    rng = np.random.default_rng(0)
    items = [(A[i], b[i]) for i in range(T)]
    while len(items) > 1:
        k = rng.integers(0, len(items) - 1)
        items[k:k + 2] = [oracle.affine_combine(*items[k], *items[k + 1])]
    G, z = items[0]
    np.testing.assert_allclose(G @ y0 + z, oracle.linrec_serial(A, b, y0)[-1], atol=1e-12)


def test_scalar_constant_coefficients_closed_form():
    a, bb, y0, T = 0.9, 0.3, 2.0, 200
    y = oracle.linrec_serial(np.full((T, 1, 1), a), np.full((T, 1), bb), np.array([y0]))
    i = np.arange(1, T + 1)
    np.testing.assert_allclose(y[:, 0], a ** i * y0 + bb * (1 - a ** i) / (1 - a), rtol=1e-12)


def test_identity_matrices_give_a_cumulative_sum():
    n, T = 4, 300
    rng = np.random.default_rng(2)
    b = rng.standard_normal((T, n))
    y0 = rng.standard_normal(n)
    A = np.broadcast_to(np.eye(n), (T, n, n))
    np.testing.assert_allclose(oracle.affine_scan(A, b, y0), y0 + np.cumsum(b, axis=0), atol=1e-12)
    np.testing.assert_allclose(oracle.linrec_serial(A, b, y0), y0 + np.cumsum(b, axis=0), atol=1e-12)
