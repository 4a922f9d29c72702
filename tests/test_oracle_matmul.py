"""Pins for the oracle's three products (CPU only).

Each pin is something other than the oracle itself: hand-computed products,
closed forms, special cases with textbook answers, numpy's own fp64 matmul,
a pure-Python brute force on tiny inputs, and the adjoint identity that follows
from the first differentiation formula of Section 3.1.2.  Shapes are kept
non-square and the test functions non-symmetric, so a transposed operand, a
swapped index or a dropped term fails at least one of them.
"""
import os

import numpy as np
import pytest

from oracle import matmul as om


def _parse_matrix(txt):
    return np.array([[float(v) for v in row.split()] for row in txt.split(";")])


def test_textbook_products(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "textbook_products.txt")):
        if line.startswith("#") or not line.strip():
            continue
        A, B, C = (_parse_matrix(p) for p in line.split("|"))
        np.testing.assert_array_equal(om.forward(A, B), C)
        # the two backward forms on the same numbers: C B^T and A^T C by hand
        # are again ordinary products, so check them through transposes
        np.testing.assert_array_equal(om.backward_dx(C, B), om.forward(C, B.T.copy()))
        np.testing.assert_array_equal(om.backward_dw(A, C), om.forward(A.T.copy(), C))
        n += 1
    assert n == 2


def test_identity_ones_and_onehot():
    rng = np.random.default_rng(7)
    X = rng.integers(-9, 10, size=(5, 7)).astype(np.float64)
    np.testing.assert_array_equal(om.forward(X, np.eye(7)), X)          # W = I
    W = rng.integers(-9, 10, size=(7, 3)).astype(np.float64)
    Y = om.forward(np.ones((4, 7)), W)                                    # X = 1
    np.testing.assert_array_equal(Y, np.tile(W.sum(axis=0), (4, 1)))
    E = np.zeros((2, 7))
    E[0, 2] = 1.0
    E[1, 5] = -2.0                                                        # one-hot rows
    np.testing.assert_array_equal(om.forward(E, W), np.stack([W[2], -2.0 * W[5]]))
    # dX with dY one-hot picks a column of W (as a row of dX)
    G = np.zeros((2, 3))
    G[0, 1] = 1.0
    G[1, 2] = 3.0
    np.testing.assert_array_equal(om.backward_dx(G, W), np.stack([W[:, 1], 3.0 * W[:, 2]]))
    # dW with X one-hot picks rows of dY
    dY = rng.integers(-9, 10, size=(2, 3)).astype(np.float64)
    R = om.backward_dw(E, dY)
    expect = np.zeros((7, 3))
    expect[2] = dY[0]
    expect[5] = -2.0 * dY[1]
    np.testing.assert_array_equal(R, expect)


def test_polynomial_closed_forms():
    M, K, N = 6, 5, 4
    r = np.arange(M)[:, None].astype(np.float64)
    t = np.arange(K).astype(np.float64)
    c = np.arange(N)[None, :].astype(np.float64)
    s1 = lambda n: n * (n - 1) / 2.0                    # sum of 0..n-1
    s2 = lambda n: (n - 1) * n * (2 * n - 1) / 6.0      # sum of squares
    # Y[r,c] = sum_t (r + 2t) * t * (c+1) = (c+1) (r S1(K) + 2 S2(K))
    X = r + 2 * t[None, :]
    W = t[:, None] * (c + 1)
    np.testing.assert_array_equal(om.forward(X, W), (c + 1) * (r * s1(K) + 2 * s2(K)))
    # dX[r,t] = sum_c (r - c)(t + 3c) = r t N + 3 r S1(N) - t S1(N) - 3 S2(N)
    dY = r - c
    W2 = t[:, None] + 3 * c
    tt = t[None, :]
    np.testing.assert_array_equal(om.backward_dx(dY, W2),
                                  r * tt * N + 3 * r * s1(N) - tt * s1(N) - 3 * s2(N))
    # dW[t,c] = sum_r (r + 2t)(r - c) = S2(M) - c S1(M) + 2t S1(M) - 2 t c M
    tc = t[:, None]
    np.testing.assert_array_equal(om.backward_dw(X, dY),
                                  s2(M) - c * s1(M) + 2 * tc * s1(M) - 2 * tc * c * M)


def test_rank_one_closed_form():
    u = np.array([1.0, -2.0, 3.0])
    v = np.array([2.0, 0.0, 1.0, -1.0])
    w = np.array([4.0, 5.0])
    z = np.array([1.0, 1.0, -3.0, 2.0])
    # (u v^T)(z w^T) = (v.z) u w^T
    Y = om.forward(np.outer(u, v), np.outer(z, w))
    np.testing.assert_array_equal(Y, (v @ z) * np.outer(u, w))


@pytest.mark.parametrize("threads", [1, 3])
def test_against_numpy_matmul(threads):
    rng = np.random.default_rng(11)
    M, K, N = 37, 29, 23
    Xi = rng.integers(-4, 5, size=(M, K)).astype(np.float64)
    Wi = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    Gi = rng.integers(-4, 5, size=(M, N)).astype(np.float64)
    np.testing.assert_array_equal(om.forward(Xi, Wi, threads), Xi @ Wi)
    np.testing.assert_array_equal(om.backward_dx(Gi, Wi, threads), Gi @ Wi.T)
    np.testing.assert_array_equal(om.backward_dw(Xi, Gi, threads), Xi.T @ Gi)
    X = rng.uniform(-1, 1, size=(M, K))
    W = rng.uniform(-1, 1, size=(K, N))
    G = rng.uniform(-1, 1, size=(M, N))
    np.testing.assert_allclose(om.forward(X, W, threads), X @ W, rtol=0, atol=1e-13)
    np.testing.assert_allclose(om.backward_dx(G, W, threads), G @ W.T, rtol=0, atol=1e-13)
    np.testing.assert_allclose(om.backward_dw(X, G, threads), X.T @ G, rtol=0, atol=1e-13)


def test_pure_python_brute_force_tiny():
    rng = np.random.default_rng(3)
    M, K, N = 8, 8, 8
    X = rng.integers(-4, 5, size=(M, K)).tolist()
    W = rng.integers(-4, 5, size=(K, N)).tolist()
    G = rng.integers(-4, 5, size=(M, N)).tolist()
    Y = [[sum(X[r][t] * W[t][c] for t in range(K)) for c in range(N)] for r in range(M)]
    dX = [[sum(G[r][c] * W[t][c] for c in range(N)) for t in range(K)] for r in range(M)]
    dW = [[sum(X[r][t] * G[r][c] for r in range(M)) for c in range(N)] for t in range(K)]
    np.testing.assert_array_equal(om.forward(X, W), np.array(Y, dtype=np.float64))
    np.testing.assert_array_equal(om.backward_dx(G, W), np.array(dX, dtype=np.float64))
    np.testing.assert_array_equal(om.backward_dw(X, G), np.array(dW, dtype=np.float64))


def test_adjoint_identity_exact_on_integers():
    # <dY, XW> = <dY W^T, X> = <X^T dY, W>
    rng = np.random.default_rng(5)
    M, K, N = 12, 20, 9
    X = rng.integers(-4, 5, size=(M, K)).astype(np.float64)
    W = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    G = rng.integers(-4, 5, size=(M, N)).astype(np.float64)
    lhs = float(np.sum(G * om.forward(X, W)))
    assert lhs == float(np.sum(om.backward_dx(G, W) * X))
    assert lhs == float(np.sum(om.backward_dw(X, G) * W))


def test_sampled_entries_match_full_and_closed_form():
    rng = np.random.default_rng(9)
    M, K, N = 10, 6, 7
    X = rng.integers(-4, 5, size=(M, K)).astype(np.float64)
    W = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    G = rng.integers(-4, 5, size=(M, N)).astype(np.float64)
    rows = np.array([0, 9, 3, 3])
    cols = np.array([6, 0, 2, 5])
    np.testing.assert_array_equal(om.forward_at(X, W, rows, cols), (X @ W)[rows, cols])
    cols_k = np.array([5, 0, 2, 4])
    np.testing.assert_array_equal(om.backward_dx_at(G, W, rows, cols_k), (G @ W.T)[rows, cols_k])
    rows_k = np.array([0, 5, 3, 3])
    np.testing.assert_array_equal(om.backward_dw_at(X, G, rows_k, cols), (X.T @ G)[rows_k, cols])
    with pytest.raises(IndexError):
        om.forward_at(X, W, np.array([M]), np.array([0]))


def test_empty_and_degenerate_shapes():
    assert om.forward(np.zeros((0, 3)), np.zeros((3, 2))).shape == (0, 2)
    Y = om.forward(np.zeros((2, 0)), np.zeros((0, 3)))       # empty contraction -> zeros
    np.testing.assert_array_equal(Y, np.zeros((2, 3)))
    np.testing.assert_array_equal(om.backward_dw(np.zeros((0, 2)), np.zeros((0, 3))), np.zeros((2, 3)))
    with pytest.raises(ValueError):
        om.forward(np.zeros((2, 3)), np.zeros((4, 2)))
