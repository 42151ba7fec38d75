"""Pins of the oracle's dense projection y = x . W^T (Sec. 3.1: H.W^Q, H.W^K, H.W^V and the feed-forward maps)."""
from fractions import Fraction

import numpy as np

import oracle


def test_small_integers_exact_against_python_loops():
    rng = np.random.default_rng(5)
    N, d, V = 3, 5, 4
    x = rng.integers(-9, 10, (N, d)).astype(np.float32)
    W = rng.integers(-9, 10, (V, d)).astype(np.float32)
    y = oracle.linear_rows(x, W)
    assert y.shape == (N, V)
    for n in range(N):
        for v in range(V):
            want = sum(Fraction(int(x[n, e])) * Fraction(int(W[v, e])) for e in range(d))
            assert Fraction(float(y[n, v])) == want


def test_non_square_against_numpy_matmul():
    # N, d, V all different: a transposed operand or swapped extent cannot pass
    rng = np.random.default_rng(6)
    x = rng.standard_normal((7, 48)).astype(np.float32)
    W = rng.standard_normal((13, 48)).astype(np.float32)
    want = x.astype(np.float64) @ W.astype(np.float64).T
    np.testing.assert_allclose(oracle.linear_rows(x, W), want, rtol=1e-13, atol=1e-13)


def test_identity_and_one_hot_rows_of_w():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((5, 16)).astype(np.float32)
    np.testing.assert_array_equal(oracle.linear_rows(x, np.eye(16, dtype=np.float32)), x.astype(np.float64))
    W = np.zeros((3, 16), np.float32)
    W[0, 4] = 1.0
    W[1, 15] = -2.0
    y = oracle.linear_rows(x, W)
    np.testing.assert_array_equal(y[:, 0], x[:, 4].astype(np.float64))
    np.testing.assert_array_equal(y[:, 1], -2.0 * x[:, 15].astype(np.float64))
    np.testing.assert_array_equal(y[:, 2], 0.0)


def test_scores_of_attention_are_projections_composed():
    # q.k of projected rows equals x (Wq^T Wk) x'^T computed directly
    rng = np.random.default_rng(8)
    x = rng.integers(-3, 4, (4, 6)).astype(np.float32)
    Wq = rng.integers(-3, 4, (5, 6)).astype(np.float32)
    Wk = rng.integers(-3, 4, (5, 6)).astype(np.float32)
    q, k = oracle.linear_rows(x, Wq), oracle.linear_rows(x, Wk)
    direct = x.astype(np.float64) @ (Wq.astype(np.float64).T @ Wk.astype(np.float64)) @ x.astype(np.float64).T
    np.testing.assert_array_equal(q @ k.T, direct)


def test_empty():
    assert oracle.linear_rows(np.zeros((0, 8), np.float32), np.zeros((3, 8), np.float32)).shape == (0, 3)
