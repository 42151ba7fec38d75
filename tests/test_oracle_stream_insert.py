"""Pins of the oracle's stream insertion, Eq. 3: S_{tj} = f(M_t) + P_j at the first multi-stream layer."""
import numpy as np

import oracle
from helpers import rows_of


def _rand(B, T, gamma, d, seed):
    rng = np.random.default_rng(seed)
    M = rng.integers(-50, 51, (B, T, d)).astype(np.float32)
    P = rng.integers(-50, 51, (gamma, d)).astype(np.float32)
    return M, P


def test_every_row_against_the_row_order_statement():
    B, T, gamma, d = 2, 5, 3, 4
    M, P = _rand(B, T, gamma, d, 1)
    X = oracle.stream_insert(M, P)
    assert X.shape == (B, T * (1 + gamma), d)
    for b in range(B):
        for r, (i, j) in enumerate(rows_of(T, gamma)):
            want = M[b, i].astype(np.float64) + (P[j - 1].astype(np.float64) if j else 0.0)
            np.testing.assert_array_equal(X[b, r], want)


def test_zero_embeddings_replicate_the_node_and_zero_states_give_the_embeddings():
    B, T, gamma, d = 1, 4, 2, 6
    M, P = _rand(B, T, gamma, d, 2)
    X = oracle.stream_insert(M, np.zeros_like(P))
    for r, (i, j) in enumerate(rows_of(T, gamma)):
        np.testing.assert_array_equal(X[0, r], M[0, i])
    X = oracle.stream_insert(np.zeros_like(M), P)
    for r, (i, j) in enumerate(rows_of(T, gamma)):
        np.testing.assert_array_equal(X[0, r], P[j - 1] if j else 0.0)


def test_transformed_states_feed_the_streams_only():
    # f(M) given: main rows keep M, stream rows take f(M) + P_j
    B, T, gamma, d = 2, 3, 2, 5
    M, P = _rand(B, T, gamma, d, 3)
    fM = 2.0 * M + 1.0
    X = oracle.stream_insert(M, P, fM=fM)
    for b in range(B):
        for r, (i, j) in enumerate(rows_of(T, gamma)):
            want = M[b, i] if j == 0 else fM[b, i].astype(np.float64) + P[j - 1]
            np.testing.assert_array_equal(X[b, r], want)
    # the identity written out as f equals the default
    np.testing.assert_array_equal(oracle.stream_insert(M, P, fM=M), oracle.stream_insert(M, P))


def test_low_rank_f_composes_with_the_projection():
    # f of rank eta as two projections (d -> eta -> d): stream rows are M.A^T.B^T + P_j
    rng = np.random.default_rng(4)
    B, T, gamma, d, eta = 1, 3, 2, 6, 2
    M, P = _rand(B, T, gamma, d, 4)
    A = rng.integers(-2, 3, (eta, d)).astype(np.float32)
    Bm = rng.integers(-2, 3, (d, eta)).astype(np.float32)
    fM = oracle.linear_rows(oracle.linear_rows(M.reshape(-1, d), A).astype(np.float32), Bm).astype(np.float32).reshape(B, T, d)
    X = oracle.stream_insert(M, P, fM=fM)
    direct = M[0].astype(np.float64) @ A.T.astype(np.float64) @ Bm.T.astype(np.float64)
    for r, (i, j) in enumerate(rows_of(T, gamma)):
        if j:
            np.testing.assert_array_equal(X[0, r], direct[i] + P[j - 1])


def test_gamma_zero_and_empty_batch():
    M = np.ones((2, 3, 4), np.float32)
    X = oracle.stream_insert(M, np.zeros((0, 4), np.float32))
    np.testing.assert_array_equal(X, M)
    assert oracle.stream_insert(np.zeros((0, 3, 4), np.float32), np.zeros((2, 4), np.float32)).shape == (0, 9, 4)
