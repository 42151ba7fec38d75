"""Pins of the oracle's stream insertion, Eq. 3: S_{tj} = f(M_t) + P_j at the first multi-stream layer."""
import numpy as np

import oracle
import pytest

from helpers import rows_of
from paper_2402_11131_amd import synth


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


# ---------------------------------------------------------------- Eq. 3 followed by a dense map (n4 + n1)
def _sil_case(seed, B=2, T=5, gamma=3, d=12, V=7, with_f=True):
    rng = synth.rng_for(seed)
    M = rng.standard_normal((B, T, d)).astype(np.float32)
    P = rng.standard_normal((gamma, d)).astype(np.float32)
    W = rng.standard_normal((V, d)).astype(np.float32)
    fM = rng.standard_normal((B, T, d)).astype(np.float32) if with_f else None
    return M, P, W, fM


@pytest.mark.parametrize("with_f", [False, True])
def test_insert_then_project_equals_numpy_on_rows_built_by_indexing(with_f):
    M, P, W, fM = _sil_case(3, with_f=with_f)
    B, T, d = M.shape
    gamma = P.shape[0]
    Y = oracle.stream_insert_linear(M, P, W, fM)
    src = (fM if with_f else M).astype(np.float64)
    X = np.concatenate([M.astype(np.float64), (src[:, :, None, :] + P.astype(np.float64)[None, None]).reshape(B, T * gamma, d)], axis=1)
    assert np.allclose(Y, X @ W.astype(np.float64).T, rtol=1e-13, atol=1e-13)


def test_insert_then_project_is_linear_in_its_parts():
    # main rows are M.W^T, and a stream row minus its node's f(M).W^T is P_j.W^T whatever the node
    M, P, W, fM = _sil_case(4)
    B, T, d = M.shape
    gamma, V = P.shape[0], W.shape[0]
    Y = oracle.stream_insert_linear(M, P, W, fM)
    YM = oracle.linear_rows(M.reshape(B * T, d), W).reshape(B, T, V)
    YF = oracle.linear_rows(fM.reshape(B * T, d), W).reshape(B, T, V)
    YP = oracle.linear_rows(P, W)
    assert np.allclose(Y[:, :T], YM, rtol=1e-13, atol=1e-13)
    S = Y[:, T:].reshape(B, T, gamma, V)
    assert np.allclose(S - YF[:, :, None, :], np.broadcast_to(YP, (B, T, gamma, V)), rtol=1e-12, atol=1e-12)


def test_insert_then_project_special_cases():
    M, P, W, fM = _sil_case(5)
    B, T, d = M.shape
    gamma, V = P.shape[0], W.shape[0]
    # zero embeddings and identity f: every stream row equals its node's main row
    Y0 = oracle.stream_insert_linear(M, np.zeros_like(P), W)
    assert np.array_equal(Y0[:, T:].reshape(B, T, gamma, V), np.broadcast_to(Y0[:, :T, None, :], (B, T, gamma, V)))
    # identity weights: the rows of Eq. 3 themselves come out
    I = np.eye(d, dtype=np.float32)
    assert np.allclose(oracle.stream_insert_linear(M, P, I, fM), oracle.stream_insert(M, P, fM), rtol=0, atol=1e-15)
    # a transposed W would not have W's shape: a non-square W with one hot row picks one feature of the rows
    W1 = np.zeros((3, d), np.float32)
    W1[1, 4] = 2.0
    Y1 = oracle.stream_insert_linear(M, P, W1, fM)
    assert np.array_equal(Y1[..., 0], np.zeros_like(Y1[..., 0])) and np.allclose(Y1[..., 1], 2.0 * oracle.stream_insert(M, P, fM)[..., 4])
