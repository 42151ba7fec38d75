"""Pins of the oracle's LM head + top-k (a3)."""
import numpy as np

import oracle
from paper_2402_11131_amd import synth


def test_matches_matmul_and_stable_argsort():
    rng = synth.rng_for(21)
    N, d, V, K = 7, 48, 301, 5
    h = rng.standard_normal((N, d)).astype(np.float32)
    W = (0.02 * rng.standard_normal((V, d))).astype(np.float32)
    idx, val, z = oracle.lm_head_topk(h, W, K, want_logits=True)
    zr = h.astype(np.float64) @ W.astype(np.float64).T          # library matmul
    assert np.allclose(z, zr, rtol=1e-12, atol=1e-15)
    order = np.argsort(-z, axis=1, kind="stable")[:, :K]        # library stable sort
    assert np.array_equal(idx, order)
    assert np.array_equal(val, np.take_along_axis(z, order, 1))
    assert np.all(np.diff(val, axis=1) <= 0)


def test_tiny_brute_force():
    h = np.array([[1.0, 2.0], [0.5, -1.0]], np.float32)
    W = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0], [-1.0, -1.0]], np.float32)
    idx, val = oracle.lm_head_topk(h, W, 3)
    # row 0 logits: 1, 2, 3, -3 ; row 1 logits: .5, -1, -.5, .5
    assert idx.tolist() == [[2, 1, 0], [0, 3, 2]]
    assert val.tolist() == [[3.0, 2.0, 1.0], [0.5, 0.5, -0.5]]


def test_planted_maximum():
    rng = synth.rng_for(22)
    N, d, V = 5, 64, 500
    h = rng.standard_normal((N, d)).astype(np.float32)
    W = (0.02 * rng.standard_normal((V, d))).astype(np.float32)
    want = [17, 499, 0, 250, 3]
    # one planted row per query: W[v] = c*h[n] makes z[n,v] = c*|h[n]|^2 the largest by far
    W2 = W.copy()
    for n, v in enumerate(want):
        W2[v] = 5.0 * h[n] / np.sqrt(d)
    idx, _ = oracle.lm_head_topk(h, W2, 1)
    # rows whose planted direction correlates with another row's h could clash only by chance
    assert idx[:, 0].tolist() == want


def test_ties_go_to_the_lower_index():
    rng = synth.rng_for(23)
    h = rng.standard_normal((3, 16)).astype(np.float32)
    W = rng.standard_normal((40, 16)).astype(np.float32)
    big = 10.0 * h[1] / 4
    W[7] = W[12] = W[31] = big          # three identical rows: exact ties
    idx, val = oracle.lm_head_topk(h, W, 4)
    assert idx[1, :3].tolist() == [7, 12, 31]
    assert val[1, 0] == val[1, 1] == val[1, 2] > val[1, 3]
