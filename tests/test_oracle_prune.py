"""Pins of the oracle's parallel tree pruning (Sec. 3.2.3, Appendix A.1 and its generation-step figure)."""
import itertools
import math

import numpy as np

import oracle
from conftest import read_golden
from helpers import all_parent_arrays, reach_closure


def _rand(B, T, d, V, seed):
    rng = np.random.default_rng(seed)
    h = rng.standard_normal((B, T, d)).astype(np.float32)
    W = rng.standard_normal((V, d)).astype(np.float32)
    parent = np.array([[-1] + [int(rng.integers(0, i)) for i in range(1, T)] for _ in range(B)], np.int32)
    tok = rng.integers(0, V, (B, T)).astype(np.int32)
    return h, W, tok, parent


def test_transition_probs_against_python_softmax():
    B, T, d, V = 2, 5, 3, 6
    h, W, tok, parent = _rand(B, T, d, V, 1)
    prob = oracle.transition_probs(h, W, tok, parent)
    for b in range(B):
        assert prob[b, 0] == 1.0
        for i in range(1, T):
            p = parent[b, i]
            z = [sum(float(h[b, p, e]) * float(W[v, e]) for e in range(d)) for v in range(V)]
            den = sum(math.exp(x) for x in z)
            assert abs(prob[b, i] - math.exp(z[tok[b, i]]) / den) <= 1e-14


def test_children_with_every_token_sum_to_one():
    # a root with one child per vocabulary token: the transition probabilities are a distribution
    d, V = 4, 9
    rng = np.random.default_rng(2)
    T = V + 1
    h = rng.standard_normal((1, T, d)).astype(np.float32)
    W = rng.standard_normal((V, d)).astype(np.float32)
    tok = np.array([[0] + list(range(V))], np.int32)
    parent = np.array([[-1] + [0] * V], np.int32)
    prob = oracle.transition_probs(h, W, tok, parent)
    assert abs(prob[0, 1:].sum() - 1.0) <= 1e-14


def test_zero_head_is_uniform_and_a_common_shift_changes_nothing():
    B, T, d, V = 1, 4, 5, 7
    h, W, tok, parent = _rand(B, T, d, V, 3)
    prob = oracle.transition_probs(h, np.zeros_like(W), tok, parent)
    np.testing.assert_allclose(prob[0, 1:], 1.0 / V, rtol=1e-15)
    # adding one vector to every row of W adds the same number to all logits of a row
    W = (np.round(W * 8) / 8).astype(np.float32)             # multiples of 1/8: the shift below is exact
    W2 = (W.astype(np.float64) + np.arange(d)[None, :] / 8.0).astype(np.float32)
    Wd = W2.astype(np.float64) - W.astype(np.float64)
    assert np.abs(Wd - Wd[0]).max() == 0.0       # exactly the same shift on every row
    np.testing.assert_allclose(oracle.transition_probs(h, W2, tok, parent), oracle.transition_probs(h, W, tok, parent),
                               rtol=1e-12)


def test_the_parent_row_decides_not_the_childs():
    # changing the hidden state of a leaf changes no probability; changing the root's changes its children's
    B, T, d, V = 1, 4, 3, 5
    h, W, tok, _ = _rand(B, T, d, V, 4)
    parent = np.array([[-1, 0, 0, 1]], np.int32)
    base = oracle.transition_probs(h, W, tok, parent)
    h2 = h.copy()
    h2[0, 3] += 1.0          # node 3 is a leaf
    np.testing.assert_array_equal(oracle.transition_probs(h2, W, tok, parent), base)
    h3 = h.copy()
    h3[0, 0] += 1.0
    other = oracle.transition_probs(h3, W, tok, parent)
    assert other[0, 1] != base[0, 1] and other[0, 2] != base[0, 2] and other[0, 3] == base[0, 3]


def test_token_outside_the_vocabulary_has_probability_zero():
    h, W, tok, parent = _rand(1, 3, 2, 4, 5)
    tok[0, 1], tok[0, 2] = -1, 4
    prob = oracle.transition_probs(h, W, tok, parent)
    assert prob[0, 1] == 0.0 and prob[0, 2] == 0.0


def test_lse_against_numpy_and_its_relation_to_the_probabilities():
    B, T, d, V = 1, 4, 6, 11
    h, W, tok, parent = _rand(B, T, d, V, 6)
    z = h[0].astype(np.float64) @ W.astype(np.float64).T
    lse = oracle.lm_head_lse(h[0], W)
    np.testing.assert_allclose(lse, np.logaddexp.reduce(z, axis=1), rtol=1e-14)
    prob = oracle.transition_probs(h, W, tok, parent)
    for i in range(1, T):
        p = parent[0, i]
        assert abs(prob[0, i] - math.exp(z[p, tok[0, i]] - lse[p])) <= 1e-14
    # large logits do not overflow
    big = oracle.lm_head_lse(1000.0 * h[0], W)
    assert np.isfinite(big).all()


def test_prune_figure_example():
    g = read_golden("tree_draft_figure.txt")
    T = len(g["parent"])
    # the transition from the root ("parameter") to m2 ("compare") is below the threshold, all others above
    prob = np.full((1, T), 0.5, np.float32)
    prob[0, 2] = 0.01
    out = oracle.tree_prune([g["tok"]], [g["parent"]], prob, 0.1)
    n = len(g["pruned_parent"])
    assert out["n_nodes"][0] == n
    assert out["keep"][0].tolist() == [1, 1, 0, 1, 1, 0, 0]          # m2, m5, m6 are pruned
    assert out["parent"][0, :n].tolist() == g["pruned_parent"]
    assert out["tok"][0, :n].tolist() == g["pruned_tok"]
    assert out["old_index"][0].tolist() == [0, 1, 3, 4, -1, -1, -1]
    assert (out["tok"][0, n:] == -1).all() and (out["parent"][0, n:] == 0).all()
    # verification of the padded pruned tree gives the figure's result: padding is never accepted
    a = np.array([g["pruned_main_argmax"] + [99] * (T - n)], np.int32)
    ver = oracle.tree_verify(out["tok"], out["parent"], a, 2)
    assert ver["n_accept"][0] == g["pruned_n_accept"][0] and ver["last"][0] == g["pruned_last"][0]
    assert ver["bonus"][0] == g["pruned_bonus"][0]


def test_prune_all_small_trees_against_the_path_statement():
    # a node stays iff every edge on its root path passes; kept nodes keep their order; parents follow
    for T in range(1, 6):
        for parent in all_parent_arrays(T):
            anc = reach_closure(parent)
            for passes in itertools.product([0, 1], repeat=T - 1):
                prob = np.array([[1.0] + [0.75 if x else 0.25 for x in passes]], np.float32)
                tok = np.arange(100, 100 + T, dtype=np.int32)[None]
                out = oracle.tree_prune(tok, [list(parent)], prob, 0.5)
                want = [all(a == 0 or passes[a - 1] for a in anc[i]) for i in range(T)]
                assert out["keep"][0].tolist() == [int(x) for x in want]
                kept = [i for i in range(T) if want[i]]
                n = len(kept)
                assert out["n_nodes"][0] == n and out["old_index"][0, :n].tolist() == kept
                assert out["tok"][0, :n].tolist() == [100 + i for i in kept]
                for j in range(1, n):
                    assert kept[out["parent"][0, j]] == parent[kept[j]] and out["parent"][0, j] < j
                assert out["parent"][0, 0] == -1
                assert (out["old_index"][0, n:] == -1).all() and (out["tok"][0, n:] == -1).all()


def test_probability_equal_to_the_threshold_is_kept():
    out = oracle.tree_prune([[1, 2, 3]], [[-1, 0, 0]], np.array([[1.0, 0.25, np.nextafter(np.float32(0.25), np.float32(0))]], np.float32), 0.25)
    assert out["keep"][0].tolist() == [1, 1, 0]
