"""Pins of the oracle's greedy tree verification (a4) and tree drafting (a5)."""
import numpy as np
import pytest

import oracle
from helpers import all_parent_arrays, enumerate_paths_verify, reach_closure
from paper_2402_11131_amd import synth


def _verify(tok, parent, a, max_depth=None):
    tok, parent, a = (np.atleast_2d(np.asarray(x, np.int32)) for x in (tok, parent, a))
    if max_depth is None:
        max_depth = parent.shape[1] - 1
    return oracle.tree_verify(tok, parent, a, max_depth)


def test_figure_example(golden):
    g = golden("tree_draft_figure.txt")
    r = _verify(g["tok"], g["parent"], g["main_argmax"], max_depth=g["gamma"][0])
    assert r["n_accept"][0] == g["n_accept"][0]
    assert r["last"][0] == g["last"][0]
    assert r["bonus"][0] == g["bonus"][0]
    assert r["path"][0].tolist()[:len(g["path"])] == g["path"]
    assert r["out_tokens"][0].tolist()[:len(g["emitted"])] == g["emitted"]
    assert r["out_tokens"][0].tolist()[len(g["emitted"]):] == [-1] * (g["gamma"][0] + 1 - len(g["emitted"]))
    # the pruned tree gives the same decision
    rp = _verify(g["pruned_tok"], g["pruned_parent"], g["pruned_main_argmax"], max_depth=g["gamma"][0])
    assert (rp["n_accept"][0], rp["last"][0], rp["bonus"][0]) == (
        g["pruned_n_accept"][0], g["pruned_last"][0], g["pruned_bonus"][0])
    # next tree: full (k,k) template filled from the streams of the last accepted node
    gamma, k, T = g["gamma"][0], g["k"][0], len(g["parent"])
    tp, tr, td = oracle.full_tree_template([k] * gamma)
    assert tp.tolist() == g["next_parent"]
    topk = np.full((1, T, gamma, k), -7, np.int32)
    topk[0, g["last"][0], 0] = g["stream1_m1"]
    topk[0, g["last"][0], 1] = g["stream2_m1"]
    nt, npar = oracle.tree_draft(topk, r["last"], r["bonus"], tp, tr)
    assert nt[0].tolist() == g["next_tok"]
    assert npar.tolist() == g["next_parent"]


@pytest.mark.parametrize("T", [1, 2, 3, 4, 5, 6, 7])
def test_exhaustive_path_enumeration(T):
    rng = synth.rng_for(100 + T)
    trees = list(all_parent_arrays(T))
    if len(trees) > 150:
        trees = [trees[i] for i in rng.choice(len(trees), 150, replace=False)]
    for parent in trees:
        for _ in range(6):
            alphabet = int(rng.integers(1, 4))
            tok = rng.integers(0, alphabet, T).tolist()
            a = rng.integers(0, alphabet, T).tolist()
            r = _verify(tok, parent, a)
            n_acc, last = enumerate_paths_verify(tok, parent, a)
            assert (r["n_accept"][0], r["last"][0]) == (n_acc, last)
            assert r["bonus"][0] == a[last]
            # invariants: path is the root path of `last`, every edge matches, and
            # no child of `last` matches (otherwise the path could be extended)
            path = [x for x in r["path"][0].tolist() if x >= 0]
            assert path[0] == 0 and path[-1] == last and len(path) == n_acc + 1
            assert set(path) == reach_closure(parent)[last]
            assert all(parent[c] == p and tok[c] == a[p] for p, c in zip(path[:-1], path[1:]))
            assert not any(parent[c] == last and tok[c] == a[last] for c in range(T))
            emitted = [x for x in r["out_tokens"][0].tolist() if x >= 0]
            assert emitted == [tok[c] for c in path[1:]] + [a[last]]


def test_chain_is_textbook_greedy_speculative_verification(golden):
    g = golden("tokens_per_pass.txt")
    gamma = g["gamma"][0]
    T = gamma + 1  # root + gamma draft tokens (k = 1)
    rng = synth.rng_for(5)
    for _ in range(200):
        tok = rng.integers(0, 3, T).tolist()
        a = rng.integers(0, 3, T).tolist()
        n = 0
        while n + 1 < T and tok[n + 1] == a[n]:   # accept while draft[i] == argmax[i-1]
            n += 1
        r = _verify(tok, synth.chain_tree(T), a, max_depth=gamma)
        assert r["n_accept"][0] == n and r["last"][0] == n and r["bonus"][0] == a[n]
        emitted = [x for x in r["out_tokens"][0].tolist() if x >= 0]
        assert 1 <= len(emitted) == n + 1 <= g["max_tokens_per_pass"][0]
    # all drafts accepted: gamma + 1 tokens in one pass
    a = [1] * T
    r = _verify([0] + [1] * gamma, synth.chain_tree(T), a, max_depth=gamma)
    assert r["n_accept"][0] == gamma and (r["out_tokens"][0] >= 0).sum() == g["max_tokens_per_pass"][0]


def test_batch_strides_and_depth_limit():
    parent = synth.make_trees(3, 4, 12, (3, 2, 2), 3)
    rng = synth.rng_for(8)
    tok = rng.integers(0, 2, parent.shape).astype(np.int32)
    a = rng.integers(0, 2, parent.shape).astype(np.int32)
    r = oracle.tree_verify(tok, parent, a, 3)
    for b in range(4):
        n_acc, last = enumerate_paths_verify(tok[b].tolist(), parent[b].tolist(), a[b].tolist())
        assert (r["n_accept"][b], r["last"][b], r["bonus"][b]) == (n_acc, last, a[b, last])
    # nodes deeper than max_depth are never accepted
    chain = synth.chain_tree(6)[None]
    r = oracle.tree_verify(np.ones((1, 6), np.int32), chain, np.ones((1, 6), np.int32), 2)
    assert r["n_accept"][0] == 2 and r["last"][0] == 2 and r["path"].shape == (1, 3)


def test_draft_template_and_tokens(golden):
    for gamma, k, nodes, _rows in golden("tree_size_closed_form.txt")[""]:
        if nodes > 64:
            continue
        tp, tr, td = oracle.full_tree_template([k] * gamma)
        assert len(tp) == nodes
        assert all(tp[i] < i for i in range(1, nodes)) and tp[0] == -1
        # depth recomputed independently; level sizes k^j; level-by-level numbering
        closure = reach_closure(tp.tolist())
        assert [len(c) - 1 for c in closure] == td.tolist()
        assert [int((td == j).sum()) for j in range(gamma + 1)] == [k ** j for j in range(gamma + 1)]
        assert np.all(np.diff(td) >= 0)
        for p in range(nodes):
            kids = [i for i in range(nodes) if tp[i] == p]
            assert len(kids) in (0, k) and [int(tr[i]) for i in kids] == list(range(len(kids)))
        # tokens
        rng = synth.rng_for(gamma * 10 + k)
        B, T, K = 3, 5, max(k, 2)
        topk = np.stack([np.stack([np.stack([rng.permutation(1000)[:K] for _ in range(gamma)])
                                   for _ in range(T)]) for _ in range(B)]).astype(np.int32)
        last = rng.integers(0, T, B).astype(np.int32)
        bonus = rng.integers(0, 1000, B).astype(np.int32)
        nt, npar = oracle.tree_draft(topk, last, bonus, tp, tr)
        assert np.array_equal(npar, tp)
        for b in range(B):
            assert nt[b, 0] == bonus[b]                                  # root = correction token
            for i in range(1, nodes):
                assert nt[b, i] == topk[b, last[b], td[i] - 1, tr[i]]    # level j <- stream j, rank r
            for p in range(nodes):
                kids = [i for i in range(nodes) if tp[i] == p]
                if kids:                                                 # k distinct tokens in rank order
                    assert nt[b, kids].tolist() == topk[b, last[b], td[kids[0]] - 1, :k].tolist()


def test_per_level_branching_and_invalid_template_entries():
    tp, tr, td = oracle.full_tree_template([4, 2, 1])
    assert len(tp) == 1 + 4 + 8 + 8
    # an entry deeper than gamma, or with rank >= K, yields -1
    topk = np.arange(2 * 3 * 2 * 2, dtype=np.int32).reshape(2, 3, 2, 2)
    tparent = np.array([-1, 0, 1, 2, 0], np.int32)   # depths 0 1 2 3 1 ; gamma = 2
    trank = np.array([0, 1, 0, 0, 2], np.int32)      # rank 2 >= K = 2
    nt, _ = oracle.tree_draft(topk, np.array([2, 0], np.int32), np.array([50, 60], np.int32), tparent, trank)
    assert nt.tolist() == [[50, topk[0, 2, 0, 1], topk[0, 2, 1, 0], -1, -1],
                           [60, topk[1, 0, 0, 1], topk[1, 0, 1, 0], -1, -1]]


def test_draft_then_verify_round_trip():
    # draft a tree, make the main stream agree along a chosen path, verify returns that path
    rng = synth.rng_for(77)
    gamma, k = 3, 2
    tp, tr, td = oracle.full_tree_template([k] * gamma)
    T2 = len(tp)
    for trial in range(20):
        topk = np.stack([rng.permutation(500)[:k] for _ in range(gamma)])[None, None].astype(np.int32)
        nt, npar = oracle.tree_draft(topk, np.zeros(1, np.int32), np.array([999], np.int32), tp, tr)
        leaf = int(rng.integers(T2))
        path = synth.root_path(npar, leaf)
        a = np.full((1, T2), -5, np.int32)
        for p, c in zip(path[:-1], path[1:]):
            a[0, p] = nt[0, c]
        r = oracle.tree_verify(nt, npar[None], a, gamma)
        assert r["last"][0] == leaf and r["n_accept"][0] == len(path) - 1
        assert [x for x in r["path"][0].tolist() if x >= 0] == path
