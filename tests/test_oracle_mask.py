"""Pins of the oracle's mask construction (a1): Eq. 1, Eq. 2, Eq. 4 and the
appendix attention-mask figure."""
import numpy as np
import pytest

import oracle
from helpers import all_parent_arrays, reach_closure, rows_of, visible_new_keys
from paper_2402_11131_amd import synth


def test_mask_figure_example(golden):
    g = golden("attn_mask_figure.txt")
    parent = np.array([g["parent"]], np.int32)
    T = parent.shape[1]
    mask, anc, depth = oracle.build_mask(parent, gamma=0)
    for i in range(T):
        want = set(g["visible %d" % i])
        got = set(np.nonzero(mask[0, i])[0].tolist())
        assert got == want
        assert int(anc[0, i]) == sum(1 << a for a in want)
    # the replicated token sees its own branch only
    assert mask[0, 3, 2] == 0 and mask[0, 4, 1] == 0 and mask[0, 3, 4] == 0 and mask[0, 4, 3] == 0
    assert depth[0].tolist() == [0, 1, 1, 2, 2]


def test_chain_without_streams_is_causal():
    for T in (1, 2, 7, 64):
        mask, anc, depth = oracle.build_mask(synth.chain_tree(T)[None], gamma=0)
        assert np.array_equal(mask[0], np.tril(np.ones((T, T), np.uint8)))
        assert depth[0].tolist() == list(range(T))
        assert [int(a) for a in anc[0]] == [(1 << (i + 1)) - 1 for i in range(T)]


@pytest.mark.parametrize("flags", [0, oracle.EXCLUDE_SELF])
def test_row_popcount_closed_form(flags):
    # row (i,j) sees depth[i]+1 main keys and j own streams (j-1 without self)
    for seed in range(5):
        parent = synth.make_trees(seed, 3, 16, (4, 2, 2), 3)
        gamma = 4
        mask, anc, depth = oracle.build_mask(parent, gamma, flags)
        for b in range(3):
            for r, (i, j) in enumerate(rows_of(16, gamma)):
                own = j if not flags else max(j - 1, 0)
                assert mask[b, r].sum() == depth[b, i] + 1 + own
                if j == 0:
                    assert mask[b, r, 16:].sum() == 0  # main rows never see stream keys


@pytest.mark.parametrize("T", [1, 2, 3, 4, 5, 6])
def test_every_small_tree_against_closure(T):
    gamma = 2
    for parent in all_parent_arrays(T):
        for flags in (0, oracle.EXCLUDE_SELF):
            mask, anc, depth = oracle.build_mask(np.array([parent], np.int32), gamma, flags)
            vis = visible_new_keys(parent, gamma, exclude_self=bool(flags))
            closure = reach_closure(parent)
            for r in range(T * (1 + gamma)):
                assert set(np.nonzero(mask[0, r])[0].tolist()) == vis[r]
            for i in range(T):
                assert int(anc[0, i]) == sum(1 << a for a in closure[i])
                assert depth[0, i] == len(closure[i]) - 1


def test_full_tree_sizes(golden):
    for gamma, k, nodes, rows in golden("tree_size_closed_form.txt")[""]:
        parent, rank, depth = oracle.full_tree_template([k] * gamma)
        assert len(parent) == nodes == 1 + sum(k ** g for g in range(1, gamma + 1))
        mask, _, _ = oracle.build_mask(parent[None], gamma)
        assert mask.shape == (1, rows, rows) and rows == (1 + gamma) * nodes


def test_bad_parent_entries_are_clamped():
    # node 0 is always the root; an out-of-range parent of i > 0 counts as 0
    bad = np.array([[5, -1, 7, 1]], np.int32)
    good = np.array([[-1, 0, 0, 1]], np.int32)
    for x, y in zip(oracle.build_mask(bad, 1), oracle.build_mask(good, 1)):
        assert np.array_equal(x, y)
