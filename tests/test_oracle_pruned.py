"""Pins of the oracle's pruned-tree variants (Sec. 3.2.3: pruning removes nodes so that the step computes less).
The definition is "the step on the smaller tree"; the pins tie it to the T-node layout the kernels work in:
with nothing pruned it is the plain step; on a tree as ss_tree_prune leaves it (kept nodes first, padding nodes
hanging off the root) the kept rows equal the plain step's rows bit for bit (padding nodes are nobody's ancestors,
so no kept row sees them); what the padding rows hold does not matter; the kept-row list is the row-order statement."""
import numpy as np
import pytest

import oracle
from helpers import rows_of, to_np_f32
from paper_2402_11131_amd import synth


def _case(seed, B=3, T=9, gamma=2, L=(0, 37, 64)):
    cfg = synth.scaled(synth.CONFIGS["c1"], B=B, H=4, Hkv=2, D=64, T=T, gamma=gamma, page=16, L_min=80, L_max=80,
                       branching=(3, 2, 2), max_depth=3)
    inp = synth.make_msa_inputs(cfg, seed)
    a = {k: (to_np_f32(v) if hasattr(v, "dtype") and v.dtype.is_floating_point else (v.numpy() if hasattr(v, "numpy") else v))
         for k, v in inp.items()}
    a["seq_lens"] = np.array(L[:B], np.int32)
    return cfg, a


def _args(a, parent=None):
    return (a["q"], a["k_new"], a["v_new"], a["k_cache"], a["v_cache"], a["block_table"], a["seq_lens"],
            a["parent"] if parent is None else parent)


def test_live_rows_is_the_row_order_statement():
    for T, gamma in ((1, 0), (5, 0), (4, 3), (9, 2)):
        R = T * (1 + gamma)
        for n_nodes in ([T], [1], [T // 2 + 1, 1, T]):
            want = [b * R + r for b, n in enumerate(n_nodes) for r, (i, j) in enumerate(rows_of(T, gamma)) if i < n]
            assert oracle.live_rows(n_nodes, T, gamma).tolist() == sorted(want)


def test_nothing_pruned_is_the_plain_step():
    cfg, a = _case(1)
    full = oracle.msa_attention(*_args(a), cfg.gamma, a["scale"])
    assert np.array_equal(oracle.msa_attention_pruned(*_args(a), cfg.gamma, a["scale"], [cfg.T] * cfg.B), full)


@pytest.mark.parametrize("flags", [0, oracle.EXCLUDE_SELF])
def test_kept_rows_equal_the_plain_step_on_the_padded_tree(flags):
    cfg, a = _case(2)
    T, gamma = cfg.T, cfg.gamma
    n_nodes = np.array([4, 9, 1], np.int32)
    parent = a["parent"].copy()
    for b, n in enumerate(n_nodes):          # as pruning leaves it: kept nodes keep their (smaller-numbered) parents,
        parent[b, n:] = 0                    # padding nodes hang off the root
    pruned = oracle.msa_attention_pruned(*_args(a, parent), gamma, a["scale"], n_nodes, flags)
    plain = oracle.msa_attention(*_args(a, parent), gamma, a["scale"], flags)
    rows = oracle.live_rows(n_nodes, T, gamma)
    R = T * (1 + gamma)
    keep = np.zeros(cfg.B * R, bool)
    keep[rows] = True
    keep = keep.reshape(cfg.B, R)
    assert np.array_equal(pruned[keep], plain[keep])
    assert not pruned[~keep].any()
    # what the padding rows hold, and the parents of padding nodes, do not matter
    b = dict(a)
    for k in ("q", "k_new", "v_new"):
        x = a[k].copy()
        x[~keep] = np.nan
        b[k] = x
    wild = parent.copy()
    for bb, n in enumerate(n_nodes):
        wild[bb, n:] = np.arange(n, T) - 1   # a chain through the padding
    again = oracle.msa_attention_pruned(*_args(b, wild), gamma, a["scale"], n_nodes, flags)
    assert np.array_equal(again, pruned)


def test_live_variants_of_the_dense_maps():
    rng = synth.rng_for(9)
    x = rng.standard_normal((10, 6)).astype(np.float32)
    W = rng.standard_normal((8, 6)).astype(np.float32)
    rows = np.array([0, 3, 4, 9])
    y = oracle.linear_rows_live(x, W, rows)
    assert np.array_equal(y[rows], oracle.linear_rows(x, W)[rows]) and not np.delete(y, rows, axis=0).any()
    idx, val = oracle.lm_head_topk_live(x, W, 3, rows)
    full = oracle.lm_head_topk(x, W, 3)
    assert np.array_equal(idx[rows], full[0][rows]) and np.array_equal(val[rows], full[1][rows])
    assert (np.delete(idx, rows, axis=0) == -1).all()
