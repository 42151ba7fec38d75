"""GPU parity, integer kernels: mask construction (a1), tree verification (a4), tree drafting (a5).
Bit-exact against the oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _trees(seed, B, T, max_depth=None):
    if T == 1:
        return np.full((B, 1), -1, np.int32)
    md = max_depth or min(T - 1, 4)
    return synth.make_trees(seed, B, T, (4, 3, 2, 2, 2, 2), md)


@pytest.mark.parametrize("T,gamma", [(1, 0), (1, 4), (8, 3), (16, 4), (32, 4), (64, 8), (64, 0), (5, 1)])
@pytest.mark.parametrize("flags", [0, api.SS_STREAM_EXCLUDE_SELF])
def test_build_mask(T, gamma, flags):
    B = 5
    parent = _trees(T * 10 + gamma, B, T)
    if T == 64:
        parent[1] = synth.chain_tree(64)          # deepest possible tree
    m_o, a_o, d_o = oracle.build_mask(parent, gamma, flags)
    mask, anc, depth = api.ss_build_mask(torch.from_numpy(parent).to(DEV), gamma, flags)
    torch.cuda.synchronize()
    assert np.array_equal(mask.cpu().numpy(), m_o)
    assert np.array_equal(anc.cpu().numpy().view(np.uint64), a_o)
    assert np.array_equal(depth.cpu().numpy(), d_o)


def test_build_mask_clamps_bad_parents():
    bad = np.array([[7, 3, -2, 1, 9, 2]], np.int32)
    m_o, a_o, d_o = oracle.build_mask(bad, 2)
    mask, anc, depth = api.ss_build_mask(torch.from_numpy(bad).to(DEV), 2)
    assert np.array_equal(mask.cpu().numpy(), m_o) and np.array_equal(depth.cpu().numpy(), d_o)


@pytest.mark.parametrize("T,max_depth", [(1, 0), (8, 3), (16, 3), (32, 4), (64, 63), (64, 5)])
def test_tree_verify(T, max_depth):
    B, V = 37, 50
    rng = synth.rng_for(1000 + T)
    parent = _trees(T, B, T, max_depth=min(max_depth, max(T - 1, 1)) if T > 1 else None)
    if T == 64 and max_depth == 63:
        parent[0] = synth.chain_tree(64)
    tok = rng.integers(0, V, (B, T)).astype(np.int32)
    a = rng.integers(0, V, (B, T)).astype(np.int32)
    # plant agreement along a random root path for most sequences (plus chance matches from the small alphabet)
    for b in range(B):
        path = synth.root_path(parent[b], int(rng.integers(T)))
        for p, c in zip(path[:-1], path[1:]):
            if rng.random() < 0.8:
                a[b, p] = tok[b, c]
    if T > 2:
        tok[3, 1:] = tok[3, 1]        # equal sibling tokens: several longest paths, lowest index wins
        a[3, :] = tok[3, 1]
    want = oracle.tree_verify(tok, parent, a, max_depth)
    # arg-max tokens handed over the way the LM head leaves them: column 0 of an [B*R, K] array
    K, R = 3, T * 2
    idx = torch.full((B * R, K), -9, dtype=torch.int32)
    idx.view(B, R, K)[:, :T, 0] = torch.from_numpy(a)
    got = api.ss_tree_verify(torch.from_numpy(tok).to(DEV), torch.from_numpy(parent).to(DEV), idx.to(DEV),
                             max_depth, batch_stride=R * K, node_stride=K)
    torch.cuda.synchronize()
    for k in want:
        assert np.array_equal(got[k].cpu().numpy(), want[k]), k
    assert want["n_accept"].max() > 0 or T == 1


@pytest.mark.parametrize("branching", [(2, 2), (4, 2, 1, 1), (3,), (1, 1, 1, 1), (2, 2, 2, 2, 2), (7, 8)])
def test_tree_draft_from_branching(branching):
    gamma, K, T, B = len(branching), max(branching), 16, 9
    rng = synth.rng_for(sum(branching) * 7)
    R = T * (1 + gamma)
    idx = rng.integers(0, 32000, (B * R, K)).astype(np.int32)            # laid out like the LM-head output
    last = rng.integers(0, T, B).astype(np.int32)
    bonus = rng.integers(0, 32000, B).astype(np.int32)
    tp, tr, td = oracle.full_tree_template(branching)
    topk = idx.reshape(B, R, K)[:, T:].reshape(B, T, gamma, K)
    want_tok, want_par = oracle.tree_draft(topk, last, bonus, tp, tr)
    got_tok, got_par = api.ss_tree_draft(torch.from_numpy(idx).to(DEV), K, torch.from_numpy(last).to(DEV),
                                         torch.from_numpy(bonus).to(DEV), T, gamma, branching=branching,
                                         batch_stride=R * K, offset=T * K)
    torch.cuda.synchronize()
    assert np.array_equal(got_tok.cpu().numpy(), want_tok)
    assert np.array_equal(got_par.cpu().numpy(), want_par)
    # host template helper agrees with the oracle's
    hp, hr, hd = api.ss_full_tree_template_host(branching)
    assert np.array_equal(hp.numpy(), tp) and np.array_equal(hr.numpy(), tr) and np.array_equal(hd.numpy(), td)


def test_tree_draft_from_device_template():
    # a pruned (irregular) template, including entries that must yield -1
    gamma, K, T, B = 3, 4, 8, 4
    rng = synth.rng_for(5)
    topk = rng.integers(0, 1000, (B, T, gamma, K)).astype(np.int32)
    last = rng.integers(0, T, B).astype(np.int32)
    bonus = rng.integers(0, 1000, B).astype(np.int32)
    tparent = np.array([-1, 0, 0, 1, 1, 2, 3, 6, 0], np.int32)      # node 7 has depth 4 > gamma
    trank = np.array([0, 0, 1, 0, 3, 2, 1, 0, 4], np.int32)         # node 8 has rank 4 >= K
    want_tok, want_par = oracle.tree_draft(topk, last, bonus, tparent, trank)
    got_tok, got_par = api.ss_tree_draft(torch.from_numpy(topk).to(DEV), K, torch.from_numpy(last).to(DEV),
                                         torch.from_numpy(bonus).to(DEV), T, gamma,
                                         tmpl_parent=torch.from_numpy(tparent).to(DEV),
                                         tmpl_rank=torch.from_numpy(trank).to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(got_tok.cpu().numpy(), want_tok)
    assert (want_tok[:, 7] == -1).all() and (want_tok[:, 8] == -1).all()
    assert np.array_equal(got_par.cpu().numpy(), want_par)


def test_empty_batch():
    e = torch.empty((0, 4), dtype=torch.int32, device=DEV)
    mask, anc, depth = api.ss_build_mask(e, 2)
    assert mask.shape == (0, 12, 12)
    r = api.ss_tree_verify(e, e, e, 3)
    assert r["n_accept"].shape == (0,)
