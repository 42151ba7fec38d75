"""GPU parity of the page allocation for the KV-cache commit (n3, Appendix A.1) against the oracle: integers,
bit-exact (the allocation order is defined, so nothing is left to scheduling); then a decode loop whose sequences
outgrow the pages their table started with: allocate, commit, attend, step after step, against the oracle chain."""
import numpy as np
import pytest
import torch

import oracle
from helpers import rel_err, to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _gpu_alloc(table, L, n_acc, page, max_depth, stack, count):
    bt = torch.from_numpy(table.copy()).to(DEV)
    cnt = torch.tensor([count], dtype=torch.int32, device=DEV)
    n_commit = api.ss_kv_alloc_pages(bt, torch.from_numpy(L).to(DEV), torch.from_numpy(n_acc).to(DEV), page, max_depth,
                                     torch.from_numpy(stack).to(DEV), cnt)
    torch.cuda.synchronize()
    return bt.cpu().numpy(), int(cnt.item()), n_commit.cpu().numpy()


@pytest.mark.parametrize("seed", range(16))
def test_random_cases_match_the_oracle(seed):
    rng = synth.rng_for(300 + seed)
    B = int(rng.choice([1, 2, 7, 64, 300, 1025, 2500]))
    page, max_pages, max_depth = int(rng.choice([16, 32, 64])), int(rng.integers(1, 7)), int(rng.integers(0, 6))
    cap = page * max_pages
    L = rng.integers(0, cap + 1, size=B).astype(np.int32)
    near = rng.random(B) < 0.6                                   # most sequences sit just below a page boundary
    L[near] = np.minimum(cap, (rng.integers(1, max_pages + 1, size=int(near.sum())) * page - rng.integers(0, 4, size=int(near.sum())))).astype(np.int32)
    n_acc = rng.integers(-1, max_depth + 2, size=B).astype(np.int32)
    table = rng.integers(0, 1000, size=(B, max_pages)).astype(np.int32)
    stack = (1000 + rng.permutation(4 * B + 8)[:int(rng.integers(0, 2 * B + 8))]).astype(np.int32)
    if stack.size == 0:
        stack = np.array([1000], np.int32)
    count = int(rng.integers(0, stack.size + 1))
    want = oracle.kv_alloc_pages(table, L, n_acc, page, max_depth, stack, count)
    got = _gpu_alloc(table, L, n_acc, page, max_depth, stack, count)
    assert np.array_equal(got[0], want[0]) and got[1] == want[1] and np.array_equal(got[2], want[2])


def test_lengths_and_counts_out_of_range_are_clamped():
    table = np.zeros((3, 2), np.int32)
    L = np.array([-5, 1000, 31], np.int32)          # below zero, beyond the capacity of 32 tokens
    n_acc = np.array([2, 2, 99], np.int32)
    stack = np.array([7, 8, 9], np.int32)
    bt, left, n_commit = _gpu_alloc(table, L, n_acc, 16, 3, stack, 3)
    want = oracle.kv_alloc_pages(table, np.clip(L, 0, 32), n_acc, 16, 3, stack, 3)
    assert np.array_equal(bt, want[0]) and left == want[1] and np.array_equal(n_commit, want[2])


def test_decode_loop_that_outgrows_its_table():
    """Three steps of a small model whose sequences start a few tokens below a page boundary with only the pages in
    use mapped.  Each step: attention, LM head, verify, draft, page allocation, commit; caches, tables, lengths,
    emitted tokens and the stack all equal the oracle's.  The stack runs dry in the last step for the last sequence."""
    T, gamma = 7, 2
    cfg = synth.scaled(synth.CONFIGS["c1"], B=3, H=4, Hkv=2, D=64, T=T, gamma=gamma, page=16, L_min=96, L_max=96,
                       branching=(2, 2, 2), max_depth=3, vocab=300, d_model=256, K=2, draft_branching=(2, 2))
    base = synth.make_msa_inputs(cfg, 21)
    W = synth.make_lm_head_inputs(cfg, 21)["W"]
    full = base["block_table"].numpy()                      # 6 logical pages per sequence
    start = np.array([14, 30, 47], np.int32)
    table = full.copy()
    free = []
    for b in range(cfg.B):
        m0 = -(-int(start[b]) // 16)
        free += full[b, m0:].tolist()
        table[b, m0:] = 0
    stack = np.array(free[:2], np.int32)                    # two free pages only: three will be asked for
    parent = synth.make_trees(21, cfg.B, T, cfg.branching, cfg.max_depth)
    tok = synth.make_draft_tokens(21, parent, cfg.vocab)
    tp, tr, _ = oracle.full_tree_template(cfg.draft_branching)
    o_kc, o_vc = to_np_f32(base["k_cache"]), to_np_f32(base["v_cache"])
    o_bt, o_len, o_cnt = table.copy(), start.copy(), stack.size
    g_kc, g_vc = base["k_cache"].to(DEV), base["v_cache"].to(DEV)
    g_bt, g_len = torch.from_numpy(table.copy()).to(DEV), torch.from_numpy(start.copy()).to(DEV)
    g_cnt = torch.tensor([stack.size], dtype=torch.int32, device=DEV)
    g_stack, g_par = torch.from_numpy(stack).to(DEV), torch.from_numpy(parent).to(DEV)
    rng = synth.rng_for(77)
    clipped = False
    for step in range(4):
        x = synth.make_msa_inputs(cfg, 200 + step)
        q, kn, vn = x["q"], x["k_new"], x["v_new"]
        o_out = oracle.msa_attention(to_np_f32(q), to_np_f32(kn), to_np_f32(vn), o_kc, o_vc, o_bt, o_len, parent, gamma, x["scale"])
        o_idx, _ = oracle.lm_head_topk(o_out.reshape(cfg.B * cfg.R, cfg.d_model).astype(np.float32), to_np_f32(W), cfg.K)
        o_idx = o_idx.reshape(cfg.B, cfg.R, cfg.K)
        for b in range(cfg.B):                              # plant agreement along one root path: every step accepts
            pth = synth.root_path(parent[b], int(rng.integers(1, T)))
            for p_, c_ in zip(pth[:-1], pth[1:]):
                tok[b, c_] = o_idx[b, p_, 0]
        o_ver = oracle.tree_verify(tok, parent, np.ascontiguousarray(o_idx[:, :T, 0]), cfg.max_depth)
        o_next, _ = oracle.tree_draft(np.ascontiguousarray(o_idx[:, T:, :].reshape(cfg.B, T, gamma, cfg.K)),
                                      o_ver["last"], o_ver["bonus"], tp, tr)
        o_bt, o_cnt, o_commit = oracle.kv_alloc_pages(o_bt, o_len, o_ver["n_accept"], 16, cfg.max_depth, stack, o_cnt)
        clipped |= bool((o_commit < o_ver["n_accept"]).any())
        o_kc, o_vc, o_len = oracle.kv_commit(to_np_f32(kn), to_np_f32(vn), o_kc, o_vc, o_bt, o_len, o_ver["path"], o_commit)

        g_tok = torch.from_numpy(tok).to(DEV)
        g_out = api.ss_msa_attention(q.to(DEV), kn.to(DEV), vn.to(DEV), g_kc, g_vc, g_bt, g_len, g_par, gamma, x["scale"])
        g_idx, _ = api.ss_lm_head_argmax_topk(g_out.view(cfg.B * cfg.R, cfg.d_model), W.to(DEV), cfg.K)
        g_ver = api.ss_tree_verify(g_tok, g_par, g_idx, cfg.max_depth, batch_stride=cfg.R * cfg.K, node_stride=cfg.K)
        g_next, _ = api.ss_tree_draft(g_idx, cfg.K, g_ver["last"], g_ver["bonus"], T, gamma, branching=cfg.draft_branching,
                                      batch_stride=cfg.R * cfg.K, offset=T * cfg.K)
        g_commit = api.ss_kv_alloc_pages(g_bt, g_len, g_ver["n_accept"], 16, cfg.max_depth, g_stack, g_cnt)
        g_len = api.ss_kv_commit(kn.to(DEV), vn.to(DEV), g_kc, g_vc, g_bt, g_len, g_ver["path"], g_commit, gamma)
        torch.cuda.synchronize()
        assert rel_err(to_np_f32(g_out), o_out) <= 1e-5, step
        assert np.array_equal(g_ver["n_accept"].cpu().numpy(), o_ver["n_accept"]), step
        assert np.array_equal(g_next.cpu().numpy(), o_next), step
        assert np.array_equal(g_commit.cpu().numpy(), o_commit) and int(g_cnt.item()) == o_cnt, step
        assert np.array_equal(g_bt.cpu().numpy(), o_bt) and np.array_equal(g_len.cpu().numpy(), o_len), step
        assert np.array_equal(to_np_f32(g_kc), o_kc) and np.array_equal(to_np_f32(g_vc), o_vc), step
        tok = o_next.astype(np.int32).copy()
    assert o_cnt == 0 and clipped            # the stack ran dry and at least one sequence had to stop short
    assert (o_len > start).all()
