"""GPU parity of the KV-cache commit (n3) against the oracle: pure copies, so everything is bit-exact;
and a short decode loop (attention -> LM head -> verify -> draft -> commit, three steps) whose integer
state has to follow the oracle's chain step by step."""
import numpy as np
import pytest
import torch

import oracle
from helpers import to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(dtype, page, B=3, T=9, gamma=2, L=(5, 40, 31), cap=80, seed=3, Hkv=2, D=64):
    cfg = synth.scaled(synth.CONFIGS["c1" if dtype == "f32" else "c2"], B=B, H=Hkv, Hkv=Hkv, D=D, T=T, gamma=gamma, page=page,
                       L_min=cap, L_max=cap, branching=(3, 2, 2), max_depth=3)
    inp = synth.make_msa_inputs(cfg, seed)
    inp["seq_lens"] = torch.tensor(list(L)[:B], dtype=torch.int32)
    par = inp["parent"].numpy()
    rng = synth.rng_for(seed + 77)
    md = cfg.max_depth
    path = -np.ones((B, md + 1), np.int32)
    n_acc = np.zeros(B, np.int32)
    for b in range(B):
        p = synth.root_path(par[b], int(rng.integers(cfg.T)))[: md + 1]
        path[b, : len(p)] = p
        n_acc[b] = len(p) - 1
    return cfg, inp, path, n_acc


def _run(cfg, inp, path, n_acc, table=None):
    bt = inp["block_table"] if table is None else table
    kc, vc = inp["k_cache"].to(DEV).clone(), inp["v_cache"].to(DEV).clone()
    lens = api.ss_kv_commit(inp["k_new"].to(DEV), inp["v_new"].to(DEV), kc, vc, bt.to(DEV), inp["seq_lens"].to(DEV),
                            torch.from_numpy(path).to(DEV), torch.from_numpy(n_acc).to(DEV), cfg.gamma)
    torch.cuda.synchronize()
    ok, ov, ol = oracle.kv_commit(to_np_f32(inp["k_new"]), to_np_f32(inp["v_new"]), to_np_f32(inp["k_cache"]),
                                  to_np_f32(inp["v_cache"]), bt.numpy(), inp["seq_lens"].numpy(), path, n_acc)
    assert np.array_equal(to_np_f32(kc), ok)
    assert np.array_equal(to_np_f32(vc), ov)
    assert np.array_equal(lens.cpu().numpy(), ol)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("page", [16, 32, 64])
def test_matches_oracle_bit_exact(dtype, page):
    _run(*_inputs(dtype, page))


def test_page_boundaries_heads_and_head_dim_128():
    # appended rows straddle a page boundary; 4 KV heads of 128 features
    _run(*_inputs("bf16", 16, B=2, L=(14, 63), Hkv=4, D=128, seed=9))


def test_capacity_cut_and_empty_batch():
    cfg, inp, path, n_acc = _inputs("f32", 16, B=1, L=(30,))
    n_acc[:] = 3
    path[0] = [0, 1, 2, 3]
    _run(cfg, inp, path, n_acc, table=inp["block_table"][:, :2].contiguous())      # capacity 32: two rows fit
    e = torch.empty((0, cfg.R, cfg.Hkv, cfg.D), device=DEV)
    z = torch.empty(0, dtype=torch.int32, device=DEV)
    out = api.ss_kv_commit(e, e, inp["k_cache"].to(DEV), inp["v_cache"].to(DEV), torch.empty((0, 5), dtype=torch.int32, device=DEV),
                           z, torch.empty((0, 4), dtype=torch.int32, device=DEV), z, cfg.gamma)
    assert out.numel() == 0


def test_new_lens_may_not_alias_seq_lens():
    cfg, inp, path, n_acc = _inputs("f32", 16)
    lens = inp["seq_lens"].to(DEV)
    with pytest.raises(api.SSError):
        api.ss_kv_commit(inp["k_new"].to(DEV), inp["v_new"].to(DEV), inp["k_cache"].to(DEV), inp["v_cache"].to(DEV),
                         inp["block_table"].to(DEV), lens, torch.from_numpy(path).to(DEV), torch.from_numpy(n_acc).to(DEV),
                         cfg.gamma, new_seq_lens=lens)


def test_three_step_decode_loop_follows_the_oracle():
    """fp32, one MSA layer whose output feeds the LM head (c1's shapes), every tree the full (2,2,1)
    template: after every step the accepted lengths, emitted tokens, next tree, cache contents and
    sequence lengths of the GPU chain equal the oracle's.  The synthetic q/k/v of a step do not depend on
    the tokens, so drafts would almost never be accepted; along one seeded root path per sequence the
    draft tokens are therefore overwritten with the oracle's arg-max tokens (both chains get the same
    tokens), which makes the commits append 1 to 4 rows."""
    tp, tr, _ = oracle.full_tree_template(synth.CONFIGS["c1"].draft_branching)
    T = len(tp)
    cfg = synth.scaled(synth.CONFIGS["c1"], B=2, L_min=160, L_max=160, T=T, gamma=3, branching=(2, 2, 1), max_depth=3)
    base = synth.make_msa_inputs(cfg, 21)
    W = synth.make_lm_head_inputs(cfg, 21)["W"]
    parent = np.broadcast_to(np.where(np.arange(T) == 0, -1, tp), (cfg.B, T)).astype(np.int32).copy()
    start = np.array([100, 117], np.int32)
    o_kc, o_vc, o_len = to_np_f32(base["k_cache"]), to_np_f32(base["v_cache"]), start.copy()
    g_kc, g_vc = base["k_cache"].to(DEV).clone(), base["v_cache"].to(DEV).clone()
    g_len = torch.from_numpy(o_len).to(DEV)
    bt = base["block_table"]
    g_par = torch.from_numpy(parent).to(DEV)
    tok = synth.make_draft_tokens(5, parent, cfg.vocab)
    rng = synth.rng_for(4321)
    accepted = []
    for step in range(3):
        x = synth.make_msa_inputs(cfg, 100 + step)          # this step's projected q / k / v (token-independent)
        q, kn, vn = x["q"], x["k_new"], x["v_new"]
        # oracle chain
        o_out = oracle.msa_attention(to_np_f32(q), to_np_f32(kn), to_np_f32(vn), o_kc, o_vc, bt.numpy(), o_len, parent,
                                     cfg.gamma, x["scale"])
        hid = o_out.reshape(cfg.B * cfg.R, cfg.d_model).astype(np.float32)
        o_idx, _ = oracle.lm_head_topk(hid, to_np_f32(W), cfg.K)
        o_idx = o_idx.reshape(cfg.B, cfg.R, cfg.K)
        for b in range(cfg.B):                              # plant agreement along one root path
            pth = synth.root_path(parent[b], int(rng.integers(1, T)))
            for e_, (p_, c_) in enumerate(zip(pth[:-1], pth[1:])):
                if e_ > 0 and rng.random() >= 0.7:          # the first edge always, later ones until a miss
                    break
                tok[b, c_] = o_idx[b, p_, 0]
        o_ver = oracle.tree_verify(tok, parent, np.ascontiguousarray(o_idx[:, :T, 0]), cfg.max_depth)
        o_next, _ = oracle.tree_draft(np.ascontiguousarray(o_idx[:, T:, :].reshape(cfg.B, T, cfg.gamma, cfg.K)),
                                      o_ver["last"], o_ver["bonus"], tp, tr)
        o_kc, o_vc, o_len = oracle.kv_commit(to_np_f32(kn), to_np_f32(vn), o_kc, o_vc, bt.numpy(), o_len, o_ver["path"],
                                             o_ver["n_accept"])
        # GPU chain (same tokens)
        g_tok = torch.from_numpy(tok).to(DEV)
        g_out = api.ss_msa_attention(q.to(DEV), kn.to(DEV), vn.to(DEV), g_kc, g_vc, bt.to(DEV), g_len, g_par, cfg.gamma, x["scale"])
        g_idx, _ = api.ss_lm_head_argmax_topk(g_out.view(cfg.B * cfg.R, cfg.d_model), W.to(DEV), cfg.K)
        g_ver = api.ss_tree_verify(g_tok, g_par, g_idx, cfg.max_depth, batch_stride=cfg.R * cfg.K, node_stride=cfg.K)
        g_next, _ = api.ss_tree_draft(g_idx, cfg.K, g_ver["last"], g_ver["bonus"], T, cfg.gamma, branching=cfg.draft_branching,
                                      batch_stride=cfg.R * cfg.K, offset=T * cfg.K)
        g_len = api.ss_kv_commit(kn.to(DEV), vn.to(DEV), g_kc, g_vc, bt.to(DEV), g_len, g_ver["path"], g_ver["n_accept"], cfg.gamma)
        torch.cuda.synchronize()
        assert np.array_equal(g_ver["n_accept"].cpu().numpy(), o_ver["n_accept"]), step
        assert np.array_equal(g_ver["out_tokens"].cpu().numpy(), o_ver["out_tokens"]), step
        assert np.array_equal(g_next.cpu().numpy(), o_next), step
        assert np.array_equal(g_len.cpu().numpy(), o_len), step
        assert np.array_equal(to_np_f32(g_kc), o_kc) and np.array_equal(to_np_f32(g_vc), o_vc), step
        accepted.append(o_ver["n_accept"].copy())
        tok = o_next.astype(np.int32).copy()                # the next step verifies the tree just drafted
    assert np.array_equal(o_len, start + np.sum(accepted, axis=0) + 3)
    assert np.sum(accepted) > 0
