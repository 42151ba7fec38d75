"""All entry points chained the way one multi-stream layer of a model uses them, on one stream:

  main-stream states of the tree nodes -> pruning layer (log-sum-exp, transition probabilities, prune) ->
  stream insertion on the pruned tree -> QKV projection -> multi-stream attention over the paged cache ->
  output projection -> LM head top-K -> verification -> next draft -> cache commit.

Every stage is compared with the oracle ON THE INPUTS THE GPU STAGE ACTUALLY HAD (stage-wise parity): what the
paper does not discuss (normalisation, rotary embedding, residuals, the feed-forward block) is left out, so the
numbers mean nothing as a model, but every interface between the calls is exercised.  Tolerances are those of
the tests of the single entry points.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import rel_err, to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _lin_ok(y, x, W):
    ref = oracle.linear_rows(to_np_f32(x), to_np_f32(W))
    S = oracle.linear_rows(np.abs(to_np_f32(x)), np.abs(to_np_f32(W)))
    return (np.abs(to_np_f32(y) - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * S).all()


def test_one_layer_all_entry_points():
    cfg = synth.scaled(synth.CONFIGS["c4"], B=3, H=4, Hkv=2, D=64, L_min=150, L_max=400, vocab=1536, d_model=256,
                       T=11, gamma=2, branching=(2, 2, 1), max_depth=3, K=2, draft_branching=(2, 2))
    B, T, g, d, H, Hkv, D, V = cfg.B, cfg.T, cfg.gamma, cfg.d_model, cfg.H, cfg.Hkv, cfg.D, cfg.vocab
    rng = synth.rng_for(77)
    bf = torch.bfloat16
    nrm = lambda shape, std: torch.from_numpy((std * rng.standard_normal(shape)).astype(np.float32)).to(bf).to(DEV)
    M = nrm((B, T, d), 1.0)                               # main-stream states of the tree nodes
    P = nrm((g, d), 0.3)                                  # stream embeddings
    W_lm = nrm((V, d), 2.0 / np.sqrt(d))                  # LM head
    W_qkv = nrm(((H + 2 * Hkv) * D, d), 1.0 / np.sqrt(d))
    W_o = nrm((d, H * D), 1.0 / np.sqrt(H * D))
    base = synth.make_msa_inputs(cfg, 9)                  # paged cache, page table, lengths, a tree
    parent = base["parent"].numpy()
    tok = synth.make_draft_tokens(9, parent, V)
    dev = lambda t: t.to(DEV)
    k_cache, v_cache = dev(base["k_cache"]), dev(base["v_cache"])
    table, lens = dev(base["block_table"]), dev(base["seq_lens"])
    tok_d, par_d = torch.from_numpy(tok).to(DEV), torch.from_numpy(parent).to(DEV)

    # ---- pruning layer on the main-stream states (o = identity here)
    lse = api.ss_lm_head_logsumexp(M.view(B * T, d), W_lm)
    prob = api.ss_transition_probs(M, W_lm, tok_d, par_d, lse)
    thr = float(prob[:, 1:].float().quantile(0.3))
    pr = api.ss_tree_prune(tok_d, par_d, prob, thr)
    # the states of the kept nodes, in the new order (padding rows repeat the root's): plumbing, a gather
    old = pr["old_index"].clamp(min=0).long()
    M2 = torch.gather(M, 1, old[:, :, None].expand(B, T, d)).contiguous()
    # ---- stream insertion, projections, attention, output projection
    X = api.ss_stream_insert(M2, P)                                          # [B,R,d]
    R = X.shape[1]
    qkv = api.ss_linear_rows(X.view(B * R, d), W_qkv).view(B, R, H + 2 * Hkv, D)
    q, k_new, v_new = qkv[:, :, :H].contiguous(), qkv[:, :, H:H + Hkv].contiguous(), qkv[:, :, H + Hkv:].contiguous()
    attn = api.ss_msa_attention(q, k_new, v_new, k_cache, v_cache, table, lens, pr["parent"], g, base["scale"])
    hid = api.ss_linear_rows(attn.view(B * R, H * D), W_o)                   # [B*R, d]
    # ---- LM head, verification, next draft, cache commit
    idx, val = api.ss_lm_head_argmax_topk(hid, W_lm, cfg.K)
    ver = api.ss_tree_verify(pr["tok"], pr["parent"], idx, cfg.max_depth, batch_stride=R * cfg.K, node_stride=cfg.K)
    nxt, npar = api.ss_tree_draft(idx, cfg.K, ver["last"], ver["bonus"], T, g, branching=cfg.draft_branching,
                                  batch_stride=R * cfg.K, offset=T * cfg.K)
    kc_before, vc_before = k_cache.clone(), v_cache.clone()
    new_lens = api.ss_kv_commit(k_new, v_new, k_cache, v_cache, table, lens, ver["path"], ver["n_accept"], g)
    torch.cuda.synchronize()

    # ---- stage-wise parity
    f = to_np_f32
    ref_lse = oracle.lm_head_lse(f(M).reshape(B * T, d), f(W_lm))
    assert (np.abs(lse.cpu().numpy() - ref_lse) <= 2e-3 * np.maximum(1.0, np.abs(ref_lse))).all()
    ref_prob = oracle.transition_probs(f(M), f(W_lm), tok, parent)
    assert (np.abs(prob.cpu().numpy() - ref_prob) <= 2e-2 * ref_prob + 1e-7).all()
    o_pr = oracle.tree_prune(tok, parent, prob.cpu().numpy(), thr)
    for k in o_pr:
        np.testing.assert_array_equal(pr[k].cpu().numpy(), o_pr[k], err_msg=k)
    assert 1 <= int(o_pr["n_nodes"].min()) and int(o_pr["n_nodes"].min()) < T          # something was pruned
    ref_X = oracle.stream_insert(f(M2), f(P))
    assert (np.abs(f(X) - ref_X) <= 2.0 ** -8 * np.abs(ref_X)).all()
    assert _lin_ok(qkv.reshape(B * R, -1), X.view(B * R, d), W_qkv)
    ref_attn = oracle.msa_attention(f(q), f(k_new), f(v_new), f(kc_before), f(vc_before), base["block_table"].numpy(),
                                    base["seq_lens"].numpy(), o_pr["parent"], g, base["scale"])
    live = np.zeros((B, R), bool)                      # rows of kept nodes: padding rows are computed and ignored
    for b in range(B):
        n = int(o_pr["n_nodes"][b])
        live[b, :n] = True
        live[b, T:T + n * g] = True
    assert rel_err(f(attn)[live], ref_attn[live]) <= 2e-2
    assert _lin_ok(hid, attn.view(B * R, H * D), W_o)
    o_idx, o_val, z = oracle.lm_head_topk(f(hid), f(W_lm), cfg.K, want_logits=True)
    g_idx = idx.cpu().numpy()
    tau = 1e-4 * np.abs(z).max()
    for n, k in zip(*np.nonzero(g_idx != o_idx)):
        assert abs(z[n, g_idx[n, k]] - o_val[n, k]) <= tau
    a = g_idx.reshape(B, R, cfg.K)[:, :T, 0]
    o_ver = oracle.tree_verify(o_pr["tok"], o_pr["parent"], a, cfg.max_depth)
    for k in o_ver:
        np.testing.assert_array_equal(ver[k].cpu().numpy(), o_ver[k], err_msg=k)
    for b in range(B):                                  # padding is never on the accepted path
        assert all(x < o_pr["n_nodes"][b] for x in o_ver["path"][b, :o_ver["n_accept"][b] + 1])
    tp, tr, _ = oracle.full_tree_template(cfg.draft_branching)
    topk = g_idx.reshape(B, R, cfg.K)[:, T:].reshape(B, T, g, cfg.K)
    o_nxt, o_par = oracle.tree_draft(topk, o_ver["last"], o_ver["bonus"], tp, tr)
    np.testing.assert_array_equal(nxt.cpu().numpy(), o_nxt)
    np.testing.assert_array_equal(npar.cpu().numpy(), o_par)
    o_kc, o_vc, o_len = oracle.kv_commit(f(k_new), f(v_new), f(kc_before), f(vc_before), base["block_table"].numpy(),
                                         base["seq_lens"].numpy(), o_ver["path"], o_ver["n_accept"])
    np.testing.assert_array_equal(f(k_cache), o_kc)
    np.testing.assert_array_equal(f(v_cache), o_vc)
    np.testing.assert_array_equal(new_lens.cpu().numpy(), o_len)
