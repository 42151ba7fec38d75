"""Parity at the full sizes of the configurations, every element: the whole c4 step (4 MSA layers, fused LM head +
verify + draft) in the launch configuration bench.py times, one full c3 layer, one full c5 sequence (all 8 KV
heads), each against the oracle on the same seeded inputs (drawn on the GPU by the seeded generator and copied
to the host for the oracle).  The oracle needs a few seconds for each."""
import numpy as np
import pytest
import torch

import oracle
from helpers import oracle_subproblem, rel_err, to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _oracle_layer(lay, parent, gamma):
    return oracle.msa_attention(to_np_f32(lay["q"]), to_np_f32(lay["k_new"]), to_np_f32(lay["v_new"]),
                                to_np_f32(lay["k_cache"]), to_np_f32(lay["v_cache"]), lay["block_table"].cpu().numpy(),
                                lay["seq_lens"].cpu().numpy(), parent.cpu().numpy(), gamma, lay["scale"])


def test_c4_whole_step_every_element():
    cfg = synth.CONFIGS["c4"]
    N = cfg.B * cfg.R
    layers = [synth.make_msa_inputs(cfg, 1, device=DEV, layer=i) for i in range(cfg.n_layers)]
    parent = layers[0]["parent"]
    max_len = layers[0]["block_table"].shape[1] * cfg.page
    assert api.ss_msa_plan(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, max_len, api.SS_BF16) == (2, 1)
    ws = api.ss_msa_workspace(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, max_len, api.SS_BF16, DEV)
    W = synth.make_lm_head_inputs(cfg, 1, device=DEV)["W"]
    tok_np = synth.make_draft_tokens(1, parent.cpu().numpy(), cfg.vocab)
    tok = torch.from_numpy(tok_np).to(DEV)
    outs = [torch.empty_like(l["q"]) for l in layers]
    # the step as bench.py enqueues it: four attention calls on one workspace, then the fused tail
    for lay, out in zip(layers, outs):
        api.ss_msa_attention(lay["q"], lay["k_new"], lay["v_new"], lay["k_cache"], lay["v_cache"], lay["block_table"],
                             lay["seq_lens"], parent, cfg.gamma, lay["scale"], out=out, workspace=ws)
    hidden = outs[-1].view(N, cfg.d_model)
    tail = api.ss_lm_head_verify_draft(hidden, W, cfg.K, tok, parent, cfg.gamma, cfg.max_depth,
                                       branching=cfg.draft_branching)
    idx, val = api.ss_lm_head_argmax_topk(hidden, W, cfg.K)
    torch.cuda.synchronize()

    # every attention output element of every layer
    for i, (lay, out) in enumerate(zip(layers, outs)):
        assert torch.isfinite(out.float()).all()
        err = rel_err(to_np_f32(out), _oracle_layer(lay, parent, cfg.gamma))
        print("c4 layer %d: err %.2e" % (i, err), flush=True)
        assert err <= 2e-2, (i, err)
    # all 320 LM-head rows over the whole vocabulary, on the hidden states the GPU produced (identical inputs)
    o_idx, o_val, z = oracle.lm_head_topk(to_np_f32(hidden), to_np_f32(W), cfg.K, want_logits=True)
    tau = 1e-4 * np.abs(z).max()
    g_idx, g_val = idx.cpu().numpy(), val.cpu().numpy()
    ties = 0
    for n, k in zip(*np.nonzero(g_idx != o_idx)):
        assert abs(z[n, g_idx[n, k]] - o_val[n, k]) <= tau, (n, k)
        ties += 1
    assert ties <= 4, ties
    assert np.max(np.abs(g_val - np.take_along_axis(z, g_idx.astype(np.int64), axis=1))) <= 2e-2 * np.sqrt(np.mean(z * z))
    for n in range(N):
        assert len(set(g_idx[n].tolist())) == cfg.K
    # verification and drafting: integers, fed the GPU's own indices on both sides -> bit-exact; the fused call
    # agrees with the three separate ones
    a = g_idx.reshape(cfg.B, cfg.R, cfg.K)[:, :cfg.T, 0]
    assert np.array_equal(tail["main_argmax"].cpu().numpy(), a)
    o_ver = oracle.tree_verify(tok_np, parent.cpu().numpy(), np.ascontiguousarray(a), cfg.max_depth)
    for k in o_ver:
        assert np.array_equal(tail[k].cpu().numpy(), o_ver[k]), k
    tp, tr, _ = oracle.full_tree_template(cfg.draft_branching)
    topk = np.ascontiguousarray(g_idx.reshape(cfg.B, cfg.R, cfg.K)[:, cfg.T:].reshape(cfg.B, cfg.T, cfg.gamma, cfg.K))
    o_nxt, o_par = oracle.tree_draft(topk, o_ver["last"], o_ver["bonus"], tp, tr)
    assert np.array_equal(tail["next_tok"].cpu().numpy(), o_nxt)
    assert np.array_equal(tail["next_parent"].cpu().numpy(), o_par)


def test_c3_one_full_layer_every_element():
    cfg = synth.CONFIGS["c3"]
    lay = synth.make_msa_inputs(cfg, 1, device=DEV, layer=2)
    max_len = lay["block_table"].shape[1] * cfg.page
    assert api.ss_msa_plan(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, max_len, api.SS_BF16) == (1, 1)
    out = api.ss_msa_attention(lay["q"], lay["k_new"], lay["v_new"], lay["k_cache"], lay["v_cache"], lay["block_table"],
                               lay["seq_lens"], lay["parent"], cfg.gamma, lay["scale"])
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    err = rel_err(to_np_f32(out), _oracle_layer(lay, lay["parent"], cfg.gamma))
    print("c3 layer: lengths %s err %.2e" % (lay["seq_lens"].tolist(), err), flush=True)
    assert err <= 2e-2, err


def test_c5_one_full_sequence_every_element():
    # the whole c5 launch on the GPU; the oracle on all 8 KV heads (32 query heads x 160 rows) of one sequence
    cfg = synth.CONFIGS["c5"]
    inp = synth.make_msa_inputs(cfg, 1, device=DEV)
    out = api.ss_msa_attention(inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["block_table"],
                               inp["seq_lens"], inp["parent"], cfg.gamma, inp["scale"])
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    b, g = 5, cfg.H // cfg.Hkv
    worst = 0.0
    for hk in range(cfg.Hkv):
        sub = oracle_subproblem(inp, b, hk, g)
        want = oracle.msa_attention(sub["q"], sub["k_new"], sub["v_new"], sub["k_cache"], sub["v_cache"],
                                    sub["block_table"], sub["seq_lens"], sub["parent"], cfg.gamma, inp["scale"])
        err = rel_err(to_np_f32(out[b:b + 1, :, hk * g:(hk + 1) * g]), want)
        worst = max(worst, err)
        assert err <= 2e-2, (hk, err)
    print("c5 sequence %d: worst err over 8 KV heads %.2e" % (b, worst), flush=True)
