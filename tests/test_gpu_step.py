"""The whole verify-and-speculate step chained on one stream through the C ABI, against the oracle
chained the same way (config c1 entire; a c4-shaped step at reduced prefix / vocabulary)."""
import numpy as np
import pytest
import torch

import oracle
from helpers import rel_err, to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_step_gpu(cfg, layers, W, tok, parent_dev):
    """N_s MSA layers (each with its own cache and q/k/v), LM head on the last layer's output,
    verify, draft: no host synchronisation in between."""
    out = None
    for lay in layers:
        out = api.ss_msa_attention(lay["q"], lay["k_new"], lay["v_new"], lay["k_cache"], lay["v_cache"],
                                   lay["block_table"], lay["seq_lens"], parent_dev, cfg.gamma, lay["scale"])
    hidden = out.view(cfg.B * cfg.R, cfg.H * cfg.D)
    idx, val = api.ss_lm_head_argmax_topk(hidden, W, cfg.K)
    ver = api.ss_tree_verify(tok, parent_dev, idx, cfg.max_depth, batch_stride=cfg.R * cfg.K, node_stride=cfg.K)
    nxt, npar = api.ss_tree_draft(idx, cfg.K, ver["last"], ver["bonus"], cfg.T, cfg.gamma,
                                  branching=cfg.draft_branching, batch_stride=cfg.R * cfg.K, offset=cfg.T * cfg.K)
    return out, idx, val, ver, nxt, npar


@pytest.mark.parametrize("name", ["c1", "c4small"])
def test_step_chain(name):
    if name == "c1":
        cfg = synth.CONFIGS["c1"]
    else:
        cfg = synth.scaled(synth.CONFIGS["c4"], B=2, H=4, Hkv=4, L_min=600, L_max=600, vocab=2000, d_model=512,
                           n_layers=2)
    assert cfg.H * cfg.D == cfg.d_model
    layers = [synth.make_msa_inputs(cfg, 1, layer=i) for i in range(cfg.n_layers)]
    parent = layers[0]["parent"]
    W = synth.make_lm_head_inputs(cfg, 1)["W"]
    tok = synth.make_draft_tokens(1, parent.numpy(), cfg.vocab)
    dl = [{k: (v.to(DEV) if isinstance(v, torch.Tensor) else v) for k, v in lay.items()} for lay in layers]
    out, idx, val, ver, nxt, npar = run_step_gpu(cfg, dl, W.to(DEV), torch.from_numpy(tok).to(DEV),
                                                 parent.to(DEV))
    torch.cuda.synchronize()

    # oracle chain: attention of the last layer -> (rounded to the storage type, as the GPU hands it on) -> LM head
    lay = layers[-1]
    o_out = oracle.msa_attention(to_np_f32(lay["q"]), to_np_f32(lay["k_new"]), to_np_f32(lay["v_new"]),
                                 to_np_f32(lay["k_cache"]), to_np_f32(lay["v_cache"]), lay["block_table"].numpy(),
                                 lay["seq_lens"].numpy(), parent.numpy(), cfg.gamma, lay["scale"])
    tol = 1e-5 if cfg.dtype == "f32" else 2e-2
    assert rel_err(to_np_f32(out), o_out) <= tol
    # the LM head is compared on the hidden states the GPU actually produced (identical inputs on both sides)
    hidden = to_np_f32(out).reshape(cfg.B * cfg.R, cfg.d_model)
    o_idx, o_val, z = oracle.lm_head_topk(hidden, to_np_f32(W), cfg.K, want_logits=True)
    tau = (1e-5 if cfg.dtype == "f32" else 1e-4) * np.abs(z).max()
    g_idx = idx.cpu().numpy()
    diff = g_idx != o_idx
    for n, k in zip(*np.nonzero(diff)):
        assert abs(z[n, g_idx[n, k]] - o_val[n, k]) <= tau
    # verify / draft: fed the GPU's own indices on both sides -> bit-exact
    a = g_idx.reshape(cfg.B, cfg.R, cfg.K)[:, :cfg.T, 0]
    o_ver = oracle.tree_verify(tok, parent.numpy(), a, cfg.max_depth)
    for k in o_ver:
        assert np.array_equal(ver[k].cpu().numpy(), o_ver[k]), k
    tp, tr, td = oracle.full_tree_template(cfg.draft_branching)
    topk = g_idx.reshape(cfg.B, cfg.R, cfg.K)[:, cfg.T:].reshape(cfg.B, cfg.T, cfg.gamma, cfg.K)
    o_nxt, o_par = oracle.tree_draft(topk, o_ver["last"], o_ver["bonus"], tp, tr)
    assert np.array_equal(nxt.cpu().numpy(), o_nxt) and np.array_equal(npar.cpu().numpy(), o_par)
    # the drafted tree is a valid input of the next step
    api.ss_check_tree_host(npar.cpu()[None], max_depth=cfg.gamma)
