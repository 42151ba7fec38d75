"""GPU parity of the fused tail of a decode step (LM head + verification + drafting in one call) against
the three separate calls (bit for bit: the same candidates are merged) and against the oracle's chain
lm_head_topk -> tree_verify -> tree_draft on the same seeded inputs (all outputs are integers: exact)."""
import numpy as np
import pytest
import torch

import oracle
from helpers import to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = [
    # dtype, B, T, tree branching, max_depth, gamma, K, draft branching, d, V
    ("f32", 2, 8, (3, 2, 2), 3, 3, 2, (2, 2, 1), 96, 1000),
    ("bf16", 4, 16, (4, 2, 2), 3, 4, 4, (4, 2, 1, 1), 256, 3000),
    ("bf16", 3, 64, (8, 4, 2), 3, 8, 8, (2, 2, 2, 1, 1, 1, 1, 1), 128, 1000),
    ("bf16", 5, 1, (1,), 1, 1, 1, (1,), 64, 129),
    ("bf16", 1, 33, (4, 3, 2, 2), 4, 2, 3, (3, 2), 512, 40000),
    ("f32", 3, 20, (3, 3, 2), 3, 5, 8, (8, 1, 1, 1, 1), 64, 300),
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_fused_tail_equals_separate_calls_and_oracle(case):
    dtype, B, T, br, md, gamma, K, dbr, d, V = CASES[case]
    cfg = synth.scaled(synth.CONFIGS["c4" if dtype == "bf16" else "c1"], B=B, T=T, branching=br, max_depth=md,
                       gamma=gamma, K=K, draft_branching=dbr, d_model=d, vocab=V)
    R = cfg.R
    inp = synth.make_lm_head_inputs(cfg, 60 + case, N=B * R)
    hidden, W = inp["hidden"], inp["W"]
    parent = synth.make_trees(70 + case, B, T, br, md)
    tok = synth.make_draft_tokens(80 + case, parent, V)
    # the oracle's chain; draft tokens agree with the main stream along one root path per sequence
    o_idx, _ = oracle.lm_head_topk(to_np_f32(hidden), to_np_f32(W), K)
    o_idx = o_idx.reshape(B, R, K)
    rng = synth.rng_for(90 + case)
    for b in range(B):
        pth = synth.root_path(parent[b], int(rng.integers(T)))
        for p_, c_ in zip(pth[:-1], pth[1:]):
            if rng.random() >= 0.8:
                break
            tok[b, c_] = o_idx[b, p_, 0]
    tp, tr, _ = oracle.full_tree_template(dbr)
    o_ver = oracle.tree_verify(tok, parent, np.ascontiguousarray(o_idx[:, :T, 0]), md)
    o_next, o_par = oracle.tree_draft(np.ascontiguousarray(o_idx[:, T:, :].reshape(B, T, gamma, K)), o_ver["last"],
                                      o_ver["bonus"], tp, tr)
    # the three calls
    g_hidden, g_W = hidden.to(DEV), W.to(DEV)
    g_tok, g_par = torch.from_numpy(tok).to(DEV), torch.from_numpy(parent).to(DEV)
    idx, _ = api.ss_lm_head_argmax_topk(g_hidden, g_W, K)
    ver = api.ss_tree_verify(g_tok, g_par, idx, md, batch_stride=R * K, node_stride=K)
    nxt, npar = api.ss_tree_draft(idx, K, ver["last"], ver["bonus"], T, gamma, branching=dbr, batch_stride=R * K,
                                  offset=T * K)
    # the fused call, twice into the same outputs (nothing may depend on what a call leaves behind)
    out = api.ss_lm_head_verify_draft(g_hidden, g_W, K, g_tok, g_par, gamma, md, branching=dbr)
    out = api.ss_lm_head_verify_draft(g_hidden, g_W, K, g_tok, g_par, gamma, md, branching=dbr, out=out)
    torch.cuda.synchronize()
    for k in ("n_accept", "last", "bonus", "path", "out_tokens"):
        assert torch.equal(out[k], ver[k]), k
        assert np.array_equal(out[k].cpu().numpy(), o_ver[k]), k
    assert torch.equal(out["next_tok"], nxt) and torch.equal(out["next_parent"], npar)
    assert torch.equal(out["main_argmax"], idx.view(B, R, K)[:, :T, 0])
    assert np.array_equal(out["next_tok"].cpu().numpy(), o_next)
    assert np.array_equal(out["next_parent"].cpu().numpy(), o_par)
    assert int(o_ver["n_accept"].max()) >= 1 or T == 1          # the planted path was found


def test_fused_tail_with_a_device_template():
    # the template as device arrays (a pruned template: one node deeper than gamma gives -1)
    dtype, B, T, br, md, gamma, K, dbr, d, V = CASES[1]
    cfg = synth.scaled(synth.CONFIGS["c4"], B=B, T=T, branching=br, max_depth=md, gamma=gamma, K=K, d_model=d, vocab=V)
    inp = synth.make_lm_head_inputs(cfg, 7, N=B * cfg.R)
    parent = synth.make_trees(8, B, T, br, md)
    tok = synth.make_draft_tokens(9, parent, V)
    tmpl_parent = np.array([-1, 0, 0, 1, 1, 2, 3, 6, 7, 8], np.int32)      # node 9 sits at depth 5 > gamma
    tmpl_rank = np.array([0, 0, 1, 0, 3, 1, 0, 2, 0, 0], np.int32)
    g = [torch.from_numpy(a).to(DEV) for a in (tok, parent, tmpl_parent, tmpl_rank)]
    out = api.ss_lm_head_verify_draft(inp["hidden"].to(DEV), inp["W"].to(DEV), K, g[0], g[1], gamma, md,
                                      tmpl_parent=g[2], tmpl_rank=g[3])
    torch.cuda.synchronize()
    o_idx, _ = oracle.lm_head_topk(to_np_f32(inp["hidden"]), to_np_f32(inp["W"]), K)
    o_idx = o_idx.reshape(B, cfg.R, K)
    o_ver = oracle.tree_verify(tok, parent, np.ascontiguousarray(o_idx[:, :T, 0]), md)
    o_next, o_par = oracle.tree_draft(np.ascontiguousarray(o_idx[:, T:, :].reshape(B, T, gamma, K)), o_ver["last"],
                                      o_ver["bonus"], tmpl_parent, tmpl_rank)
    assert np.array_equal(out["next_tok"].cpu().numpy(), o_next)
    assert (out["next_tok"][:, 9] == -1).all()
    assert np.array_equal(out["out_tokens"].cpu().numpy(), o_ver["out_tokens"])


def test_c4_full_size_fused_tail():
    # workload c4 at full size (320 x 4096 x 32000), acceptance planted in the hidden states: the fused call
    # equals the three calls bit for bit, finds the planted accepted lengths, and the rows it merged (the main
    # rows, the stream rows of the last accepted node) agree with the oracle's logits for those rows
    cfg = synth.CONFIGS["c4"]
    B, T, R, K, gamma = cfg.B, cfg.T, cfg.R, cfg.K, cfg.gamma
    inp = synth.make_lm_head_inputs(cfg, 3)
    parent = synth.make_trees(3, B, T, cfg.branching, cfg.max_depth)
    tok = synth.make_draft_tokens(3, parent, cfg.vocab)
    planted = synth.plant_acceptance(3, parent, tok, inp["hidden"], inp["W"], R, p_match=0.8)
    g_h, g_W = inp["hidden"].to(DEV), inp["W"].to(DEV)
    g_tok, g_par = torch.from_numpy(tok).to(DEV), torch.from_numpy(parent).to(DEV)
    idx, _ = api.ss_lm_head_argmax_topk(g_h, g_W, K)
    ver = api.ss_tree_verify(g_tok, g_par, idx, cfg.max_depth, batch_stride=R * K, node_stride=K)
    nxt, npar = api.ss_tree_draft(idx, K, ver["last"], ver["bonus"], T, gamma, branching=cfg.draft_branching,
                                  batch_stride=R * K, offset=T * K)
    out = api.ss_lm_head_verify_draft(g_h, g_W, K, g_tok, g_par, gamma, cfg.max_depth, branching=cfg.draft_branching)
    torch.cuda.synchronize()
    for k in ("n_accept", "last", "bonus", "path", "out_tokens"):
        assert torch.equal(out[k], ver[k]), k
    assert torch.equal(out["next_tok"], nxt) and torch.equal(out["next_parent"], npar)
    assert np.array_equal(out["n_accept"].cpu().numpy(), planted) and planted.max() >= 1
    # oracle on the rows the tail read: B*T main rows (arg-max) and B*gamma stream rows (top-K)
    last = out["last"].cpu().numpy()
    h32, w32 = to_np_f32(inp["hidden"]), to_np_f32(inp["W"])
    main_rows = np.array([b * R + i for b in range(B) for i in range(T)])
    stream_rows = np.array([b * R + T + last[b] * gamma + j for b in range(B) for j in range(gamma)])
    o_main, o_mval, z_main = oracle.lm_head_topk(h32[main_rows], w32, 1, want_logits=True)
    tau = 1e-4 * np.abs(z_main).max()
    g_main = out["main_argmax"].cpu().numpy().reshape(-1)
    for n in np.nonzero(g_main != o_main[:, 0])[0]:
        assert abs(z_main[n, g_main[n]] - o_mval[n, 0]) <= tau
    o_top, o_tval, z_s = oracle.lm_head_topk(h32[stream_rows], w32, K, want_logits=True)
    tp, tr, td = oracle.full_tree_template(cfg.draft_branching)
    g_next = out["next_tok"].cpu().numpy()
    for b in range(B):
        assert g_next[b, 0] == out["bonus"][b].item()
        for i in range(1, len(tp)):
            j, want = td[i] - 1, o_top[b * gamma + td[i] - 1, tr[i]]
            if g_next[b, i] != want:      # a near tie inside tau may swap two ranks
                assert abs(z_s[b * gamma + j, g_next[b, i]] - o_tval[b * gamma + j, tr[i]]) <= tau
