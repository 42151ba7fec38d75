"""Pruned trees on the GPU (Sec. 3.2.3): the calls that take n_nodes, or the list of kept rows, against the
oracle's pruned-tree variants; kept rows equal what the plain calls give for them, rows of padding nodes are left untouched; and pruning pays: with half the nodes gone the attention of a long GQA
tree and the LM head take measurably less time."""
import numpy as np
import pytest
import torch

import oracle
from helpers import rel_err, to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _padded_parents(parent, n_nodes):
    p = parent.clone()
    for b, n in enumerate(n_nodes.tolist()):
        p[b, n:] = 0            # as ss_tree_prune leaves padding nodes: children of the root
    return p


def _timed(fn, iters=60, warm=20):
    for _ in range(warm):
        fn()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    s.record()
    for _ in range(iters):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) * 1000.0 / iters


def test_live_rows_match_the_oracle():
    for B, T, gamma in ((1, 1, 0), (3, 7, 2), (5, 64, 8), (40, 16, 4)):
        n = synth.rng_for(B * 100 + T).integers(-2, T + 3, size=B).astype(np.int32)      # out-of-range counts are clamped
        rows, n_live = api.ss_live_rows(torch.from_numpy(n).to(DEV), T, gamma)
        want = oracle.live_rows(n, T, gamma)
        assert int(n_live.item()) == want.size and np.array_equal(rows.cpu().numpy()[:want.size], want)


@pytest.mark.parametrize("case", ["f32", "bf16_unsplit", "bf16_two_splits", "bf16_many_splits", "bf16_gqa_chunks"])
def test_attention_on_pruned_trees(case):
    if case == "f32":
        cfg, split = synth.scaled(synth.CONFIGS["c1"], B=3, T=8, gamma=3, L_min=0, L_max=300), 0
    elif case == "bf16_gqa_chunks":
        cfg, split = synth.scaled(synth.CONFIGS["c5"], B=2, L_min=300, L_max=900), 0                 # 160 rows x 4 heads: 8 row chunks
    else:
        cfg = synth.scaled(synth.CONFIGS["c2"], B=3, H=4, Hkv=2, T=16, gamma=4, L_min=100, L_max=700)
        split = {"bf16_unsplit": 4096, "bf16_two_splits": 352, "bf16_many_splits": 64}[case]
    inp = synth.make_msa_inputs(cfg, 31)
    n_nodes = torch.tensor([[5, cfg.T, 1], [cfg.T // 2, 3]][cfg.B == 2][:cfg.B], dtype=torch.int32)
    parent = _padded_parents(inp["parent"], n_nodes)
    d = {k: (v.to(DEV) if isinstance(v, torch.Tensor) else v) for k, v in inp.items()}
    args = (d["q"], d["k_new"], d["v_new"], d["k_cache"], d["v_cache"], d["block_table"], d["seq_lens"], parent.to(DEV),
            cfg.gamma, d["scale"])
    prev = api.ss_msa_set_split_keys(split)
    try:
        got = api.ss_msa_attention(*args, n_nodes=n_nodes.to(DEV), out=torch.full_like(d["q"], 3.0))
        plain = api.ss_msa_attention(*args)
        torch.cuda.synchronize()
    finally:
        api.ss_msa_set_split_keys(prev)
    f = to_np_f32
    want = oracle.msa_attention_pruned(f(inp["q"]), f(inp["k_new"]), f(inp["v_new"]), f(inp["k_cache"]), f(inp["v_cache"]),
                                       inp["block_table"].numpy(), inp["seq_lens"].numpy(), parent.numpy(), cfg.gamma,
                                       inp["scale"], n_nodes.numpy())
    R = cfg.R
    keep = np.zeros(cfg.B * R, bool)
    keep[oracle.live_rows(n_nodes.numpy(), cfg.T, cfg.gamma)] = True
    keep = keep.reshape(cfg.B, R)
    tol = 1e-5 if cfg.dtype == "f32" else 2e-2
    assert rel_err(f(got)[keep], want[keep]) <= tol
    assert rel_err(f(got)[keep], f(plain)[keep]) <= tol    # the plain call's kept rows, up to summation order
    assert bool((got[torch.from_numpy(~keep).to(DEV)] == 3.0).all())   # rows of padding nodes: untouched


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dense_maps_on_the_kept_rows(dtype):
    cfg = synth.scaled(synth.CONFIGS["c4"], dtype=dtype, B=3, T=9, gamma=3, vocab=1003, d_model=192, K=3)
    N, K = cfg.B * cfg.R, cfg.K
    lm = synth.make_lm_head_inputs(cfg, 17, device=DEV)
    n_nodes = torch.tensor([4, 9, 1], dtype=torch.int32, device=DEV)
    live = api.ss_live_rows(n_nodes, cfg.T, cfg.gamma)
    rows = oracle.live_rows(n_nodes.cpu().numpy(), cfg.T, cfg.gamma)
    dead = np.setdiff1d(np.arange(N), rows)
    # (launches with one row chunk start every vocabulary tile at another feature block, which changes the order of
    # the fp32 sums; with that switched off the kept rows are bit-identical whatever the launch is shaped for)
    api.ss_lm_set_stagger(0)
    for plan in (0, 32, 64):                                  # shaped for all rows, for fewer than are kept, for about as many
        y = torch.full((N, cfg.vocab), 7.0, dtype=cfg.torch_dtype, device=DEV)
        api.ss_linear_rows(lm["hidden"], lm["W"], y=y, live=live, plan_rows=plan)
        full = api.ss_linear_rows(lm["hidden"], lm["W"])
        torch.cuda.synchronize()
        assert torch.equal(y[rows], full[rows]) and bool((y[dead] == 7.0).all())
        idx = torch.full((N, K), -5, dtype=torch.int32, device=DEV)
        val = torch.full((N, K), -5.0, dtype=torch.float32, device=DEV)
        api.ss_lm_head_argmax_topk(lm["hidden"], lm["W"], K, idx=idx, val=val, live=live, plan_rows=plan)
        fidx, fval = api.ss_lm_head_argmax_topk(lm["hidden"], lm["W"], K)
        torch.cuda.synchronize()
        assert torch.equal(idx[rows], fidx[rows]) and torch.equal(val[rows], fval[rows])
        assert bool((idx[dead] == -5).all()) and bool((val[dead] == -5.0).all())
    api.ss_lm_set_stagger(-1)
    # against the oracle's variant (the plain calls are checked against the plain oracle elsewhere)
    o_idx, o_val, z = oracle.lm_head_topk_live(to_np_f32(lm["hidden"]), to_np_f32(lm["W"]), K, rows, want_logits=True)
    tau = (1e-5 if dtype == "f32" else 1e-4) * np.abs(z).max()
    g = idx.cpu().numpy()
    for n, k in zip(*np.nonzero(g[rows] != o_idx[rows])):
        assert abs(z[rows[n], g[rows[n], k]] - o_val[rows[n], k]) <= tau
    y_ref = oracle.linear_rows_live(to_np_f32(lm["hidden"]), to_np_f32(lm["W"]), rows)
    assert rel_err(to_np_f32(y)[rows], y_ref[rows]) <= (1e-5 if dtype == "f32" else 2e-2)


def test_fused_tail_on_a_pruned_tree_equals_the_chain():
    cfg = synth.scaled(synth.CONFIGS["c4"], B=3, T=9, gamma=3, branching=(3, 2, 2), max_depth=3, vocab=1500, d_model=256, K=2,
                       draft_branching=(2, 2, 1))
    N = cfg.B * cfg.R
    lm = synth.make_lm_head_inputs(cfg, 23, device=DEV)
    parent0 = synth.make_trees(23, cfg.B, cfg.T, cfg.branching, cfg.max_depth)
    tok0 = synth.make_draft_tokens(23, parent0, cfg.vocab)
    prob = torch.rand(cfg.B, cfg.T, generator=torch.Generator().manual_seed(3)).to(DEV)
    pr = api.ss_tree_prune(torch.from_numpy(tok0).to(DEV), torch.from_numpy(parent0).to(DEV), prob, 0.35)
    live = api.ss_live_rows(pr["n_nodes"], cfg.T, cfg.gamma)
    assert 0 < int(live[1].item()) < N
    a = api.ss_lm_head_verify_draft(lm["hidden"], lm["W"], cfg.K, pr["tok"], pr["parent"], cfg.gamma, cfg.max_depth,
                                    branching=cfg.draft_branching, live=live, plan_rows=int(live[1].item()))
    b = api.ss_lm_head_verify_draft(lm["hidden"], lm["W"], cfg.K, pr["tok"], pr["parent"], cfg.gamma, cfg.max_depth,
                                    branching=cfg.draft_branching)
    torch.cuda.synchronize()
    for k in ("n_accept", "last", "bonus", "path", "out_tokens", "next_tok", "next_parent"):
        assert torch.equal(a[k], b[k]), k
    n = pr["n_nodes"].cpu().numpy()
    am_a, am_b = a["main_argmax"].cpu().numpy(), b["main_argmax"].cpu().numpy()
    for bb in range(cfg.B):
        assert np.array_equal(am_a[bb, :n[bb]], am_b[bb, :n[bb]])      # arg-max of kept nodes (the others are not computed)


def test_pruning_pays():
    """Half of every tree pruned away: the compute-bound attention of long GQA trees (c5's shape at a quarter of its
    prefix) and the c4 LM head shaped for the surviving rows both get faster."""
    cfg = synth.scaled(synth.CONFIGS["c5"], L_min=8192, L_max=8192)
    inp = synth.make_msa_inputs(cfg, 5, device=DEV)
    n_nodes = torch.full((cfg.B,), cfg.T // 2, dtype=torch.int32, device=DEV)
    parent = _padded_parents(inp["parent"].cpu(), n_nodes.cpu()).to(DEV)
    out = torch.empty_like(inp["q"])
    ws = api.ss_msa_workspace(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, inp["block_table"].shape[1] * cfg.page, api.SS_BF16, DEV)
    call = lambda nn: api.ss_msa_attention(inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["block_table"],
                                           inp["seq_lens"], parent, cfg.gamma, inp["scale"], out=out, workspace=ws, n_nodes=nn)
    t_full, t_half = _timed(lambda: call(None)), _timed(lambda: call(n_nodes))
    print("attention, c5 shape at prefix 8192: all nodes %.1f us, half pruned %.1f us" % (t_full, t_half), flush=True)
    assert t_half < 0.85 * t_full

    c4 = synth.CONFIGS["c4"]
    N = c4.B * c4.R
    lm = synth.make_lm_head_inputs(c4, 1, device=DEV)
    nn = torch.full((c4.B,), c4.T // 2, dtype=torch.int32, device=DEV)
    live = api.ss_live_rows(nn, c4.T, c4.gamma)
    idx = torch.empty((N, c4.K), dtype=torch.int32, device=DEV)
    val = torch.empty((N, c4.K), dtype=torch.float32, device=DEV)
    lws = torch.empty(api.ss_lm_head_workspace_bytes(N, c4.d_model, c4.vocab, c4.K, api.SS_BF16), dtype=torch.uint8, device=DEV)
    t_all = _timed(lambda: api.ss_lm_head_argmax_topk(lm["hidden"], lm["W"], c4.K, idx=idx, val=val, workspace=lws))
    t_live = _timed(lambda: api.ss_lm_head_argmax_topk(lm["hidden"], lm["W"], c4.K, idx=idx, val=val, workspace=lws, live=live,
                                                        plan_rows=N // 2))
    print("LM head 320 x 4096 x 32000: all rows %.1f us, half of them listed %.1f us" % (t_all, t_live), flush=True)
    assert t_live < 0.85 * t_all
