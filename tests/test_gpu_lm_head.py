"""GPU parity of the LM head with fused arg-max / top-K (a3) against the oracle.

Indices must match the oracle exactly wherever the oracle's logits separate the competing tokens
by more than tau = 1e-5 * max|z| (fp32) or 1e-4 * max|z| (bf16 storage, fp32 accumulation over d in
a different order than the oracle's double sum); inside tau either order is accepted and such
positions are counted.  Values: |val - z[idx]| <= tau.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _compare(hidden, W, K, rows=None, tau_rel=None):
    idx, val = api.ss_lm_head_argmax_topk(hidden.to(DEV), W.to(DEV), K)
    torch.cuda.synchronize()
    idx, val = idx.cpu().numpy(), val.cpu().numpy()
    rows = np.arange(hidden.shape[0]) if rows is None else np.asarray(rows)
    h32, w32 = to_np_f32(hidden)[rows], to_np_f32(W)
    o_idx, o_val, z = oracle.lm_head_topk(h32, w32, K, want_logits=True)
    if tau_rel is None:
        tau_rel = 1e-5 if hidden.dtype == torch.float32 else 1e-4
    tau = tau_rel * np.abs(z).max()
    near_ties = 0
    for j, n in enumerate(rows):
        assert len(set(idx[n].tolist())) == K                      # K distinct tokens
        for k in range(K):
            zi = z[j, idx[n, k]]
            assert abs(val[n, k] - zi) <= tau, (n, k)
            if idx[n, k] != o_idx[j, k]:
                assert abs(zi - o_val[j, k]) <= tau, (n, k, idx[n, k], o_idx[j, k])
                near_ties += 1
    return near_ties


def test_c1_fp32():
    cfg = synth.CONFIGS["c1"]
    inp = synth.make_lm_head_inputs(cfg, 1)
    assert _compare(inp["hidden"], inp["W"], cfg.K) == 0


@pytest.mark.parametrize("N,d,V,K", [(1, 32, 5, 5), (33, 100, 1000, 8), (7, 257, 64, 1), (70, 64, 129, 3)])
def test_fp32_shapes(N, d, V, K):
    cfg = synth.scaled(synth.CONFIGS["c1"], vocab=V, d_model=d)
    inp = synth.make_lm_head_inputs(cfg, 2, N=N)
    assert _compare(inp["hidden"], inp["W"], K) == 0


@pytest.mark.parametrize("N,d,V,K", [(80, 512, 3000, 4), (1, 64, 128, 1), (100, 1024, 777, 8), (320, 256, 1000, 2),
                                      (400, 128, 300, 4), (17, 4096, 500, 4),
                                      (50, 128, 700, 4), (64, 192, 520, 3)])    # 2 and 3 feature blocks, one row chunk
def test_bf16_shapes(N, d, V, K):
    cfg = synth.scaled(synth.CONFIGS["c4"], vocab=V, d_model=d)
    inp = synth.make_lm_head_inputs(cfg, 3, N=N)
    assert _compare(inp["hidden"], inp["W"], K) <= 1


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_exact_ties_go_to_lower_index(dtype):
    rng = synth.rng_for(4)
    N, d, V, K = 40, 128, 700, 4
    h = torch.from_numpy(rng.standard_normal((N, d)).astype(np.float32)).to(dtype)
    W = torch.from_numpy((0.02 * rng.standard_normal((V, d))).astype(np.float32)).to(dtype)
    # identical weight rows give bit-identical logits on both sides; plant them as each row's maximum,
    # inside one vocabulary tile and across tiles
    for n in range(N):
        t = (h[n].float() * 0.5).to(dtype)
        for v in ((3 * n + 1) % V, (3 * n + 2) % V, (3 * n + 300) % V):
            W[v] = t
    idx, val = api.ss_lm_head_argmax_topk(h.to(DEV), W.to(DEV), K)
    torch.cuda.synchronize()
    o_idx, o_val = oracle.lm_head_topk(to_np_f32(h), to_np_f32(W), K)
    got = idx.cpu().numpy()
    for n in range(N):
        want3 = sorted([(3 * n + 1) % V, (3 * n + 2) % V, (3 * n + 300) % V])
        if o_idx[n, :3].tolist() == want3:      # the planted rows won (they do unless a later row overwrote them)
            assert got[n, :3].tolist() == want3
            assert val[n, 0] == val[n, 1] == val[n, 2]


def test_c4_bf16_full_size_sampled_rows():
    # the whole 320 x 4096 x 32000 GEMM runs on the GPU; the oracle checks 48 sampled rows over all 32000 tokens
    cfg = synth.CONFIGS["c4"]
    inp = synth.make_lm_head_inputs(cfg, 1)
    rows = synth.rng_for(77).choice(cfg.B * cfg.R, 48, replace=False)
    ties = _compare(inp["hidden"], inp["W"], cfg.K, rows=np.sort(rows))
    print("near ties inside tau: %d of %d" % (ties, 48 * cfg.K), flush=True)
    assert ties <= 2


def test_planted_argmax_is_found():
    cfg = synth.scaled(synth.CONFIGS["c4"], B=2, vocab=5000, d_model=1024)
    inp = synth.make_lm_head_inputs(cfg, 5)
    parent = synth.make_trees(5, cfg.B, cfg.T, cfg.branching, cfg.max_depth)
    tok = synth.make_draft_tokens(5, parent, cfg.vocab)
    planted = synth.plant_acceptance(5, parent, tok, inp["hidden"], inp["W"], cfg.R, p_match=1.0)
    idx, _ = api.ss_lm_head_argmax_topk(inp["hidden"].to(DEV), inp["W"].to(DEV), 1)
    a = idx.cpu().numpy().reshape(cfg.B, cfg.R)[:, :cfg.T]
    r = oracle.tree_verify(tok, parent, a, cfg.max_depth)
    assert np.array_equal(r["n_accept"], planted) and planted.max() >= 1


def test_candidates_only_is_a_profiling_aid_that_leaves_the_outputs_alone():
    # while it is on the call stops after the matrix kernel: idx / val keep what they held; off again, same results as before
    cfg = synth.scaled(synth.CONFIGS["c4"], vocab=1500, d_model=256)
    inp = synth.make_lm_head_inputs(cfg, 5, N=96)
    h, W = inp["hidden"].to(DEV), inp["W"].to(DEV)
    want_idx, want_val = api.ss_lm_head_argmax_topk(h, W, 4)
    idx = torch.full_like(want_idx, -7)
    val = torch.full_like(want_val, -7.0)
    assert api.ss_lm_set_candidates_only(True) is False
    try:
        api.ss_lm_head_argmax_topk(h, W, 4, idx=idx, val=val)
        torch.cuda.synchronize()
        assert (idx == -7).all() and (val == -7.0).all()
    finally:
        assert api.ss_lm_set_candidates_only(False) is True
    api.ss_lm_head_argmax_topk(h, W, 4, idx=idx, val=val)
    assert torch.equal(idx, want_idx) and torch.equal(val, want_val)
