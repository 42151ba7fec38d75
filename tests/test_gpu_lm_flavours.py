"""Every shape of the MFMA LM-head kernel (4 waves x 1..6 row tiles, 8 waves x 1..5 row tiles) behind its three
epilogues, forced through the tuning variables, against the oracle.  The host plan picks only some of them for
the sizes the other tests use; this one makes sure all are right.  Tolerances as in the tests of the entry points."""

import numpy as np
import pytest
import torch

import oracle
from helpers import to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FLAVOURS = ["1", "2", "3", "4", "5", "6", "1w", "2w", "3w", "4w", "5w"]


@pytest.fixture(scope="module")
def problem():
    # 200 rows (several row chunks for small tiles, a ragged last chunk), 5 feature blocks (more than the buffers
    # of either shape), 1000 outputs (ragged last tile of 128 and of 256)
    cfg = synth.scaled(synth.CONFIGS["c4"], vocab=1000, d_model=320)
    inp = synth.make_lm_head_inputs(cfg, 41, N=200)
    x, W = inp["hidden"], inp["W"]
    x32, w32 = to_np_f32(x), to_np_f32(W)
    ref = dict(z=oracle.linear_rows(x32, w32), S=oracle.linear_rows(np.abs(x32), np.abs(w32)),
               lse=oracle.lm_head_lse(x32, w32))
    ref["idx"], ref["val"], _ = oracle.lm_head_topk(x32, w32, 4, want_logits=True)
    return x.to(DEV), W.to(DEV), ref


@pytest.fixture(autouse=True)
def _automatic_again():
    yield
    api.ss_lm_set_flavour(False, None)
    api.ss_lm_set_flavour(True, None)
    api.ss_lm_set_stagger(-1)


@pytest.mark.parametrize("flavour", FLAVOURS)
def test_projection(problem, flavour):
    x, W, ref = problem
    api.ss_lm_set_flavour(True, flavour)
    y = to_np_f32(api.ss_linear_rows(x, W).cpu()).astype(np.float64)
    assert (np.abs(y - ref["z"]) <= 2.0 ** -8 * np.abs(ref["z"]) + 1e-5 * ref["S"]).all()


@pytest.mark.parametrize("flavour", FLAVOURS)
def test_top_k(problem, flavour):
    x, W, ref = problem
    api.ss_lm_set_flavour(False, flavour)
    idx, val = api.ss_lm_head_argmax_topk(x, W, 4)
    torch.cuda.synchronize()
    idx, val = idx.cpu().numpy(), val.cpu().numpy()
    tau = 1e-4 * np.abs(ref["z"]).max()
    z_at = np.take_along_axis(ref["z"], idx.astype(np.int64), axis=1)
    assert (np.abs(val - z_at) <= tau).all()
    differs = idx != ref["idx"]
    assert (np.abs(z_at - ref["val"])[differs] <= tau).all() and differs.sum() <= 1


@pytest.mark.parametrize("flavour", FLAVOURS)
def test_log_sum_exp(problem, flavour):
    x, W, ref = problem
    api.ss_lm_set_flavour(False, flavour)
    lse = api.ss_lm_head_logsumexp(x, W).cpu().numpy()
    assert (np.abs(lse - ref["lse"]) <= 2e-3 * np.maximum(1.0, np.abs(ref["lse"]))).all()


@pytest.mark.parametrize("K", [1, 8])
@pytest.mark.parametrize("flavour", ["2", "6", "1w", "3w", "5w"])
def test_top_1_and_top_8(problem, flavour, K):
    # the other two widths of the candidate lists (K = 1 and K = 5..8) in both shapes
    x, W, ref = problem
    api.ss_lm_set_flavour(False, flavour)
    idx, val = api.ss_lm_head_argmax_topk(x, W, K)
    torch.cuda.synchronize()
    idx, val = idx.cpu().numpy(), val.cpu().numpy()
    o_idx, o_val = oracle.lm_head_topk(to_np_f32(x.cpu()), to_np_f32(W.cpu()), K)[:2]
    tau = 1e-4 * np.abs(ref["z"]).max()
    z_at = np.take_along_axis(ref["z"], idx.astype(np.int64), axis=1)
    assert (np.abs(val - z_at) <= tau).all()
    differs = idx != o_idx
    assert (np.abs(z_at - o_val)[differs] <= tau).all() and differs.sum() <= 2
    for n in range(idx.shape[0]):
        assert len(set(idx[n].tolist())) == K


@pytest.mark.parametrize("stagger", [1, 3, 7])
@pytest.mark.parametrize("flavour", ["1", "3", "6", "2w", "5w"])
def test_staggered_starting_blocks(problem, flavour, stagger):
    # every vocabulary tile walks the 5 feature blocks from its own start and wraps around (the host does this only
    # for launches with one row chunk; here it is forced for all shapes): same results within the same bounds
    x, W, ref = problem
    api.ss_lm_set_flavour(False, flavour)
    api.ss_lm_set_flavour(True, flavour)
    api.ss_lm_set_stagger(stagger)
    y = to_np_f32(api.ss_linear_rows(x, W).cpu()).astype(np.float64)
    assert (np.abs(y - ref["z"]) <= 2.0 ** -8 * np.abs(ref["z"]) + 1e-5 * ref["S"]).all()
    lse = api.ss_lm_head_logsumexp(x, W).cpu().numpy()
    assert (np.abs(lse - ref["lse"]) <= 2e-3 * np.maximum(1.0, np.abs(ref["lse"]))).all()
    idx, val = api.ss_lm_head_argmax_topk(x, W, 4)
    idx, val = idx.cpu().numpy(), val.cpu().numpy()
    tau = 1e-4 * np.abs(ref["z"]).max()
    z_at = np.take_along_axis(ref["z"], idx.astype(np.int64), axis=1)
    assert (np.abs(val - z_at) <= tau).all()
    differs = idx != ref["idx"]
    assert (np.abs(z_at - ref["val"])[differs] <= tau).all() and differs.sum() <= 1
