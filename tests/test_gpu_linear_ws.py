"""GPU parity of the dense projection with a workspace (n1, feature dimension cut between workgroups) against the
oracle, with the tolerance of test_gpu_linear.py: the operation is the same, only the order of the fp32 sum differs.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(N, d, V, dtype, seed):
    cfg = synth.scaled(synth.CONFIGS["c4" if dtype == "bf16" else "c1"], vocab=V, d_model=d)
    inp = synth.make_lm_head_inputs(cfg, seed, N=N)
    return inp["hidden"], inp["W"]


def _check(x, W, rows=None, want_cut=None):
    N, d = x.shape
    V = W.shape[0]
    code = api.SS_BF16 if x.dtype == torch.bfloat16 else api.SS_F32
    cut = api.ss_linear_rows_splits(N, d, V, code)
    if want_cut is not None:
        assert (cut > 1) == want_cut, cut
    y = api.ss_linear_rows_ws(x.to(DEV), W.to(DEV))
    torch.cuda.synchronize()
    assert y.dtype == x.dtype and tuple(y.shape) == (N, V)
    y = to_np_f32(y.cpu()).astype(np.float64)
    rows = np.arange(N) if rows is None else np.asarray(rows)
    x32, w32 = to_np_f32(x)[rows], to_np_f32(W)
    ref = oracle.linear_rows(x32, w32)
    S = oracle.linear_rows(np.abs(x32), np.abs(w32))
    tol = 1e-5 * S + (2.0 ** -8 * np.abs(ref) if x.dtype == torch.bfloat16 else 0.0)
    err = np.abs(y[rows] - ref)
    bad = np.argwhere(err > tol)
    assert bad.size == 0, (bad[:5], err.max())
    return cut


# few outputs, many features: cut.  Rows: one tile, ragged chunks; outputs: below a tile, not a multiple of 4 or 8
@pytest.mark.parametrize("N,d,V", [(96, 2048, 250), (17, 4096, 500), (320, 4096, 1000), (33, 8192, 129), (200, 2048, 64),
                                    (1, 4096, 8), (161, 4096, 257)])
def test_cut_shapes(N, d, V):
    _check(*_inputs(N, d, V, "bf16", 31), want_cut=True)


@pytest.mark.parametrize("N,d,V", [(100, 1024, 777), (320, 256, 12288), (64, 64, 128)])
def test_uncut_shapes_equal_the_plain_call_bit_for_bit(N, d, V):
    x, W = _inputs(N, d, V, "bf16", 32)
    assert _check(x, W, want_cut=False) == 1
    a = api.ss_linear_rows_ws(x.to(DEV), W.to(DEV))
    b = api.ss_linear_rows(x.to(DEV), W.to(DEV))
    assert torch.equal(a, b)


def test_fp32_goes_through_the_plain_kernel():
    x, W = _inputs(33, 100, 1000, "f32", 33)
    _check(x, W, want_cut=False)


def test_c4_down_and_output_maps_every_row():
    # the two maps of a layer that the cut is for: 11008 -> 4096 and 4096 -> 4096 on the 320 rows of a step
    cfg = synth.CONFIGS["c4"]
    N = cfg.B * cfg.R
    for d, V, seed in ((11008, 4096, 34), (4096, 4096, 35)):
        x, W = _inputs(N, d, V, "bf16", seed)
        assert _check(x, W, want_cut=True) == 4


def test_small_integers_bit_exact_and_deterministic():
    # every product sum is an integer below 2^8 in magnitude: exact in fp32 and in bf16, in any order
    rng = np.random.default_rng(36)
    N, d, V = 130, 2048, 200
    x = torch.from_numpy((rng.random((N, d)) < 0.02).astype(np.float32) * rng.integers(-1, 2, (N, d))).to(torch.bfloat16)
    W = torch.from_numpy(rng.integers(-2, 3, (V, d)).astype(np.float32)).to(torch.bfloat16)
    assert api.ss_linear_rows_splits(N, d, V, api.SS_BF16) > 1
    y = api.ss_linear_rows_ws(x.to(DEV), W.to(DEV)).cpu()
    ref = oracle.linear_rows(to_np_f32(x), to_np_f32(W))
    assert np.abs(ref).max() <= 256
    np.testing.assert_array_equal(to_np_f32(y).astype(np.float64), ref)
    x2, W2 = _inputs(96, 2048, 250, "bf16", 37)
    a = api.ss_linear_rows_ws(x2.to(DEV), W2.to(DEV))
    b = api.ss_linear_rows_ws(x2.to(DEV), W2.to(DEV))
    assert torch.equal(a, b)


def test_workspace_is_checked_and_guard_bytes_survive():
    x, W = _inputs(96, 2048, 250, "bf16", 38)
    need = api.ss_linear_rows_workspace_bytes(96, 2048, 250, api.SS_BF16)
    assert need > 256
    with pytest.raises(api.SSError) as e:
        api.ss_linear_rows_ws(x.to(DEV), W.to(DEV), workspace=torch.empty(need - 1, dtype=torch.uint8, device=DEV))
    assert e.value.code == 4  # SS_ERR_WORKSPACE
    guard = 4096
    ws = torch.full((need + 2 * guard,), 0xA5, dtype=torch.uint8, device=DEV)
    ybuf = torch.full((96 + 2, 250), 7.0, dtype=torch.bfloat16, device=DEV)
    y = api.ss_linear_rows_ws(x.to(DEV), W.to(DEV), y=ybuf[1:97], workspace=ws[guard:guard + need])
    torch.cuda.synchronize()
    assert (ws[:guard] == 0xA5).all() and (ws[guard + need:] == 0xA5).all()
    assert (ybuf[0] == 7.0).all() and (ybuf[97] == 7.0).all()
    assert torch.equal(y, api.ss_linear_rows_ws(x.to(DEV), W.to(DEV)))
