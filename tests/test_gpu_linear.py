"""GPU parity of the dense projection y = x . W^T (n1) against the oracle.

Tolerance.  The kernel multiplies exactly (bf16 or fp32 inputs), accumulates in fp32 in an order of
its own and rounds a bf16 result once.  With S[n,v] = sum_e |x[n,e] W[v,e]|:
  fp32: |y - ref| <= 1e-5 * S        (d * 2^-24 is below 1e-5 for every d used here)
  bf16: |y - ref| <= 2^-8 * |ref| + 1e-5 * S   (one rounding to 8 significant bits, plus the sum)
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check(x, W, rows=None):
    y = api.ss_linear_rows(x.to(DEV), W.to(DEV))
    torch.cuda.synchronize()
    assert y.dtype == x.dtype and tuple(y.shape) == (x.shape[0], W.shape[0])
    y = to_np_f32(y.cpu()).astype(np.float64)
    rows = np.arange(x.shape[0]) if rows is None else np.asarray(rows)
    x32, w32 = to_np_f32(x)[rows], to_np_f32(W)
    ref = oracle.linear_rows(x32, w32)
    S = oracle.linear_rows(np.abs(x32), np.abs(w32))
    tol = 1e-5 * S + (2.0 ** -8 * np.abs(ref) if x.dtype == torch.bfloat16 else 0.0)
    err = np.abs(y[rows] - ref)
    bad = np.argwhere(err > tol)
    assert bad.size == 0, (bad[:5], err.max())


def _inputs(N, d, V, dtype, seed):
    cfg = synth.scaled(synth.CONFIGS["c4" if dtype == "bf16" else "c1"], vocab=V, d_model=d)
    inp = synth.make_lm_head_inputs(cfg, seed, N=N)
    return inp["hidden"], inp["W"]


@pytest.mark.parametrize("N,d,V", [(1, 32, 5), (33, 100, 1000), (7, 257, 64), (70, 64, 129), (5, 48, 13)])
def test_fp32_shapes(N, d, V):
    _check(*_inputs(N, d, V, "f32", 11))


# rows: one tile, a ragged second chunk of 320, several row tiles; outputs: below one tile, ragged, not a
# multiple of 8 (scalar stores), several tiles
@pytest.mark.parametrize("N,d,V", [(1, 64, 8), (40, 256, 100), (64, 128, 128), (65, 512, 136), (320, 256, 1000),
                                    (321, 64, 264), (700, 128, 300), (17, 4096, 504), (200, 1024, 1001)])
def test_bf16_shapes(N, d, V):
    _check(*_inputs(N, d, V, "bf16", 12))


def test_bf16_small_integers_bit_exact():
    # every product sum is an integer below 2^8 in magnitude: exact in fp32 and in bf16, any order
    rng = np.random.default_rng(13)
    N, d, V = 130, 64, 200
    x = torch.from_numpy(rng.integers(-1, 2, (N, d)).astype(np.float32)).to(torch.bfloat16)
    W = torch.from_numpy(rng.integers(-2, 3, (V, d)).astype(np.float32)).to(torch.bfloat16)
    y = api.ss_linear_rows(x.to(DEV), W.to(DEV)).cpu()
    ref = oracle.linear_rows(to_np_f32(x), to_np_f32(W))
    assert np.abs(ref).max() <= 128
    np.testing.assert_array_equal(to_np_f32(y).astype(np.float64), ref)


def test_c4_feed_forward_and_qkv_shapes_sampled_rows():
    # the rows of one step (B*R = 320) through the layer's maps: 4096 -> 11008, 11008 -> 4096 and 4096 -> 3*4096
    cfg = synth.CONFIGS["c4"]
    N = cfg.B * cfg.R
    for d, V, seed in ((4096, 11008, 21), (11008, 4096, 22), (4096, 12288, 23)):
        x, W = _inputs(N, d, V, "bf16", seed)
        _check(x, W, rows=[0, 63, 64, 191, 319])


def test_output_tensor_is_used_and_rows_past_n_untouched():
    x, W = _inputs(70, 128, 72, "bf16", 14)
    y = torch.full((71, 72), 7.0, dtype=torch.bfloat16, device=DEV)
    out = api.ss_linear_rows(x.to(DEV), W.to(DEV), y[:70])
    torch.cuda.synchronize()
    assert out.data_ptr() == y.data_ptr()
    assert (y[70] == 7.0).all()
    ref = oracle.linear_rows(to_np_f32(x), to_np_f32(W))
    np.testing.assert_allclose(to_np_f32(y[:70].cpu()), ref, rtol=2.0 ** -7, atol=1e-3)


def test_empty_and_rejected_arguments():
    W = torch.zeros(16, 64, dtype=torch.bfloat16, device=DEV)
    y = api.ss_linear_rows(torch.zeros(0, 64, dtype=torch.bfloat16, device=DEV), W)
    assert tuple(y.shape) == (0, 16)
    with pytest.raises(api.SSError):      # bf16 needs d % 64 == 0
        api.ss_linear_rows(torch.zeros(4, 48, dtype=torch.bfloat16, device=DEV), torch.zeros(16, 48, dtype=torch.bfloat16, device=DEV))
    with pytest.raises(ValueError):
        api.ss_linear_rows(torch.zeros(4, 64, dtype=torch.bfloat16, device=DEV), torch.zeros(16, 128, dtype=torch.bfloat16, device=DEV))
