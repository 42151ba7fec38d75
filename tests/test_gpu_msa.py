"""GPU parity of multi-stream attention (a2) against the oracle on the same seeded inputs.

Tolerances (per tensor, err = max |gpu-ref| / (|ref| + rms(ref))):
  fp32: 1e-5.   bf16 storage: 2e-2 (observed ~4e-3: output rounding 2^-9 plus bf16 probabilities).
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import oracle_subproblem, rel_err, to_np_f32
from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"f32": 1e-5, "bf16": 2e-2}


def _to_dev(inp):
    return {k: (v.to(DEV) if isinstance(v, torch.Tensor) else v) for k, v in inp.items()}


def _gpu(inp, gamma, flags=0):
    d = _to_dev(inp)
    out = api.ss_msa_attention(d["q"], d["k_new"], d["v_new"], d["k_cache"], d["v_cache"], d["block_table"],
                               d["seq_lens"], d["parent"], gamma, d["scale"], flags)
    torch.cuda.synchronize()
    return out


def _oracle(inp, gamma, flags=0):
    return oracle.msa_attention(to_np_f32(inp["q"]), to_np_f32(inp["k_new"]), to_np_f32(inp["v_new"]),
                                to_np_f32(inp["k_cache"]), to_np_f32(inp["v_cache"]), inp["block_table"].numpy(),
                                inp["seq_lens"].numpy(), inp["parent"].numpy(), gamma, inp["scale"], flags)


def _check(cfg, seed, flags=0, lens=None, split=0):
    inp = synth.make_msa_inputs(cfg, seed)
    if lens is not None:
        inp["seq_lens"] = torch.tensor(lens, dtype=torch.int32)
    prev = api.ss_msa_set_split_keys(split)
    try:
        got = _gpu(inp, cfg.gamma, flags)
    finally:
        api.ss_msa_set_split_keys(prev)
    want = _oracle(inp, cfg.gamma, flags)
    assert torch.isfinite(got.float()).all()
    err = rel_err(to_np_f32(got), want)
    assert err <= TOL[cfg.dtype], (cfg.name, err)
    return err


# ---------------------------------------------------------------- fp32 path
def test_c1_fp32_full():
    _check(synth.CONFIGS["c1"], 1)


@pytest.mark.parametrize("flags", [0, api.SS_STREAM_EXCLUDE_SELF])
@pytest.mark.parametrize("D,H,Hkv", [(64, 4, 4), (128, 4, 2), (64, 6, 1)])
def test_fp32_shapes(D, H, Hkv, flags):
    cfg = synth.scaled(synth.CONFIGS["c1"], B=2, D=D, H=H, Hkv=Hkv, L_min=40, L_max=200, T=11, gamma=2)
    _check(cfg, 2, flags)


@pytest.mark.parametrize("lens", [[0, 1], [63, 64], [65, 130], [200, 7]])
def test_fp32_ragged_and_empty_prefix(lens):
    cfg = synth.scaled(synth.CONFIGS["c1"], B=2, L_min=200, L_max=200, T=5, gamma=3)
    _check(cfg, 3, lens=lens)


def test_fp32_split_invariance():
    cfg = synth.scaled(synth.CONFIGS["c1"], B=2, L_min=300, L_max=700, T=8, gamma=3)
    errs = [_check(cfg, 4, split=s) for s in (0, 128, 256, 1024)]
    assert max(errs) <= 1e-5


# ---------------------------------------------------------------- bf16 MFMA path
def test_c2_bf16_full():
    # the whole config: 32 heads x 128, prefix 2048, 16-node tree x 4 streams, 16-token pages
    _check(synth.CONFIGS["c2"], 1)


@pytest.mark.parametrize("T,gamma", [(1, 0), (1, 4), (3, 1), (4, 3), (5, 4), (7, 4), (13, 4), (16, 4), (20, 4), (64, 8)])
def test_bf16_row_tilings(T, gamma):
    # R = 1 .. 576 rows: every query-tile count of the kernel, padded tiles and several row chunks
    md = max(1, min(T - 1, 4))
    cfg = synth.scaled(synth.CONFIGS["c2"], B=2, H=4, Hkv=4, L_min=100, L_max=300, T=T, gamma=gamma,
                       branching=(4, 3, 2, 2), max_depth=md)
    _check(cfg, 10 + T)


@pytest.mark.parametrize("lens", [[0, 0], [1, 31], [32, 33], [127, 128], [129, 1000], [4095, 4096]])
def test_bf16_ragged_lengths(lens):
    cfg = synth.scaled(synth.CONFIGS["c2"], B=2, H=2, Hkv=2, L_min=4096, L_max=4096)
    _check(cfg, 5, lens=lens)


@pytest.mark.parametrize("page", [16, 32, 64])
@pytest.mark.parametrize("split", [0, 96, 128, 384, 736, 8192])
def test_bf16_pages_and_splits(page, split):
    cfg = synth.scaled(synth.CONFIGS["c2"], B=3, H=4, Hkv=4, L_min=500, L_max=1500, page=page)
    _check(cfg, 6, split=split)


@pytest.mark.parametrize("flags", [0, api.SS_STREAM_EXCLUDE_SELF])
def test_bf16_gqa_folded_rows(flags):
    # c5's shape at a short prefix: 4 query heads per KV head, 32-node trees -> 640 folded rows in 8 chunks
    cfg = synth.scaled(synth.CONFIGS["c5"], B=2, H=8, Hkv=2, L_min=700, L_max=1100)
    _check(cfg, 7, flags)


def test_bf16_head_dim_64():
    cfg = synth.scaled(synth.CONFIGS["c2"], B=2, H=4, Hkv=2, D=64, L_min=300, L_max=900, T=9, gamma=3)
    _check(cfg, 8)


def test_bf16_deterministic_and_page_order_invariant():
    cfg = synth.scaled(synth.CONFIGS["c2"], B=2, H=4, Hkv=4, L_min=777, L_max=777)
    inp = synth.make_msa_inputs(cfg, 9)
    a = _gpu(inp, cfg.gamma)
    b = _gpu(inp, cfg.gamma)
    assert torch.equal(a, b)                                   # run-to-run bitwise identical
    # move every page to a different physical slot: same logical cache, same result bit for bit
    perm = torch.from_numpy(synth.rng_for(99).permutation(inp["k_cache"].shape[0]))
    inv = torch.empty_like(perm)
    inv[perm] = torch.arange(perm.numel())
    moved = dict(inp)
    moved["k_cache"] = inp["k_cache"][perm]
    moved["v_cache"] = inp["v_cache"][perm]
    moved["block_table"] = inv[inp["block_table"].long()].to(torch.int32)
    assert torch.equal(_gpu(moved, cfg.gamma), a)


def test_bf16_unused_cache_slots_may_hold_nan():
    # memory past the end of a sequence (rest of the last page, unused pages) is never allowed to leak
    cfg = synth.scaled(synth.CONFIGS["c2"], B=2, H=2, Hkv=2, L_min=100, L_max=100)
    inp = synth.make_msa_inputs(cfg, 11)
    inp["seq_lens"] = torch.tensor([37, 91], dtype=torch.int32)
    base = _gpu(inp, cfg.gamma)
    bad = dict(inp)
    kc, vc = inp["k_cache"].clone(), inp["v_cache"].clone()
    used = set()
    for b, L in enumerate([37, 91]):
        for t in range(L):
            used.add((int(inp["block_table"][b, t // cfg.page]), t % cfg.page))
    for pg in range(kc.shape[0]):
        for s in range(cfg.page):
            if (pg, s) not in used:
                kc[pg, :, s, :] = float("nan")
                vc[pg, :, :, s] = float("nan")
    bad["k_cache"], bad["v_cache"] = kc, vc
    assert torch.equal(_gpu(bad, cfg.gamma), base)


# ---------------------------------------------------------------- full-size configs, sampled (sequence, KV head) pairs
@pytest.mark.parametrize("name,n_pairs", [("c3", 3), ("c4", 2), ("c5", 1)])
def test_full_size_sampled_pairs(name, n_pairs):
    cfg = synth.CONFIGS[name]
    inp = synth.make_msa_inputs(cfg, 1, device=DEV)            # drawn on the GPU: too large for the CPU generator
    got = api.ss_msa_attention(inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"],
                               inp["block_table"], inp["seq_lens"], inp["parent"], cfg.gamma, inp["scale"])
    torch.cuda.synchronize()
    assert torch.isfinite(got.float()).all()
    host = {k: (v.cpu() if isinstance(v, torch.Tensor) and v.dtype == torch.int32 else v) for k, v in inp.items()}
    rng = synth.rng_for(4242)
    g = cfg.H // cfg.Hkv
    lens = host["seq_lens"].numpy()
    picks = [(int(np.argmax(lens)), 0)] + [(int(rng.integers(cfg.B)), int(rng.integers(cfg.Hkv)))
                                             for _ in range(n_pairs - 1)]
    for b, hk in picks:
        sub = oracle_subproblem(host, b, hk, g)
        want = oracle.msa_attention(sub["q"], sub["k_new"], sub["v_new"], sub["k_cache"], sub["v_cache"],
                                    sub["block_table"], sub["seq_lens"], sub["parent"], cfg.gamma, inp["scale"])
        err = rel_err(to_np_f32(got[b:b + 1, :, hk * g:(hk + 1) * g]), want)
        print("%s pair (b=%d, hk=%d, L=%d): err %.2e" % (name, b, hk, lens[b], err), flush=True)
        assert err <= TOL["bf16"], (name, b, hk, err)


def test_attention_kernel_and_split_merge_as_two_calls():
    # SS_MSA_PARTIALS_ONLY then SS_MSA_MERGE_ONLY on the same workspace is the full call, bit for bit
    cfg = synth.scaled(synth.CONFIGS["c2"], B=2, H=4, Hkv=4, L_min=900, L_max=1300)
    inp = synth.make_msa_inputs(cfg, 11, device=DEV)
    args = (inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["block_table"], inp["seq_lens"],
            inp["parent"], cfg.gamma, inp["scale"])
    prev = api.ss_msa_set_split_keys(256)          # several splits
    try:
        need = api.ss_msa_workspace_bytes(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D,
                                          inp["block_table"].shape[1] * cfg.page, api.SS_BF16)
        ws = torch.zeros(need, dtype=torch.uint8, device=DEV)
        full = api.ss_msa_attention(*args, workspace=ws).clone()
        out = torch.zeros_like(full)
        api.ss_msa_attention(*args, flags=api.SS_MSA_PARTIALS_ONLY, out=out, workspace=ws)
        api.ss_msa_attention(*args, flags=api.SS_MSA_MERGE_ONLY, out=out, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(out, full)
        with pytest.raises(api.SSError):
            api.ss_msa_attention(*args, flags=api.SS_MSA_PARTIALS_ONLY | api.SS_MSA_MERGE_ONLY, out=out, workspace=ws)
    finally:
        api.ss_msa_set_split_keys(prev)


@pytest.mark.parametrize("name", ["c4", "c4short", "gqa"])
def test_merge_in_kernel_equals_merge_kernel(name):
    # two splits merged inside the attention kernel (default) against the separate merge kernel: bit for bit,
    # call after call (the arrival counters must come back to zero), also for sequences with one active split
    if name == "c4":
        cfg, lens = synth.CONFIGS["c4"], None
    elif name == "c4short":
        cfg, lens = synth.CONFIGS["c4"], [4096, 900, 0, 2500]     # 900 and 0: a single active split
    else:
        cfg, lens = synth.scaled(synth.CONFIGS["c5"], B=4, H=16, Hkv=4, L_min=2000, L_max=3000), None   # 8 row chunks
    inp = synth.make_msa_inputs(cfg, 12, device=DEV)
    if lens is not None:
        inp["seq_lens"] = torch.tensor(lens, dtype=torch.int32, device=DEV)
    args = (inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["block_table"], inp["seq_lens"],
            inp["parent"], cfg.gamma, inp["scale"])
    prev = api.ss_msa_set_merge_in_kernel(False)
    try:
        ref = api.ss_msa_attention(*args).clone()
        api.ss_msa_set_merge_in_kernel(True)
        for _ in range(3):
            got = api.ss_msa_attention(*args)
            torch.cuda.synchronize()
            assert torch.equal(got, ref)
    finally:
        api.ss_msa_set_merge_in_kernel(prev)


SWEEP = [
    # (B, H, Hkv, D, page, T, gamma, branching, max_depth, L_min, L_max)
    (1, 4, 4, 128, 16, 1, 0, (1,), 1, 300, 300),
    (3, 8, 2, 128, 16, 5, 1, (2, 2), 2, 64, 700),
    (2, 8, 1, 128, 32, 16, 4, (4, 2, 2), 3, 500, 1500),
    (5, 4, 4, 64, 16, 33, 2, (4, 3, 2, 2), 4, 0, 900),
    (2, 8, 8, 64, 64, 64, 1, (8, 4, 2), 3, 700, 1100),
    (4, 16, 4, 128, 64, 12, 8, (3, 2, 2), 3, 100, 2100),
    (2, 4, 2, 128, 16, 64, 8, (8, 4, 2), 3, 257, 800),
    (7, 2, 2, 64, 32, 7, 3, (2, 2, 2), 3, 31, 640),
]


@pytest.mark.parametrize("case", range(len(SWEEP)))
def test_two_split_merge_in_kernel_over_shapes(case):
    # exactly two key splits forced on shapes with one and several row chunks, both head dims, all page
    # sizes, GQA groups 1..8, ragged lengths down to 0: merged in the kernel = merged by the merge kernel,
    # bit for bit, on three calls in a row; and the result is the oracle's
    B, H, Hkv, D, page, T, gamma, br, md, lo, hi = SWEEP[case]
    cfg = synth.scaled(synth.CONFIGS["c2"], B=B, H=H, Hkv=Hkv, D=D, page=page, T=T, gamma=gamma, branching=br,
                       max_depth=md, L_min=lo, L_max=hi)
    inp = synth.make_msa_inputs(cfg, 40 + case, device=DEV)
    args = (inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["block_table"], inp["seq_lens"],
            inp["parent"], cfg.gamma, inp["scale"])
    max_len = inp["block_table"].shape[1] * page
    prev_keys = api.ss_msa_set_split_keys(max(64, (max_len // 2 + 31) // 32 * 32))
    prev = api.ss_msa_set_merge_in_kernel(False)
    try:
        ws = torch.zeros(api.ss_msa_workspace_bytes(B, T, gamma, H, Hkv, D, max_len, api.SS_BF16), dtype=torch.uint8,
                         device=DEV)
        ref = api.ss_msa_attention(*args, workspace=ws).clone()
        api.ss_msa_set_merge_in_kernel(True)
        for _ in range(3):
            got = api.ss_msa_attention(*args, workspace=ws)
            torch.cuda.synchronize()
            assert torch.equal(got, ref), SWEEP[case]
    finally:
        api.ss_msa_set_merge_in_kernel(prev)
        api.ss_msa_set_split_keys(prev_keys)
    want = _oracle({k: (v.cpu() if isinstance(v, torch.Tensor) else v) for k, v in inp.items()}, cfg.gamma)
    err = rel_err(to_np_f32(ref), want)
    print("sweep case", SWEEP[case], "err %.2e" % err, flush=True)
    assert err <= TOL["bf16"]
