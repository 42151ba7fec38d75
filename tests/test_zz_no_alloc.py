"""The entry point that allocates nothing (ss_msa_attention_static) against ss_msa_attention: two calls in a
row on one GPU, the second on a smaller input, both bit for bit; then the size limit."""
import pytest
import torch

from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(seed, **kw):
    cfg = synth.scaled(synth.CONFIGS["c4"], **kw)
    inp = synth.make_msa_inputs(cfg, seed, device=DEV)
    args = (inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["block_table"], inp["seq_lens"],
            inp["parent"], cfg.gamma, inp["scale"])
    max_len = inp["block_table"].shape[1] * cfg.page
    plan = api.ss_msa_plan(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, max_len, api.SS_BF16)
    return cfg, args, plan


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    # first call: 4 sequences x 32 heads x 1500..2000 cached tokens -> two splits merged inside the kernel
    # (partial results and arrival counters in the library's array); second call: a smaller problem that
    # is split too, on the array as the first call left it
    big = _case(5, L_min=1500, L_max=2000)
    small = _case(6, B=1, H=4, Hkv=4, L_min=520, L_max=700)
    assert big[2] == (2, 1) and small[2][0] >= 2, (big[2], small[2])
    refs = [api.ss_msa_attention(*c[1]).clone() for c in (big, small)]
    outs = [torch.zeros_like(r) for r in refs]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for c, out in zip((big, small), outs):
        api.ss_msa_attention_static(*c[1], out=out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for got, ref in zip(outs, refs):
        assert torch.equal(got, ref)
    # and once more in the other order, with the merge kernel instead of the in-kernel merge
    prev = api.ss_msa_set_merge_in_kernel(False)
    try:
        for c, ref in zip((small, big), refs[::-1]):
            out = torch.zeros_like(ref)
            api.ss_msa_attention_static(*c[1], out=out)
            torch.cuda.synchronize()
            assert torch.equal(out, ref)
    finally:
        api.ss_msa_set_merge_in_kernel(prev)


def test_static_scratch_unsplit_and_fp32():
    cfg = synth.CONFIGS["c1"]
    inp = synth.make_msa_inputs(cfg, 3, device=DEV)
    args = (inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["block_table"], inp["seq_lens"],
            inp["parent"], cfg.gamma, inp["scale"])
    ref = api.ss_msa_attention(*args)
    out = torch.zeros_like(ref)
    api.ss_msa_attention_static(*args, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


def test_static_scratch_rejects_what_does_not_fit():
    cap = api.ss_msa_static_scratch_bytes()
    assert cap == 32 << 20
    # c5 split into many parts needs more partial rows than the array holds
    cfg = synth.CONFIGS["c5"]
    prev = api.ss_msa_set_split_keys(1024)
    try:
        need = api.ss_msa_workspace_bytes(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, 32768, api.SS_BF16)
        assert need > cap
        lib = api.load_library()
        dummy = torch.zeros(64, dtype=torch.uint8, device=DEV).data_ptr()
        rc = lib.ss_msa_attention_static(dummy, dummy, dummy, dummy, dummy, dummy, 32768 // cfg.page, 1, dummy, dummy,
                                         cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, cfg.page, 0.1, api.SS_BF16, 0,
                                         dummy, None)
        assert rc == 2 and b"scratch" in lib.ss_last_error()
    finally:
        api.ss_msa_set_split_keys(prev)
