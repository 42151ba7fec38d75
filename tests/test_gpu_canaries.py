"""Every entry point once with its outputs (and workspaces) embedded in guard bytes: after the call the guards
must be untouched.  Shapes are ragged on purpose (rows, outputs and lengths that fill no tile).  Values are
checked by the parity tests; this file only looks for writes outside the arrays."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
PAD = 4096
PATTERN = 0xA5


class Guarded:
    """A tensor of the given shape and type inside a byte buffer whose first and last PAD bytes are guards."""

    def __init__(self, shape, dtype):
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        self.n = n
        self.buf = torch.full((2 * PAD + max(n, 1),), PATTERN, dtype=torch.uint8, device=DEV)
        self.t = self.buf[PAD:PAD + n].view(dtype).view(shape) if n else torch.empty(shape, dtype=dtype, device=DEV)

    def fill_from(self, src):
        self.t.copy_(src)
        return self

    def check(self, what):
        torch.cuda.synchronize()
        assert bool((self.buf[:PAD] == PATTERN).all()), "%s: bytes before the array were written" % what
        assert bool((self.buf[PAD + self.n:] == PATTERN).all()), "%s: bytes behind the array were written" % what


def _check_all(guards, what):
    for i, g in enumerate(guards):
        g.check("%s (output %d)" % (what, i))


def _msa_case(cfg, seed, split_keys=0, merge_in_kernel=True):
    inp = synth.make_msa_inputs(cfg, seed, device=DEV)
    out = Guarded(tuple(inp["q"].shape), inp["q"].dtype)
    prev_k = api.ss_msa_set_split_keys(split_keys)
    prev_m = api.ss_msa_set_merge_in_kernel(merge_in_kernel)
    try:
        code = api.SS_BF16 if cfg.dtype == "bf16" else api.SS_F32
        need = api.ss_msa_workspace_bytes(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D,
                                          inp["block_table"].shape[1] * cfg.page, code)
        ws = Guarded((need,), torch.uint8)
        ws.t.zero_()
        for _ in range(2):
            api.ss_msa_attention(inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["block_table"],
                                 inp["seq_lens"], inp["parent"], cfg.gamma, inp["scale"], out=out.t, workspace=ws.t)
        _check_all([out, ws], "ss_msa_attention %s split_keys=%d" % (cfg.name, split_keys))
        assert torch.isfinite(out.t.float()).all()
    finally:
        api.ss_msa_set_split_keys(prev_k)
        api.ss_msa_set_merge_in_kernel(prev_m)


def test_attention_outputs_and_workspace():
    c1 = synth.CONFIGS["c1"]
    _msa_case(synth.scaled(c1, T=7, gamma=2, L_min=0, L_max=200, B=3), 2)               # fp32, unsplit and ragged
    _msa_case(synth.scaled(c1, T=7, gamma=2, L_min=100, L_max=200, B=2), 3, 64)         # fp32, several splits
    c2 = synth.CONFIGS["c2"]
    small = synth.scaled(c2, B=3, H=4, Hkv=2, T=7, gamma=3, branching=(3, 2, 2), L_min=1, L_max=700)
    _msa_case(small, 4)                                                                  # bf16, plan's choice
    _msa_case(small, 5, 352)                                                             # two splits merged in the kernel
    _msa_case(small, 6, 352, merge_in_kernel=False)                                      # ... and by the merge kernel
    _msa_case(small, 7, 64)                                                              # many splits
    one_page = synth.scaled(c2, B=2, H=2, Hkv=2, T=3, gamma=1, branching=(2, 2), max_depth=2, L_min=5, L_max=16)
    _msa_case(one_page, 8)                                                               # a table of one 16-token page


def test_page_table_of_one_page_is_not_read_past_its_end():
    # capacity of 16 tokens: the kernel's page-id gather must not look at entry 1 of a one-entry table
    cfg = synth.scaled(synth.CONFIGS["c2"], B=2, H=2, Hkv=2, T=3, gamma=1, branching=(2, 2), max_depth=2, L_min=16, L_max=16)
    inp = synth.make_msa_inputs(cfg, 9, device=DEV)
    assert inp["block_table"].shape == (2, 1)
    # the table sits at the very end of its allocation's used part, followed by page ids that do not exist
    tab = Guarded((2, 1), torch.int32)
    tab.buf.view(torch.int32)[:] = 0x7fffffff
    tab.t.copy_(inp["block_table"])
    ref = api.ss_msa_attention(inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["block_table"],
                               inp["seq_lens"], inp["parent"], cfg.gamma, inp["scale"])
    got = api.ss_msa_attention(inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], tab.t,
                               inp["seq_lens"], inp["parent"], cfg.gamma, inp["scale"])
    torch.cuda.synchronize()
    assert torch.equal(got, ref)


def test_lm_head_tail_and_projection():
    cfg = synth.scaled(synth.CONFIGS["c4"], B=3, T=5, gamma=2, branching=(2, 2), max_depth=2, vocab=1003, d_model=192,
                       K=3, draft_branching=(3, 2))
    N, K = cfg.B * cfg.R, cfg.K
    lm = synth.make_lm_head_inputs(cfg, 3, device=DEV)
    parent = torch.from_numpy(synth.make_trees(3, cfg.B, cfg.T, cfg.branching, cfg.max_depth)).to(DEV)
    tok = torch.from_numpy(synth.make_draft_tokens(3, parent.cpu().numpy(), cfg.vocab)).to(DEV)
    i32, f32 = torch.int32, torch.float32
    idx, val = Guarded((N, K), i32), Guarded((N, K), f32)
    ws = Guarded((api.ss_lm_head_workspace_bytes(N, cfg.d_model, cfg.vocab, K, api.SS_BF16),), torch.uint8)
    api.ss_lm_head_argmax_topk(lm["hidden"], lm["W"], K, idx=idx.t, val=val.t, workspace=ws.t)
    _check_all([idx, val, ws], "ss_lm_head_argmax_topk")
    T2 = 1 + 3 + 6
    out = dict(n_accept=Guarded((cfg.B,), i32), last=Guarded((cfg.B,), i32), bonus=Guarded((cfg.B,), i32),
               path=Guarded((cfg.B, cfg.max_depth + 1), i32), out_tokens=Guarded((cfg.B, cfg.max_depth + 1), i32),
               next_tok=Guarded((cfg.B, T2), i32), next_parent=Guarded((T2,), i32), main_argmax=Guarded((cfg.B, cfg.T), i32))
    api.ss_lm_head_verify_draft(lm["hidden"], lm["W"], K, tok, parent, cfg.gamma, cfg.max_depth, branching=cfg.draft_branching,
                                workspace=ws.t, out={k: g.t for k, g in out.items()})
    _check_all(list(out.values()) + [ws], "ss_lm_head_verify_draft")
    ver = {k: out[k] for k in ("n_accept", "last", "bonus", "path", "out_tokens")}
    api.ss_tree_verify(tok, parent, idx.t, cfg.max_depth, batch_stride=cfg.R * K, node_stride=K, out={k: g.t for k, g in ver.items()})
    _check_all(list(ver.values()), "ss_tree_verify")
    nt, npar = Guarded((cfg.B, T2), i32), Guarded((T2,), i32)
    api.ss_tree_draft(idx.t, K, ver["last"].t, ver["bonus"].t, cfg.T, cfg.gamma, branching=cfg.draft_branching,
                      batch_stride=cfg.R * K, offset=cfg.T * K, out=(nt.t, npar.t))
    _check_all([nt, npar], "ss_tree_draft")
    for flav in (None, "2", "3w"):
        api.ss_lm_set_flavour(True, flav)
        try:
            y = Guarded((N, cfg.vocab), torch.bfloat16)
            api.ss_linear_rows(lm["hidden"], lm["W"], y=y.t)
            y.check("ss_linear_rows flavour %s" % flav)
        finally:
            api.ss_lm_set_flavour(True, None)
    lse = Guarded((N,), f32)
    api.ss_lm_head_logsumexp(lm["hidden"], lm["W"], lse=lse.t, workspace=ws.t)
    _check_all([lse, ws], "ss_lm_head_logsumexp")
    h = lm["hidden"][:cfg.B * cfg.T].view(cfg.B, cfg.T, cfg.d_model)
    prob = Guarded((cfg.B, cfg.T), f32)
    api.ss_transition_probs(h, lm["W"], tok, parent, lse.t[:cfg.B * cfg.T].contiguous(), prob=prob.t)
    prob.check("ss_transition_probs")
    lib = api.load_library()
    pr = [Guarded((cfg.B, cfg.T), i32) for _ in range(4)] + [Guarded((cfg.B,), i32)]
    rc = lib.ss_tree_prune(tok.data_ptr(), parent.data_ptr(), prob.t.data_ptr(), ctypes.c_float(0.3), cfg.B, cfg.T,
                           *[g.t.data_ptr() for g in pr], torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    _check_all(pr, "ss_tree_prune")
    R = cfg.R
    mask, anc, depth = Guarded((cfg.B, R, R), torch.uint8), Guarded((cfg.B, cfg.T), torch.int64), Guarded((cfg.B, cfg.T), i32)
    rc = lib.ss_build_mask(parent.data_ptr(), cfg.B, cfg.T, cfg.gamma, 0, mask.t.data_ptr(), anc.t.data_ptr(),
                           depth.t.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    _check_all([mask, anc, depth], "ss_build_mask")


def test_fp32_lm_head_and_projection():
    cfg = synth.scaled(synth.CONFIGS["c1"], vocab=77, d_model=40, K=2)
    N = 37
    lm = synth.make_lm_head_inputs(cfg, 5, device=DEV, N=N)
    idx, val = Guarded((N, 2), torch.int32), Guarded((N, 2), torch.float32)
    ws = Guarded((api.ss_lm_head_workspace_bytes(N, cfg.d_model, cfg.vocab, 2, api.SS_F32),), torch.uint8)
    api.ss_lm_head_argmax_topk(lm["hidden"], lm["W"], 2, idx=idx.t, val=val.t, workspace=ws.t)
    y = Guarded((N, cfg.vocab), torch.float32)
    api.ss_linear_rows(lm["hidden"], lm["W"], y=y.t)
    lse = Guarded((N,), torch.float32)
    api.ss_lm_head_logsumexp(lm["hidden"], lm["W"], lse=lse.t, workspace=ws.t)
    _check_all([idx, val, ws, y, lse], "fp32 LM head / projection / log-sum-exp")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stream_insert_value_rotate_and_cache_commit(dtype):
    cfg = synth.scaled(synth.CONFIGS["c2"], dtype=dtype, B=3, H=4, Hkv=2, D=64, T=5, gamma=3, branching=(2, 2, 2), L_min=1, L_max=90)
    dt = cfg.torch_dtype
    d = 72
    M = torch.randn(cfg.B, cfg.T, d, device=DEV).to(dt)
    P = torch.randn(cfg.gamma, d, device=DEV).to(dt)
    X = Guarded((cfg.B, cfg.R, d), dt)
    api.ss_stream_insert(M, P, X=X.t)
    X.check("ss_stream_insert")
    inp = synth.make_msa_inputs(cfg, 7, device=DEV)
    v = Guarded(tuple(inp["v_new"].shape), dt).fill_from(inp["v_new"])
    api.ss_value_rotate(v.t, cfg.T, cfg.gamma, 0.01)
    v.check("ss_value_rotate")
    # commit: the caches themselves are the outputs; rows past the table's capacity must be dropped, not written
    kc = Guarded(tuple(inp["k_cache"].shape), dt).fill_from(inp["k_cache"])
    vc = Guarded(tuple(inp["v_cache"].shape), dt).fill_from(inp["v_cache"])
    cap = inp["block_table"].shape[1] * cfg.page
    lens = torch.tensor([cap - 1, 3, cap], dtype=torch.int32, device=DEV)
    path = torch.tensor([[0, 1, 3, 4], [0, 2, -1, -1], [0, 1, 2, 3]], dtype=torch.int32, device=DEV)
    n_acc = torch.tensor([3, 1, 3], dtype=torch.int32, device=DEV)
    new_lens = Guarded((cfg.B,), torch.int32)
    api.ss_kv_commit(inp["k_new"], inp["v_new"], kc.t, vc.t, inp["block_table"], lens, path, n_acc, cfg.gamma,
                     new_seq_lens=new_lens.t)
    _check_all([kc, vc, new_lens], "ss_kv_commit")
    assert new_lens.t.tolist() == [cap, 5, cap]
