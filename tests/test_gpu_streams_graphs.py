"""The calls are asynchronous on the stream they are given: the same step on a side stream, on two streams at
once, and captured into a HIP graph that is replayed several times with eager work in between, all against the
result of the default stream (bit for bit: every kernel is deterministic)."""
import pytest
import torch

from paper_2402_11131_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _setup(seed):
    # two key splits (merged inside the attention kernel) and the fused tail
    cfg = synth.scaled(synth.CONFIGS["c4"], B=2, H=4, Hkv=4, L_min=900, L_max=1200, vocab=3000, d_model=512, n_layers=1)
    lay = synth.make_msa_inputs(cfg, seed, device=DEV)
    W = synth.make_lm_head_inputs(cfg, seed, device=DEV)["W"]
    tok = torch.from_numpy(synth.make_draft_tokens(seed, lay["parent"].cpu().numpy(), cfg.vocab)).to(DEV)
    max_len = lay["block_table"].shape[1] * cfg.page
    ws = torch.zeros(api.ss_msa_workspace_bytes(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, max_len, api.SS_BF16),
                     dtype=torch.uint8, device=DEV)
    lm_ws = torch.empty(api.ss_lm_head_workspace_bytes(cfg.B * cfg.R, cfg.d_model, cfg.vocab, cfg.K, api.SS_BF16),
                        dtype=torch.uint8, device=DEV)
    out = torch.empty_like(lay["q"])
    return dict(cfg=cfg, lay=lay, W=W, tok=tok, ws=ws, lm_ws=lm_ws, out=out, tail=None)


def _step(s):
    cfg, lay = s["cfg"], s["lay"]
    api.ss_msa_attention(lay["q"], lay["k_new"], lay["v_new"], lay["k_cache"], lay["v_cache"], lay["block_table"],
                         lay["seq_lens"], lay["parent"], cfg.gamma, lay["scale"], out=s["out"], workspace=s["ws"])
    s["tail"] = api.ss_lm_head_verify_draft(s["out"].view(cfg.B * cfg.R, cfg.d_model), s["W"], cfg.K, s["tok"],
                                            lay["parent"], cfg.gamma, cfg.max_depth, branching=cfg.draft_branching,
                                            workspace=s["lm_ws"], out=s["tail"])


def _result(s):
    return [s["out"].clone()] + [s["tail"][k].clone() for k in ("n_accept", "out_tokens", "next_tok", "main_argmax")]


def _same(a, b):
    return all(torch.equal(x, y) for x, y in zip(a, b))


@pytest.fixture(scope="module")
def prev_split():
    prev = api.ss_msa_set_split_keys(640)       # two splits for these lengths
    yield
    api.ss_msa_set_split_keys(prev)


def test_side_stream_and_two_streams_at_once(prev_split):
    a, b = _setup(1), _setup(2)
    assert api.ss_msa_plan(a["cfg"].B, a["cfg"].T, a["cfg"].gamma, a["cfg"].H, a["cfg"].Hkv, a["cfg"].D,
                           a["lay"]["block_table"].shape[1] * a["cfg"].page, api.SS_BF16) == (2, 1)
    _step(a), _step(b)
    torch.cuda.synchronize()
    ref_a, ref_b = _result(a), _result(b)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(5):
        a["out"].zero_(), b["out"].zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(s1):
            _step(a)
        with torch.cuda.stream(s2):
            _step(b)
        torch.cuda.synchronize()
        assert _same(_result(a), ref_a) and _same(_result(b), ref_b), rep


def test_graph_replays_equal_the_eager_step(prev_split):
    a, other = _setup(3), _setup(4)
    _step(a)
    torch.cuda.synchronize()
    ref = _result(a)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _step(a)
    for rep in range(4):
        a["out"].zero_()
        _step(other)                            # eager work of the program's own between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert _same(_result(a), ref), rep
