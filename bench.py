#!/usr/bin/env python3
"""Benchmark of the verify-and-speculate step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that
is already resident in HBM: N_s multi-stream-attention layers (each with its own
paged KV cache and q/k/v), the LM head with fused arg-max/top-k on the last
layer's output, greedy tree verification and tree drafting, all enqueued on one
stream through the C ABI with no host synchronisation in between.

Default workload: c4 (4 sequences, 32x128 heads, prefix 4096, 16-node trees x 4
streams, 4 MSA layers, LM head 320 x 4096 x 32000, top-4): the only configuration
that contains every part of the path.  `--workload c2|c3|c5` time the attention
layer(s) of the other configurations (no LM head in those).

Prints ONE JSON line.  `value` is microseconds per step.  `roofline` describes the
dominant kernel (the bf16 MSA kernel): algorithmic bytes per launch divided by the
kernel's own average duration, measured here with events on the launch stream
around a loop of launches with the split-merge kernel switched off (rotating
input sets).  `kernels.msa_kernel_in_step_with_events_us` is the same kernel
bracketed by events launch by launch inside the steps.  `cpu_baseline` times the
CPU oracle on whole steps of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, vendor figure

# HBM traffic of one launch of the MSA kernel, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE; KiB
# per dispatch), each scaled by what the same counter reads for the 256 MiB device copy of --calibrate-copy
# (FETCH_SIZE reads half of the bytes the copy fetches: factor 2.0; WRITE_SIZE factor 1.0).  c4, the launch
# the steps make (two splits merged inside the kernel): 139168 KiB x 2.0 fetched (the cache once + one split's
# partial rows read back) + 15608 KiB written (both splits' fp32 partials + the output).  Summaries are under
# profiles/.
MSA_TRAFFIC_BYTES = {"c4": int((139168.0 * 2.0 + 15608.0) * 1024), "c2": None, "c3": None, "c5": None}


def msa_bytes(cfg, seq_lens):
    """Algorithmic bytes of one MSA launch: K and V prefix once, the step's new K/V block, q in, out."""
    e = 2 if cfg.dtype == "bf16" else 4
    kv = sum(2 * int(L) * cfg.Hkv * cfg.D * e for L in seq_lens)
    new = cfg.B * 2 * cfg.R * cfg.Hkv * cfg.D * e
    io = cfg.B * 2 * cfg.R * cfg.H * cfg.D * e
    table = sum(((int(L) + cfg.page - 1) // cfg.page) * 4 for L in seq_lens)
    return kv + new + io + table


def msa_flops(cfg, seq_lens):
    return sum(4 * cfg.R * (int(L) + cfg.R) * cfg.H * cfg.D for L in seq_lens)


def timed(fn, iters, torch):
    """Average microseconds of fn() over iters calls, events on the current stream."""
    start = torch.cuda.Event(enable_timing=True)
    end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(iters):
        fn(i)
    end.record()
    torch.cuda.synchronize()
    return start.elapsed_time(end) * 1000.0 / iters


def cpu_baseline(cfg, synth, seq_lens):
    """The oracle on the same workload, whole steps (every MSA layer on its own inputs, the LM head, verify,
    draft), repeated until about 10 s of CPU time have been spent (at most 8 steps); the mean step is reported."""
    import numpy as np
    import oracle
    oracle.build()
    f32 = lambda t: t.float().numpy()
    layers = []
    for i in range(cfg.n_layers):
        inp = synth.make_msa_inputs(cfg, 4242, layer=i)
        layers.append((f32(inp["q"]), f32(inp["k_new"]), f32(inp["v_new"]), f32(inp["k_cache"]), f32(inp["v_cache"]),
                       inp["block_table"].numpy(), inp["seq_lens"].numpy(), inp["parent"].numpy(), cfg.gamma, inp["scale"]))
    par = layers[0][7]
    if cfg.vocab:
        lm = synth.make_lm_head_inputs(cfg, 4242)
        hidden, W = f32(lm["hidden"]), f32(lm["W"])
        tok = synth.make_draft_tokens(4242, par, cfg.vocab)
        tp, tr, _ = oracle.full_tree_template(cfg.draft_branching)
    reps, t_all = 0, 0.0
    while reps < 8 and t_all < 10.0:
        t0 = time.perf_counter()
        for a in layers:
            oracle.msa_attention(*a)
        if cfg.vocab:
            idx, _ = oracle.lm_head_topk(hidden, W, cfg.K)
            idx = np.ascontiguousarray(idx.reshape(cfg.B, cfg.R, cfg.K))
            ver = oracle.tree_verify(tok, par, np.ascontiguousarray(idx[:, :cfg.T, 0]), cfg.max_depth)
            topk = np.ascontiguousarray(idx[:, cfg.T:, :].reshape(cfg.B, cfg.T, cfg.gamma, cfg.K))
            oracle.tree_draft(topk, ver["last"], ver["bonus"], tp, tr)
        t_all += time.perf_counter() - t0
        reps += 1
    return {"value": round(t_all / reps * 1e6, 1), "unit": "us", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d whole steps of the same workload (%d MSA layers + LM head + verify + draft each), %.1f s in all; "
                      "mean step" % (reps, cfg.n_layers, t_all)}


def calibrate_copy(torch, dev):
    """A plain device-to-device copy of known size (256 MiB read, 256 MiB written per call), so that a
    rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this script has a kernel to scale the counters by."""
    src = torch.ones(128 * 1024 * 1024, dtype=torch.bfloat16, device=dev)
    dst = torch.empty_like(src)
    for _ in range(4):
        dst.copy_(src)
    torch.cuda.synchronize()


def time_rows_after_hot_path(api, synth, torch, cfg, dev, N, it, lm, lm_ws, tok, parent, extra):
    """Rows after the hot path (not part of `value`), each in a loop of its own; fills `extra`."""
    # Dense projections of one MSA layer on the step's N rows (the row after the hot path: not part of
    # `value`): fused QKV, attention output, fused gate+up and down of a 4096/11008 feed-forward block.
    dm, dff = cfg.d_model, 11008
    dense = {}
    total = 0.0
    for name, (din, dout) in (("qkv", (dm, 3 * cfg.H * cfg.D)), ("attn_out", (cfg.H * cfg.D, dm)),
                              ("gate_up", (dm, 2 * dff)), ("down", (dff, dm))):
        xs = [synth.make_lm_head_inputs(synth.scaled(cfg, vocab=dout, d_model=din), 50 + j, device=dev, N=N)
              for j in range(2)]
        y = torch.empty(N, dout, dtype=xs[0]["hidden"].dtype, device=dev)
        for j in range(2):
            api.ss_linear_rows(xs[j]["hidden"], xs[j]["W"], y)
        us = timed(lambda i: api.ss_linear_rows(xs[i % 2]["hidden"], xs[i % 2]["W"], y), it, torch)
        total += us
        dense[name] = {"d_in": din, "d_out": dout, "us": round(us, 2),
                       "tflops": round(2.0 * N * din * dout / (us * 1e-6) / 1e12, 1),
                       "hbm_gbps": round((din * dout + N * din + N * dout) * 2 / (us * 1e-6) / 1e9, 1)}
        del xs, y
    dense["layer_total_us"] = round(total, 2)
    extra["linear_rows"] = dense
    # The pruning layer (also after the hot path): log-sum-exp of the early-exit logits of the B*T main
    # rows over the whole vocabulary, transition probabilities, pruning decision and compaction.
    hm = synth.make_lm_head_inputs(cfg, 60, device=dev, N=cfg.B * cfg.T)["hidden"].view(cfg.B, cfg.T, dm)
    w_copies = [lm["W"], lm["W"].clone()]
    lse = torch.empty(cfg.B * cfg.T, dtype=torch.float32, device=dev)
    prob = torch.empty(cfg.B, cfg.T, dtype=torch.float32, device=dev)

    def prune_layer(i):
        api.ss_lm_head_logsumexp(hm.view(cfg.B * cfg.T, dm), w_copies[i & 1], lse=lse, workspace=lm_ws)
        api.ss_transition_probs(hm, w_copies[i & 1], tok, parent, lse, prob=prob)
        return api.ss_tree_prune(tok, parent, prob, 0.01)
    prune_layer(0)
    us_prune = timed(prune_layer, it, torch)
    us_lse = timed(lambda i: api.ss_lm_head_logsumexp(hm.view(cfg.B * cfg.T, dm), w_copies[i & 1], lse=lse,
                                                      workspace=lm_ws), it, torch)
    # Stream insertion (Eq. 3) for the same batch: elementwise, B*R*d elements
    P_emb = synth.make_lm_head_inputs(synth.scaled(cfg, vocab=64, d_model=dm), 61, device=dev, N=cfg.gamma)["hidden"]
    X_rows = torch.empty(cfg.B, cfg.R, dm, dtype=hm.dtype, device=dev)
    api.ss_stream_insert(hm, P_emb, X=X_rows)
    us_ins = timed(lambda i: api.ss_stream_insert(hm, P_emb, X=X_rows), it, torch)
    extra["stream_insert_us"] = round(us_ins, 2)
    # The appendix's value-rotation variant on one layer's value block [B,R,Hkv,D], in place
    v_blk = X_rows.view(cfg.B, cfg.R, cfg.Hkv, dm // cfg.Hkv) if dm % cfg.Hkv == 0 and (dm // cfg.Hkv) % 2 == 0 else None
    if v_blk is not None:
        api.ss_value_rotate(v_blk, cfg.T, cfg.gamma, 1e-4)
        extra["value_rotate_us"] = round(timed(lambda i: api.ss_value_rotate(v_blk, cfg.T, cfg.gamma, 1e-4), it, torch), 2)
    extra["prune_layer"] = {"us": round(us_prune, 2), "logsumexp_us": round(us_lse, 2),
                            "logsumexp_hbm_gbps": round(cfg.vocab * dm * 2 / (us_lse * 1e-6) / 1e9, 1)}
    del w_copies


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c4", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--split-keys", type=int, default=0, help="KV split length of the MSA kernel (0 = automatic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-tail", action="store_true",
                    help="LM head, verification and drafting as three calls instead of the fused one")
    ap.add_argument("--in-step-events", action="store_true",
                    help="also time the attention kernel inside the steps with a pair of events per launch")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step's launches once into a HIP graph and replay it (measured: no faster "
                         "than launching from the host, the step is bound by the kernels, not by launches)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 256 MiB device copy (reference kernel for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (the path uses no collectives; "
              "sequences, heads or vocabulary slices would be sharded, one small exchange per step)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2402_11131_amd import api, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    api.load_library()
    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    if args.split_keys:
        api.ss_msa_set_split_keys(args.split_keys)

    # ---- inputs.  Each MSA layer has its own caches; input sets are rotated so that one rotation
    # touches more than 512 MB and the 256 MB last-level cache cannot serve repeats.
    seq_lens = synth.seq_lens_for(cfg, 1)
    per_layer = msa_bytes(cfg, seq_lens)
    n_sets = max(cfg.n_layers, int(np.ceil(768e6 / per_layer)))
    n_sets = ((n_sets + cfg.n_layers - 1) // cfg.n_layers) * cfg.n_layers
    layers = [synth.make_msa_inputs(cfg, 1, device=dev, layer=i) for i in range(n_sets)]
    outs = [torch.empty_like(layers[0]["q"]) for _ in range(cfg.n_layers)]
    ws_bytes = api.ss_msa_workspace_bytes(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D,
                                          layers[0]["block_table"].shape[1] * cfg.page, api.SS_BF16)
    msa_ws = torch.zeros(max(ws_bytes, 1), dtype=torch.uint8, device=dev)
    parent = layers[0]["parent"]
    has_lm = cfg.vocab > 0
    if has_lm:
        N = cfg.B * cfg.R
        lm = synth.make_lm_head_inputs(cfg, 1, device=dev)
        tok_np = synth.make_draft_tokens(1, parent.cpu().numpy(), cfg.vocab)
        tok = torch.from_numpy(tok_np).to(dev)
        idx = torch.empty((N, cfg.K), dtype=torch.int32, device=dev)
        val = torch.empty((N, cfg.K), dtype=torch.float32, device=dev)
        lm_ws = torch.empty(api.ss_lm_head_workspace_bytes(N, cfg.d_model, cfg.vocab, cfg.K, api.SS_BF16),
                            dtype=torch.uint8, device=dev)

    def msa_call(layer, out, flags=0):
        api.ss_msa_attention(layer["q"], layer["k_new"], layer["v_new"], layer["k_cache"], layer["v_cache"],
                             layer["block_table"], layer["seq_lens"], parent, cfg.gamma, layer["scale"],
                             flags=flags, out=out, workspace=msa_ws)

    state = {}

    def step(i, kernel_events=None):
        base = (i * cfg.n_layers) % n_sets
        for j in range(cfg.n_layers):
            if kernel_events is None:
                msa_call(layers[base + j], outs[j])
            else:
                # the same two kernels as two calls, with a pair of events around the attention kernel alone
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                msa_call(layers[base + j], outs[j], api.SS_MSA_PARTIALS_ONLY)
                e1.record()
                msa_call(layers[base + j], outs[j], api.SS_MSA_MERGE_ONLY)
                kernel_events.append((e0, e1))
        if has_lm:
            hidden = outs[-1].view(N, cfg.d_model)
            if args.separate_tail:
                # a3, a4 and a5 as three calls (four kernels)
                api.ss_lm_head_argmax_topk(hidden, lm["W"], cfg.K, idx=idx, val=val, workspace=lm_ws)
                ver = api.ss_tree_verify(tok, parent, idx, cfg.max_depth, batch_stride=cfg.R * cfg.K, node_stride=cfg.K)
                nxt = api.ss_tree_draft(idx, cfg.K, ver["last"], ver["bonus"], cfg.T, cfg.gamma,
                                        branching=cfg.draft_branching, batch_stride=cfg.R * cfg.K, offset=cfg.T * cfg.K)
                state["ver"], state["nxt"], state["argmax"] = ver, nxt, idx.view(cfg.B, cfg.R, cfg.K)[:, :cfg.T, 0]
            else:
                # the same three rows in one call (two kernels): the candidate merge happens in the kernel
                # that verifies and drafts, for the rows those steps read
                t = api.ss_lm_head_verify_draft(hidden, lm["W"], cfg.K, tok, parent, cfg.gamma, cfg.max_depth,
                                                branching=cfg.draft_branching, workspace=lm_ws, out=state.get("tail"))
                state["tail"] = t
                state["ver"], state["nxt"], state["argmax"] = t, (t["next_tok"], t["next_parent"]), t["main_argmax"]

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if has_lm and n_sets == cfg.n_layers:
        # Every step sees the same inputs, so the main stream's arg-max tokens are known after the warm-up.
        # Plant the draft the way a decode loop would have produced it: along one seeded root path per
        # sequence each draft token equals the main stream's token at its parent with probability 0.7
        # (until the first miss), which gives the accepted lengths the paper's call-reduction ratios imply.
        a = state["argmax"].cpu().numpy()
        par = parent.cpu().numpy()
        rng = synth.rng_for(99)
        for b in range(cfg.B):
            path = synth.root_path(par[b], int(rng.integers(cfg.T)))
            for p_, c_ in zip(path[:-1], path[1:]):
                if rng.random() >= 0.7:
                    break
                tok_np[b, c_] = a[b, p_]
        tok.copy_(torch.from_numpy(tok_np))
        step(0)
        torch.cuda.synchronize()
    # Optionally the step's launches are captured once into a HIP graph and replayed (only when every
    # step sees the same input sets; replays are checked against the eager result before anything is timed).
    use_graph = args.graph and n_sets == cfg.n_layers
    run_step = step
    if use_graph:
        eager = [state["ver"]["out_tokens"].clone(), state["nxt"][0].clone(), state["argmax"].clone()] if has_lm else [o.clone() for o in outs]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(0)
        for _ in range(3):
            graph.replay()
            torch.cuda.synchronize()
            now = [state["ver"]["out_tokens"], state["nxt"][0], state["argmax"]] if has_lm else outs
            for e_, n_ in zip(eager, now):
                if not torch.equal(e_, n_):
                    print("bench.py: a graph replay differs from the eager step", file=sys.stderr)
                    sys.exit(1)
        run_step = lambda i: graph.replay()
    t_wall0 = time.perf_counter()
    us_step = timed(run_step, args.steps, torch)
    wall_s = time.perf_counter() - t_wall0

    # ---- per-kernel figures (each in its own timed loop, same rotation of inputs)
    it = max(20, args.steps)
    us_msa_call = timed(lambda i: msa_call(layers[i % n_sets], outs[0]), it, torch)
    us_msa_partials = timed(lambda i: msa_call(layers[i % n_sets], outs[0], api.SS_MSA_PARTIALS_ONLY), it, torch)
    # The roofline is that of the attention kernel as the step launches it.  A full call is that kernel alone
    # when the prefix is unsplit or its two splits are merged inside the kernel (c4): then the loop of whole
    # calls times it; otherwise a merge kernel follows and the loop that leaves the merge out does.
    max_len = layers[0]["block_table"].shape[1] * cfg.page
    n_splits, n_kernels = api.ss_msa_plan(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, max_len,
                                          api.SS_BF16 if cfg.dtype == "bf16" else api.SS_F32)
    us_msa_kernel = us_msa_call if n_kernels == 1 else us_msa_partials
    kern = {"msa_call_us": round(us_msa_call, 2), "msa_kernel_us": round(us_msa_kernel, 2),
            "msa_kernel_without_split_merge_us": round(us_msa_partials, 2), "msa_splits": n_splits,
            "msa_kernels_per_call": n_kernels}
    if args.in_step_events:
        # The attention kernel inside the step, for comparison with a kernel trace: the timed steps again, every
        # attention call made in its two halves (kernel, then split merge as a kernel of its own) with a pair of
        # events around the first.  This figure includes what the two events cost themselves.
        evs = []
        for i in range(args.steps):
            step(i, evs)
        torch.cuda.synchronize()
        kern["msa_kernel_in_step_with_events_us"] = round(sum(a_.elapsed_time(b_) for a_, b_ in evs) * 1000.0 / len(evs), 2)
        del evs
    b_msa = msa_bytes(cfg, seq_lens)
    f_msa = msa_flops(cfg, seq_lens)
    gbps = b_msa / (us_msa_kernel * 1e-6) / 1e9
    tflops = f_msa / (us_msa_kernel * 1e-6) / 1e12
    # Which roofline binds the kernel on this workload: the matrix cores if its FLOP per byte exceed the
    # machine's ridge (long GQA trees: c5), HBM otherwise.  Both figures are reported either way.
    if f_msa / b_msa > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBPS * 1e9):
        roofline = {"kernel": "msa_bf16_kernel", "bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                    "traffic": MSA_TRAFFIC_BYTES.get(args.workload), "algorithmic_flops": f_msa, "hbm_gbps": round(gbps, 1)}
    else:
        roofline = {"kernel": "msa_bf16_kernel", "bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4),
                    "traffic": MSA_TRAFFIC_BYTES.get(args.workload), "algorithmic_bytes": b_msa,
                    "mfma_tflops": round(tflops, 1)}
    # The read rate this GPU reaches with plain 16-byte loads over 1 GiB (four times the last-level cache), next to
    # the published peak the fraction is taken against
    probe_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_()
    probe_sink = torch.zeros(1, dtype=torch.int32, device=dev)
    roofline["measured_read_ceiling_gbps"] = {
        "plain": round((1 << 30) / (timed(lambda i: api.ss_probe_hbm_read(probe_buf, False, probe_sink), 20, torch) * 1e-6) / 1e9, 1),
        "streaming": round((1 << 30) / (timed(lambda i: api.ss_probe_hbm_read(probe_buf, True, probe_sink), 20, torch) * 1e-6) / 1e9, 1)}
    del probe_buf
    if n_kernels == 1 and n_splits > 1:
        # for comparison: the same kernel when it leaves the split merge to a second kernel
        roofline["without_split_merge"] = {"us": round(us_msa_partials, 2),
                                           "frac": round(b_msa / (us_msa_partials * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
    extra = {}
    if has_lm:
        hidden = outs[-1].view(N, cfg.d_model)
        # two copies of W in turn: a single 262 MB matrix would partly stay in the last-level cache between
        # calls, which it cannot inside a step (the MSA layers stream more than a gigabyte in between)
        w_copies = [lm["W"], lm["W"].clone()]
        us_lm = timed(lambda i: api.ss_lm_head_argmax_topk(hidden, w_copies[i & 1], cfg.K, idx=idx, val=val,
                                                           workspace=lm_ws), it, torch)
        tail_out = state.get("tail")
        us_tail = timed(lambda i: api.ss_lm_head_verify_draft(hidden, w_copies[i & 1], cfg.K, tok, parent, cfg.gamma,
                                                              cfg.max_depth, branching=cfg.draft_branching,
                                                              workspace=lm_ws, out=tail_out), it, torch)
        del w_copies
        us_ver = timed(lambda i: api.ss_tree_verify(tok, parent, idx, cfg.max_depth, batch_stride=cfg.R * cfg.K,
                                                    node_stride=cfg.K), it, torch)
        ver = state["ver"]
        us_draft = timed(lambda i: api.ss_tree_draft(idx, cfg.K, ver["last"], ver["bonus"], cfg.T, cfg.gamma,
                                                     branching=cfg.draft_branching, batch_stride=cfg.R * cfg.K,
                                                     offset=cfg.T * cfg.K), it, torch)
        # KV-cache commit of the accepted path (the row after the hot path: not part of `value`), all layers
        cap = layers[0]["block_table"].shape[1] * cfg.page
        short = torch.clamp(layers[0]["seq_lens"], max=cap - cfg.max_depth - 1)
        new_lens = torch.empty_like(short)
        us_commit = timed(lambda i: [api.ss_kv_commit(l["k_new"], l["v_new"], l["k_cache"], l["v_cache"], l["block_table"], short,
                                                       ver["path"], ver["n_accept"], cfg.gamma, new_seq_lens=new_lens)
                                     for l in layers[:cfg.n_layers]], it, torch)
        kern.update({"lm_head_call_us": round(us_lm, 2), "lm_head_verify_draft_call_us": round(us_tail, 2), "verify_us": round(us_ver, 2), "draft_us": round(us_draft, 2),
                     "kv_commit_all_layers_us": round(us_commit, 2)})
        f_lm = 2.0 * N * cfg.vocab * cfg.d_model
        tf = f_lm / (us_lm * 1e-6) / 1e12
        mfma_sink = torch.zeros(1, dtype=torch.float32, device=dev)
        mfma_flops = api.ss_probe_mfma_bf16(1000, mfma_sink)
        us_mfma = timed(lambda i: api.ss_probe_mfma_bf16(1000, mfma_sink), 20, torch)
        extra["roofline_lm_head"] = {"kernel": "lm_head_bf16_kernel + lm_head_reduce_kernel", "bound": "mfma", "achieved": round(tf, 1),
                                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                                     "hbm_gbps": round((cfg.vocab * cfg.d_model * 2 + N * cfg.d_model * 2) /
                                                       (us_lm * 1e-6) / 1e9, 1),
                                     # register-only matrix-core work on the whole chip, at the clock it is granted
                                     "measured_mfma_ceiling_tflops": round(mfma_flops / (us_mfma * 1e-6) / 1e12, 1)}
        extra["accepted_per_sequence"] = state["ver"]["n_accept"].tolist()
        if args.workload == "c4":
            try:
                time_rows_after_hot_path(api, synth, torch, cfg, dev, N, it, lm, lm_ws, tok, parent, extra)
            except Exception as e:  # the headline measurement must survive a failure here
                extra["rows_after_hot_path_error"] = "%s: %s" % (type(e).__name__, e)

    result = {
        "metric": "verify+speculate step time (MSA layers + LM-head argmax/top-k + verify + draft)",
        "value": round(us_step, 2), "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us_step / 1000.0, 5), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: B=%d, %dx%d heads (%d KV), prefix %s, %d-node trees x %d streams (%d rows/seq), "
                               "%d-token pages, %d MSA layer(s)%s" % (
                                   cfg.name, cfg.B, cfg.H, cfg.D, cfg.Hkv,
                                   cfg.L_min if cfg.L_min == cfg.L_max else "%d..%d" % (cfg.L_min, cfg.L_max),
                                   cfg.T, cfg.gamma, cfg.R, cfg.page, cfg.n_layers,
                                   ", LM head %dx%dx%d top-%d" % (cfg.B * cfg.R, cfg.d_model, cfg.vocab, cfg.K)
                                   if has_lm else ""),
                   "input_sets_rotated": n_sets, "split_keys": args.split_keys or "auto",
                   "launch": "hip graph replay" if use_graph else "eager"},
        "roofline": roofline, "kernels": kern, "timed_wall_s": round(wall_s, 3),
    }
    result.update(extra)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, synth, seq_lens)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
