#!/usr/bin/env python3
"""Benchmark of the verify-and-speculate step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that
is already resident in HBM: N_s multi-stream-attention layers (each with its own
paged KV cache and q/k/v), the LM head with fused arg-max/top-k on the last
layer's output, greedy tree verification and tree drafting, all enqueued on one
stream through the C ABI with no host synchronisation in between.

Headline workload: c4 (4 sequences, 32x128 heads, prefix 4096, 16-node trees x 4
streams, 4 MSA layers, LM head 320 x 4096 x 32000, top-4), the only configuration
that contains every part of the path.  `--workload c2|c3|c5` time the attention
layer(s) of another configuration instead (no LM head in those); the default,
`--workload all`, reports c4 and appends the attention rooflines of c2, c3 and c5
as `other_workloads`.

Prints ONE JSON line.  `value` is microseconds per step.  `roofline` describes the
dominant kernel (the bf16 MSA kernel): algorithmic bytes per launch divided by the
kernel's own average duration, measured here with events on the launch stream
around a loop of that launch alone (rotating input sets).  Every timed per-kernel
loop has a fixed length (KERNEL_ITERS launches after KERNEL_WARMUP untimed ones)
whatever --steps says, and the GPU is brought to its working clock by
PREWARM_SECONDS of untimed steps before anything is timed.  `cpu_baseline` times
the CPU oracle on whole steps of the same inputs.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, vendor figure
KERNEL_ITERS = 200            # launches per timed per-kernel loop
KERNEL_WARMUP = 50            # untimed launches before each such loop
PREWARM_SECONDS = 0.4         # untimed steps before the warm-up steps (the first milliseconds of work run slower)
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "msa_kernel_hbm_traffic.md")


def msa_traffic_bytes(workload):
    """HBM bytes of one launch of the MSA kernel as the counters saw them: the row of this workload in the table
    of profiles/msa_kernel_hbm_traffic.md (`| workload | FETCH_SIZE KiB | fetch scale | WRITE_SIZE KiB | write
    scale |`, the scale factors being what the same counters read for a copy of known size).  None if the table
    has no such row."""
    try:
        text = open(TRAFFIC_TABLE).read()
    except OSError:
        return None
    for line in text.splitlines():
        m = re.match(r"\|\s*%s\s*\|\s*([0-9.]+)\s*\|\s*([0-9.]+)\s*\|\s*([0-9.]+)\s*\|\s*([0-9.]+)\s*\|" % re.escape(workload), line)
        if m:
            fetch, fs, write, wsc = (float(x) for x in m.groups())
            return int((fetch * fs + write * wsc) * 1024)
    return None


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


def timed(fn, iters, torch, warmup=0):
    """Average microseconds of fn(i) over iters calls, events on the current stream."""
    for i in range(warmup):
        fn(i)
    start = torch.cuda.Event(enable_timing=True)
    end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(iters):
        fn(i)
    end.record()
    torch.cuda.synchronize()
    return start.elapsed_time(end) * 1000.0 / iters


def kernel_timed(fn, torch):
    return timed(fn, KERNEL_ITERS, torch, KERNEL_WARMUP)


def describe(cfg, has_lm):
    return "%s: B=%d, %dx%d heads (%d KV), prefix %s, %d-node trees x %d streams (%d rows/seq), %d-token pages, %d MSA layer(s)%s" % (
        cfg.name, cfg.B, cfg.H, cfg.D, cfg.Hkv, cfg.L_min if cfg.L_min == cfg.L_max else "%d..%d" % (cfg.L_min, cfg.L_max),
        cfg.T, cfg.gamma, cfg.R, cfg.page, cfg.n_layers,
        ", LM head %dx%dx%d top-%d" % (cfg.B * cfg.R, cfg.d_model, cfg.vocab, cfg.K) if has_lm else "")


class MsaWorkload:
    """The attention layers of one configuration: rotating input sets on the GPU, one workspace, one output per layer."""

    def __init__(self, cfg, api, synth, torch, np, dev):
        self.cfg, self.api, self.torch = cfg, api, torch
        self.seq_lens = synth.seq_lens_for(cfg, 1)
        per_layer = msa_bytes(cfg, self.seq_lens)
        # Each MSA layer has its own caches; input sets are rotated so that one rotation touches more than
        # 512 MB and the 256 MB last-level cache cannot serve repeats.
        n_sets = max(cfg.n_layers, int(np.ceil(768e6 / per_layer)))
        self.n_sets = ((n_sets + cfg.n_layers - 1) // cfg.n_layers) * cfg.n_layers
        self.layers = [synth.make_msa_inputs(cfg, 1, device=dev, layer=i) for i in range(self.n_sets)]
        self.outs = [torch.empty_like(self.layers[0]["q"]) for _ in range(cfg.n_layers)]
        self.max_len = self.layers[0]["block_table"].shape[1] * cfg.page
        self.code = api.SS_BF16 if cfg.dtype == "bf16" else api.SS_F32
        self.ws = api.ss_msa_workspace(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, self.max_len, self.code, dev)
        self.parent = self.layers[0]["parent"]

    def call(self, layer, out, flags=0):
        c = self.cfg
        self.api.ss_msa_attention(layer["q"], layer["k_new"], layer["v_new"], layer["k_cache"], layer["v_cache"],
                                  layer["block_table"], layer["seq_lens"], self.parent, c.gamma, layer["scale"],
                                  flags=flags, out=out, workspace=self.ws)

    def layers_of_step(self, i):
        base = (i * self.cfg.n_layers) % self.n_sets
        return self.layers[base:base + self.cfg.n_layers]

    def roofline(self, workload_name):
        """Times the attention call and the attention kernel alone; returns (roofline, kernel timings)."""
        api, torch, cfg = self.api, self.torch, self.cfg
        us_call = kernel_timed(lambda i: self.call(self.layers[i % self.n_sets], self.outs[0]), torch)
        us_partials = kernel_timed(lambda i: self.call(self.layers[i % self.n_sets], self.outs[0], api.SS_MSA_PARTIALS_ONLY), torch)
        # The roofline is that of the attention kernel as the step launches it.  A full call is that kernel alone
        # when the prefix is unsplit or its two splits are merged inside the kernel (c4): then the loop of whole
        # calls times it; otherwise a merge kernel follows and the loop that leaves the merge out does.
        n_splits, n_kernels = api.ss_msa_plan(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, self.max_len, self.code)
        us_kernel = us_call if n_kernels == 1 else us_partials
        kern = {"msa_call_us": round(us_call, 2), "msa_kernel_us": round(us_kernel, 2),
                "msa_kernel_without_split_merge_us": round(us_partials, 2), "msa_splits": n_splits,
                "msa_kernels_per_call": n_kernels}
        b_msa, f_msa = msa_bytes(cfg, self.seq_lens), msa_flops(cfg, self.seq_lens)
        gbps = b_msa / (us_kernel * 1e-6) / 1e9
        tflops = f_msa / (us_kernel * 1e-6) / 1e12
        # Which roofline binds the kernel on this workload: the matrix cores if its FLOP per byte exceed the
        # machine's ridge (long GQA trees: c5), HBM otherwise.  Both figures are reported either way.
        if f_msa / b_msa > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBPS * 1e9):
            roof = {"kernel": "msa_bf16_kernel", "bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                    "traffic": msa_traffic_bytes(workload_name), "algorithmic_flops": f_msa, "hbm_gbps": round(gbps, 1)}
        else:
            roof = {"kernel": "msa_bf16_kernel", "bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": msa_traffic_bytes(workload_name),
                    "algorithmic_bytes": b_msa, "mfma_tflops": round(tflops, 1)}
        roof["kernel_us"] = round(us_kernel, 2)
        if n_kernels == 1 and n_splits > 1:
            # for comparison: the same kernel when it leaves the split merge to a second kernel
            roof["without_split_merge"] = {"us": round(us_partials, 2),
                                           "frac": round(b_msa / (us_partials * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
        return roof, kern


def cpu_baseline(cfg, synth, work, lm, tok_np, torch):
    """The oracle on the inputs the GPU steps ran on (the first step's input sets, copied to the host; the LM head
    on the oracle's own last-layer output rounded to the storage type, as the GPU's is), whole steps (every MSA
    layer, the LM head, verify, draft), repeated until about 10 s of CPU time have been spent (at most 8 steps);
    the mean step is reported."""
    import numpy as np
    import oracle
    oracle.build()
    f32 = lambda t: t.float().cpu().numpy()
    layers = []
    for inp in work.layers[:cfg.n_layers]:
        layers.append((f32(inp["q"]), f32(inp["k_new"]), f32(inp["v_new"]), f32(inp["k_cache"]), f32(inp["v_cache"]),
                       inp["block_table"].cpu().numpy(), inp["seq_lens"].cpu().numpy(), work.parent.cpu().numpy(),
                       cfg.gamma, inp["scale"]))
    par = layers[0][7]
    if cfg.vocab:
        W = f32(lm["W"])
        tp, tr, _ = oracle.full_tree_template(cfg.draft_branching)
    reps, t_all = 0, 0.0
    while reps < 8 and t_all < 10.0:
        t0 = time.perf_counter()
        for a in layers:
            out = oracle.msa_attention(*a)
        if cfg.vocab:
            hidden = torch.from_numpy(np.ascontiguousarray(out, dtype=np.float32)).to(cfg.torch_dtype).float().numpy()
            idx, _ = oracle.lm_head_topk(hidden.reshape(cfg.B * cfg.R, cfg.d_model), W, cfg.K)
            idx = np.ascontiguousarray(idx.reshape(cfg.B, cfg.R, cfg.K))
            ver = oracle.tree_verify(tok_np, par, np.ascontiguousarray(idx[:, :cfg.T, 0]), cfg.max_depth)
            topk = np.ascontiguousarray(idx[:, cfg.T:, :].reshape(cfg.B, cfg.T, cfg.gamma, cfg.K))
            oracle.tree_draft(topk, ver["last"], ver["bonus"], tp, tr)
        t_all += time.perf_counter() - t0
        reps += 1
    return {"value": round(t_all / reps * 1e6, 1), "unit": "us", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d whole steps on the GPU steps' own input sets (%d MSA layers + LM head + verify + draft each), "
                      "%.1f s in all; mean step" % (reps, cfg.n_layers, t_all)}


def calibrate_copy(torch, dev):
    """A plain device-to-device copy of known size (256 MiB read, 256 MiB written per call), so that a
    rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this script has a kernel to scale the counters by."""
    src = torch.ones(128 * 1024 * 1024, dtype=torch.bfloat16, device=dev)
    dst = torch.empty_like(src)
    for _ in range(4):
        dst.copy_(src)
    torch.cuda.synchronize()


def weight_copies(nbytes, footprint=1 << 30):
    """Copies of a weight matrix to use in turn so that no cache (256 MB last level) can hold them."""
    return max(2, -(-footprint // nbytes))


def time_rows_after_hot_path(api, synth, torch, cfg, dev, N, lm, lm_ws, tok, parent, extra):
    """Rows after the hot path (not part of `value`), each in a loop of its own; fills `extra`."""
    # Dense projections of one MSA layer on the step's N rows: fused QKV, attention output, fused gate+up and
    # down of a 4096/11008 feed-forward block.
    dm, dff = cfg.d_model, 11008
    dense = {}
    total = total_plain = 0.0
    for name, (din, dout) in (("qkv", (dm, 3 * cfg.H * cfg.D)), ("attn_out", (cfg.H * cfg.D, dm)),
                              ("gate_up", (dm, 2 * dff)), ("down", (dff, dm))):
        # Weights come from HBM in a model (a layer's 400 MB, 13 GB for all layers): as many copies in turn as
        # make up 1 GB, four times the last-level cache.  With two copies of a 90 MB matrix the cache serves
        # them and the map reads 40 % faster than it ever would in a layer sequence.
        copies = weight_copies(din * dout * 2)
        x0 = synth.make_lm_head_inputs(synth.scaled(cfg, vocab=dout, d_model=din), 50, device=dev, N=N)
        xs = [x0] + [{"hidden": x0["hidden"], "W": x0["W"].clone()} for _ in range(copies - 1)]
        y = torch.empty(N, dout, dtype=xs[0]["hidden"].dtype, device=dev)
        us_plain = kernel_timed(lambda i: api.ss_linear_rows(xs[i % copies]["hidden"], xs[i % copies]["W"], y), torch)
        # the same map with a workspace: few outputs and many features are cut along the feature dimension
        slices = api.ss_linear_rows_splits(N, din, dout, api.SS_BF16)
        lin_ws = torch.empty(api.ss_linear_rows_workspace_bytes(N, din, dout, api.SS_BF16), dtype=torch.uint8, device=dev)
        us = kernel_timed(lambda i: api.ss_linear_rows_ws(xs[i % copies]["hidden"], xs[i % copies]["W"], y, workspace=lin_ws),
                          torch) if slices > 1 else us_plain
        total += us
        total_plain += us_plain
        dense[name] = {"d_in": din, "d_out": dout, "us": round(us, 2), "feature_slices": slices,
                       "us_without_workspace": round(us_plain, 2), "weight_copies_in_turn": copies,
                       "tflops": round(2.0 * N * din * dout / (us * 1e-6) / 1e12, 1),
                       "hbm_gbps": round((din * dout + N * din + N * dout) * 2 / (us * 1e-6) / 1e9, 1)}
        del xs, y, lin_ws
    dense["layer_total_us"] = round(total, 2)
    dense["layer_total_without_workspace_us"] = round(total_plain, 2)
    extra["linear_rows"] = dense
    # The pruning layer: log-sum-exp of the early-exit logits of the B*T main rows over the whole vocabulary,
    # transition probabilities, pruning decision and compaction.
    hm = synth.make_lm_head_inputs(cfg, 60, device=dev, N=cfg.B * cfg.T)["hidden"].view(cfg.B, cfg.T, dm)
    w_copies = [lm["W"], lm["W"].clone()]
    lse = torch.empty(cfg.B * cfg.T, dtype=torch.float32, device=dev)
    prob = torch.empty(cfg.B, cfg.T, dtype=torch.float32, device=dev)

    def prune_layer(i):
        api.ss_lm_head_logsumexp(hm.view(cfg.B * cfg.T, dm), w_copies[i & 1], lse=lse, workspace=lm_ws)
        api.ss_transition_probs(hm, w_copies[i & 1], tok, parent, lse, prob=prob)
        return api.ss_tree_prune(tok, parent, prob, 0.01)
    us_prune = kernel_timed(prune_layer, torch)
    us_lse = kernel_timed(lambda i: api.ss_lm_head_logsumexp(hm.view(cfg.B * cfg.T, dm), w_copies[i & 1], lse=lse,
                                                             workspace=lm_ws), torch)
    # Stream insertion (Eq. 3) for the same batch: elementwise, B*R*d elements
    P_emb = synth.make_lm_head_inputs(synth.scaled(cfg, vocab=64, d_model=dm), 61, device=dev, N=cfg.gamma)["hidden"]
    X_rows = torch.empty(cfg.B, cfg.R, dm, dtype=hm.dtype, device=dev)
    extra["stream_insert_us"] = round(kernel_timed(lambda i: api.ss_stream_insert(hm, P_emb, X=X_rows), torch), 2)
    # ... and Eq. 3 through the QKV projection of the first multi-stream layer: rows written out and projected, against
    # the one call that projects the B*T states and the gamma embeddings only and adds the results
    dq = 3 * cfg.H * cfg.D
    wq = [synth.make_lm_head_inputs(synth.scaled(cfg, vocab=dq, d_model=dm), 62, device=dev, N=8)["W"]]
    n_wq = weight_copies(dq * dm * 2)
    wq += [wq[0].clone() for _ in range(n_wq - 1)]
    Yq = torch.empty(cfg.B, cfg.R, dq, dtype=hm.dtype, device=dev)
    sil_ws = torch.empty(api.load_library().ss_stream_insert_linear_workspace_bytes(cfg.B, cfg.T, cfg.gamma, dm, dq, api.SS_BF16, 0),
                         dtype=torch.uint8, device=dev)

    def unfused(i):
        api.ss_stream_insert(hm, P_emb, X=X_rows)
        api.ss_linear_rows(X_rows.view(cfg.B * cfg.R, dm), wq[i % n_wq], Yq.view(cfg.B * cfg.R, dq))
    extra["stream_insert_qkv"] = {
        "insert_then_project_us": round(kernel_timed(unfused, torch), 2),
        "one_call_us": round(kernel_timed(lambda i: api.ss_stream_insert_linear(hm, P_emb, wq[i % n_wq], Y=Yq, workspace=sil_ws), torch), 2)}
    del wq, Yq
    # The appendix's value-rotation variant on one layer's value block [B,R,Hkv,D], in place
    v_blk = X_rows.view(cfg.B, cfg.R, cfg.Hkv, dm // cfg.Hkv) if dm % cfg.Hkv == 0 and (dm // cfg.Hkv) % 2 == 0 else None
    if v_blk is not None:
        extra["value_rotate_us"] = round(kernel_timed(lambda i: api.ss_value_rotate(v_blk, cfg.T, cfg.gamma, 1e-4), torch), 2)
    extra["prune_layer"] = {"us": round(us_prune, 2), "logsumexp_us": round(us_lse, 2),
                            "logsumexp_hbm_gbps": round(cfg.vocab * dm * 2 / (us_lse * 1e-6) / 1e9, 1)}
    del w_copies


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="all", choices=["all", "c2", "c3", "c4", "c5"],
                    help="all (default): c4 as the headline plus the attention rooflines of c2, c3 and c5")
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
    headline = "c4" if args.workload == "all" else args.workload
    cfg = synth.CONFIGS[headline]
    api.load_library()
    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    if args.split_keys:
        api.ss_msa_set_split_keys(args.split_keys)

    work = MsaWorkload(cfg, api, synth, torch, np, dev)
    parent = work.parent
    outs = work.outs
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
    else:
        lm, tok_np = None, None

    state = {}

    def step(i, kernel_events=None):
        for j, layer in enumerate(work.layers_of_step(i)):
            if kernel_events is None:
                work.call(layer, outs[j])
            else:
                # the same two kernels as two calls, with a pair of events around the attention kernel alone
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                work.call(layer, outs[j], api.SS_MSA_PARTIALS_ONLY)
                e1.record()
                work.call(layer, outs[j], api.SS_MSA_MERGE_ONLY)
                kernel_events.append((e0, e1))
        if has_lm:
            hidden = outs[-1].view(N, cfg.d_model)
            if args.separate_tail:
                # a3, a4 and a5 as three calls (four kernels)
                api.ss_lm_head_argmax_topk(hidden, lm["W"], cfg.K, idx=idx, val=val, workspace=lm_ws)
                ver = api.ss_tree_verify(tok, parent, idx, cfg.max_depth, batch_stride=cfg.R * cfg.K, node_stride=cfg.K,
                                         out=state.get("ver_out"))
                nxt = api.ss_tree_draft(idx, cfg.K, ver["last"], ver["bonus"], cfg.T, cfg.gamma,
                                        branching=cfg.draft_branching, batch_stride=cfg.R * cfg.K, offset=cfg.T * cfg.K,
                                        out=state.get("nxt_out"))
                state["ver_out"], state["nxt_out"] = ver, nxt
                state["ver"], state["nxt"], state["argmax"] = ver, nxt, idx.view(cfg.B, cfg.R, cfg.K)[:, :cfg.T, 0]
            else:
                # the same three rows in one call (two kernels): the candidate merge happens in the kernel
                # that verifies and drafts, for the rows those steps read
                t = api.ss_lm_head_verify_draft(hidden, lm["W"], cfg.K, tok, parent, cfg.gamma, cfg.max_depth,
                                                branching=cfg.draft_branching, workspace=lm_ws, out=state.get("tail"))
                state["tail"] = t
                state["ver"], state["nxt"], state["argmax"] = t, (t["next_tok"], t["next_parent"]), t["main_argmax"]

    # ---- the GPU reaches its working clock only after some milliseconds of work: untimed steps first
    step(0)
    torch.cuda.synchronize()
    t_pre = time.perf_counter()
    n_pre = 0
    while time.perf_counter() - t_pre < PREWARM_SECONDS:
        for i in range(50):
            step(n_pre + i)
        n_pre += 50
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if has_lm and work.n_sets == cfg.n_layers:
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
    use_graph = args.graph and work.n_sets == cfg.n_layers
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

    # ---- per-kernel figures (each in its own timed loop of fixed length, same rotation of inputs)
    roofline, kern = work.roofline(headline)
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
    # The read rate this GPU reaches with plain 16-byte loads over 1 GiB (four times the last-level cache), next to
    # the published peak the fraction is taken against
    probe_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_()
    probe_sink = torch.zeros(1, dtype=torch.int32, device=dev)
    roofline["measured_read_ceiling_gbps"] = {
        "plain": round((1 << 30) / (timed(lambda i: api.ss_probe_hbm_read(probe_buf, False, probe_sink), 20, torch, 5) * 1e-6) / 1e9, 1),
        "streaming": round((1 << 30) / (timed(lambda i: api.ss_probe_hbm_read(probe_buf, True, probe_sink), 20, torch, 5) * 1e-6) / 1e9, 1)}
    del probe_buf
    extra = {}
    if has_lm:
        hidden = outs[-1].view(N, cfg.d_model)
        # two copies of W in turn: a single 262 MB matrix would partly stay in the last-level cache between
        # calls, which it cannot inside a step (the MSA layers stream more than a gigabyte in between)
        w_copies = [lm["W"], lm["W"].clone()]
        us_lm = kernel_timed(lambda i: api.ss_lm_head_argmax_topk(hidden, w_copies[i & 1], cfg.K, idx=idx, val=val,
                                                                  workspace=lm_ws), torch)
        # the matrix kernel alone (the call stops before the kernel that merges the tiles' candidates)
        api.ss_lm_set_candidates_only(True)
        try:
            us_lm_kernel = kernel_timed(lambda i: api.ss_lm_head_argmax_topk(hidden, w_copies[i & 1], cfg.K, idx=idx, val=val,
                                                                             workspace=lm_ws), torch)
        finally:
            api.ss_lm_set_candidates_only(False)
        api.ss_lm_head_argmax_topk(hidden, w_copies[0], cfg.K, idx=idx, val=val, workspace=lm_ws)  # idx / val valid again
        tail_out = state.get("tail") or api.ss_lm_head_verify_draft(hidden, lm["W"], cfg.K, tok, parent, cfg.gamma, cfg.max_depth,
                                                                    branching=cfg.draft_branching, workspace=lm_ws)
        us_tail = kernel_timed(lambda i: api.ss_lm_head_verify_draft(hidden, w_copies[i & 1], cfg.K, tok, parent, cfg.gamma,
                                                                     cfg.max_depth, branching=cfg.draft_branching,
                                                                     workspace=lm_ws, out=tail_out), torch)
        del w_copies
        # a4 and a5 as calls of their own, with preallocated outputs (what is timed is the kernel and its launch)
        ver = api.ss_tree_verify(tok, parent, idx, cfg.max_depth, batch_stride=cfg.R * cfg.K, node_stride=cfg.K)
        us_ver = kernel_timed(lambda i: api.ss_tree_verify(tok, parent, idx, cfg.max_depth, batch_stride=cfg.R * cfg.K,
                                                           node_stride=cfg.K, out=ver), torch)
        nxt = api.ss_tree_draft(idx, cfg.K, ver["last"], ver["bonus"], cfg.T, cfg.gamma, branching=cfg.draft_branching,
                                batch_stride=cfg.R * cfg.K, offset=cfg.T * cfg.K)
        us_draft = kernel_timed(lambda i: api.ss_tree_draft(idx, cfg.K, ver["last"], ver["bonus"], cfg.T, cfg.gamma,
                                                            branching=cfg.draft_branching, batch_stride=cfg.R * cfg.K,
                                                            offset=cfg.T * cfg.K, out=nxt), torch)
        # KV-cache commit of the accepted path (the row after the hot path: not part of `value`), all layers
        cap = work.max_len
        short = torch.clamp(work.layers[0]["seq_lens"], max=cap - cfg.max_depth - 1)
        new_lens = torch.empty_like(short)
        us_commit = kernel_timed(lambda i: [api.ss_kv_commit(l["k_new"], l["v_new"], l["k_cache"], l["v_cache"], l["block_table"], short,
                                                              ver["path"], ver["n_accept"], cfg.gamma, new_seq_lens=new_lens)
                                            for l in work.layers[:cfg.n_layers]], torch)
        kern.update({"lm_head_call_us": round(us_lm, 2), "lm_head_kernel_us": round(us_lm_kernel, 2),
                     "lm_head_verify_draft_call_us": round(us_tail, 2),
                     "verify_us": round(us_ver, 2), "draft_us": round(us_draft, 2),
                     "kv_commit_all_layers_us": round(us_commit, 2)})
        f_lm = 2.0 * N * cfg.vocab * cfg.d_model
        tf = f_lm / (us_lm * 1e-6) / 1e12
        mfma_sink = torch.zeros(1, dtype=torch.float32, device=dev)
        mfma_flops = api.ss_probe_mfma_bf16(1000, mfma_sink)
        us_mfma = timed(lambda i: api.ss_probe_mfma_bf16(1000, mfma_sink), 20, torch, 5)
        ceiling = mfma_flops / (us_mfma * 1e-6) / 1e12
        extra["roofline_lm_head"] = {"kernel": "lm_head_bf16_kernel + lm_head_reduce_kernel", "bound": "mfma", "achieved": round(tf, 1),
                                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                                     # lm_head_bf16_kernel alone, as a kernel trace shows it
                                     "matrix_kernel_alone": {"us": round(us_lm_kernel, 2),
                                                             "frac": round(f_lm / (us_lm_kernel * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)},
                                     "hbm_gbps": round((cfg.vocab * cfg.d_model * 2 + N * cfg.d_model * 2) /
                                                       (us_lm * 1e-6) / 1e9, 1),
                                     # register-only matrix-core work on the whole chip, at the clock it is granted
                                     "measured_mfma_ceiling_tflops": round(ceiling, 1),
                                     "frac_of_measured_ceiling": round(tf / ceiling, 4)}
        extra["accepted_per_sequence"] = state["ver"]["n_accept"].tolist()
        if headline == "c4":
            try:
                time_rows_after_hot_path(api, synth, torch, cfg, dev, N, lm, lm_ws, tok, parent, extra)
            except Exception as e:  # the headline measurement must survive a failure here
                extra["rows_after_hot_path_error"] = "%s: %s" % (type(e).__name__, e)

    result = {
        "metric": "verify+speculate step time (MSA layers + LM-head argmax/top-k + verify + draft)",
        "value": round(us_step, 2), "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us_step / 1000.0, 5), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": describe(cfg, has_lm), "input_sets_rotated": work.n_sets,
                   "split_keys": args.split_keys or "auto", "launch": "hip graph replay" if use_graph else "eager",
                   "untimed_prewarm_steps": n_pre, "kernel_loop_iters": KERNEL_ITERS, "kernel_loop_warmup": KERNEL_WARMUP},
        "roofline": roofline, "kernels": kern, "timed_wall_s": round(wall_s, 3),
    }
    result.update(extra)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, synth, work, lm, tok_np, torch)
    if args.workload == "all":
        # the attention layers of the other configurations, each in loops of its own (no LM head in those)
        del work, outs
        others = {}
        for name in ("c2", "c3", "c5"):
            try:
                torch.cuda.empty_cache()
                ocfg = synth.CONFIGS[name]
                w2 = MsaWorkload(ocfg, api, synth, torch, np, dev)
                us_layers = kernel_timed(lambda i: [w2.call(l, w2.outs[j]) for j, l in enumerate(w2.layers_of_step(i))], torch)
                roof, k2 = w2.roofline(name)
                roof["workload"] = describe(ocfg, False)
                roof["all_layers_us"] = round(us_layers, 2)
                roof["call_us"] = k2["msa_call_us"]
                roof["splits"], roof["kernels_per_call"] = k2["msa_splits"], k2["msa_kernels_per_call"]
                others[name] = roof
                del w2
            except Exception as e:  # the headline measurement must survive a failure here
                others[name] = {"error": "%s: %s" % (type(e).__name__, e)}
        result["other_workloads"] = others
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
