"""Python binding of libss.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/ss.h),
takes torch tensors that already live on the GPU, checks their shapes / dtypes /
contiguity, and passes raw device pointers plus the current HIP stream.  Output
tensors and workspaces are allocated here with torch when the caller does not
pass them; no arithmetic of the method happens in Python.  There is no CPU
fallback: if libss.so has not been built, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libss.so")

SS_OK = 0
SS_F32, SS_BF16 = 0, 1
SS_STREAM_EXCLUDE_SELF = 1
SS_MSA_PARTIALS_ONLY = 2
SS_MSA_MERGE_ONLY = 4
SS_MAX_T, SS_MAX_GAMMA, SS_MAX_K = 64, 8, 8

EXPORTS = (
    "ss_version", "ss_last_error", "ss_probe_hbm_read", "ss_probe_mfma_bf16", "ss_check_tree_host", "ss_build_mask", "ss_msa_workspace_bytes",
    "ss_msa_attention", "ss_msa_workspace_init", "ss_msa_attention_static", "ss_msa_static_scratch_bytes", "ss_msa_plan", "ss_msa_set_split_keys", "ss_msa_set_merge_in_kernel", "ss_lm_head_workspace_bytes", "ss_lm_set_flavour", "ss_lm_set_stagger", "ss_lm_set_candidates_only", "ss_lm_head_argmax_topk", "ss_lm_head_verify_draft",
    "ss_tree_verify", "ss_tree_draft", "ss_full_tree_template_host", "ss_kv_commit", "ss_kv_alloc_pages", "ss_linear_rows", "ss_linear_rows_ws", "ss_linear_rows_workspace_bytes", "ss_linear_rows_splits", "ss_stream_insert", "ss_stream_insert_linear", "ss_stream_insert_linear_workspace_bytes", "ss_value_rotate",
    "ss_lm_head_logsumexp", "ss_transition_probs", "ss_tree_prune", "ss_live_rows", "ss_msa_attention_pruned",
    "ss_linear_rows_live", "ss_lm_head_argmax_topk_live", "ss_lm_head_verify_draft_live",
)

_lib = None


class SSError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("libss error %d: %s" % (code, msg))
        self.code = code


def load_library() -> ctypes.CDLL:
    """Loads libss.so (after torch, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libss.so is not built (%s missing): run `python -m paper_2402_11131_amd.build` "
            "or __graft_entry__.build(); there is no fallback path" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i32, u32, sz, lng = c.c_void_p, c.c_int, c.c_uint32, c.c_size_t, c.c_long
    lib.ss_version.restype = i32
    lib.ss_last_error.restype = c.c_char_p
    lib.ss_check_tree_host.argtypes = [vp, i32, i32, i32]
    lib.ss_probe_hbm_read.argtypes = [vp, sz, i32, vp, vp]
    lib.ss_probe_mfma_bf16.argtypes = [i32, c.POINTER(c.c_double), vp, vp]
    lib.ss_build_mask.argtypes = [vp, i32, i32, i32, u32, vp, vp, vp, vp]
    lib.ss_msa_workspace_bytes.argtypes = [i32] * 8
    lib.ss_msa_workspace_bytes.restype = sz
    lib.ss_msa_plan.argtypes = [i32] * 8 + [ctypes.POINTER(ctypes.c_int)] * 2
    lib.ss_msa_plan.restype = i32
    lib.ss_msa_attention.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, i32, i32, i32, i32, i32, i32,
                                     c.c_float, i32, u32, vp, vp, sz, vp]
    lib.ss_msa_workspace_init.argtypes = [vp, sz, vp]
    lib.ss_msa_attention_static.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, i32, i32, i32, i32, i32, i32,
                                            c.c_float, i32, u32, vp, vp]
    lib.ss_msa_static_scratch_bytes.restype = sz
    lib.ss_msa_set_split_keys.argtypes = [i32]
    lib.ss_msa_set_merge_in_kernel.argtypes = [i32]
    lib.ss_lm_head_workspace_bytes.argtypes = [i32] * 5
    lib.ss_lm_set_flavour.argtypes = [i32, i32, i32]
    lib.ss_lm_set_stagger.argtypes = [i32]
    lib.ss_lm_set_candidates_only.argtypes = [i32]
    lib.ss_lm_head_workspace_bytes.restype = sz
    lib.ss_lm_head_argmax_topk.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.ss_tree_verify.argtypes = [vp, vp, vp, lng, lng, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.ss_lm_head_verify_draft.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, i32, i32, i32, i32, vp, vp, vp, i32] + [vp] * 9 + [sz, vp]
    lib.ss_tree_draft.argtypes = [vp, lng, i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
    lib.ss_full_tree_template_host.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.ss_kv_commit.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.ss_kv_alloc_pages.argtypes = [vp, i32, vp, vp, i32, i32, i32, vp, vp, vp, vp]
    lib.ss_linear_rows.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp]
    lib.ss_linear_rows_ws.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.ss_linear_rows_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.ss_linear_rows_workspace_bytes.restype = sz
    lib.ss_linear_rows_splits.argtypes = [i32, i32, i32, i32]
    lib.ss_stream_insert.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
    lib.ss_stream_insert_linear_workspace_bytes.argtypes = [i32] * 7
    lib.ss_stream_insert_linear_workspace_bytes.restype = sz
    lib.ss_stream_insert_linear.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.ss_value_rotate.argtypes = [vp, i32, i32, i32, i32, i32, c.c_float, i32, vp]
    lib.ss_lm_head_logsumexp.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.ss_transition_probs.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
    lib.ss_tree_prune.argtypes = [vp, vp, vp, c.c_float, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.ss_live_rows.argtypes = [vp, i32, i32, i32, vp, vp, vp]
    lib.ss_msa_attention_pruned.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32,
                                            c.c_float, i32, u32, vp, vp, sz, vp]
    lib.ss_linear_rows_live.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, i32, vp]
    lib.ss_lm_head_argmax_topk_live.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.ss_lm_head_verify_draft_live.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, i32, i32, i32, i32, vp, vp, vp, i32] + [vp] * 8 + [vp, vp, i32, vp, sz, vp]
    for name in EXPORTS:
        getattr(lib, name)
    _lib = lib
    return lib


def _check(rc: int):
    if rc != SS_OK:
        raise SSError(rc, load_library().ss_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError("%s must be a contiguous GPU tensor of dtype %s" % (name, dtype))
    return t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SS_F32
    if t.dtype == torch.bfloat16:
        return SS_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def ss_probe_hbm_read(buf: torch.Tensor, streaming: bool, sink: torch.Tensor) -> None:
    """Measurement aid: one pass of 16-byte loads over `buf` (a contiguous GPU tensor), nothing written."""
    _check(load_library().ss_probe_hbm_read(buf.data_ptr(), buf.numel() * buf.element_size(), 1 if streaming else 0,
                                            sink.data_ptr(), _stream()))


def ss_probe_mfma_bf16(iters: int, sink: torch.Tensor) -> float:
    """Measurement aid: register-only bf16 matrix-core work on the whole chip; returns the launch's FLOPs."""
    fl = ctypes.c_double(0.0)
    _check(load_library().ss_probe_mfma_bf16(int(iters), ctypes.byref(fl), sink.data_ptr(), _stream()))
    return fl.value


def ss_version() -> int:
    return load_library().ss_version()


def ss_check_tree_host(parent, max_depth: int = -1) -> None:
    """parent: CPU int32 tensor [B,T].  Raises SSError on a malformed tree."""
    p = parent.to(torch.int32).contiguous().cpu()
    B, T = p.shape
    _check(load_library().ss_check_tree_host(p.data_ptr(), B, T, max_depth))


def ss_build_mask(parent: torch.Tensor, gamma: int, flags: int = 0, want_mask: bool = True):
    """a1.  parent [B,T] int32 -> (mask [B,R,R] uint8 or None, anc [B,T] int64 (bit pattern of the
    uint64 ancestor sets), depth [B,T] int32)."""
    lib = load_library()
    B, T = parent.shape
    R = T * (1 + gamma)
    dev = parent.device
    mask = torch.empty((B, R, R), dtype=torch.uint8, device=dev) if want_mask else None
    anc = torch.empty((B, T), dtype=torch.int64, device=dev)
    depth = torch.empty((B, T), dtype=torch.int32, device=dev)
    _check(lib.ss_build_mask(_dev(parent, torch.int32, "parent"), B, T, gamma, flags,
                             mask.data_ptr() if want_mask else None, anc.data_ptr(), depth.data_ptr(), _stream()))
    return mask, anc, depth


def ss_msa_workspace_bytes(B, T, gamma, H, Hkv, D, max_seq_len, dtype_code) -> int:
    return load_library().ss_msa_workspace_bytes(B, T, gamma, H, Hkv, D, max_seq_len, dtype_code)


def ss_msa_plan(B, T, gamma, H, Hkv, D, max_seq_len, dtype_code):
    """(n_splits, n_kernels) of a full ss_msa_attention call of this shape, as currently tuned."""
    ns, nk = ctypes.c_int(0), ctypes.c_int(0)
    _check(load_library().ss_msa_plan(B, T, gamma, H, Hkv, D, max_seq_len, dtype_code, ctypes.byref(ns), ctypes.byref(nk)))
    return ns.value, nk.value


def ss_msa_set_split_keys(split_keys: int) -> int:
    return load_library().ss_msa_set_split_keys(int(split_keys))


def ss_msa_set_merge_in_kernel(on: bool) -> bool:
    """Tuning knob: merge two KV splits inside the attention kernel (default on).  Returns the previous setting."""
    return bool(load_library().ss_msa_set_merge_in_kernel(1 if on else 0))


def ss_msa_workspace(B, T, gamma, H, Hkv, D, max_seq_len, dtype_code, device) -> torch.Tensor:
    """A zero-filled workspace for ss_msa_attention calls of this shape (the arrival counters of the in-kernel
    split merge must be zero before the first call; every call leaves them zero)."""
    need = ss_msa_workspace_bytes(B, T, gamma, H, Hkv, D, max_seq_len, dtype_code)
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device=device)
    ss_msa_workspace_init(ws)
    return ws


def ss_msa_workspace_init(workspace: torch.Tensor) -> torch.Tensor:
    _check(load_library().ss_msa_workspace_init(_dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()))
    return workspace


def _msa_shapes(q, k_new, v_new, k_cache, v_cache, block_table, seq_lens, parent, gamma):
    B, R, H, D = q.shape
    Hkv = k_new.shape[2]
    T = parent.shape[1]
    P, _, page, _ = k_cache.shape
    if R != T * (1 + gamma) or tuple(k_new.shape) != (B, R, Hkv, D) or tuple(v_new.shape) != (B, R, Hkv, D):
        raise ValueError("q / k_new / v_new shapes do not match B,R,H,Hkv,D")
    if tuple(k_cache.shape) != (P, Hkv, page, D) or tuple(v_cache.shape) != (P, Hkv, D, page):
        raise ValueError("k_cache must be [P,Hkv,page,D] and v_cache [P,Hkv,D,page]")
    if block_table.shape[0] != B or tuple(seq_lens.shape) != (B,) or parent.shape[0] != B:
        raise ValueError("block_table / seq_lens / parent batch size mismatch")
    return B, R, H, D, Hkv, T, P, page, block_table.shape[1]


def ss_msa_attention(q, k_new, v_new, k_cache, v_cache, block_table, seq_lens, parent, gamma: int, scale: float,
                     flags: int = 0, out: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, n_nodes: Optional[torch.Tensor] = None) -> torch.Tensor:
    """a2.  q [B,R,H,D]; k_new, v_new [B,R,Hkv,D]; k_cache [P,Hkv,page,D]; v_cache [P,Hkv,D,page];
    block_table [B,max_pages] int32; seq_lens [B] int32; parent [B,T] int32.  Returns out [B,R,H,D].
    `workspace`: a tensor from ss_msa_workspace (zero-filled once); made here if not given.
    `n_nodes` [B] int32 (after pruning): ss_msa_attention_pruned is called, rows of padding nodes are left untouched."""
    lib = load_library()
    dt = q.dtype
    code = _dtype_code(q)
    B, R, H, D, Hkv, T, P, page, max_pages = _msa_shapes(q, k_new, v_new, k_cache, v_cache, block_table, seq_lens,
                                                          parent, gamma)
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = ss_msa_workspace(B, T, gamma, H, Hkv, D, max_pages * page, code, q.device)
    if n_nodes is not None:
        if tuple(n_nodes.shape) != (B,):
            raise ValueError("n_nodes must be [B]")
        _check(lib.ss_msa_attention_pruned(
            _dev(q, dt, "q"), _dev(k_new, dt, "k_new"), _dev(v_new, dt, "v_new"), _dev(k_cache, dt, "k_cache"),
            _dev(v_cache, dt, "v_cache"), _dev(block_table, torch.int32, "block_table"), max_pages, P,
            _dev(seq_lens, torch.int32, "seq_lens"), _dev(parent, torch.int32, "parent"), _dev(n_nodes, torch.int32, "n_nodes"),
            B, T, gamma, H, Hkv, D, page, float(scale), code, flags, _dev(out, dt, "out"),
            _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()))
        return out
    _check(lib.ss_msa_attention(
        _dev(q, dt, "q"), _dev(k_new, dt, "k_new"), _dev(v_new, dt, "v_new"), _dev(k_cache, dt, "k_cache"),
        _dev(v_cache, dt, "v_cache"), _dev(block_table, torch.int32, "block_table"), max_pages, P,
        _dev(seq_lens, torch.int32, "seq_lens"), _dev(parent, torch.int32, "parent"), B, T, gamma, H, Hkv, D, page,
        float(scale), code, flags, _dev(out, dt, "out"), _dev(workspace, torch.uint8, "workspace"),
        workspace.numel(), _stream()))
    return out


def ss_live_rows(n_nodes: torch.Tensor, T: int, gamma: int, live_rows: Optional[torch.Tensor] = None,
                 n_live: Optional[torch.Tensor] = None):
    """Rows of the kept nodes after pruning: (live_rows [B*R] int32, of which the first n_live[0] count; n_live [1])."""
    B = n_nodes.shape[0]
    i32 = torch.int32
    if live_rows is None:
        live_rows = torch.empty(max(B * T * (1 + gamma), 1), dtype=i32, device=n_nodes.device)
    if n_live is None:
        n_live = torch.empty(1, dtype=i32, device=n_nodes.device)
    _check(load_library().ss_live_rows(_dev(n_nodes, i32, "n_nodes"), B, T, gamma, _dev(live_rows, i32, "live_rows"),
                                       _dev(n_live, i32, "n_live"), _stream()))
    return live_rows, n_live


def ss_msa_static_scratch_bytes() -> int:
    return load_library().ss_msa_static_scratch_bytes()


def ss_msa_attention_static(q, k_new, v_new, k_cache, v_cache, block_table, seq_lens, parent, gamma: int,
                            scale: float, out: torch.Tensor, flags: int = 0) -> torch.Tensor:
    """a2 without a workspace: the scratch memory is the library's own array.  `out` must be given: this
    binding allocates nothing either."""
    lib = load_library()
    dt = q.dtype
    code = _dtype_code(q)
    B, R, H, D, Hkv, T, P, page, max_pages = _msa_shapes(q, k_new, v_new, k_cache, v_cache, block_table, seq_lens,
                                                          parent, gamma)
    _check(lib.ss_msa_attention_static(
        _dev(q, dt, "q"), _dev(k_new, dt, "k_new"), _dev(v_new, dt, "v_new"), _dev(k_cache, dt, "k_cache"),
        _dev(v_cache, dt, "v_cache"), _dev(block_table, torch.int32, "block_table"), max_pages, P,
        _dev(seq_lens, torch.int32, "seq_lens"), _dev(parent, torch.int32, "parent"), B, T, gamma, H, Hkv, D, page,
        float(scale), code, flags, _dev(out, dt, "out"), _stream()))
    return out


def ss_lm_head_workspace_bytes(N, d, V, K, dtype_code) -> int:
    return load_library().ss_lm_head_workspace_bytes(N, d, V, K, dtype_code)


def ss_lm_set_flavour(linear: bool, flavour) -> int:
    """Tuning knob: kernel shape of the LM head (linear=False) or of ss_linear_rows (linear=True): "<row tiles>"
    (4 waves, 1..6 tiles of 32 rows per workgroup), "<row tiles>w" (8 waves, 1..5) or None (automatic)."""
    if flavour is None:
        return load_library().ss_lm_set_flavour(1 if linear else 0, 0, 0)
    f = str(flavour)
    wide = f.endswith("w")
    return load_library().ss_lm_set_flavour(1 if linear else 0, int(f[:-1] if wide else f), 1 if wide else 0)


def ss_lm_set_stagger(blocks: int) -> int:
    """Tuning knob: feature blocks between the starting blocks of neighbouring vocabulary tiles (-1 = automatic)."""
    return load_library().ss_lm_set_stagger(int(blocks))


def ss_lm_set_candidates_only(on: bool) -> bool:
    """Profiling aid: while on, ss_lm_head_argmax_topk stops after the matrix kernel (idx / val are not written)."""
    return bool(load_library().ss_lm_set_candidates_only(1 if on else 0))


def ss_lm_head_argmax_topk(hidden, W, K: int, idx=None, val=None, workspace=None, live=None, plan_rows: int = 0):
    """a3.  hidden [N,d], W [V,d] -> (idx [N,K] int32, val [N,K] float32).  `live` = (live_rows, n_live) from
    ss_live_rows: only those rows are computed (the others of idx / val are left as they are)."""
    lib = load_library()
    dt = hidden.dtype
    code = _dtype_code(hidden)
    N, d = hidden.shape
    V = W.shape[0]
    if W.shape[1] != d:
        raise ValueError("hidden and W disagree on d")
    if idx is None:
        idx = torch.empty((N, K), dtype=torch.int32, device=hidden.device)
    if val is None:
        val = torch.empty((N, K), dtype=torch.float32, device=hidden.device)
    need = lib.ss_lm_head_workspace_bytes(N, d, V, K, code)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=hidden.device)
    if live is not None:
        _check(lib.ss_lm_head_argmax_topk_live(_dev(hidden, dt, "hidden"), _dev(W, dt, "W"), N, d, V, K, code,
                                               _dev(idx, torch.int32, "idx"), _dev(val, torch.float32, "val"),
                                               _dev(live[0], torch.int32, "live_rows"), _dev(live[1], torch.int32, "n_live"),
                                               int(plan_rows), _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                               _stream()))
        return idx, val
    _check(lib.ss_lm_head_argmax_topk(_dev(hidden, dt, "hidden"), _dev(W, dt, "W"), N, d, V, K, code,
                                      _dev(idx, torch.int32, "idx"), _dev(val, torch.float32, "val"),
                                      _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()))
    return idx, val


def ss_tree_verify(tok, parent, main_argmax, max_depth: int, batch_stride: Optional[int] = None,
                   node_stride: Optional[int] = None, offset: int = 0, out: Optional[dict] = None) -> dict:
    """a4.  tok, parent [B,T] int32.  main_argmax: int32 GPU tensor; the arg-max token of main row i
    of sequence b is element offset + b*batch_stride + i*node_stride of its storage (defaults: a
    contiguous [B,T] tensor).  `out` (the dict of an earlier call of the same shape) is reused if given."""
    lib = load_library()
    B, T = tok.shape
    if batch_stride is None:
        batch_stride, node_stride = T, 1
    dev = tok.device
    i32 = torch.int32
    if out is None:
        out = dict(n_accept=torch.empty(B, dtype=i32, device=dev), last=torch.empty(B, dtype=i32, device=dev),
                   bonus=torch.empty(B, dtype=i32, device=dev),
                   path=torch.empty((B, max_depth + 1), dtype=i32, device=dev),
                   out_tokens=torch.empty((B, max_depth + 1), dtype=i32, device=dev))
    elif out["n_accept"].shape != (B,) or out["path"].shape != (B, max_depth + 1) or out["out_tokens"].shape != (B, max_depth + 1):
        raise ValueError("`out` was made for another shape")
    res = out
    need = offset + (B - 1) * batch_stride + (T - 1) * node_stride + 1 if B > 0 else 0
    if main_argmax.numel() < need:
        raise ValueError("main_argmax too small for the given strides")
    _check(lib.ss_tree_verify(_dev(tok, i32, "tok"), _dev(parent, i32, "parent"),
                              _dev(main_argmax, i32, "main_argmax") + 4 * offset, batch_stride, node_stride, B, T,
                              max_depth, _dev(res["n_accept"], i32, "n_accept"), _dev(res["last"], i32, "last"),
                              _dev(res["bonus"], i32, "bonus"), _dev(res["path"], i32, "path"),
                              _dev(res["out_tokens"], i32, "out_tokens"), _stream()))
    return res


def ss_full_tree_template_host(branching: Sequence[int], capacity: int = SS_MAX_T):
    """Host helper: full tree with per-level branching -> (parent, rank, depth) CPU int32 tensors."""
    lib = load_library()
    br = torch.tensor(list(branching), dtype=torch.int32)
    par = torch.zeros(SS_MAX_T, dtype=torch.int32)
    rank = torch.zeros(SS_MAX_T, dtype=torch.int32)
    dep = torch.zeros(SS_MAX_T, dtype=torch.int32)
    n = lib.ss_full_tree_template_host(br.data_ptr(), len(branching), capacity, par.data_ptr(), rank.data_ptr(),
                                       dep.data_ptr())
    if n < 0:
        raise SSError(2, lib.ss_last_error().decode())
    return par[:n].clone(), rank[:n].clone(), dep[:n].clone()


def ss_tree_draft(stream_topk, K: int, last, bonus, T: int, gamma: int, tmpl_parent=None, tmpl_rank=None,
                  branching: Optional[Sequence[int]] = None, T2: Optional[int] = None,
                  batch_stride: Optional[int] = None, offset: int = 0, out=None):
    """a5.  stream_topk: int32 GPU tensor; rank-th token of stream j of node i of sequence b is element
    offset + b*batch_stride + ((i*gamma)+(j-1))*K + rank (default: contiguous [B,T,gamma,K]).
    Template: device tensors tmpl_parent/tmpl_rank [T2], or per-level `branching`.
    Returns (next_tok [B,T2], next_parent [T2]); `out` (the pair of an earlier call) is reused if given."""
    lib = load_library()
    B = last.shape[0]
    i32 = torch.int32
    if batch_stride is None:
        batch_stride = T * gamma * K
    br_ptr = None
    br = None
    if tmpl_parent is None:
        if branching is None:
            raise ValueError("give a template or per-level branching")
        br = torch.tensor(list(branching), dtype=i32)
        br_ptr = br.data_ptr()
        if T2 is None:
            T2 = 1
            width = 1
            for k in branching:
                width *= int(k)
                T2 += width
    else:
        T2 = tmpl_parent.shape[0]
    dev = last.device
    if out is None:
        next_tok = torch.empty((B, T2), dtype=i32, device=dev)
        next_parent = torch.empty(T2, dtype=i32, device=dev)
    else:
        next_tok, next_parent = out
        if next_tok.shape != (B, T2) or next_parent.shape != (T2,):
            raise ValueError("`out` was made for another shape")
    need = offset + (B - 1) * batch_stride + T * gamma * K if B > 0 else 0
    if stream_topk.numel() < need:
        raise ValueError("stream_topk too small for the given strides")
    _check(lib.ss_tree_draft(_dev(stream_topk, i32, "stream_topk") + 4 * offset, batch_stride, K,
                             _dev(last, i32, "last"), _dev(bonus, i32, "bonus"),
                             None if tmpl_parent is None else _dev(tmpl_parent, i32, "tmpl_parent"),
                             None if tmpl_rank is None else _dev(tmpl_rank, i32, "tmpl_rank"), br_ptr, B, T, gamma,
                             T2, _dev(next_tok, i32, "next_tok"), _dev(next_parent, i32, "next_parent"), _stream()))
    return next_tok, next_parent


def ss_lm_head_verify_draft(hidden, W, K: int, tok, parent, gamma: int, max_depth: int, tmpl_parent=None,
                            tmpl_rank=None, branching: Optional[Sequence[int]] = None, T2: Optional[int] = None,
                            workspace=None, out: Optional[dict] = None, live=None, plan_rows: int = 0) -> dict:
    """a3 + a4 + a5 in one call.  hidden [B*T*(1+gamma), d] (main rows of a sequence first, then its stream
    rows node by node), W [V,d], tok/parent [B,T] int32.  Returns the outputs of ss_tree_verify plus next_tok
    [B,T2], next_parent [T2] and main_argmax [B,T]; `out` (a dict from an earlier call) is reused if given."""
    lib = load_library()
    dt = hidden.dtype
    code = _dtype_code(hidden)
    N, d = hidden.shape
    V = W.shape[0]
    B, T = tok.shape
    if W.shape[1] != d:
        raise ValueError("hidden and W disagree on d")
    if N != B * T * (1 + gamma):
        raise ValueError("hidden has %d rows, expected B*T*(1+gamma) = %d" % (N, B * T * (1 + gamma)))
    i32 = torch.int32
    br = None
    br_ptr = None
    if tmpl_parent is None:
        if branching is None:
            raise ValueError("give a template or per-level branching")
        br = torch.tensor(list(branching), dtype=i32)
        br_ptr = br.data_ptr()
        if T2 is None:
            T2, width = 1, 1
            for k in branching:
                width *= int(k)
                T2 += width
    else:
        T2 = tmpl_parent.shape[0]
    dev = hidden.device
    if out is None:
        out = dict(n_accept=torch.empty(B, dtype=i32, device=dev), last=torch.empty(B, dtype=i32, device=dev),
                   bonus=torch.empty(B, dtype=i32, device=dev),
                   path=torch.empty((B, max_depth + 1), dtype=i32, device=dev),
                   out_tokens=torch.empty((B, max_depth + 1), dtype=i32, device=dev),
                   next_tok=torch.empty((B, T2), dtype=i32, device=dev),
                   next_parent=torch.empty(T2, dtype=i32, device=dev),
                   main_argmax=torch.empty((B, T), dtype=i32, device=dev))
    elif out["next_tok"].shape != (B, T2) or out["path"].shape != (B, max_depth + 1) or out["main_argmax"].shape != (B, T):
        raise ValueError("`out` was made for another shape")
    need = lib.ss_lm_head_workspace_bytes(N, d, V, K, code)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
    head = (_dev(hidden, dt, "hidden"), _dev(W, dt, "W"), d, V, K, code, _dev(tok, i32, "tok"), _dev(parent, i32, "parent"),
            B, T, gamma, max_depth, None if tmpl_parent is None else _dev(tmpl_parent, i32, "tmpl_parent"),
            None if tmpl_rank is None else _dev(tmpl_rank, i32, "tmpl_rank"), br_ptr, T2,
            *[_dev(out[k], i32, k) for k in ("n_accept", "last", "bonus", "path", "out_tokens", "next_tok", "next_parent",
                                            "main_argmax")])
    if live is not None:
        _check(lib.ss_lm_head_verify_draft_live(*head, _dev(live[0], i32, "live_rows"), _dev(live[1], i32, "n_live"),
                                                int(plan_rows), _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                                _stream()))
    else:
        _check(lib.ss_lm_head_verify_draft(*head, _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()))
    return out


def ss_kv_commit(k_new, v_new, k_cache, v_cache, block_table, seq_lens, path, n_accept, gamma: int,
                 new_seq_lens: Optional[torch.Tensor] = None, want_lens: bool = True):
    """n3.  Appends the main-row keys/values of the accepted path (path [B,max_depth+1], n_accept [B] from
    ss_tree_verify) to the paged caches IN PLACE.  Returns new_seq_lens [B] int32 (None if want_lens is False
    and no tensor was given)."""
    lib = load_library()
    code = _dtype_code(k_new)
    dt = k_new.dtype
    B, R, Hkv, D = k_new.shape
    P, _, page, _ = k_cache.shape
    if R % (1 + gamma):
        raise ValueError("k_new has %d rows, not a multiple of 1+gamma" % R)
    T = R // (1 + gamma)
    if tuple(v_new.shape) != (B, R, Hkv, D) or tuple(k_cache.shape) != (P, Hkv, page, D) or tuple(v_cache.shape) != (P, Hkv, D, page):
        raise ValueError("k_new/v_new must be [B,R,Hkv,D], k_cache [P,Hkv,page,D], v_cache [P,Hkv,D,page]")
    if block_table.shape[0] != B or tuple(seq_lens.shape) != (B,) or path.shape[0] != B or tuple(n_accept.shape) != (B,):
        raise ValueError("block_table / seq_lens / path / n_accept batch size mismatch")
    i32 = torch.int32
    if new_seq_lens is None and want_lens:
        new_seq_lens = torch.empty(B, dtype=i32, device=k_new.device)
    _check(lib.ss_kv_commit(_dev(k_new, dt, "k_new"), _dev(v_new, dt, "v_new"), _dev(k_cache, dt, "k_cache"),
                            _dev(v_cache, dt, "v_cache"), _dev(block_table, i32, "block_table"), block_table.shape[1], P,
                            _dev(seq_lens, i32, "seq_lens"), _dev(path, i32, "path"), _dev(n_accept, i32, "n_accept"),
                            B, T, gamma, Hkv, D, page, path.shape[1] - 1, code,
                            None if new_seq_lens is None else _dev(new_seq_lens, i32, "new_seq_lens"), _stream()))
    return new_seq_lens



def ss_kv_alloc_pages(block_table, seq_lens, n_accept, page: int, max_depth: int, free_pages, free_count,
                      n_commit: Optional[torch.Tensor] = None) -> torch.Tensor:
    """n3, page allocation.  block_table [B,max_pages] int32 is updated IN PLACE with pages popped from the stack
    free_pages (int32, top at index free_count-1; free_count: int32 GPU tensor of one element, lowered in place).
    Returns n_commit [B] int32: n_accept clipped to the path rows that have a page."""
    lib = load_library()
    i32 = torch.int32
    B, max_pages = block_table.shape
    if tuple(seq_lens.shape) != (B,) or tuple(n_accept.shape) != (B,) or free_count.numel() != 1:
        raise ValueError("seq_lens / n_accept must be [B], free_count one element")
    if n_commit is None:
        n_commit = torch.empty(B, dtype=i32, device=block_table.device)
    _check(lib.ss_kv_alloc_pages(_dev(block_table, i32, "block_table"), max_pages, _dev(seq_lens, i32, "seq_lens"),
                                 _dev(n_accept, i32, "n_accept"), B, page, max_depth, _dev(free_pages, i32, "free_pages"),
                                 _dev(free_count, i32, "free_count"), _dev(n_commit, i32, "n_commit"), _stream()))
    return n_commit


def ss_linear_rows(x: torch.Tensor, W: torch.Tensor, y: Optional[torch.Tensor] = None, live=None,
                   plan_rows: int = 0) -> torch.Tensor:
    """n1.  y [N,V] = x [N,d] . W[V,d]^T in the inputs' dtype (fp32 or bf16).  `live` = (live_rows, n_live) from
    ss_live_rows: only those rows are computed (the others of y are left as they are)."""
    lib = load_library()
    code = _dtype_code(x)
    dt = x.dtype
    N, d = x.shape
    V = W.shape[0]
    if tuple(W.shape) != (V, d):
        raise ValueError("W must be [V,%d]" % d)
    if y is None:
        y = torch.empty(N, V, dtype=dt, device=x.device)
    elif tuple(y.shape) != (N, V):
        raise ValueError("y must be [%d,%d]" % (N, V))
    if live is not None:
        _check(lib.ss_linear_rows_live(_dev(x, dt, "x"), _dev(W, dt, "W"), N, d, V, code, _dev(y, dt, "y"),
                                       _dev(live[0], torch.int32, "live_rows"), _dev(live[1], torch.int32, "n_live"),
                                       int(plan_rows), _stream()))
        return y
    _check(lib.ss_linear_rows(_dev(x, dt, "x"), _dev(W, dt, "W"), N, d, V, code, _dev(y, dt, "y"), _stream()))
    return y


def ss_linear_rows_workspace_bytes(N: int, d: int, V: int, dtype_code: int) -> int:
    return int(load_library().ss_linear_rows_workspace_bytes(N, d, V, dtype_code))


def ss_linear_rows_splits(N: int, d: int, V: int, dtype_code: int) -> int:
    """Slices of the feature dimension ss_linear_rows_ws uses for this shape (1 = the map is not cut)."""
    return int(load_library().ss_linear_rows_splits(N, d, V, dtype_code))


def ss_linear_rows_ws(x: torch.Tensor, W: torch.Tensor, y: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """n1 with a workspace: the same map as ss_linear_rows; maps with few outputs and many features are cut along
    the feature dimension (fp32 partial products in the workspace, added by a second kernel)."""
    lib = load_library()
    code = _dtype_code(x)
    dt = x.dtype
    N, d = x.shape
    V = W.shape[0]
    if tuple(W.shape) != (V, d):
        raise ValueError("W must be [V,%d]" % d)
    if y is None:
        y = torch.empty(N, V, dtype=dt, device=x.device)
    elif tuple(y.shape) != (N, V):
        raise ValueError("y must be [%d,%d]" % (N, V))
    if workspace is None:
        workspace = torch.empty(max(ss_linear_rows_workspace_bytes(N, d, V, code), 1), dtype=torch.uint8, device=x.device)
    _check(lib.ss_linear_rows_ws(_dev(x, dt, "x"), _dev(W, dt, "W"), N, d, V, code, _dev(y, dt, "y"),
                                 _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()))
    return y


def ss_stream_insert(M: torch.Tensor, P: torch.Tensor, fM: Optional[torch.Tensor] = None,
                     X: Optional[torch.Tensor] = None) -> torch.Tensor:
    """n4 (Eq. 3).  M [B,T,d], P [gamma,d], fM = f(M) or None (identity) -> X [B, T*(1+gamma), d]."""
    lib = load_library()
    code = _dtype_code(M)
    dt = M.dtype
    B, T, d = M.shape
    gamma = P.shape[0]
    if tuple(P.shape) != (gamma, d):
        raise ValueError("P must be [gamma,%d]" % d)
    if fM is not None and tuple(fM.shape) != (B, T, d):
        raise ValueError("fM must have M's shape")
    R = T * (1 + gamma)
    if X is None:
        X = torch.empty(B, R, d, dtype=dt, device=M.device)
    elif tuple(X.shape) != (B, R, d):
        raise ValueError("X must be [%d,%d,%d]" % (B, R, d))
    _check(lib.ss_stream_insert(_dev(M, dt, "M"), None if fM is None else _dev(fM, dt, "fM"), _dev(P, dt, "P"),
                                B, T, gamma, d, code, _dev(X, dt, "X"), _stream()))
    return X


def ss_stream_insert_linear(M: torch.Tensor, P: torch.Tensor, W: torch.Tensor, fM: Optional[torch.Tensor] = None,
                            Y: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """n4 + n1 (Eq. 3 through a dense map).  M [B,T,d], P [gamma,d], W [V,d], fM = f(M) or None -> Y [B, T*(1+gamma), V]."""
    lib = load_library()
    code = _dtype_code(M)
    dt = M.dtype
    B, T, d = M.shape
    gamma, V = P.shape[0], W.shape[0]
    if tuple(P.shape) != (gamma, d) or tuple(W.shape) != (V, d):
        raise ValueError("P must be [gamma,%d] and W [V,%d]" % (d, d))
    if fM is not None and tuple(fM.shape) != (B, T, d):
        raise ValueError("fM must have M's shape")
    R = T * (1 + gamma)
    if Y is None:
        Y = torch.empty(B, R, V, dtype=dt, device=M.device)
    elif tuple(Y.shape) != (B, R, V):
        raise ValueError("Y must be [%d,%d,%d]" % (B, R, V))
    need = lib.ss_stream_insert_linear_workspace_bytes(B, T, gamma, d, V, code, 0 if fM is None else 1)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=M.device)
    _check(lib.ss_stream_insert_linear(_dev(M, dt, "M"), None if fM is None else _dev(fM, dt, "fM"), _dev(P, dt, "P"),
                                       _dev(W, dt, "W"), B, T, gamma, d, V, code, _dev(Y, dt, "Y"),
                                       _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()))
    return Y


def ss_value_rotate(v_new: torch.Tensor, T: int, gamma: int, eps: float) -> torch.Tensor:
    """Value rotation (appendix ablation).  v_new [B,R,Hkv,D], IN PLACE: the stream rows become the node's main-row
    value times e^{i eps n}, features paired (2m, 2m+1).  Returns v_new."""
    lib = load_library()
    B, R, Hkv, D = v_new.shape
    if R != T * (1 + gamma):
        raise ValueError("v_new has %d rows per sequence, expected T*(1+gamma) = %d" % (R, T * (1 + gamma)))
    _check(lib.ss_value_rotate(_dev(v_new, v_new.dtype, "v_new"), B, T, gamma, Hkv, D, float(eps), _dtype_code(v_new),
                               _stream()))
    return v_new


def ss_lm_head_logsumexp(hidden: torch.Tensor, W: torch.Tensor, lse: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """n2.  lse [N] f32 = log-sum-exp over the vocabulary of hidden [N,d] . W[V,d]^T."""
    lib = load_library()
    code = _dtype_code(hidden)
    dt = hidden.dtype
    N, d = hidden.shape
    V = W.shape[0]
    if tuple(W.shape) != (V, d):
        raise ValueError("W must be [V,%d]" % d)
    if lse is None:
        lse = torch.empty(N, dtype=torch.float32, device=hidden.device)
    need = ss_lm_head_workspace_bytes(N, d, V, 1, code)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=hidden.device)
    _check(lib.ss_lm_head_logsumexp(_dev(hidden, dt, "hidden"), _dev(W, dt, "W"), N, d, V, code,
                                    _dev(lse, torch.float32, "lse"), workspace.data_ptr(), workspace.numel(), _stream()))
    return lse


def ss_transition_probs(h: torch.Tensor, W: torch.Tensor, tok: torch.Tensor, parent: torch.Tensor,
                        lse: torch.Tensor, prob: Optional[torch.Tensor] = None) -> torch.Tensor:
    """n2.  prob [B,T] f32: softmax of the parent's early-exit logits at each node's token (root: 1)."""
    lib = load_library()
    code = _dtype_code(h)
    dt = h.dtype
    B, T, d = h.shape
    V = W.shape[0]
    if tuple(W.shape) != (V, d) or tuple(tok.shape) != (B, T) or tuple(parent.shape) != (B, T) or lse.numel() != B * T:
        raise ValueError("W must be [V,d], tok/parent [B,T], lse [B*T]")
    if prob is None:
        prob = torch.empty(B, T, dtype=torch.float32, device=h.device)
    i32 = torch.int32
    _check(lib.ss_transition_probs(_dev(h, dt, "h"), _dev(W, dt, "W"), _dev(tok, i32, "tok"), _dev(parent, i32, "parent"),
                                   _dev(lse, torch.float32, "lse"), B, T, d, V, code, _dev(prob, torch.float32, "prob"),
                                   _stream()))
    return prob


def ss_tree_prune(tok: torch.Tensor, parent: torch.Tensor, prob: torch.Tensor, threshold: float) -> dict:
    """n2.  Returns dict(keep, tok, parent, old_index [B,T] int32, n_nodes [B] int32) of the pruned, compacted and
    padded trees."""
    lib = load_library()
    B, T = tok.shape
    if tuple(parent.shape) != (B, T) or tuple(prob.shape) != (B, T):
        raise ValueError("parent and prob must be [B,T]")
    i32 = torch.int32
    out = {k: torch.empty(B, T, dtype=i32, device=tok.device) for k in ("keep", "tok", "parent", "old_index")}
    out["n_nodes"] = torch.empty(B, dtype=i32, device=tok.device)
    _check(lib.ss_tree_prune(_dev(tok, i32, "tok"), _dev(parent, i32, "parent"), _dev(prob, torch.float32, "prob"),
                             float(threshold), B, T, _dev(out["keep"], i32, "keep"), _dev(out["tok"], i32, "tok"),
                             _dev(out["parent"], i32, "parent"), _dev(out["old_index"], i32, "old_index"),
                             _dev(out["n_nodes"], i32, "n_nodes"), _stream()))
    return out
