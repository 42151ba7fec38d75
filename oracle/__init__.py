"""CPU oracle of the Speculative Streaming verify-and-speculate step.

TEST INFRASTRUCTURE ONLY.  This package wraps ``ss_oracle.c`` (plain C, double
precision, written from the paper) with numpy.  Only ``tests/``, the smoke check
and the CPU-baseline leg of ``bench.py`` may use it; the product never does, and
this package imports nothing from the product.

Array layouts are those of the C ABI of the HIP library (row order: main rows
first, then stream rows; paged K cache token-major, V cache feature-major).
Floating-point inputs are float32 arrays holding the stored values exactly
(bf16 tensors are up-cast by the caller); outputs are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ss_oracle.c")
_LIB = os.path.join(_HERE, "libss_oracle.so")

EXCLUDE_SELF = 1

_lib = None


def build(force: bool = False) -> str:
    """Compile ss_oracle.c with gcc (-O2 -fopenmp).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.ora_full_tree_template.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle use (OMP_NUM_THREADS or all cores)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return max(1, int(v.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def build_mask(parent, gamma: int, flags: int = 0):
    """a1.  parent [B,T] -> (mask [B,R,R] uint8, anc [B,T] uint64, depth [B,T] int32)."""
    parent = _i32(parent)
    B, T = parent.shape
    R = T * (1 + gamma)
    mask = np.zeros((B, R, R), np.uint8)
    anc = np.zeros((B, T), np.uint64)
    depth = np.zeros((B, T), np.int32)
    _load().ora_build_mask(_p(parent), B, T, gamma, ctypes.c_uint32(flags), _p(mask), _p(anc), _p(depth))
    return mask, anc, depth


def msa_attention(q, k_new, v_new, k_cache, v_cache, block_table, seq_lens, parent, gamma: int,
                  scale: float, flags: int = 0):
    """a2.  Returns out [B,R,H,D] float64."""
    q, k_new, v_new = _f32(q), _f32(k_new), _f32(v_new)
    k_cache, v_cache = _f32(k_cache), _f32(v_cache)
    block_table, seq_lens, parent = _i32(block_table), _i32(seq_lens), _i32(parent)
    B, R, H, D = q.shape
    Hkv = k_new.shape[2]
    T = parent.shape[1]
    assert R == T * (1 + gamma) and k_new.shape == (B, R, Hkv, D) and v_new.shape == k_new.shape
    page = k_cache.shape[2]
    assert k_cache.shape[1] == Hkv and k_cache.shape[3] == D
    assert v_cache.shape == (k_cache.shape[0], Hkv, D, page)
    assert block_table.shape[0] == B and seq_lens.shape == (B,)
    if block_table.size:
        assert block_table.min() >= 0 and block_table.max() < k_cache.shape[0]
    out = np.zeros((B, R, H, D), np.float64)
    _load().ora_msa_attention(
        _p(q), _p(k_new), _p(v_new), _p(k_cache), _p(v_cache), _p(block_table),
        int(block_table.shape[1]), _p(seq_lens), _p(parent), B, T, gamma, H, Hkv, D, page,
        ctypes.c_double(scale), ctypes.c_uint32(flags), _p(out))
    return out


def lm_head_topk(hidden, W, K: int, want_logits: bool = False):
    """a3.  Returns (idx [N,K] int32, val [N,K] float64[, logits [N,V] float64])."""
    hidden, W = _f32(hidden), _f32(W)
    N, d = hidden.shape
    V = W.shape[0]
    assert W.shape[1] == d and 1 <= K <= V
    idx = np.zeros((N, K), np.int32)
    val = np.zeros((N, K), np.float64)
    logits = np.zeros((N, V), np.float64) if want_logits else None
    _load().ora_lm_head_topk(_p(hidden), _p(W), N, d, V, K, _p(idx), _p(val), _p(logits))
    return (idx, val, logits) if want_logits else (idx, val)


def linear_rows(x, W):
    """n1.  y [N,V] (float64) = x [N,d] . W[V,d]^T."""
    x, W = _f32(x), _f32(W)
    N, d = x.shape
    V = W.shape[0]
    assert W.shape == (V, d)
    y = np.zeros((N, V), np.float64)
    _load().ora_linear_rows(_p(x), _p(W), N, d, V, _p(y))
    return y


def stream_insert(M, P, fM=None):
    """n4 (Eq. 3).  M [B,T,d] main-stream hidden states of the tree nodes, P [gamma,d] stream embeddings,
    fM = f(M) or None for the identity.  Returns X [B,R,d] float64."""
    M, P = _f32(M), _f32(P)
    B, T, d = M.shape
    gamma = P.shape[0]
    assert P.shape == (gamma, d)
    if fM is not None:
        fM = _f32(fM)
        assert fM.shape == M.shape
    X = np.zeros((B, T * (1 + gamma), d), np.float64)
    _load().ora_stream_insert(_p(M), _p(fM), _p(P), B, T, gamma, d, _p(X))
    return X


def value_rotate(v, T: int, gamma: int, eps: float):
    """Value-rotation ablation of the appendix.  v [B,R,Hkv,D] (only its main rows are read) -> float64 copy
    whose stream rows hold the node's main-row value times e^{i eps n}, features paired (2m, 2m+1)."""
    v = _f32(v)
    B, R, Hkv, D = v.shape
    assert R == T * (1 + gamma) and D % 2 == 0
    out = np.zeros(v.shape, np.float64)
    lib = _load()
    lib.ora_value_rotate.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int, ctypes.c_double, ctypes.c_void_p]
    lib.ora_value_rotate(_p(v), B, T, gamma, Hkv, D, float(eps), _p(out))
    return out


def tree_verify(tok, parent, main_argmax, max_depth: int):
    """a4.  tok, parent, main_argmax [B,T] -> dict(n_accept, last, bonus, path, out_tokens)."""
    tok, parent, a = _i32(tok), _i32(parent), _i32(main_argmax)
    B, T = tok.shape
    assert parent.shape == (B, T) and a.shape == (B, T) and T <= 64
    n_accept = np.zeros(B, np.int32)
    last = np.zeros(B, np.int32)
    bonus = np.zeros(B, np.int32)
    path = np.zeros((B, max_depth + 1), np.int32)
    out_tokens = np.zeros((B, max_depth + 1), np.int32)
    _load().ora_tree_verify(_p(tok), _p(parent), _p(a), ctypes.c_long(T), ctypes.c_long(1), B, T,
                            max_depth, _p(n_accept), _p(last), _p(bonus), _p(path), _p(out_tokens))
    return dict(n_accept=n_accept, last=last, bonus=bonus, path=path, out_tokens=out_tokens)


def full_tree_template(branching):
    """Full tree of Sec. 3.2.3 with per-level branching -> (parent, rank, depth) int32 arrays."""
    br = _i32(branching)
    cap = 1 << 16
    parent = np.zeros(cap, np.int32)
    rank = np.zeros(cap, np.int32)
    depth = np.zeros(cap, np.int32)
    n = _load().ora_full_tree_template(_p(br), int(br.size), cap, _p(parent), _p(rank), _p(depth))
    if n < 0:
        raise ValueError("tree too large")
    return parent[:n].copy(), rank[:n].copy(), depth[:n].copy()


def tree_draft(stream_topk, last, bonus, tmpl_parent, tmpl_rank):
    """a5.  stream_topk [B,T,gamma,K] -> (next_tok [B,T2], next_parent [T2])."""
    tk = _i32(stream_topk)
    B, T, gamma, K = tk.shape
    last, bonus = _i32(last), _i32(bonus)
    tp, tr = _i32(tmpl_parent), _i32(tmpl_rank)
    T2 = tp.shape[0]
    next_tok = np.zeros((B, T2), np.int32)
    next_parent = np.zeros(T2, np.int32)
    _load().ora_tree_draft(_p(tk), ctypes.c_long(T * gamma * K), K, _p(last), _p(bonus), _p(tp),
                           _p(tr), B, T, gamma, T2, _p(next_tok), _p(next_parent))
    return next_tok, next_parent


def lm_head_lse(h, W):
    """n2.  log-sum-exp over the vocabulary of every row's logits h.W^T -> [N] float64."""
    h, W = _f32(h), _f32(W)
    N, d = h.shape
    lse = np.zeros(N, np.float64)
    _load().ora_lm_head_lse(_p(h), _p(W), N, d, W.shape[0], _p(lse))
    return lse


def transition_probs(h, W, tok, parent):
    """n2.  h [B,T,d] = o(M) of the tree nodes, W [V,d]; prob[b,i] = softmax(h[b,parent[i]].W^T)[tok[b,i]],
    prob[b,0] = 1.  Returns [B,T] float64."""
    h, W, tok, parent = _f32(h), _f32(W), _i32(tok), _i32(parent)
    B, T, d = h.shape
    assert tok.shape == (B, T) and parent.shape == (B, T) and W.shape[1] == d
    prob = np.zeros((B, T), np.float64)
    _load().ora_transition_probs(_p(h), _p(W), _p(tok), _p(parent), B, T, d, W.shape[0], _p(prob))
    return prob


def tree_prune(tok, parent, prob, threshold: float):
    """n2.  Drops every child with prob < threshold and its sub-tree; compacts.  prob is taken in single
    precision.  Returns dict(keep, tok, parent, old_index [B,T] int32, n_nodes [B] int32)."""
    tok, parent = _i32(tok), _i32(parent)
    prob = _f32(prob)
    B, T = tok.shape
    assert T <= 64 and parent.shape == (B, T) and prob.shape == (B, T)
    out = {k: np.zeros((B, T), np.int32) for k in ("keep", "tok", "parent", "old_index")}
    out["n_nodes"] = np.zeros(B, np.int32)
    _load().ora_tree_prune(_p(tok), _p(parent), _p(prob), ctypes.c_float(threshold), B, T, _p(out["keep"]),
                           _p(out["tok"]), _p(out["parent"]), _p(out["old_index"]), _p(out["n_nodes"]))
    return out


def kv_commit(k_new, v_new, k_cache, v_cache, block_table, seq_lens, path, n_accept):
    """n3.  Appends the main-row keys/values of the accepted path (path [B,max_depth+1], n_accept [B]
    as verification returns them) to copies of the caches.  Returns (k_cache, v_cache, new_seq_lens)."""
    k_new, v_new = _f32(k_new), _f32(v_new)
    kc, vc = _f32(k_cache).copy(), _f32(v_cache).copy()
    bt, sl, path, na = _i32(block_table), _i32(seq_lens), _i32(path), _i32(n_accept)
    B, R, Hkv, D = k_new.shape
    P, _, page, _ = kc.shape
    assert v_new.shape == k_new.shape and vc.shape == (P, Hkv, D, page)
    assert bt.shape[0] == B and sl.shape == (B,) and na.shape == (B,) and path.shape[0] == B
    new_lens = np.zeros(B, np.int32)
    _load().ora_kv_commit(_p(k_new), _p(v_new), _p(kc), _p(vc), _p(bt), bt.shape[1], _p(sl), _p(path), _p(na),
                          B, R, Hkv, D, page, path.shape[1] - 1, _p(new_lens))
    return kc, vc, new_lens


def kv_alloc_pages(block_table, seq_lens, n_accept, page, max_depth, free_pages, free_count):
    """n3, page allocation.  Returns (block_table with the new pages written in, free_count left, n_commit [B])."""
    bt = _i32(block_table).copy()
    sl, na, fp = _i32(seq_lens), _i32(n_accept), _i32(free_pages)
    B, max_pages = bt.shape
    assert sl.shape == (B,) and na.shape == (B,) and 0 <= free_count <= fp.size
    cnt = np.array([free_count], np.int32)
    n_commit = np.zeros(B, np.int32)
    _load().ora_kv_alloc_pages(_p(bt), max_pages, _p(sl), _p(na), B, page, max_depth, _p(fp), _p(cnt), _p(n_commit))
    return bt, int(cnt[0]), n_commit


def stream_insert_linear(M, P, W, fM=None):
    """n4 + n1: the rows of Eq. 3 through a dense map, Y [B,R,V] float64 = (rows of stream_insert) . W^T with
    nothing rounded in between.  M [B,T,d], P [gamma,d], W [V,d], fM = f(M) or None."""
    M, P, W = _f32(M), _f32(P), _f32(W)
    B, T, d = M.shape
    gamma, V = P.shape[0], W.shape[0]
    assert P.shape == (gamma, d) and W.shape == (V, d)
    if fM is not None:
        fM = _f32(fM)
        assert fM.shape == M.shape
    Y = np.zeros((B, T * (1 + gamma), V), np.float64)
    _load().ora_stream_insert_linear(_p(M), _p(fM), _p(P), _p(W), B, T, gamma, d, V, _p(Y))
    return Y


# ------------------------------------------------------------------ pruned trees (Sec. 3.2.3)
# After pruning, sequence b keeps the nodes 0 .. n_nodes[b]-1 of its (compacted) tree; the other entries of the
# T-node arrays are padding.  The step on a pruned tree IS the step on the smaller tree: these functions cut every
# sequence down to its kept nodes, run the definitions above on that, and put the rows back where the T-node row
# order has them; rows of padding nodes come back as zeros (the kernels leave them untouched: tests compare the
# kept rows).

def live_rows(n_nodes, T: int, gamma: int):
    """Row numbers b*R + r (ascending) of the rows whose node is kept: main rows r = i and stream rows
    r = T + i*gamma + (j-1) of the nodes i < n_nodes[b]."""
    R = T * (1 + gamma)
    rows = []
    for b, n in enumerate(np.asarray(n_nodes).tolist()):
        n = max(1, min(int(n), T))
        rows += [b * R + i for i in range(n)]
        rows += [b * R + T + i * gamma + j for i in range(n) for j in range(gamma)]
    return np.asarray(rows, np.int32)


def msa_attention_pruned(q, k_new, v_new, k_cache, v_cache, block_table, seq_lens, parent, gamma: int, scale: float,
                         n_nodes, flags: int = 0):
    """a2 on pruned trees.  Arrays as for msa_attention (T-node layout); n_nodes [B].  Returns out [B,R,H,D]
    float64, zero in the rows of padding nodes."""
    q, k_new, v_new = _f32(q), _f32(k_new), _f32(v_new)
    block_table, seq_lens, parent = _i32(block_table), _i32(seq_lens), _i32(parent)
    B, R, H, D = q.shape
    T = parent.shape[1]
    out = np.zeros((B, R, H, D), np.float64)
    for b in range(B):
        n = max(1, min(int(n_nodes[b]), T))
        rows = live_rows([n], T, gamma)                      # rows of this sequence, in the order of the n-node tree
        sub = msa_attention(q[b:b + 1, rows], k_new[b:b + 1, rows], v_new[b:b + 1, rows], k_cache, v_cache,
                            block_table[b:b + 1], seq_lens[b:b + 1], parent[b:b + 1, :n], gamma, scale, flags)
        out[b, rows] = sub[0]
    return out


def linear_rows_live(x, W, rows):
    """n1 on the kept rows only: y [N,V] float64, zero elsewhere."""
    x = _f32(x)
    y = np.zeros((x.shape[0], np.asarray(W).shape[0]), np.float64)
    rows = np.asarray(rows, np.int64)
    if rows.size:
        y[rows] = linear_rows(x[rows], W)
    return y


def lm_head_topk_live(hidden, W, K: int, rows, want_logits: bool = False):
    """a3 on the kept rows only: (idx, val[, logits]) with idx -1 and val / logits 0 in the other rows."""
    hidden = _f32(hidden)
    N, V = hidden.shape[0], np.asarray(W).shape[0]
    rows = np.asarray(rows, np.int64)
    idx = -np.ones((N, K), np.int32)
    val = np.zeros((N, K), np.float64)
    z = np.zeros((N, V), np.float64) if want_logits else None
    if rows.size:
        r = lm_head_topk(hidden[rows], W, K, want_logits=want_logits)
        idx[rows], val[rows] = r[0], r[1]
        if want_logits:
            z[rows] = r[2]
    return (idx, val, z) if want_logits else (idx, val)
