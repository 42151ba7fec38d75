"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and moves data between layouts; it holds
none of the method's arithmetic (no attention, no softmax, no argmax, no tree
walk beyond what is needed to *generate* a tree) and imports neither the HIP
binding nor the oracle, so that both can be fed from it.

The paper evaluates on fine-tuned OPT / Phi / OpenLlama models over three text
datasets (Sec. 4); none of that is available here, so these inputs stand in for
it: 7B-shaped heads and widths, vocab 32000, gamma = 3..4 streams, pruned draft
trees of a few tens of nodes (Sec. 3.2.3), N(0,1) activations, N(0,0.02) LM-head
weights, and draft tokens planted so that the number of accepted tokens per step
falls in the range the paper's call-reduction ratios imply (Table 1).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Sequence

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    dtype: str          # "f32" | "bf16": storage type of q/k/v/hidden/W
    B: int              # sequences
    H: int              # query heads
    Hkv: int            # KV heads
    D: int              # head dim
    L_min: int          # cached prefix length (uniform in [L_min, L_max] per sequence)
    L_max: int
    T: int              # tree nodes per sequence
    gamma: int          # speculative streams per node
    branching: tuple    # max children per node at depth 0,1,...
    max_depth: int
    page: int           # tokens per KV page
    n_layers: int = 1   # MSA layers in the step (N_s)
    vocab: int = 0      # LM head: 0 = config has none
    d_model: int = 0
    K: int = 0          # top-k width of the draft
    draft_branching: tuple = ()  # template of the next tree (per level)

    @property
    def R(self) -> int:
        return self.T * (1 + self.gamma)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


# The five workloads (smallest first).  c1 is the correctness case the oracle
# finishes in seconds; c4 is the full step (4 MSA layers + LM head + verify + draft).
CONFIGS = {
    "c1": Config("c1", "f32", 1, 4, 4, 64, 128, 128, 8, 3, (8, 8, 8), 3, 16, 1, 1000, 256, 2, (2, 2, 1)),
    "c2": Config("c2", "bf16", 1, 32, 32, 128, 2048, 2048, 16, 4, (4, 2, 2), 3, 16),
    "c3": Config("c3", "bf16", 16, 32, 32, 128, 1024, 4096, 16, 4, (4, 2, 2), 3, 16, 4),
    "c4": Config("c4", "bf16", 4, 32, 32, 128, 4096, 4096, 16, 4, (4, 2, 2), 3, 16, 4, 32000, 4096, 4,
                 (4, 2, 1, 1)),
    "c5": Config("c5", "bf16", 8, 32, 8, 128, 32768, 32768, 32, 4, (4, 2, 2, 2), 4, 64),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of cfg with some fields replaced (used for reduced test sizes)."""
    return replace(cfg, **kw)


def rng_for(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


# --------------------------------------------------------------------- trees

def make_tree(rng: np.random.Generator, T: int, branching: Sequence[int], max_depth: int) -> np.ndarray:
    """A pruned draft tree: grow from the root by attaching each new node to a
    random eligible parent (depth < max_depth, fewer children than
    branching[depth]), then number the nodes level by level so parent[i] < i."""
    parent = [-1]
    depth = [0]
    nchild = [0]
    while len(parent) < T:
        elig = [n for n in range(len(parent))
                if depth[n] < max_depth and nchild[n] < branching[min(depth[n], len(branching) - 1)]]
        if not elig:
            raise ValueError("tree cannot reach %d nodes with branching %r" % (T, tuple(branching)))
        p = int(elig[int(rng.integers(len(elig)))])
        parent.append(p)
        depth.append(depth[p] + 1)
        nchild.append(0)
        nchild[p] += 1
    order = sorted(range(T), key=lambda n: (depth[n], n))
    new_id = {old: new for new, old in enumerate(order)}
    out = np.full(T, -1, np.int32)
    for old in range(T):
        if parent[old] >= 0:
            out[new_id[old]] = new_id[parent[old]]
    return out


def make_trees(seed: int, B: int, T: int, branching, max_depth: int) -> np.ndarray:
    rng = rng_for(seed)
    return np.stack([make_tree(rng, T, branching, max_depth) for _ in range(B)]).astype(np.int32)


def chain_tree(T: int) -> np.ndarray:
    return np.arange(-1, T - 1, dtype=np.int32)


# --------------------------------------------------------------------- tensors

def _normal(gen, shape, std, dtype, device):
    """N(0, std) in fp32, rounded to the storage dtype."""
    if isinstance(gen, np.random.Generator):
        x = torch.from_numpy(gen.standard_normal(size=shape, dtype=np.float32))
        if std != 1.0:
            x = x * std
        return x.to(dtype)
    x = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    if std != 1.0:
        x = x * std
    return x.to(dtype)


def seq_lens_for(cfg: Config, seed: int) -> np.ndarray:
    rng = rng_for(seed ^ 0x5EED)
    if cfg.L_min == cfg.L_max:
        return np.full(cfg.B, cfg.L_min, np.int32)
    return rng.integers(cfg.L_min, cfg.L_max + 1, size=cfg.B).astype(np.int32)


def make_page_table(seed: int, seq_lens: np.ndarray, page: int, slack: float = 1.25):
    """Seeded random placement of every sequence's logical pages in a pool of
    ceil(slack * needed) physical pages.  Unused table entries are 0."""
    rng = rng_for(seed ^ 0xB10C)
    need = [(int(L) + page - 1) // page for L in seq_lens]
    total = int(sum(need))
    num_pages = max(1, int(np.ceil(total * slack)))
    perm = rng.permutation(num_pages)[:total]
    max_pages = max(1, max(need) if need else 1)
    table = np.zeros((len(seq_lens), max_pages), np.int32)
    o = 0
    for b, n in enumerate(need):
        table[b, :n] = perm[o:o + n]
        o += n
    return table, num_pages


def make_msa_inputs(cfg: Config, seed: int, device: Optional[str] = None, layer: int = 0) -> dict:
    """Inputs of one MSA layer.  With device=None everything is drawn with numpy
    (Philox) on the CPU; with a device string the large tensors are drawn there
    with torch's seeded generator (for sizes that would take too long on the CPU).
    Returns torch tensors (floating tensors in cfg's storage dtype)."""
    dt = cfg.torch_dtype
    s = seed * 1000 + layer
    seq_lens = seq_lens_for(cfg, seed)
    table, num_pages = make_page_table(seed, seq_lens, cfg.page)
    parent = make_trees(seed ^ 0x7EE, cfg.B, cfg.T, cfg.branching, cfg.max_depth)
    if device is None:
        gen = rng_for(s)
        dev = "cpu"
    else:
        gen = torch.Generator(device=device)
        gen.manual_seed(s)
        dev = device
    B, R, H, Hkv, D, P = cfg.B, cfg.R, cfg.H, cfg.Hkv, cfg.D, cfg.page
    out = dict(
        q=_normal(gen, (B, R, H, D), 1.0, dt, dev),
        k_new=_normal(gen, (B, R, Hkv, D), 1.0, dt, dev),
        v_new=_normal(gen, (B, R, Hkv, D), 1.0, dt, dev),
        k_cache=_normal(gen, (num_pages, Hkv, P, D), 1.0, dt, dev),
        v_cache=_normal(gen, (num_pages, Hkv, D, P), 1.0, dt, dev),
        block_table=torch.from_numpy(table).to(dev),
        seq_lens=torch.from_numpy(seq_lens).to(dev),
        parent=torch.from_numpy(parent).to(dev),
        scale=1.0 / float(np.sqrt(D)),
    )
    return out


def pack_paged(k: np.ndarray, v: np.ndarray, page: int, seed: int, slack: float = 1.5):
    """Move contiguous caches k, v [B,L,Hkv,D] into a paged pool with a seeded
    random page table.  Returns (k_cache [P,Hkv,page,D], v_cache [P,Hkv,D,page],
    block_table [B,max_pages]).  Unused slots hold 1e3 so that a read past the
    end of a sequence shows."""
    B, L, Hkv, D = k.shape
    lens = np.full(B, L, np.int32)
    table, num_pages = make_page_table(seed, lens, page, slack)
    kc = np.full((num_pages, Hkv, page, D), 1e3, np.float32)
    vc = np.full((num_pages, Hkv, D, page), 1e3, np.float32)
    for b in range(B):
        for t in range(L):
            pg = table[b, t // page]
            kc[pg, :, t % page, :] = k[b, t]
            vc[pg, :, :, t % page] = v[b, t]
    return kc, vc, table


# --------------------------------------------------------------------- LM head / tokens

def make_lm_head_inputs(cfg: Config, seed: int, device: Optional[str] = None, N: Optional[int] = None) -> dict:
    """hidden [N,d] ~ N(0,1), W [V,d] ~ N(0,0.02) in cfg's storage dtype."""
    dt = cfg.torch_dtype
    N = cfg.B * cfg.R if N is None else N
    if device is None:
        gen = rng_for(seed * 1000 + 77)
        dev = "cpu"
    else:
        gen = torch.Generator(device=device)
        gen.manual_seed(seed * 1000 + 77)
        dev = device
    return dict(hidden=_normal(gen, (N, cfg.d_model), 1.0, dt, dev),
                W=_normal(gen, (cfg.vocab, cfg.d_model), 0.02, dt, dev))


def root_path(parent_row: np.ndarray, node: int):
    path = [int(node)]
    while parent_row[path[-1]] >= 0:
        path.append(int(parent_row[path[-1]]))
    return path[::-1]


def make_draft_tokens(seed: int, parent: np.ndarray, vocab: int) -> np.ndarray:
    """Random draft tokens [B,T]; siblings get distinct tokens (they are the
    top-k of one stream, hence distinct)."""
    rng = rng_for(seed ^ 0x70C)
    B, T = parent.shape
    tok = rng.integers(0, vocab, size=(B, T)).astype(np.int32)
    for b in range(B):
        for p in range(T):
            kids = [i for i in range(T) if parent[b, i] == p]
            seen = set()
            for i in kids:
                while int(tok[b, i]) in seen:
                    tok[b, i] = (int(tok[b, i]) + 1) % vocab
                seen.add(int(tok[b, i]))
    return tok


def plant_acceptance(seed: int, parent: np.ndarray, tok: np.ndarray, hidden: torch.Tensor, W: torch.Tensor,
                     R: int, p_match: float = 0.7, beta: Optional[float] = None):
    """Make the main stream agree with the draft along one seeded root path per
    sequence: for each edge (p -> c) of the path, with probability p_match until
    the first miss, add beta * W[tok[c]] to the hidden state of main row p, which
    makes tok[c] the arg-max logit of that row by a wide margin.  Draft tokens do
    not feed the synthetic hidden states, so this is a free choice of input.
    Returns the planted number of accepted tokens per sequence."""
    rng = rng_for(seed ^ 0xACC)
    B, T = parent.shape
    d = W.shape[1]
    if beta is None:
        # logit noise has std ~ sqrt(d)*0.02; the planted logit gains beta*d*0.02^2
        beta = 12.0 / (0.02 * float(np.sqrt(d)))
    planted = np.zeros(B, np.int32)
    for b in range(B):
        leaf = int(rng.integers(T))
        path = root_path(parent[b], leaf)
        for p, c in zip(path[:-1], path[1:]):
            if rng.random() >= p_match:
                break
            row = b * R + p
            upd = hidden[row].float() + beta * W[int(tok[b, c])].float().to(hidden.device)
            hidden[row] = upd.to(hidden.dtype)
            planted[b] += 1
    return planted
