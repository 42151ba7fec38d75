"""Independent little re-statements used to pin the oracle (pure Python, tiny
inputs only).  Nothing here is imported by the oracle or by the product."""
import itertools
import math


def all_parent_arrays(T):
    """Every tree on T nodes with parent[0] = -1 and parent[i] < i."""
    for tail in itertools.product(*[range(i) for i in range(1, T)]):
        yield (-1,) + tuple(tail)


def reach_closure(parent):
    """anc[i] = set of nodes on the root..i path, by transitive closure of the
    child relation (Warshall), not by walking parent pointers."""
    T = len(parent)
    reach = [[a == i for i in range(T)] for a in range(T)]  # reach[a][i]: a is anc-or-self of i
    for i in range(T):
        if parent[i] >= 0:
            reach[parent[i]][i] = True
    for k in range(T):
        for a in range(T):
            if reach[a][k]:
                for i in range(T):
                    if reach[k][i]:
                        reach[a][i] = True
    return [set(a for a in range(T) if reach[a][i]) for i in range(T)]


def rows_of(T, gamma):
    """(node, stream) of each row in ABI order."""
    return [(i, 0) for i in range(T)] + [(i, j) for i in range(T) for j in range(1, gamma + 1)]


def visible_new_keys(parent, gamma, exclude_self=False):
    """For each row the set of new-block column indices it may attend, from the
    statement of Eq. 1 / Eq. 2 / the mask figure."""
    T = len(parent)
    anc = reach_closure(parent)
    rows = rows_of(T, gamma)
    col = {rc: c for c, rc in enumerate(rows)}
    vis = []
    for (i, j) in rows:
        s = set(col[(a, 0)] for a in anc[i])          # main rows of the path root..i
        if j > 0:
            top = j - 1 if exclude_self else j
            s |= set(col[(i, jj)] for jj in range(1, top + 1))  # own streams
        vis.append(s)
    return vis


def softmax_attend(qv, keys, vals, scale):
    """One row of attention over explicit key / value lists (lists of floats)."""
    s = [scale * sum(a * b for a, b in zip(qv, k)) for k in keys]
    m = max(s)
    e = [math.exp(x - m) for x in s]
    z = sum(e)
    D = len(vals[0])
    return [sum(e[c] / z * vals[c][d] for c in range(len(keys))) for d in range(D)]


def enumerate_paths_verify(tok, parent, a):
    """Longest root path all of whose edges match, by listing every root->node
    path and checking each edge; ties -> lowest last node."""
    T = len(parent)
    best = (0, 0)
    for n in range(T):
        path = [n]
        while parent[path[-1]] >= 0:
            path.append(parent[path[-1]])
        path = path[::-1]
        if all(tok[c] == a[p] for p, c in zip(path[:-1], path[1:])):
            if len(path) - 1 > best[0]:
                best = (len(path) - 1, n)
    return best  # (n_accept, last)


# ---------------------------------------------------------------- GPU-vs-oracle comparison helpers
def rel_err(got, ref):
    """The error the tolerances are stated in: the larger of
      max over all elements of |got-ref| / (|ref| + rms(ref))       (plain relative error is meaningless at
                                                                     zero crossings), and
      max over the elements with |ref| >= rms(ref) of |got-ref| / |ref|     (the plain relative error, where
                                                                     it means something)."""
    import numpy as np
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) or 1.0
    d = np.abs(got - ref)
    err = float(np.max(d / (np.abs(ref) + rms))) if d.size else 0.0
    big = np.abs(ref) >= rms
    if big.any():
        err = max(err, float(np.max(d[big] / np.abs(ref[big]))))
    return err


def to_np_f32(t):
    """torch tensor (any float dtype, any device) -> float32 numpy holding the stored values."""
    return t.detach().float().cpu().numpy()


def oracle_subproblem(inp, b, hk, g):
    """Inputs of one (sequence, KV head) of a batched MSA problem as a B=1, Hkv=1, H=g problem,
    with only that sequence's pages gathered (so that large configs stay small on the CPU)."""
    import numpy as np
    page = inp["k_cache"].shape[2]
    L = int(inp["seq_lens"][b])
    npg = max(1, (L + page - 1) // page)
    pages = inp["block_table"][b, :npg].long()
    sub = dict(
        q=to_np_f32(inp["q"][b:b + 1, :, hk * g:(hk + 1) * g]),
        k_new=to_np_f32(inp["k_new"][b:b + 1, :, hk:hk + 1]),
        v_new=to_np_f32(inp["v_new"][b:b + 1, :, hk:hk + 1]),
        k_cache=to_np_f32(inp["k_cache"][pages, hk:hk + 1]),
        v_cache=to_np_f32(inp["v_cache"][pages, hk:hk + 1]),
        block_table=np.arange(npg, dtype=np.int32)[None],
        seq_lens=np.array([L], np.int32),
        parent=inp["parent"][b:b + 1].cpu().numpy(),
    )
    return sub
