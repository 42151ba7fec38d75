// Greedy tree verification and top-k tree drafting of ONE sequence (Sec. 3.2.2, Appendix A.1) as device
// functions: the bodies of the two stand-alone kernels and of the fused tail of the LM head.  Thread i of
// the workgroup owns tree node i (T <= 64); threads beyond the first wavefront only take part in the
// barriers, so every thread of the workgroup must make the call.
#pragma once
#include "ss_common.h"

namespace ss {

// Template of the next tree, passed by value when the caller gives per-level branching.
struct TemplateArg {
  int8_t parent[SS_MAX_T];
  int8_t rank[SS_MAX_T];
};

struct VerifyLds {
  int par[64];
  int edge_ok[64];
  int tk[64];
  int pth[64];
  int res[3];
};

// Acceptance is a property of a node's whole root path: every edge on it must match.  Lane i walks its
// path through LDS copies of parent / edge-match flags; the deepest accepted node is then picked with a
// wave-wide max of (depth, 63 - index) so that ties go to the lowest index.  `a[n * node_stride]` is the
// main stream's arg-max token at node n (global memory or LDS).  On return every thread holds the last
// accepted node and the bonus token.
// `p`, `my_tok`: node i's parent and token from verify_load (a caller with other memory work to do
// first issues these loads early).
SS_DEV void verify_load(int i, int b, const int32_t* __restrict__ tok, const int32_t* __restrict__ parent, int T,
                        int& p, int& my_tok) {
  p = -1;
  my_tok = -1;
  if (i < T) {
    p = clamp_parent(parent[(size_t)b * T + i], i);
    my_tok = tok[(size_t)b * T + i];
  }
}

SS_DEV void verify_sequence(int i, int b, int p, int my_tok, const int32_t* a, long node_stride, int T, int max_depth,
                            int32_t* __restrict__ n_accept, int32_t* __restrict__ last, int32_t* __restrict__ bonus,
                            int32_t* __restrict__ path, int32_t* __restrict__ out_tokens, VerifyLds& s,
                            int& last_node, int& bonus_tok) {
  if (i < T) {
    s.par[i] = p;
    s.tk[i] = my_tok;
    s.edge_ok[i] = (i == 0) ? 1 : (my_tok == a[(size_t)p * node_stride]);
  }
  if (i <= max_depth) s.pth[i] = -1;
  __syncthreads();
  int depth = 0, ok = (i < T);
  if (i < T) {
    int n = i;
    for (int step = 0; step < 64 && n > 0; ++step) {
      ok &= s.edge_ok[n];
      n = s.par[n];
      ++depth;
    }
    ok &= (depth <= max_depth);
  }
  // key: depth * 64 + (63 - i) for accepted nodes; the root (always accepted) gives key >= 63
  int key = ok ? depth * 64 + (63 - i) : -1;
  for (int off = 32; off > 0; off >>= 1) key = max(key, __shfl_xor(key, off, 64));
  if (i == 0) {  // the first wavefront holds all nodes: its result is the sequence's
    const int best = 63 - (key & 63);
    const int best_depth = key >> 6;
    const int bon = a[(size_t)best * node_stride];
    n_accept[b] = best_depth;
    last[b] = best;
    bonus[b] = bon;
    s.res[0] = best;
    s.res[1] = bon;
    s.res[2] = best_depth;
    int n = best;
    for (int k = best_depth; k >= 0 && n >= 0; --k) {
      s.pth[k] = n;
      n = s.par[n];
    }
  }
  __syncthreads();
  last_node = s.res[0];
  bonus_tok = s.res[1];
  const int best_depth = s.res[2];
  // path / emitted tokens: thread k < max_depth+1 writes slot k
  if (i <= max_depth) {
    const int node = s.pth[i];
    path[(size_t)b * (max_depth + 1) + i] = node;
    int t = -1;
    if (i < best_depth) t = s.tk[s.pth[i + 1]];
    else if (i == best_depth) t = bonus_tok;
    out_tokens[(size_t)b * (max_depth + 1) + i] = t;
  }
}

// The next tree: node i of the template takes the token of rank `rank[i]` of stream `level(i)` of the
// last accepted node; the root takes the bonus token.  `topk_of_node[(j-1) * K + r]` is the token of
// rank r of stream j of that node (global memory or LDS).
// `p`, `rank`: template entry i from draft_load (may be issued early).
SS_DEV void draft_load(int i, const int32_t* __restrict__ tmpl_parent, const int32_t* __restrict__ tmpl_rank,
                       const TemplateArg& targ, int T2, int& p, int& rank) {
  p = 0;
  rank = 0;
  if (i < T2) {
    p = tmpl_parent ? tmpl_parent[i] : (int)targ.parent[i];
    rank = tmpl_rank ? tmpl_rank[i] : (int)targ.rank[i];
  }
}

SS_DEV void draft_sequence(int i, int b, int p, int rank, const int32_t* topk_of_node, int K, int bonus_tok, int gamma,
                           int T2, int32_t* __restrict__ next_tok, int32_t* __restrict__ next_parent,
                           int* par /* LDS, 64 ints */) {
  if (i < T2) par[i] = clamp_parent(p, i);
  __syncthreads();
  if (i >= T2) return;
  int level = 0;
  for (int n = i, step = 0; step < 64 && n > 0; ++step) {
    n = par[n];
    ++level;
  }
  int t;
  if (i == 0) t = bonus_tok;
  else if (level >= 1 && level <= gamma && rank >= 0 && rank < K) t = topk_of_node[(size_t)(level - 1) * K + rank];
  else t = -1;
  next_tok[(size_t)b * T2 + i] = t;
  if (next_parent && b == 0) next_parent[i] = par[i];
}

// Host: the template argument of a draft call from per-level branching (checks it against K and T2).
int draft_template_from_branching(const char* fn, const int32_t* branching, int gamma, int K, int T2, TemplateArg* targ);

}  // namespace ss
