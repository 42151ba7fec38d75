// a4 / a5: greedy tree verification and top-k tree drafting (Sec. 3.2.2,
// Appendix A.1).  One wavefront per sequence; lane i owns tree node i (T <= 64).
#include <string.h>

#include "ss_common.h"

namespace ss {

// Acceptance is a property of a node's whole root path: every edge on it must
// match.  Lane i walks its path through LDS copies of parent / edge-match flags;
// the deepest accepted node is then picked with a wave-wide max of
// (depth, 63 - index) so that ties go to the lowest index.
__global__ __launch_bounds__(64) void tree_verify_kernel(const int32_t* __restrict__ tok,
                                                         const int32_t* __restrict__ parent,
                                                         const int32_t* __restrict__ main_argmax,
                                                         long batch_stride, long node_stride, int T, int max_depth,
                                                         int32_t* __restrict__ n_accept, int32_t* __restrict__ last,
                                                         int32_t* __restrict__ bonus, int32_t* __restrict__ path,
                                                         int32_t* __restrict__ out_tokens) {
  __shared__ int par[64];
  __shared__ int edge_ok[64];
  __shared__ int tk[64];
  const int b = blockIdx.x, i = threadIdx.x;
  const int32_t* a = main_argmax + (size_t)b * batch_stride;
  int p = -1, my_tok = -1;
  if (i < T) {
    p = clamp_parent(parent[(size_t)b * T + i], i);
    my_tok = tok[(size_t)b * T + i];
    par[i] = p;
    tk[i] = my_tok;
    edge_ok[i] = (i == 0) ? 1 : (my_tok == a[(size_t)p * node_stride]);
  }
  __syncthreads();
  int depth = 0, ok = (i < T);
  if (i < T) {
    int n = i;
    for (int step = 0; step < 64 && n > 0; ++step) {
      ok &= edge_ok[n];
      n = par[n];
      ++depth;
    }
    ok &= (depth <= max_depth);
  }
  // key: depth * 64 + (63 - i) for accepted nodes; the root (always accepted) gives key >= 63
  int key = ok ? depth * 64 + (63 - i) : -1;
  for (int off = 32; off > 0; off >>= 1) key = max(key, __shfl_xor(key, off, 64));
  const int best = 63 - (key & 63);
  const int best_depth = key >> 6;
  const int bon = a[(size_t)best * node_stride];
  if (i == 0) {
    n_accept[b] = best_depth;
    last[b] = best;
    bonus[b] = bon;
  }
  // path / emitted tokens: lane k < max_depth+1 writes slot k
  __shared__ int pth[64];
  if (i <= max_depth) pth[i] = -1;
  __syncthreads();
  if (i == 0) {
    int n = best;
    for (int k = best_depth; k >= 0 && n >= 0; --k) {
      pth[k] = n;
      n = par[n];
    }
  }
  __syncthreads();
  if (i <= max_depth) {
    const int node = pth[i];
    path[(size_t)b * (max_depth + 1) + i] = node;
    int t = -1;
    if (i < best_depth) t = tk[pth[i + 1]];
    else if (i == best_depth) t = bon;
    out_tokens[(size_t)b * (max_depth + 1) + i] = t;
  }
}

// Template passed by value when the caller gives per-level branching.
struct TemplateArg {
  int8_t parent[SS_MAX_T];
  int8_t rank[SS_MAX_T];
};

__global__ __launch_bounds__(64) void tree_draft_kernel(const int32_t* __restrict__ stream_topk, long batch_stride,
                                                        int K, const int32_t* __restrict__ last,
                                                        const int32_t* __restrict__ bonus,
                                                        const int32_t* __restrict__ tmpl_parent,
                                                        const int32_t* __restrict__ tmpl_rank, TemplateArg targ,
                                                        int T, int gamma, int T2, int32_t* __restrict__ next_tok,
                                                        int32_t* __restrict__ next_parent) {
  __shared__ int par[64];
  const int b = blockIdx.x, i = threadIdx.x;
  int rank = 0;
  if (i < T2) {
    const int p = tmpl_parent ? tmpl_parent[i] : (int)targ.parent[i];
    rank = tmpl_rank ? tmpl_rank[i] : (int)targ.rank[i];
    par[i] = clamp_parent(p, i);
  }
  __syncthreads();
  if (i >= T2) return;
  int level = 0;
  for (int n = i, step = 0; step < 64 && n > 0; ++step) {
    n = par[n];
    ++level;
  }
  int node = last[b];
  node = min(max(node, 0), T - 1);
  int t;
  if (i == 0) t = bonus[b];
  else if (level >= 1 && level <= gamma && rank >= 0 && rank < K)
    t = stream_topk[(size_t)b * batch_stride + ((size_t)node * gamma + (level - 1)) * K + rank];
  else t = -1;
  next_tok[(size_t)b * T2 + i] = t;
  if (next_parent && b == 0) next_parent[i] = par[i];
}

}  // namespace ss

extern "C" {

int ss_tree_verify(const int32_t* tok, const int32_t* parent, const int32_t* main_argmax, long argmax_batch_stride,
                   long argmax_node_stride, int B, int T, int max_depth, int32_t* n_accept, int32_t* last,
                   int32_t* bonus, int32_t* path, int32_t* out_tokens, void* stream) {
  ss::clear_error();
  SS_REQUIRE(B == 0 || (tok && parent && main_argmax && n_accept && last && bonus && path && out_tokens),
             SS_ERR_INVALID_ARG, "ss_tree_verify: NULL argument");
  SS_REQUIRE(B >= 0 && argmax_node_stride >= 1 && argmax_batch_stride >= 0, SS_ERR_INVALID_ARG,
             "ss_tree_verify: bad B or strides");
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "ss_tree_verify: T=%d outside [1,%d]", T, SS_MAX_T);
  SS_REQUIRE(max_depth >= 0 && max_depth < SS_MAX_T, SS_ERR_UNSUPPORTED, "ss_tree_verify: max_depth=%d outside [0,%d)",
             max_depth, SS_MAX_T);
  if (B == 0) return SS_OK;
  hipLaunchKernelGGL(ss::tree_verify_kernel, dim3(B), dim3(64), 0, (hipStream_t)stream, tok, parent, main_argmax,
                     argmax_batch_stride, argmax_node_stride, T, max_depth, n_accept, last, bonus, path, out_tokens);
  return ss::check_launch("ss_tree_verify");
}

int ss_tree_draft(const int32_t* stream_topk, long topk_batch_stride, int K, const int32_t* last,
                  const int32_t* bonus, const int32_t* tmpl_parent, const int32_t* tmpl_rank,
                  const int32_t* branching, int B, int T, int gamma, int T2, int32_t* next_tok, int32_t* next_parent,
                  void* stream) {
  ss::clear_error();
  SS_REQUIRE(B == 0 || (stream_topk && last && bonus && next_tok), SS_ERR_INVALID_ARG,
             "ss_tree_draft: NULL argument");
  SS_REQUIRE(B >= 0 && topk_batch_stride >= 0, SS_ERR_INVALID_ARG, "ss_tree_draft: bad B or stride");
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T && T2 >= 1 && T2 <= SS_MAX_T, SS_ERR_UNSUPPORTED,
             "ss_tree_draft: T=%d or T2=%d outside [1,%d]", T, T2, SS_MAX_T);
  SS_REQUIRE(gamma >= 0 && gamma <= SS_MAX_GAMMA, SS_ERR_UNSUPPORTED, "ss_tree_draft: gamma=%d outside [0,%d]", gamma,
             SS_MAX_GAMMA);
  SS_REQUIRE(K >= 1 && K <= SS_MAX_K, SS_ERR_UNSUPPORTED, "ss_tree_draft: K=%d outside [1,%d]", K, SS_MAX_K);
  SS_REQUIRE((tmpl_parent == nullptr) == (tmpl_rank == nullptr), SS_ERR_INVALID_ARG,
             "ss_tree_draft: tmpl_parent and tmpl_rank must both be given or both be NULL");
  ss::TemplateArg targ;
  for (int i = 0; i < SS_MAX_T; ++i) targ.parent[i] = targ.rank[i] = 0;
  if (!tmpl_parent) {
    SS_REQUIRE(branching != nullptr, SS_ERR_INVALID_ARG, "ss_tree_draft: neither a template nor branching given");
    int32_t par[SS_MAX_T], rnk[SS_MAX_T];
    const int n = ss_full_tree_template_host(branching, gamma, SS_MAX_T, par, rnk, nullptr);
    SS_REQUIRE(n > 0, SS_ERR_UNSUPPORTED, "ss_tree_draft: full tree exceeds %d nodes", SS_MAX_T);
    SS_REQUIRE(n == T2, SS_ERR_INVALID_ARG, "ss_tree_draft: branching gives %d nodes but T2=%d", n, T2);
    for (int i = 0; i < n; ++i) {
      SS_REQUIRE(rnk[i] < K, SS_ERR_INVALID_ARG, "ss_tree_draft: branching %d exceeds K=%d", rnk[i] + 1, K);
      targ.parent[i] = (int8_t)par[i];
      targ.rank[i] = (int8_t)rnk[i];
    }
  }
  if (B == 0) return SS_OK;
  hipLaunchKernelGGL(ss::tree_draft_kernel, dim3(B), dim3(64), 0, (hipStream_t)stream, stream_topk, topk_batch_stride,
                     K, last, bonus, tmpl_parent, tmpl_rank, targ, T, gamma, T2, next_tok, next_parent);
  return ss::check_launch("ss_tree_draft");
}

}  // extern "C"
