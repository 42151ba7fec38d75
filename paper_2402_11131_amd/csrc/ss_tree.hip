// a4 / a5: greedy tree verification and top-k tree drafting (Sec. 3.2.2,
// Appendix A.1).  One wavefront per sequence; lane i owns tree node i (T <= 64).
#include <string.h>

#include "ss_tree.h"

namespace ss {

__global__ __launch_bounds__(64) void tree_verify_kernel(const int32_t* __restrict__ tok,
                                                         const int32_t* __restrict__ parent,
                                                         const int32_t* __restrict__ main_argmax,
                                                         long batch_stride, long node_stride, int T, int max_depth,
                                                         int32_t* __restrict__ n_accept, int32_t* __restrict__ last,
                                                         int32_t* __restrict__ bonus, int32_t* __restrict__ path,
                                                         int32_t* __restrict__ out_tokens) {
  __shared__ VerifyLds s;
  const int b = blockIdx.x;
  int p, my_tok, last_node, bonus_tok;
  verify_load(threadIdx.x, b, tok, parent, T, p, my_tok);
  verify_sequence(threadIdx.x, b, p, my_tok, main_argmax + (size_t)b * batch_stride, node_stride, T, max_depth,
                  n_accept, last, bonus, path, out_tokens, s, last_node, bonus_tok);
}

__global__ __launch_bounds__(64) void tree_draft_kernel(const int32_t* __restrict__ stream_topk, long batch_stride,
                                                        int K, const int32_t* __restrict__ last,
                                                        const int32_t* __restrict__ bonus,
                                                        const int32_t* __restrict__ tmpl_parent,
                                                        const int32_t* __restrict__ tmpl_rank, TemplateArg targ,
                                                        int T, int gamma, int T2, int32_t* __restrict__ next_tok,
                                                        int32_t* __restrict__ next_parent) {
  __shared__ int par[64];
  const int b = blockIdx.x;
  const int node = min(max(last[b], 0), T - 1);
  int p, rank;
  draft_load(threadIdx.x, tmpl_parent, tmpl_rank, targ, T2, p, rank);
  draft_sequence(threadIdx.x, b, p, rank, stream_topk + (size_t)b * batch_stride + (size_t)node * gamma * K, K, bonus[b],
                 gamma, T2, next_tok, next_parent, par);
}

int draft_template_from_branching(const char* fn, const int32_t* branching, int gamma, int K, int T2,
                                  TemplateArg* targ) {
  for (int i = 0; i < SS_MAX_T; ++i) targ->parent[i] = targ->rank[i] = 0;
  SS_REQUIRE(branching != nullptr, SS_ERR_INVALID_ARG, "%s: neither a template nor branching given", fn);
  int32_t par[SS_MAX_T], rnk[SS_MAX_T];
  const int n = ss_full_tree_template_host(branching, gamma, SS_MAX_T, par, rnk, nullptr);
  SS_REQUIRE(n > 0, SS_ERR_UNSUPPORTED, "%s: full tree exceeds %d nodes", fn, SS_MAX_T);
  SS_REQUIRE(n == T2, SS_ERR_INVALID_ARG, "%s: branching gives %d nodes but T2=%d", fn, n, T2);
  for (int i = 0; i < n; ++i) {
    SS_REQUIRE(rnk[i] < K, SS_ERR_INVALID_ARG, "%s: branching %d exceeds K=%d", fn, rnk[i] + 1, K);
    targ->parent[i] = (int8_t)par[i];
    targ->rank[i] = (int8_t)rnk[i];
  }
  return SS_OK;
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
  if (!tmpl_parent)
    if (int rc = ss::draft_template_from_branching("ss_tree_draft", branching, gamma, K, T2, &targ)) return rc;
  if (B == 0) return SS_OK;
  hipLaunchKernelGGL(ss::tree_draft_kernel, dim3(B), dim3(64), 0, (hipStream_t)stream, stream_topk, topk_batch_stride,
                     K, last, bonus, tmpl_parent, tmpl_rank, targ, T, gamma, T2, next_tok, next_parent);
  return ss::check_launch("ss_tree_draft");
}

}  // extern "C"
