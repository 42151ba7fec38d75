// n2: parallel tree pruning (Sec. 3.2.3, Appendix A.1).  Two small kernels around the LM head's
// log-sum-exp: the transition probability of every child from its parent's early-exit logits, and
// the removal of low-probability sub-trees with compaction of the tree.
#include <math.h>

#include "ss_common.h"

namespace ss {

struct ProbArgs {
  const void* h;          // [B,T,d] o(M): main-stream hidden states after the low-rank map
  const void* W;          // [V,d] LM head
  const int32_t* tok;     // [B,T]
  const int32_t* parent;  // [B,T]
  const float* lse;       // [B*T] log-sum-exp of every node's early-exit logits
  float* prob;            // [B,T]
  int B, T, d, V;
};

// One wavefront per (sequence, node): the early-exit logit of the PARENT's row at the node's token is
// a dot product of length d; prob = exp(logit - lse[parent]).
template <bool BF16>
__global__ __launch_bounds__(64) void transition_prob_kernel(ProbArgs a) {
  const int b = blockIdx.x / a.T, i = blockIdx.x % a.T, lane = threadIdx.x;
  float* out = a.prob + (size_t)b * a.T + i;
  if (i == 0) {
    if (lane == 0) *out = 1.f;
    return;
  }
  const int p = clamp_parent(a.parent[(size_t)b * a.T + i], i);
  const int c = a.tok[(size_t)b * a.T + i];
  if (c < 0 || c >= a.V) {
    if (lane == 0) *out = 0.f;
    return;
  }
  const size_t hr = ((size_t)b * a.T + p) * a.d, wr = (size_t)c * a.d;
  float acc = 0.f;
  constexpr int PER = BF16 ? 8 : 4;  // elements per 16-byte piece
  const bool vec = a.d % PER == 0 && (((uintptr_t)a.h | (uintptr_t)a.W) & 15) == 0;
  if (vec) {
    const uintx4* hv = reinterpret_cast<const uintx4*>((const unsigned char*)a.h + hr * (BF16 ? 2 : 4));
    const uintx4* wv = reinterpret_cast<const uintx4*>((const unsigned char*)a.W + wr * (BF16 ? 2 : 4));
    for (int c0 = lane; c0 < a.d / PER; c0 += 64) {
      const uintx4 x = hv[c0], y = wv[c0];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if constexpr (BF16) {
          acc = fmaf(bf16_bits_to_f32(x[q] & 0xffffu), bf16_bits_to_f32(y[q] & 0xffffu), acc);
          acc = fmaf(bf16_bits_to_f32(x[q] >> 16), bf16_bits_to_f32(y[q] >> 16), acc);
        } else {
          acc = fmaf(__uint_as_float(x[q]), __uint_as_float(y[q]), acc);
        }
      }
    }
  } else
  for (int e = lane; e < a.d; e += 64) {
    float x, y;
    if constexpr (BF16) {
      x = bf16_bits_to_f32(((const uint16_t*)a.h)[hr + e]);
      y = bf16_bits_to_f32(((const uint16_t*)a.W)[wr + e]);
    } else {
      x = ((const float*)a.h)[hr + e];
      y = ((const float*)a.W)[wr + e];
    }
    acc = fmaf(x, y, acc);
  }
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (lane == 0) *out = expf(acc - a.lse[(size_t)b * a.T + p]);
}

struct PruneArgs {
  const int32_t* tok;
  const int32_t* parent;
  const float* prob;
  float threshold;
  int32_t* keep;
  int32_t* new_tok;
  int32_t* new_parent;
  int32_t* old_index;
  int32_t* n_nodes;
  int B, T;
};

// One wavefront per sequence, lane i = node i (T <= 64).  An edge passes unless its probability is
// below the threshold; a node stays iff every edge on its root path passes, i.e. iff its ancestor set
// holds no failed node.  New numbers are ranks among the kept nodes (prefix count of the kept mask).
__global__ __launch_bounds__(64) void tree_prune_kernel(PruneArgs a) {
  __shared__ int par_lds[64];
  __shared__ uint64_t anc[64];
  const int b = blockIdx.x, i = threadIdx.x, T = a.T;
  const bool live = i < T;
  const int par = live ? clamp_parent(a.parent[(size_t)b * T + i], i) : -1;
  par_lds[i] = par;
  __syncthreads();
  compute_anc(par_lds, T, anc, i);
  __syncthreads();
  const bool fails = live && i > 0 && (a.prob[(size_t)b * T + i] < a.threshold);
  const uint64_t failed = __ballot(fails);
  const bool kept = live && (anc[live ? i : 0] & failed) == 0;
  const uint64_t kept_mask = __ballot(kept);
  const int n = __popcll(kept_mask);
  if (live) {
    a.keep[(size_t)b * T + i] = kept ? 1 : 0;
    if (kept) {
      const int me = __popcll(kept_mask & ((1ull << i) - 1ull));
      a.new_tok[(size_t)b * T + me] = a.tok[(size_t)b * T + i];
      a.new_parent[(size_t)b * T + me] = i == 0 ? -1 : __popcll(kept_mask & ((1ull << par) - 1ull));
      a.old_index[(size_t)b * T + me] = i;
    }
    if (i >= n) {  // padding: a token that matches no prediction
      a.new_tok[(size_t)b * T + i] = -1;
      a.new_parent[(size_t)b * T + i] = 0;
      a.old_index[(size_t)b * T + i] = -1;
    }
  }
  if (i == 0) a.n_nodes[b] = n;
}

// The rows of the kept nodes, ascending, for the calls that skip the rows of padding nodes: sequence b
// contributes its main rows b*R + i and its stream rows b*R + T + i*gamma + (j-1) of the nodes i < n_nodes[b].
// One workgroup: thread 0 lays the sequences' offsets down in batch order, then all threads write the rows.
struct LiveArgs {
  const int32_t* n_nodes;
  int32_t* live_rows;
  int32_t* n_live;
  int B, T, gamma;
};
__global__ __launch_bounds__(256) void live_rows_kernel(LiveArgs a) {
  const int R = a.T * (1 + a.gamma);
  int off = 0;
  for (int b = 0; b < a.B; ++b) {
    const int n = min(max(a.n_nodes[b], 1), a.T);
    const int per = n * (1 + a.gamma);
    for (int r = threadIdx.x; r < per; r += 256)
      a.live_rows[off + r] = b * R + (r < n ? r : a.T + (r - n));  // stream rows of kept nodes are T .. T + n*gamma - 1
    off += per;
  }
  if (threadIdx.x == 0) *a.n_live = off;
}

}  // namespace ss

extern "C" {

int ss_transition_probs(const void* h, const void* W, const int32_t* tok, const int32_t* parent, const float* lse,
                        int B, int T, int d, int V, int dtype, float* prob, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_transition_probs";
  SS_REQUIRE(B >= 0 && d >= 1 && V >= 1, SS_ERR_INVALID_ARG, "%s: B=%d d=%d V=%d", fn, B, d, V);
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: T=%d outside [1,%d]", fn, T, SS_MAX_T);
  SS_REQUIRE(dtype == SS_F32 || dtype == SS_BF16, SS_ERR_UNSUPPORTED, "%s: dtype %d", fn, dtype);
  SS_REQUIRE(B == 0 || (h && W && tok && parent && lse && prob), SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  SS_REQUIRE((long)B * T <= 0x7fffffffL, SS_ERR_UNSUPPORTED, "%s: grid too large", fn);
  if (B == 0) return SS_OK;
  ProbArgs a;
  a.h = h; a.W = W; a.tok = tok; a.parent = parent; a.lse = lse; a.prob = prob;
  a.B = B; a.T = T; a.d = d; a.V = V;
  const dim3 grid((unsigned)(B * T));
  if (dtype == SS_F32) hipLaunchKernelGGL(transition_prob_kernel<false>, grid, dim3(64), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(transition_prob_kernel<true>, grid, dim3(64), 0, (hipStream_t)stream, a);
  return check_launch(fn);
}

int ss_tree_prune(const int32_t* tok, const int32_t* parent, const float* prob, float threshold, int B, int T,
                  int32_t* keep, int32_t* new_tok, int32_t* new_parent, int32_t* old_index, int32_t* n_nodes,
                  void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_tree_prune";
  SS_REQUIRE(B >= 0, SS_ERR_INVALID_ARG, "%s: B=%d", fn, B);
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: T=%d outside [1,%d]", fn, T, SS_MAX_T);
  SS_REQUIRE(B == 0 || (tok && parent && prob && keep && new_tok && new_parent && old_index && n_nodes),
             SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  SS_REQUIRE(new_tok != tok && new_parent != parent, SS_ERR_INVALID_ARG, "%s: outputs must not be the input arrays", fn);
  if (B == 0) return SS_OK;
  PruneArgs a;
  a.tok = tok; a.parent = parent; a.prob = prob; a.threshold = threshold;
  a.keep = keep; a.new_tok = new_tok; a.new_parent = new_parent; a.old_index = old_index; a.n_nodes = n_nodes;
  a.B = B; a.T = T;
  hipLaunchKernelGGL(tree_prune_kernel, dim3((unsigned)B), dim3(64), 0, (hipStream_t)stream, a);
  return check_launch(fn);
}

int ss_live_rows(const int32_t* n_nodes, int B, int T, int gamma, int32_t* live_rows, int32_t* n_live, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_live_rows";
  SS_REQUIRE(B >= 0, SS_ERR_INVALID_ARG, "%s: B=%d", fn, B);
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: T=%d outside [1,%d]", fn, T, SS_MAX_T);
  SS_REQUIRE(gamma >= 0 && gamma <= SS_MAX_GAMMA, SS_ERR_UNSUPPORTED, "%s: gamma=%d outside [0,%d]", fn, gamma, SS_MAX_GAMMA);
  SS_REQUIRE((long)B * T * (1 + gamma) <= 0x7fffffffL, SS_ERR_UNSUPPORTED, "%s: too many rows", fn);
  SS_REQUIRE(n_live != nullptr && (B == 0 || (n_nodes && live_rows)), SS_ERR_INVALID_ARG, "%s: NULL argument", fn);
  LiveArgs a;
  a.n_nodes = n_nodes; a.live_rows = live_rows; a.n_live = n_live; a.B = B; a.T = T; a.gamma = gamma;
  hipLaunchKernelGGL(live_rows_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, a);
  return check_launch(fn);
}

}  // extern "C"
