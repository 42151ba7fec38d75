// Shared declarations of the multi-stream attention kernels (a2).
#pragma once

#include "ss_common.h"

namespace ss {

// Everything a workgroup needs; passed by value.
struct MsaArgs {
  const void* q;
  const void* k_new;
  const void* v_new;
  const void* k_cache;
  const void* v_cache;
  const int32_t* block_table;
  const int32_t* seq_lens;
  const int32_t* parent;
  const int32_t* n_nodes;  // [B] kept nodes per sequence after pruning (rows of the others are not computed), or NULL
  void* out;
  float* part_o;    // [B,H,S,R,D]  per-split outputs, already divided by their own sum
  float* part_lse;  // [B,H,S,R]    log2-domain log-sum-exp of each split
  int B, T, gamma, R, H, Hkv, g, D;
  int page, page_shift, max_pages, num_pages;
  int split_keys;  // cached tokens per split (multiple of 32; of 64 for the fp32 kernel)
  int split0_keys; // cached tokens of split 0 (MFMA path: shorter, that split also scans the step's own rows)
  int n_splits;    // S: upper bound on splits per sequence
  int n_qc;        // query-row chunks per (sequence, KV head) (MFMA path)
  int groups;      // wave groups per workgroup the plan asks for (MFMA path)
  int stages;      // ring stages per wave group the plan asks for (MFMA path)
  unsigned int* arrive;  // MFMA path, two splits merged inside the kernel: arrival counters [B,Hkv,n_qc,kArriveTiles] in the
                         // workspace (zero before the call, zero again after it), else NULL
  float scale_log2;  // softmax scale times log2(e)
  uint32_t flags;
};

// A sequence of L cached tokens has active_splits(L) splits; every sequence has at least one (split 0, which
// also scans the step's new keys).  Split 0 takes the tokens [0, min(L, split0_keys)), split s > 0 the
// tokens [split_begin(s), min(L, split_begin(s) + split_keys)).
SS_DEV int clamp_len(int L, const MsaArgs& a) { return min(max(L, 0), a.max_pages * a.page); }
SS_DEV int active_splits(int L, const MsaArgs& a) {
  return L <= a.split0_keys ? 1 : 1 + (L - a.split0_keys + a.split_keys - 1) / a.split_keys;
}
// Kept nodes of sequence b: all T unless the call passes n_nodes (clamped to [1,T]).
SS_DEV int kept_nodes(int b, const MsaArgs& a) { return a.n_nodes ? min(max(a.n_nodes[b], 1), a.T) : a.T; }
SS_DEV int split_begin(int s, const MsaArgs& a) { return s == 0 ? 0 : a.split0_keys + (s - 1) * a.split_keys; }
SS_DEV int split_len(int s, const MsaArgs& a) { return s == 0 ? a.split0_keys : a.split_keys; }

// Arrival counters of the in-kernel split merge: one per (sequence, KV head, row chunk, query tile of at most
// kArriveTiles per chunk).
constexpr int kArriveTiles = 8;

// MFMA path (bf16, D = 64 or 128).  Returns SS_OK or an error code.
int launch_msa_bf16(const MsaArgs& a, hipStream_t stream);
// Query rows per workgroup chunk the MFMA path uses for F = g*R folded rows.
int msa_bf16_rows_per_chunk(int F);

}  // namespace ss
