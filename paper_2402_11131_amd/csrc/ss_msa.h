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
  void* out;
  float* part_o;    // [B,H,S,R,D]  per-split outputs, already divided by their own sum
  float* part_lse;  // [B,H,S,R]    log2-domain log-sum-exp of each split
  int B, T, gamma, R, H, Hkv, g, D;
  int page, page_shift, max_pages, num_pages;
  int split_keys;  // cached tokens per split (multiple of 32; of 64 for the fp32 kernel)
  int n_splits;    // S: upper bound on splits per sequence
  int n_qc;        // query-row chunks per (sequence, KV head) (MFMA path)
  int groups;      // wave groups per workgroup the plan asks for (MFMA path)
  int arrive_region;  // MFMA path, split launches: region of the arrival counters for the in-kernel merge, or -1
  float scale_log2;  // softmax scale times log2(e)
  uint32_t flags;
};

// A sequence of L cached tokens has active_splits(L) splits; every sequence has at least one (it
// also scans the step's new keys).  Split s takes the tokens [s*split_keys, min(L,(s+1)*split_keys)).
SS_DEV int clamp_len(int L, const MsaArgs& a) { return min(max(L, 0), a.max_pages * a.page); }
SS_DEV int active_splits(int L, const MsaArgs& a) { return max(1, (L + a.split_keys - 1) / a.split_keys); }

// Arrival counters of the in-kernel split merge: kArriveRegions regions (calls take them in turn, so that calls
// in flight on different streams do not share one) of kArriveSlots counters, one per (sequence, KV head, row
// chunk, query tile).
constexpr int kArriveRegions = 32;
constexpr int kArriveSlots = 8192;

// MFMA path (bf16, D = 64 or 128).  Returns SS_OK or an error code.
int launch_msa_bf16(const MsaArgs& a, hipStream_t stream);
// Query rows per workgroup chunk the MFMA path uses for F = g*R folded rows.
int msa_bf16_rows_per_chunk(int F);

}  // namespace ss
