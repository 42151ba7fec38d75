// n3: KV-cache commit after verification (Sec. 3.2.1, Appendix A.1).  Of the step's own rows only the
// main rows of the accepted path are appended to the paged cache; stream rows and rejected nodes are
// dropped.  A few KB per sequence: one workgroup per (sequence, path position, KV head), pure copies.
#include "ss_common.h"

namespace ss {

struct KvArgs {
  const void* k_new;
  const void* v_new;
  void* k_cache;
  void* v_cache;
  const int32_t* block_table;
  const int32_t* seq_lens;
  const int32_t* path;
  const int32_t* n_accept;
  int32_t* new_seq_lens;
  int B, T, R, Hkv, D, page, page_shift, max_pages, num_pages, max_depth;
};

// E = element type of the tensors as an unsigned integer of the same size (the copy is bit-exact).
template <typename E>
__global__ __launch_bounds__(128) void kv_commit_kernel(KvArgs a) {
  const int b = blockIdx.x / (a.max_depth + 1), j = blockIdx.x % (a.max_depth + 1);
  const int cap = a.max_pages * a.page;
  const int L = min(max(a.seq_lens[b], 0), cap);
  const int n_acc = min(max(a.n_accept[b], -1), a.max_depth);  // -1: nothing of this sequence is appended
  if (j == 0 && blockIdx.y == 0 && threadIdx.x == 0 && a.new_seq_lens) a.new_seq_lens[b] = min(L + n_acc + 1, cap);
  const int pos = L + j;
  if (j > n_acc || pos >= cap) return;
  const int node = min(max(a.path[(size_t)b * (a.max_depth + 1) + j], 0), a.T - 1);
  const int pg = min(max(a.block_table[(size_t)b * a.max_pages + (pos >> a.page_shift)], 0), a.num_pages - 1);
  const int slot = pos & (a.page - 1);
  const E* ks = (const E*)a.k_new + ((size_t)b * a.R + node) * a.Hkv * a.D;
  const E* vs = (const E*)a.v_new + ((size_t)b * a.R + node) * a.Hkv * a.D;
  E* kd = (E*)a.k_cache + (size_t)pg * a.Hkv * a.page * a.D + (size_t)slot * a.D;  // + h*page*D + d
  E* vd = (E*)a.v_cache + (size_t)pg * a.Hkv * a.D * a.page + slot;                // + (h*D + d)*page
  const int h = blockIdx.y;  // one workgroup per (sequence, path position, KV head)
  for (int d = threadIdx.x; d < a.D; d += 128) {
    const int e = h * a.D + d;
    kd[(size_t)h * a.page * a.D + d] = ks[e];
    vd[(size_t)e * a.page] = vs[e];
  }
}

// Page allocation (Appendix A.1: the cache grows by the accepted tokens after every step).  One workgroup:
// thread b works out how many logical pages beyond the ceil(L/page) in use sequence b's accepted rows need, an
// exclusive prefix sum over the batch gives its place below the top of the stack of free pages (sequences are
// served in batch order, pages in logical order, exactly as a sequential allocator would), and the thread
// writes its pages into the block table.  A sequence stops growing at the table's capacity or when the stack
// is empty; n_commit tells how many of its path rows have a page.
struct AllocArgs {
  int32_t* block_table;
  const int32_t* seq_lens;
  const int32_t* n_accept;
  const int32_t* free_pages;
  int32_t* free_count;
  int32_t* n_commit;
  int B, page, page_shift, max_pages, max_depth;
};

__global__ __launch_bounds__(1024) void kv_alloc_pages_kernel(AllocArgs a) {
  __shared__ int wave_sum[16];
  __shared__ int carry_s;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int cap = a.max_pages * a.page;
  const int count = max(*a.free_count, 0);
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int b0 = 0; b0 < a.B; b0 += 1024) {
    const int b = b0 + tid;
    int L = 0, acc = -1, mapped0 = 0, need = 0;
    if (b < a.B) {
      L = min(max(a.seq_lens[b], 0), cap);
      acc = min(max(a.n_accept[b], -1), a.max_depth);
      mapped0 = (L + a.page - 1) >> a.page_shift;
      if (acc >= 0) need = max(min((L + acc) >> a.page_shift, a.max_pages - 1) + 1 - mapped0, 0);
    }
    // exclusive prefix sum of `need` over this round's 1024 sequences, plus what earlier rounds took
    int incl = need;
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) wave_sum[w] = incl;
    __syncthreads();
    int before = carry_s;
    for (int j = 0; j < w; ++j) before += wave_sum[j];
    const int off = before + incl - need;
    if (b < a.B) {
      const int granted = min(max(count - off, 0), need);
      for (int k = 0; k < granted; ++k)
        a.block_table[(size_t)b * a.max_pages + mapped0 + k] = a.free_pages[count - 1 - (off + k)];
      const int room = min(cap, (mapped0 + granted) * a.page);  // tokens the mapped pages hold
      a.n_commit[b] = acc < 0 ? -1 : max(min(acc, room - 1 - L), -1);
    }
    __syncthreads();
    if (tid == 1023) carry_s = before + incl;
    __syncthreads();
  }
  if (tid == 0) *a.free_count = count - min(carry_s, count);
}

}  // namespace ss

extern "C" int ss_kv_alloc_pages(int32_t* block_table, int max_pages_per_seq, const int32_t* seq_lens,
                                 const int32_t* n_accept, int B, int page_size, int max_depth,
                                 const int32_t* free_pages, int32_t* free_count, int32_t* n_commit, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_kv_alloc_pages";
  SS_REQUIRE(B >= 0, SS_ERR_INVALID_ARG, "%s: B=%d", fn, B);
  SS_REQUIRE(page_size == 16 || page_size == 32 || page_size == 64, SS_ERR_UNSUPPORTED,
             "%s: page_size %d not in {16,32,64}", fn, page_size);
  SS_REQUIRE(max_pages_per_seq >= 1, SS_ERR_INVALID_ARG, "%s: max_pages_per_seq=%d", fn, max_pages_per_seq);
  SS_REQUIRE((long)max_pages_per_seq * page_size <= (1L << 30), SS_ERR_UNSUPPORTED, "%s: sequence capacity too large", fn);
  SS_REQUIRE(max_depth >= 0 && max_depth < SS_MAX_T, SS_ERR_INVALID_ARG, "%s: max_depth=%d", fn, max_depth);
  SS_REQUIRE(B == 0 || (block_table && seq_lens && n_accept && free_pages && free_count && n_commit), SS_ERR_INVALID_ARG,
             "%s: NULL argument", fn);
  if (B == 0) return SS_OK;
  AllocArgs a;
  a.block_table = block_table; a.seq_lens = seq_lens; a.n_accept = n_accept; a.free_pages = free_pages;
  a.free_count = free_count; a.n_commit = n_commit;
  a.B = B; a.page = page_size; a.page_shift = page_size == 16 ? 4 : (page_size == 32 ? 5 : 6);
  a.max_pages = max_pages_per_seq; a.max_depth = max_depth;
  hipLaunchKernelGGL(kv_alloc_pages_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, a);
  return check_launch(fn);
}

extern "C" int ss_kv_commit(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                            const int32_t* block_table, int max_pages_per_seq, int num_pages,
                            const int32_t* seq_lens, const int32_t* path, const int32_t* n_accept, int B, int T,
                            int gamma, int Hkv, int D, int page_size, int max_depth, int dtype,
                            int32_t* new_seq_lens, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_kv_commit";
  SS_REQUIRE(B >= 0, SS_ERR_INVALID_ARG, "%s: B=%d", fn, B);
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: T=%d outside [1,%d]", fn, T, SS_MAX_T);
  SS_REQUIRE(gamma >= 0 && gamma <= SS_MAX_GAMMA, SS_ERR_UNSUPPORTED, "%s: gamma=%d outside [0,%d]", fn, gamma,
             SS_MAX_GAMMA);
  SS_REQUIRE(Hkv >= 1 && D >= 1, SS_ERR_INVALID_ARG, "%s: Hkv=%d D=%d", fn, Hkv, D);
  SS_REQUIRE(dtype == SS_F32 || dtype == SS_BF16, SS_ERR_UNSUPPORTED, "%s: dtype %d", fn, dtype);
  SS_REQUIRE(page_size == 16 || page_size == 32 || page_size == 64, SS_ERR_UNSUPPORTED,
             "%s: page_size %d not in {16,32,64}", fn, page_size);
  SS_REQUIRE(max_pages_per_seq >= 1 && num_pages >= 1, SS_ERR_INVALID_ARG, "%s: max_pages_per_seq=%d num_pages=%d", fn,
             max_pages_per_seq, num_pages);
  SS_REQUIRE((long)max_pages_per_seq * page_size <= (1L << 30), SS_ERR_UNSUPPORTED, "%s: sequence capacity too large",
             fn);
  SS_REQUIRE(max_depth >= 0 && max_depth < SS_MAX_T, SS_ERR_INVALID_ARG, "%s: max_depth=%d", fn, max_depth);
  SS_REQUIRE(B == 0 || (k_new && v_new && k_cache && v_cache && block_table && seq_lens && path && n_accept),
             SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  SS_REQUIRE(new_seq_lens == nullptr || new_seq_lens != seq_lens, SS_ERR_INVALID_ARG,
             "%s: new_seq_lens must not be the seq_lens array", fn);
  SS_REQUIRE((long)B * (max_depth + 1) <= 0x7fffffffL, SS_ERR_UNSUPPORTED, "%s: grid too large", fn);
  if (B == 0) return SS_OK;
  KvArgs a;
  a.k_new = k_new; a.v_new = v_new; a.k_cache = k_cache; a.v_cache = v_cache;
  a.block_table = block_table; a.seq_lens = seq_lens; a.path = path; a.n_accept = n_accept;
  a.new_seq_lens = new_seq_lens;
  a.B = B; a.T = T; a.R = T * (1 + gamma); a.Hkv = Hkv; a.D = D; a.page = page_size;
  a.page_shift = page_size == 16 ? 4 : (page_size == 32 ? 5 : 6);
  a.max_pages = max_pages_per_seq; a.num_pages = num_pages; a.max_depth = max_depth;
  SS_REQUIRE(Hkv <= 65535, SS_ERR_UNSUPPORTED, "%s: Hkv=%d", fn, Hkv);
  const dim3 grid((unsigned)(B * (max_depth + 1)), (unsigned)Hkv);
  if (dtype == SS_F32) hipLaunchKernelGGL(kv_commit_kernel<uint32_t>, grid, dim3(128), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(kv_commit_kernel<uint16_t>, grid, dim3(128), 0, (hipStream_t)stream, a);
  return check_launch(fn);
}
