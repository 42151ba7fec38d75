// a2: multi-stream attention (Eq. 1 main rows, Eq. 2 stream rows) over a paged
// KV cache.  This file holds the entry point, the split planning, the fp32
// kernel and the kernel that merges the per-split partial results.
#include <math.h>
#include <stdlib.h>

#include <atomic>
#include <mutex>

#include "ss_msa.h"

namespace ss {

// ------------------------------------------------------------------ fp32 kernel
//
// One workgroup = (row chunk of 32 rows, split, sequence, head); wave w owns 8 of
// the rows.  Keys are taken 64 at a time: the K tile sits in LDS token-major
// (padded), the V tile feature-major (padded); in the score phase a lane owns a
// key, in the P.V phase it owns output features.  Softmax is the usual running
// max / running sum in the log2 domain.
template <int D>
__global__ __launch_bounds__(256) void msa_f32_kernel(MsaArgs a) {
  constexpr int RC = 32, RW = 8, KT = 64, DL = D / 64;
  __shared__ float Qs[RC][D];
  __shared__ float Ks[KT][D + 1];
  __shared__ float Vs[D][KT + 1];
  __shared__ float Ps[4][RW][KT];
  __shared__ int par[SS_MAX_T];
  __shared__ uint64_t anc[SS_MAX_T];

  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int chunk = blockIdx.x, s = blockIdx.y;
  const int b = blockIdx.z / a.H, h = blockIdx.z % a.H, hk = h / a.g;
  const int L = clamp_len(a.seq_lens[b], a);
  const int n_active = active_splits(L, a);
  if (s >= n_active) return;
  const bool is_last = (s == n_active - 1);
  const int k0 = split_begin(s, a);
  const int n_prefix = max(0, min(L, k0 + split_len(s, a)) - k0);
  const int n_new = is_last ? a.R : 0;
  const int total = n_prefix + n_new;
  const int r0 = chunk * RC;
  const int R = a.R, T = a.T;
  const int n_kept = kept_nodes(b, a);

  const float* q = (const float*)a.q;
  const float* k_new = (const float*)a.k_new;
  const float* v_new = (const float*)a.v_new;
  const float* k_cache = (const float*)a.k_cache;
  const float* v_cache = (const float*)a.v_cache;

  if (tid < T) par[tid] = clamp_parent(a.parent[(size_t)b * T + tid], tid);
  for (int e = tid; e < RC * D; e += 256) {
    const int r = e / D, d = e % D;
    Qs[r][d] = (r0 + r < R) ? q[(((size_t)b * R + r0 + r) * a.H + h) * D + d] : 0.f;
  }
  __syncthreads();
  compute_anc(par, T, anc, tid);
  __syncthreads();

  RowVis vis[RW];
  float m[RW], l[RW], o[RW][DL];
#pragma unroll
  for (int i = 0; i < RW; ++i) {
    vis[i] = make_row_vis(min(r0 + w * RW + i, R - 1), T, a.gamma, anc, (a.flags & SS_STREAM_EXCLUDE_SELF) != 0);
    m[i] = -1e30f;
    l[i] = 0.f;
#pragma unroll
    for (int dd = 0; dd < DL; ++dd) o[i][dd] = 0.f;
  }

  for (int t0 = 0; t0 < total; t0 += KT) {
    __syncthreads();  // the previous tile has been consumed
    // K tile: consecutive threads take consecutive features of one key
    for (int e = tid; e < KT * D; e += 256) {
      const int kk = e / D, d = e % D, u = t0 + kk;
      float v = 0.f;
      if (u < n_prefix) {
        const int tok = k0 + u;
        int pg = a.block_table[(size_t)b * a.max_pages + (tok >> a.page_shift)];
        pg = min(max(pg, 0), a.num_pages - 1);
        v = k_cache[(((size_t)pg * a.Hkv + hk) * a.page + (tok & (a.page - 1))) * D + d];
      } else if (u < total) {
        v = k_new[(((size_t)b * R + (u - n_prefix)) * a.Hkv + hk) * D + d];
      }
      Ks[kk][d] = v;
    }
    // V tile: consecutive threads take consecutive tokens (contiguous inside a feature-major page)
    for (int e = tid; e < KT * D; e += 256) {
      const int kk = e % KT, d = e / KT, u = t0 + kk;
      float v = 0.f;
      if (u < n_prefix) {
        const int tok = k0 + u;
        int pg = a.block_table[(size_t)b * a.max_pages + (tok >> a.page_shift)];
        pg = min(max(pg, 0), a.num_pages - 1);
        v = v_cache[(((size_t)pg * a.Hkv + hk) * D + d) * a.page + (tok & (a.page - 1))];
      } else if (u < total) {
        v = v_new[(((size_t)b * R + (u - n_prefix)) * a.Hkv + hk) * D + d];
      }
      Vs[d][kk] = v;
    }
    __syncthreads();

    // scores of this lane's key against the wave's 8 rows
    float sc[RW];
#pragma unroll
    for (int i = 0; i < RW; ++i) sc[i] = 0.f;
#pragma unroll 4
    for (int d = 0; d < D; ++d) {
      const float kd = Ks[lane][d];
#pragma unroll
      for (int i = 0; i < RW; ++i) sc[i] = fmaf(Qs[w * RW + i][d], kd, sc[i]);
    }
    const int u = t0 + lane;
#pragma unroll
    for (int i = 0; i < RW; ++i) {
      bool vis_ok = u < total;
      if (u >= n_prefix) vis_ok = vis_ok && row_sees(vis[i], u - n_prefix, T);
      const float sv = vis_ok ? sc[i] * a.scale_log2 : -INFINITY;
      float mx = sv;
      for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      const float m_new = fmaxf(m[i], mx);
      const float alpha = exp2f(m[i] - m_new);
      const float p = exp2f(sv - m_new);
      float ps = p;
      for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off, 64);
      l[i] = l[i] * alpha + ps;
      m[i] = m_new;
#pragma unroll
      for (int dd = 0; dd < DL; ++dd) o[i][dd] *= alpha;
      Ps[w][i][lane] = p;
    }
    // P.V: a lane owns output features lane, lane+64; the probabilities of the wave's
    // rows are read back from LDS (same address for all lanes: a broadcast)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll 4
    for (int kk = 0; kk < KT; ++kk) {
      float vk[DL];
#pragma unroll
      for (int dd = 0; dd < DL; ++dd) vk[dd] = Vs[lane + 64 * dd][kk];
#pragma unroll
      for (int i = 0; i < RW; ++i) {
        const float pk = Ps[w][i][kk];
#pragma unroll
        for (int dd = 0; dd < DL; ++dd) o[i][dd] = fmaf(pk, vk[dd], o[i][dd]);
      }
    }
  }

#pragma unroll
  for (int i = 0; i < RW; ++i) {
    const int row = r0 + w * RW + i;
    if (row >= R) continue;
    if ((row < T ? row : (row - T) / max(a.gamma, 1)) >= n_kept) continue;  // rows of removed nodes are not written
    const float inv = l[i] > 0.f ? 1.f / l[i] : 0.f;
    if (a.n_splits == 1) {
      float* out = (float*)a.out + (((size_t)b * R + row) * a.H + h) * D;
#pragma unroll
      for (int dd = 0; dd < DL; ++dd) out[lane + 64 * dd] = o[i][dd] * inv;
    } else {
      const size_t pr = (((size_t)b * a.H + h) * a.n_splits + s) * R + row;
#pragma unroll
      for (int dd = 0; dd < DL; ++dd) a.part_o[pr * D + lane + 64 * dd] = o[i][dd] * inv;
      if (lane == 0) a.part_lse[pr] = m[i] + log2f(l[i]);
    }
  }
}

// ------------------------------------------------------------------ merge of splits
//
// out = sum_s w_s * o_s with w_s = 2^(lse_s - max) / sum.  One thread per (sequence, row, head,
// 4 features).  The partial outputs are fetched four splits at a time without waiting for the
// log-sum-exps (their addresses do not depend on them) and folded in with a running maximum, so the
// kernel is one round of independent loads deep; splits a sequence does not use are never read.
template <bool BF16>
__global__ __launch_bounds__(256) void msa_combine_kernel(MsaArgs a) {
  const int dq = a.D >> 2;  // threads per row
  const long t = (long)blockIdx.x * 256 + threadIdx.x;
  const long item = t / dq;
  const int d0 = (int)(t % dq) * 4;
  if (item >= (long)a.B * a.R * a.H) return;
  const int h = item % a.H;
  const int r = (item / a.H) % a.R;
  const int b = item / ((long)a.H * a.R);
  if ((r < a.T ? r : (r - a.T) / max(a.gamma, 1)) >= kept_nodes(b, a)) return;  // rows of removed nodes: no partials, not written
  const int n_active = active_splits(clamp_len(a.seq_lens[b], a), a);
  const size_t base = (((size_t)b * a.H + h) * a.n_splits) * a.R + r;
  float m = -INFINITY, wsum = 0.f;
  floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < n_active; s0 += 4) {
    floatx4 v[4];
    float l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int s = min(s0 + i, n_active - 1);
      const size_t row = base + (size_t)s * a.R;
      v[i] = *reinterpret_cast<const floatx4*>(a.part_o + row * a.D + d0);
      l[i] = a.part_lse[row];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (s0 + i < n_active && l[i] > -INFINITY) {
        const float m_new = fmaxf(m, l[i]);
        const float keep = exp2f(m - m_new), w = exp2f(l[i] - m_new);
        acc = merge_step(acc, keep, v[i], w);
        wsum = __builtin_fmaf(wsum, keep, w);
        m = m_new;
      }
    }
  }
  const float inv = wsum > 0.f ? 1.f / wsum : 0.f;
  acc *= inv;
  const size_t oidx = (((size_t)b * a.R + r) * a.H + h) * a.D + d0;
  if (BF16) {
    *reinterpret_cast<uintx2*>((uint16_t*)a.out + oidx) = uintx2{pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3])};
  } else {
    *reinterpret_cast<floatx4*>((float*)a.out + oidx) = acc;
  }
}

// ------------------------------------------------------------------ planning (host)

static std::atomic<int> g_split_keys_override{0};
static std::atomic<int> g_merge_in_kernel{1};

struct MsaPlan {
  int split_keys, split0_keys, n_splits, n_qc, groups, stages;
  size_t part_o_bytes, part_lse_bytes, arrive_bytes, total_bytes;
};

// Chooses the split length from the shape alone (sequence lengths live on the device).  Every split
// costs a workgroup set-up and fp32 partial results that are read back, so the plan uses as few as fill
// the chip; no split is shorter than 256 cached tokens.
//   fp32 kernel: splits for about 512 workgroups.
//   MFMA kernel: with 512 or more (sequence, KV head, row chunk) items one workgroup of one wave group
//   each with a two-stage ring, three resident per compute unit (measured best when lengths vary: the
//   hardware evens them out); with fewer, two wave groups per workgroup (the prefix split again inside the
//   workgroup and merged through LDS) with three ring stages each, and splits for about 256 workgroups;
//   three wave groups when a sequence has several row chunks (long GQA trees: the kernel is then bound by
//   the matrix cores and more waves hide more latency).  Split 0 also scans the step's own rows and gets
//   that much less of the prefix.
// Tuning aid: blocks' worth of time, beyond its ceil(R/32) blocks, that scanning the step's own rows costs
// split 0 (SS_MSA_SPLIT0_EXTRA, read once).
static int split0_extra_blocks() {
  static const int v = []() {
    const char* e = getenv("SS_MSA_SPLIT0_EXTRA");
    const int x = e ? atoi(e) : 2;
    return x < -64 ? -64 : (x > 64 ? 64 : x);
  }();
  return v;
}

static MsaPlan make_plan(int B, int R, int H, int Hkv, int D, int max_len, int dtype) {
  MsaPlan p;
  const int g = H / Hkv;
  int base;
  p.groups = 1;
  p.stages = 2;
  if (dtype == SS_BF16) {
    const int rows = msa_bf16_rows_per_chunk(g * R);
    p.n_qc = ceil_div(g * R, rows);
    base = B * Hkv * p.n_qc;
  } else {
    p.n_qc = ceil_div(R, 32);
    base = B * H * p.n_qc;
  }
  if (base < 1) base = 1;
  const int len = max_len < 1 ? 1 : max_len;
  const int unit = dtype == SS_BF16 ? 32 : 64;  // the MFMA kernel works in 32-key blocks, the fp32 kernel in 64-key tiles
  int split_keys = g_split_keys_override.load();
  const bool overridden = split_keys > 0;
  int want_wgs = 512;
  if (dtype == SS_BF16) {
    if (base < 512) {
      p.groups = 2;
      p.stages = 3;
      want_wgs = 256;
    } else if (p.n_qc > 1) {
      p.groups = 3;
      p.stages = 3;
    }
    if (p.n_qc > 1) p.groups = msa_bf16_rows_per_chunk(g * R) == 128 ? 2 : 3;  // 16 or 15 waves per workgroup
  }
  if (split_keys <= 0) {
    int n = ceil_div(want_wgs, base);
    const int n_cap = len / 256 < 1 ? 1 : len / 256;
    if (n > n_cap) n = n_cap;
    if (dtype == SS_BF16 && p.n_qc > 1 && base >= 256) {
      // Several row chunks, one workgroup per compute unit: whole rounds of 256 workgroups matter more than
      // anything else.  The fewest splits (of at least 1024 tokens) that waste the least of the last round:
      // 320 items -> 4 splits = 5 rounds exactly (c5: 845 us; unsplit, in 2 rounds of which the second is a
      // quarter full: 1120 us).
      int best_n = 1;
      double best_waste = 0.0;
      for (int cand = 1; cand <= 8 && (cand == 1 || len / cand >= 1024); ++cand) {
        const double wgs = (double)base * cand, waste = ceil(wgs / 256.0) * 256.0 / wgs;
        if (cand == 1 || waste < best_waste - 1e-9) {
          best_n = cand;
          best_waste = waste;
        }
      }
      n = best_n;
    }
    split_keys = ceil_div(ceil_div(len, unit), n) * unit;
  }
  split_keys = (int)align_up((size_t)(split_keys < 64 ? 64 : split_keys), unit);
  p.split_keys = p.split0_keys = split_keys;
  p.n_splits = ceil_div(len, split_keys);
  if (dtype == SS_BF16 && p.n_splits > 1 && !overridden) {
    // Split 0 also scans the step's own rows: masked blocks with transposing reads, about `extra` blocks'
    // worth of time.  It gets that much less of the prefix; the others take whole iterations of all wave
    // groups where that leaves split 0 something.
    const int nu = ceil_div(len, 32), n = p.n_splits, extra = ceil_div(R, 32) + split0_extra_blocks();
    int rest = (nu + extra + n / 2) / n;
    rest = (rest + p.groups / 2) / p.groups * p.groups;
    if (rest >= 2 && nu - (n - 1) * rest >= 1) {
      p.split_keys = 32 * rest;
      p.split0_keys = 32 * (nu - (n - 1) * rest);
    }
  }
  if (p.n_splits > 1) {
    p.part_o_bytes = align_up((size_t)B * H * p.n_splits * R * D * sizeof(float), 256);
    p.part_lse_bytes = align_up((size_t)B * H * p.n_splits * R * sizeof(float), 256);
    p.arrive_bytes = (dtype == SS_BF16 && p.n_splits == 2)
                         ? align_up((size_t)B * Hkv * p.n_qc * kArriveTiles * sizeof(unsigned int), 256) : 0;
  } else {
    p.part_o_bytes = p.part_lse_bytes = p.arrive_bytes = 0;
  }
  p.total_bytes = p.part_o_bytes + p.part_lse_bytes + p.arrive_bytes + 256;
  return p;
}

// Whether a full call folds its two splits inside the attention kernel (see ss_msa_attention).
static bool merges_in_kernel(const MsaPlan& plan, int dtype) {
  return g_merge_in_kernel.load() && dtype == SS_BF16 && plan.n_splits == 2;
}

static int check_shape(const char* fn, int B, int T, int gamma, int H, int Hkv, int D, int dtype) {
  SS_REQUIRE(B >= 0, SS_ERR_INVALID_ARG, "%s: B=%d", fn, B);
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: T=%d outside [1,%d]", fn, T, SS_MAX_T);
  SS_REQUIRE(gamma >= 0 && gamma <= SS_MAX_GAMMA, SS_ERR_UNSUPPORTED, "%s: gamma=%d outside [0,%d]", fn, gamma,
             SS_MAX_GAMMA);
  SS_REQUIRE(H >= 1 && Hkv >= 1 && H % Hkv == 0, SS_ERR_INVALID_ARG, "%s: H=%d must be a multiple of Hkv=%d", fn, H,
             Hkv);
  SS_REQUIRE(D == 64 || D == 128, SS_ERR_UNSUPPORTED, "%s: head dim %d not in {64,128}", fn, D);
  SS_REQUIRE(dtype == SS_F32 || dtype == SS_BF16, SS_ERR_UNSUPPORTED, "%s: dtype %d", fn, dtype);
  return SS_OK;
}

// Zero fill by a kernel (a memset node must not be recorded into a captured graph): 16 bytes per thread over
// the aligned middle, thread 0 also takes the unaligned ends.
__global__ __launch_bounds__(256) void zero_bytes_kernel(unsigned char* p, size_t head, size_t chunks, size_t tail) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < chunks) reinterpret_cast<uintx4*>(p + head)[i] = uintx4{0u, 0u, 0u, 0u};
  if (i == 0) {
    for (size_t j = 0; j < head; ++j) p[j] = 0;
    for (size_t j = 0; j < tail; ++j) p[head + 16 * chunks + j] = 0;
  }
}
static int zero_bytes(unsigned char* p, size_t bytes, hipStream_t st, const char* fn) {
  if (bytes == 0) return SS_OK;
  size_t head = (16 - ((uintptr_t)p & 15)) & 15;
  if (head > bytes) head = bytes;
  const size_t chunks = (bytes - head) / 16, tail = bytes - head - 16 * chunks;
  const size_t blocks = chunks / 256 + 1;
  SS_REQUIRE(blocks <= 0x7fffffffUL, SS_ERR_UNSUPPORTED, "%s: %zu bytes are too many for one fill", fn, bytes);
  hipLaunchKernelGGL(zero_bytes_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, head, chunks, tail);
  return check_launch(fn);
}

// Scratch memory of ss_msa_attention_static: the per-split partial results and the arrival counters of a
// call, for callers that cannot provide a workspace.  Every GPU the library runs on holds its own copy of
// the array; host code reaches it only through the address hipGetSymbolAddress reports for the device that
// is current, looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char g_msa_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];  // guarded by g_scratch_mutex

static int static_scratch(const char* fn, void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) SS_FAIL(SS_ERR_HIP, "%s: hipGetDevice: %s", fn, hipGetErrorString(e));
  SS_REQUIRE(dev >= 0 && dev < kMaxDevices, SS_ERR_UNSUPPORTED, "%s: device %d outside [0,%d)", fn, dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_msa_scratch));
    if (e != hipSuccess || p == nullptr)
      SS_FAIL(SS_ERR_HIP, "%s: hipGetSymbolAddress: %s", fn, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return SS_OK;
}

// The body of ss_msa_attention and ss_msa_attention_static.  `library_scratch`: the workspace is the library's
// own array, whose size is a limit of the call (not a caller's mistake) and whose arrival counters are cleared
// here on every call.
static int msa_run(const char* fn, const void* q, const void* k_new, const void* v_new, const void* k_cache,
                   const void* v_cache, const int32_t* block_table, int max_pages_per_seq, int num_pages,
                   const int32_t* seq_lens, const int32_t* parent, const int32_t* n_nodes, int B, int T, int gamma, int H,
                   int Hkv, int D, int page_size, float scale, int dtype, uint32_t flags, void* out, void* workspace,
                   size_t workspace_bytes, bool library_scratch, void* stream) {
  if (int rc = check_shape(fn, B, T, gamma, H, Hkv, D, dtype)) return rc;
  SS_REQUIRE(B == 0 || (q && k_new && v_new && k_cache && v_cache && block_table && seq_lens && parent && out),
             SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  SS_REQUIRE(page_size == 16 || page_size == 32 || page_size == 64, SS_ERR_UNSUPPORTED,
             "%s: page_size %d not in {16,32,64}", fn, page_size);
  SS_REQUIRE(max_pages_per_seq >= 1 && num_pages >= 1, SS_ERR_INVALID_ARG, "%s: max_pages_per_seq=%d num_pages=%d", fn,
             max_pages_per_seq, num_pages);
  SS_REQUIRE((long)max_pages_per_seq * page_size <= (1L << 30), SS_ERR_UNSUPPORTED, "%s: sequence capacity too large",
             fn);
  // the MFMA kernel keeps a page's offset in units of 256 bytes in 32 bits
  SS_REQUIRE(dtype != SS_BF16 || (double)num_pages * Hkv * page_size * D * 2.0 <= 1099511627776.0, SS_ERR_UNSUPPORTED,
             "%s: a cache of more than 1 TiB per tensor (num_pages=%d)", fn, num_pages);
  SS_REQUIRE(scale > 0.f && isfinite(scale), SS_ERR_INVALID_ARG, "%s: scale must be positive and finite", fn);
  SS_REQUIRE((flags & ~(SS_STREAM_EXCLUDE_SELF | SS_MSA_PARTIALS_ONLY | SS_MSA_MERGE_ONLY)) == 0, SS_ERR_INVALID_ARG,
             "%s: unknown flags 0x%x", fn, flags);
  SS_REQUIRE((flags & (SS_MSA_PARTIALS_ONLY | SS_MSA_MERGE_ONLY)) != (SS_MSA_PARTIALS_ONLY | SS_MSA_MERGE_ONLY),
             SS_ERR_INVALID_ARG, "%s: SS_MSA_PARTIALS_ONLY and SS_MSA_MERGE_ONLY exclude each other", fn);
  if (B == 0) return SS_OK;

  const int R = T * (1 + gamma);
  const int max_len = max_pages_per_seq * page_size;
  const MsaPlan plan = make_plan(B, R, H, Hkv, D, max_len, dtype);
  if (library_scratch) {
    SS_REQUIRE(plan.total_bytes <= workspace_bytes, SS_ERR_UNSUPPORTED,
               "%s: this shape needs %zu bytes of scratch memory, the library's array holds %zu; use "
               "ss_msa_attention with a workspace", fn, plan.total_bytes, workspace_bytes);
  } else {
    SS_REQUIRE(plan.n_splits == 1 || (workspace != nullptr && workspace_bytes >= plan.total_bytes), SS_ERR_WORKSPACE,
               "%s: workspace of %zu bytes needed, %zu given", fn, plan.total_bytes, workspace_bytes);
  }

  MsaArgs a;
  a.q = q; a.k_new = k_new; a.v_new = v_new; a.k_cache = k_cache; a.v_cache = v_cache;
  a.block_table = block_table; a.seq_lens = seq_lens; a.parent = parent; a.n_nodes = n_nodes; a.out = out;
  char* ws = (char*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  a.part_o = (float*)ws;
  a.part_lse = (float*)(ws + plan.part_o_bytes);
  a.B = B; a.T = T; a.gamma = gamma; a.R = R; a.H = H; a.Hkv = Hkv; a.g = H / Hkv; a.D = D;
  a.page = page_size; a.page_shift = page_size == 16 ? 4 : (page_size == 32 ? 5 : 6);
  a.max_pages = max_pages_per_seq; a.num_pages = num_pages;
  a.split_keys = plan.split_keys; a.split0_keys = plan.split0_keys; a.n_splits = plan.n_splits; a.n_qc = plan.n_qc; a.groups = plan.groups; a.stages = plan.stages;
  a.scale_log2 = scale * 1.4426950408889634f;
  // In-kernel merge (MFMA path, two splits): the second split of a (sequence, head) to finish adds the other's
  // partial rows to its own and writes the output, which saves the merge kernel and its kernel boundary.  With
  // more splits the partial rows would be fetched one split after the other and the merge kernel is faster.
  a.arrive = nullptr;
  if (merges_in_kernel(plan, dtype) && !(flags & SS_MSA_MERGE_ONLY))
    a.arrive = (unsigned int*)(ws + plan.part_o_bytes + plan.part_lse_bytes);
  a.flags = flags;
  hipStream_t st = (hipStream_t)stream;

  if (library_scratch && a.arrive != nullptr)
    if (int rc = zero_bytes((unsigned char*)a.arrive, plan.arrive_bytes, st, fn)) return rc;
  if (flags & SS_MSA_MERGE_ONLY) {
    // the attention kernel ran in an earlier call with SS_MSA_PARTIALS_ONLY
  } else if (dtype == SS_F32) {
    dim3 grid(plan.n_qc, plan.n_splits, B * H);
    SS_REQUIRE((long)B * H <= 65535 && plan.n_splits <= 65535, SS_ERR_UNSUPPORTED, "%s: grid too large", fn);
    if (D == 64) hipLaunchKernelGGL(msa_f32_kernel<64>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(msa_f32_kernel<128>, grid, dim3(256), 0, st, a);
    if (int rc = check_launch(fn)) return rc;
  } else {
    if (int rc = launch_msa_bf16(a, st)) return rc;
  }
  if (plan.n_splits > 1 && !(flags & SS_MSA_PARTIALS_ONLY) && a.arrive == nullptr) {
    const long threads = (long)B * R * H * (D / 4);
    dim3 grid((unsigned)((threads + 255) / 256));
    if (dtype == SS_F32) hipLaunchKernelGGL(msa_combine_kernel<false>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(msa_combine_kernel<true>, grid, dim3(256), 0, st, a);
    if (int rc = check_launch(fn)) return rc;
  }
  return SS_OK;
}

}  // namespace ss

extern "C" {

int ss_msa_set_split_keys(int split_keys) {
  return ss::g_split_keys_override.exchange(split_keys > 0 ? split_keys : 0);
}

int ss_msa_set_merge_in_kernel(int on) { return ss::g_merge_in_kernel.exchange(on ? 1 : 0); }

int ss_msa_plan(int B, int T, int gamma, int H, int Hkv, int D, int max_seq_len, int dtype, int* n_splits,
                int* n_kernels) {
  ss::clear_error();
  if (int rc = ss::check_shape("ss_msa_plan", B, T, gamma, H, Hkv, D, dtype)) return rc;
  if (max_seq_len < 0) max_seq_len = 0;
  const ss::MsaPlan plan = ss::make_plan(B, T * (1 + gamma), H, Hkv, D, max_seq_len, dtype);
  if (n_splits) *n_splits = plan.n_splits;
  if (n_kernels) *n_kernels = (plan.n_splits > 1 && !ss::merges_in_kernel(plan, dtype)) ? 2 : 1;
  return SS_OK;
}

size_t ss_msa_workspace_bytes(int B, int T, int gamma, int H, int Hkv, int D, int max_seq_len, int dtype) {
  ss::clear_error();
  if (ss::check_shape("ss_msa_workspace_bytes", B, T, gamma, H, Hkv, D, dtype) != SS_OK) return 0;
  if (max_seq_len < 0) max_seq_len = 0;
  return ss::make_plan(B, T * (1 + gamma), H, Hkv, D, max_seq_len, dtype).total_bytes;
}

int ss_msa_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  ss::clear_error();
  SS_REQUIRE(workspace != nullptr || workspace_bytes == 0, SS_ERR_INVALID_ARG, "ss_msa_workspace_init: NULL workspace");
  return ss::zero_bytes((unsigned char*)workspace, workspace_bytes, (hipStream_t)stream, "ss_msa_workspace_init");
}

int ss_msa_attention(const void* q, const void* k_new, const void* v_new, const void* k_cache, const void* v_cache,
                     const int32_t* block_table, int max_pages_per_seq, int num_pages, const int32_t* seq_lens,
                     const int32_t* parent, int B, int T, int gamma, int H, int Hkv, int D, int page_size, float scale,
                     int dtype, uint32_t flags, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  ss::clear_error();
  return ss::msa_run("ss_msa_attention", q, k_new, v_new, k_cache, v_cache, block_table, max_pages_per_seq, num_pages,
                     seq_lens, parent, nullptr, B, T, gamma, H, Hkv, D, page_size, scale, dtype, flags, out, workspace,
                     workspace_bytes, false, stream);
}

int ss_msa_attention_pruned(const void* q, const void* k_new, const void* v_new, const void* k_cache,
                            const void* v_cache, const int32_t* block_table, int max_pages_per_seq, int num_pages,
                            const int32_t* seq_lens, const int32_t* parent, const int32_t* n_nodes, int B, int T,
                            int gamma, int H, int Hkv, int D, int page_size, float scale, int dtype, uint32_t flags,
                            void* out, void* workspace, size_t workspace_bytes, void* stream) {
  ss::clear_error();
  SS_REQUIRE(B == 0 || n_nodes != nullptr, SS_ERR_INVALID_ARG, "ss_msa_attention_pruned: NULL n_nodes");
  return ss::msa_run("ss_msa_attention_pruned", q, k_new, v_new, k_cache, v_cache, block_table, max_pages_per_seq,
                     num_pages, seq_lens, parent, n_nodes, B, T, gamma, H, Hkv, D, page_size, scale, dtype, flags, out,
                     workspace, workspace_bytes, false, stream);
}

size_t ss_msa_static_scratch_bytes(void) { return ss::kStaticScratchBytes; }

int ss_msa_attention_static(const void* q, const void* k_new, const void* v_new, const void* k_cache,
                            const void* v_cache, const int32_t* block_table, int max_pages_per_seq, int num_pages,
                            const int32_t* seq_lens, const int32_t* parent, int B, int T, int gamma, int H, int Hkv,
                            int D, int page_size, float scale, int dtype, uint32_t flags, void* out, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_msa_attention_static";
  void* scratch = nullptr;
  if (int rc = static_scratch(fn, &scratch)) return rc;
  return msa_run(fn, q, k_new, v_new, k_cache, v_cache, block_table, max_pages_per_seq, num_pages, seq_lens, parent,
                 nullptr, B, T, gamma, H, Hkv, D, page_size, scale, dtype, flags, out, scratch, kStaticScratchBytes, true, stream);
}

}  // extern "C"
