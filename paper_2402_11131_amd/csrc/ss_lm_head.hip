// a3: LM head with fused arg-max / top-K (Sec. 3.2.1, 3.2.2).  logits = hidden . W^T
// are produced tile by tile in registers and reduced to K candidates per (row,
// vocabulary tile) in the same kernel; a second, tiny kernel merges the
// candidates of all tiles.  The logits themselves never reach memory.
//
// Order everywhere: larger logit first, equal logits -> lower token id first.
#include <limits.h>
#include <math.h>
#include <stdlib.h>

#include <atomic>
#include <mutex>

#include "ss_common.h"
#include "ss_tree.h"

namespace ss {

struct LmArgs {
  const void* hidden;  // [N,d]
  const void* W;       // [V,d]
  int N, d, V, K;
  int n_tiles;         // vocabulary tiles
  int n_chunks;        // row chunks (bf16 kernel)
  int k_stagger;       // feature blocks between the starting blocks of neighbouring vocabulary tiles (bf16 kernel)
  uint64_t* cand_key;  // [N, n_tiles, K] candidates as ordered keys
  int32_t* idx;        // [N,K]
  float* val;          // [N,K]
  void* y;             // [N,V], plain-projection flavour only (same type as the inputs)
  float* lse;          // [N], log-sum-exp flavour only; its parts (max, sum) per (row, tile) use cand_key's memory
  const int32_t* live_rows;  // rows to compute, ascending ([N], the first *n_live entries count), or NULL = all N rows
  const int32_t* n_live;     // [1] device, or NULL
  int n_ksplit;        // workgroups that share a tile's feature dimension (bf16 projection with a workspace), else 1
  float* part;         // [n_ksplit, N, V] fp32 partial products of those workgroups, else NULL
};

// Rows a launch computes, and the row of `hidden` / of the outputs that its r-th computed row is (r is clamped
// to the last computed row, ids to [0,N): addresses formed from them are always valid).
SS_DEV int lm_rows(const LmArgs& a) { return a.n_live ? min(max(*a.n_live, 0), a.N) : a.N; }
SS_DEV int lm_row_id(const LmArgs& a, int r, int n_rows) {
  const int rc = min(r, n_rows - 1);
  return a.live_rows ? min(max(a.live_rows[rc], 0), a.N - 1) : rc;
}

SS_DEV bool cand_better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }
SS_DEV bool cand_after(float v, int i, float pv, int pi) { return v < pv || (v == pv && i > pi); }

// (max, sum of exp(x - max)) of two sets of logits -> of their union.  An empty set is (-inf, 0).
SS_DEV float2 lse_merge(float2 p, float2 q) {
  const float m = fmaxf(p.x, q.x);
  const float sp = p.x == -INFINITY ? 0.f : p.y * __expf(p.x - m);
  const float sq = q.x == -INFINITY ? 0.f : q.y * __expf(q.x - m);
  return make_float2(m, sp + sq);
}

// A candidate as one 64-bit key whose unsigned order is the candidate order: the logit mapped to an
// order-preserving unsigned pattern in the high word, the complement of the token id in the low word
// (equal logits -> lower id first).  Key 0 ranks below every real candidate.
SS_DEV uint64_t cand_key(float v, int id) {
  v += 0.f;  // -0 -> +0, so that the two zeros tie
  const uint32_t u = __float_as_uint(v);
  const uint32_t o = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((uint64_t)o << 32) | (uint32_t)(0xffffffffu - (uint32_t)id);
}
SS_DEV float key_value(uint64_t k) {
  const uint32_t o = (uint32_t)(k >> 32);
  return k == 0 ? -INFINITY : __uint_as_float((o & 0x80000000u) ? (o ^ 0x80000000u) : ~o);
}
SS_DEV int key_id(uint64_t k) { return k == 0 ? INT_MAX : (int)(0xffffffffu - (uint32_t)k); }


// ------------------------------------------------------------------ fp32 kernel (small problems)
//
// Workgroup tile 32 rows x 64 vocabulary columns, feature chunks of 32 through
// LDS; thread (wave w, lane c) accumulates rows w, w+4, ... of column c.
//
// MODE 0: top-K search.  MODE 1: the plain projection, the tile is written to y.  MODE 2: (max, sum of
// exp) of the tile's logits per row, for the log-sum-exp over the vocabulary.
template <int MODE>
__global__ __launch_bounds__(256) void lm_head_f32_kernel(LmArgs a) {
  constexpr int BM = 32, BN = 64, BK = 32;
  __shared__ float As[BM][BK + 1];
  __shared__ float Ws[BN][BK + 1];
  __shared__ float Z[BM][BN + 1];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int v0 = blockIdx.x * BN, r0 = blockIdx.y * BM;
  const int n_rows = lm_rows(a);
  if (r0 >= n_rows) return;
  const float* hidden = (const float*)a.hidden;
  const float* W = (const float*)a.W;
  float acc[BM / 4];
#pragma unroll
  for (int i = 0; i < BM / 4; ++i) acc[i] = 0.f;
  for (int k0 = 0; k0 < a.d; k0 += BK) {
    __syncthreads();
    for (int e = tid; e < BM * BK; e += 256) {
      const int r = e / BK, kk = e % BK;
      As[r][kk] = (r0 + r < n_rows && k0 + kk < a.d) ? hidden[(size_t)lm_row_id(a, r0 + r, n_rows) * a.d + k0 + kk] : 0.f;
    }
    for (int e = tid; e < BN * BK; e += 256) {
      const int cc = e / BK, kk = e % BK;
      Ws[cc][kk] = (v0 + cc < a.V && k0 + kk < a.d) ? W[(size_t)(v0 + cc) * a.d + k0 + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < BK; ++kk) {
      const float wv = Ws[lane][kk];
#pragma unroll
      for (int i = 0; i < BM / 4; ++i) acc[i] = fmaf(As[w + 4 * i][kk], wv, acc[i]);
    }
  }
  if constexpr (MODE == 1) {
#pragma unroll
    for (int i = 0; i < BM / 4; ++i) {
      const int row = r0 + w + 4 * i, col = v0 + lane;
      if (row < n_rows && col < a.V) ((float*)a.y)[(size_t)lm_row_id(a, row, n_rows) * a.V + col] = acc[i];
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < BM / 4; ++i) Z[w + 4 * i][lane] = acc[i];
  __syncthreads();
  if constexpr (MODE == 2) {
    for (int rr = w; rr < BM; rr += 4) {
      if (r0 + rr >= n_rows) break;
      const int row = lm_row_id(a, r0 + rr, n_rows);
      float2 p = v0 + lane < a.V ? make_float2(Z[rr][lane], 1.f) : make_float2(-INFINITY, 0.f);
      for (int off = 32; off > 0; off >>= 1)
        p = lse_merge(p, make_float2(__shfl_xor(p.x, off, 64), __shfl_xor(p.y, off, 64)));
      if (lane == 0) reinterpret_cast<float2*>(a.cand_key)[(size_t)row * a.n_tiles + blockIdx.x] = p;
    }
    return;
  }
  // wave w selects for rows w, w+4, ...: K rounds of a wave-wide arg-max over the 64 columns
  for (int rr = w; rr < BM; rr += 4) {
    if (r0 + rr >= n_rows) break;
    const int row = lm_row_id(a, r0 + rr, n_rows);
    const int col = v0 + lane;
    const float v = col < a.V ? Z[rr][lane] : -INFINITY;
    const int ci = col < a.V ? col : INT_MAX;
    float pv = INFINITY;
    int pi = -1;
    for (int k = 0; k < a.K; ++k) {
      float bv = -INFINITY;
      int bi = INT_MAX;
      if (cand_after(v, ci, pv, pi)) {
        bv = v;
        bi = ci;
      }
      for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(bv, off, 64);
        const int oi = __shfl_xor(bi, off, 64);
        if (cand_better(ov, oi, bv, bi)) {
          bv = ov;
          bi = oi;
        }
      }
      if (lane == 0) {
        const size_t o = ((size_t)row * a.n_tiles + blockIdx.x) * a.K + k;
        a.cand_key[o] = bi == INT_MAX ? 0 : cand_key(bv, bi);
      }
      pv = bv;
      pi = bi;
    }
  }
}

// ------------------------------------------------------------------ bf16 MFMA kernel
//
// The product is computed transposed, logits^T = W . hidden^T, with
// v_mfma_f32_32x32x16_bf16 (A = 32 token ids x 16 features, B = 16 features x 32
// rows).  In the 32x32 result a lane holds 16 token ids of ONE row, so the top-K
// over the vocabulary is mostly a per-lane affair: no logit is ever exchanged
// between lanes, only K-entry candidate lists.
//
// Workgroup = NW waves (4 or 8); tile = 32*NW token ids x 32*NRT rows; wave w owns
// ids [32*w, 32*w+32) and all rows of the tile: NRT accumulator tiles.  Rows beyond
// one tile go in equal chunks; the grid is one-dimensional and XCD-aware (below).
// Features go in blocks of 64 (one 128-byte line per row).  Both operands reach LDS
// by direct global->LDS loads (no staging registers and no ds_write: LDS stores of
// this size run at a quarter of the read rate).  Such a load writes lane l's 16
// bytes to (base + 16*l), so the LDS image is row-major; the chunks of a row are
// XOR-swizzled on the global side (lane (row r, position q) fetches chunk
// q ^ ((r >> 1) & 7)), which makes the operand reads (32 rows x one chunk, 16 lanes
// per LDS cycle over 64 banks) conflict free.  These loads are inline assembly (the
// compiler would drain the memory counter before every LDS read if it knew of
// them), so the wait for them is written by hand; loads complete in order.
//
// An earlier version fed W straight into operand registers (every lane 16 bytes of
// its own row: one instruction touches 32 lines for 32 bytes each) and kept all 320
// rows of the headline workload in one workgroup.  Taking loads out one kind at a
// time showed it bound by exactly those W loads (the L1 spends its tag lookups on
// them), most of all with few rows per workgroup; W through LDS with whole lines
// took the projection 4096 -> 4096 on 320 rows from 42 to 23 us and, as the
// 8-wave tile of 256 ids x 160 rows, the 320 x 4096 x 32000 LM head from 112 to 92 us.
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

// 16 bytes per lane from (sbase + voff) to LDS address lds_addr + 16*lane.
SS_DEV void load_to_lds16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0" ::"s"(sbase), "v"(voff), "s"(lds_addr) : "memory", "m0");
}
// The same with the streaming hint, for data that no other workgroup will ask for.
SS_DEV void load_to_lds16_stream(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0 nt" ::"s"(sbase), "v"(voff), "s"(lds_addr) : "memory", "m0");
}

// The KT best (logit, id) pairs of candidates that arrive in increasing id order: an equal logit
// never displaces an earlier entry, so a strict float compare implements "lower id first".
template <int KT>
struct TopAsc {
  float v[KT];
  int i[KT];
  SS_DEV void clear() {
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      v[j] = -INFINITY;
      i[j] = INT_MAX;
    }
  }
  SS_DEV void insert(float cv, int ci) {
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      const bool up = cv > v[j];
      const float nv = fmaxf(v[j], cv), ov = fminf(v[j], cv);
      const int ni = up ? ci : i[j], oi = up ? i[j] : ci;
      v[j] = nv;
      i[j] = ni;
      cv = ov;
      ci = oi;
    }
  }
};

// Median of three unsigned numbers (one instruction on this hardware).
SS_DEV uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
  const uint32_t lo = a < b ? a : b, hi = a < b ? b : a;
  const uint32_t m = hi < c ? hi : c;
  return lo > m ? lo : m;
}

template <int KT>
struct TopList {  // the KT best keys seen so far, best first
  uint64_t k[KT];
  SS_DEV void clear() {
#pragma unroll
    for (int j = 0; j < KT; ++j) k[j] = 0;
  }
  SS_DEV void insert(uint64_t c) {
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      const uint64_t hi = k[j] > c ? k[j] : c, lo = k[j] > c ? c : k[j];
      k[j] = hi;
      c = lo;
    }
  }
};

// The epilogue of both MFMA kernels.  acc[rt][e] on lane (ln, lh) is the logit of row row0 + 32*rt + ln
// and token id v0 + 8*(e/4) + 4*lh + e%4.  `hbuf` (64*NW + 16 bytes per row of the tile) must be free:
// the callers end their loops with a barrier.
template <int NRT, int KT, int NW>  // NW waves of 32 ids each
SS_DEV void lm_epilogue(const LmArgs& a, floatx16 (&acc)[NRT], unsigned char* hbuf, int tile, int row0, int n_rows, int v0,
                        int w, int tid) {
  constexpr int ROWS = 32 * NRT;
  constexpr int TI = 32 * NW;  // ids per tile
  const int lane = tid & 63, ln = lane & 31, lh = lane >> 5;
  if constexpr (KT == -1) {
    // Log-sum-exp: (max, sum of exp) of this lane's 16 logits of a row, of the row's two lanes, of the
    // NW waves through LDS; one thread per row leaves the tile's pair.
    float2* pairs = reinterpret_cast<float2*>(hbuf);  // [ROWS][NW]
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      float m = -INFINITY;
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (v0 + 8 * (e >> 2) + 4 * lh + (e & 3) < a.V) m = fmaxf(m, acc[rt][e]);
      float sum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (v0 + 8 * (e >> 2) + 4 * lh + (e & 3) < a.V) sum += __expf(acc[rt][e] - m);
      float2 p = make_float2(m, sum);
      p = lse_merge(p, make_float2(__shfl_xor(p.x, 32, 64), __shfl_xor(p.y, 32, 64)));
      if (lh == 0) pairs[(32 * rt + ln) * NW + w] = p;
    }
    __syncthreads();
    for (int r = tid; r < ROWS; r += 64 * NW) {
      float2 p = pairs[r * NW];
#pragma unroll
      for (int j = 1; j < NW; ++j) p = lse_merge(p, pairs[r * NW + j]);
      if (row0 + r < n_rows) reinterpret_cast<float2*>(a.cand_key)[(size_t)lm_row_id(a, row0 + r, n_rows) * a.n_tiles + tile] = p;
    }
    return;
  } else if constexpr (KT == -2) {
    // Partial product of one slice of the feature dimension: the fp32 tile is turned round through LDS in two
    // halves of the rows (a whole tile of 160 x 256 floats would not fit beside nothing) and leaves in 16-byte
    // pieces, 4*TI contiguous bytes per row, into this slice's plane of the workspace.
    constexpr int YS = 4 * TI + 16;
    constexpr int HALF = (NRT + 1) / 2;  // row tiles per pass
    const int ks = a.n_ksplit > 1 ? (int)((blockIdx.x >> 3) % (a.n_chunks * a.n_ksplit)) / a.n_chunks : 0;
    float* plane = a.part + (size_t)ks * a.N * a.V;
    const bool vec_ok = (a.V % 4) == 0 && ((uintptr_t)a.part & 15) == 0;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      if (pass == 1) __syncthreads();
#pragma unroll
      for (int rt = pass * HALF; rt < NRT && rt < (pass + 1) * HALF; ++rt)
#pragma unroll
        for (int eg = 0; eg < 4; ++eg) {
          const floatx4 v = floatx4{acc[rt][4 * eg], acc[rt][4 * eg + 1], acc[rt][4 * eg + 2], acc[rt][4 * eg + 3]};
          *reinterpret_cast<floatx4*>(hbuf + (32 * (rt - pass * HALF) + ln) * YS + (32 * w + 8 * eg + 4 * lh) * 4) = v;
        }
      __syncthreads();
      const int rows_here = 32 * ((pass == 0 ? HALF : NRT - HALF));
      for (int p = tid; p < rows_here * (TI / 4); p += 64 * NW) {
        const int r = p / (TI / 4), ch = p % (TI / 4);
        const int id0 = tile * TI + 4 * ch, rr = row0 + 32 * pass * HALF + r;
        if (rr >= n_rows || id0 >= a.V) continue;
        const floatx4 piece = *reinterpret_cast<const floatx4*>(hbuf + r * YS + ch * 16);
        float* dst = plane + (size_t)lm_row_id(a, rr, n_rows) * a.V + id0;
        if (vec_ok) {
          *reinterpret_cast<floatx4*>(dst) = piece;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (id0 + j < a.V) dst[j] = piece[j];
        }
      }
    }
    return;
  } else if constexpr (KT == 0) {
    // Plain projection: the tile is rounded to bf16 and turned round through LDS ([ROWS] rows of TI
    // outputs, padded by 16 bytes so that the 8-byte writes of 32 rows spread over the banks), then
    // leaves in 16-byte pieces, 2*TI contiguous bytes per row.
    constexpr int YS = 2 * TI + 16;
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int eg = 0; eg < 4; ++eg) {
        uintx2 pk;
        pk[0] = pack_bf16x2(acc[rt][4 * eg], acc[rt][4 * eg + 1]);
        pk[1] = pack_bf16x2(acc[rt][4 * eg + 2], acc[rt][4 * eg + 3]);
        *reinterpret_cast<uintx2*>(hbuf + (32 * rt + ln) * YS + (32 * w + 8 * eg + 4 * lh) * 2) = pk;
      }
    __syncthreads();
    const bool vec_ok = (a.V % 8) == 0 && ((uintptr_t)a.y & 15) == 0;  // rows of y are 16-byte aligned
    uint16_t* y = (uint16_t*)a.y;
    for (int p = tid; p < ROWS * (TI / 8); p += 64 * NW) {
      const int r = p / (TI / 8), ch = p % (TI / 8);
      const int id0 = tile * TI + 8 * ch;
      if (row0 + r >= n_rows || id0 >= a.V) continue;
      const int row = lm_row_id(a, row0 + r, n_rows);
      const uintx4 piece = *reinterpret_cast<const uintx4*>(hbuf + r * YS + ch * 16);
      uint16_t* dst = y + (size_t)row * a.V + id0;
      if (vec_ok) {
        *reinterpret_cast<uintx4*>(dst) = piece;  // V % 8 == 0 and id0 < V: the whole piece is inside
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (id0 + j < a.V) dst[j] = (uint16_t)(piece[j >> 1] >> (16 * (j & 1)));
      }
    }
    return;
  } else {
  // Per row: the KT best of this lane's 16 logits, then of the row's two lanes (32 token ids), are found on
  // 32-bit keys: the logit's order-preserving pattern with its five lowest bits replaced by 31 - (position of
  // the id among the wave's 32), so that one unsigned maximum / median per list entry inserts a candidate
  // (equal patterns -> lower id first) and no index travels beside the value.  The five bits cost 2^-18 of a
  // logit's magnitude in resolution: logits closer than that are ordered by id, and the values reported
  // carry those bits cleared.  The waves' lists (64-bit keys from here on: pattern, complement of the id) meet
  // in LDS, and one thread per row merges them by taking the best head KT times (every list is sorted).
  uint64_t* lists = reinterpret_cast<uint64_t*>(hbuf);  // [ROWS][NW waves][KT]
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    uint32_t top[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) top[k] = 0;  // ranks below every real candidate
    auto insert = [&](uint32_t x) {
#pragma unroll
      for (int k = KT - 1; k >= 1; --k) top[k] = umed3(top[k - 1], top[k], x);
      top[0] = top[0] > x ? top[0] : x;
    };
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int off = 8 * (e >> 2) + 4 * lh + (e & 3);
      const uint32_t u = __float_as_uint(acc[rt][e] + 0.f);  // -0 -> +0, so that the two zeros tie
      const uint32_t o = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      insert(v0 + off < a.V ? ((o & ~31u) | (uint32_t)(31 - off)) : 0u);
    }
    uint32_t other[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) other[k] = __shfl_xor(top[k], 32, 64);
#pragma unroll
    for (int k = 0; k < KT; ++k) insert(other[k]);
    if (lh == 0) {
#pragma unroll
      for (int k = 0; k < KT; ++k)
        lists[((32 * rt + ln) * NW + w) * KT + k] =
            top[k] == 0 ? 0 : (((uint64_t)(top[k] & ~31u) << 32) | (uint32_t)(0xffffffffu - (uint32_t)(v0 + 31 - (int)(top[k] & 31u))));
    }
  }
  __syncthreads();
  for (int r = tid; r < ROWS; r += 64 * NW) {
    const uint64_t* L = lists + (size_t)r * NW * KT;
    uint64_t head[NW];
    int pos[NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) {
      head[j] = L[j * KT];
      pos[j] = 0;
    }
    const bool row_ok = row0 + r < n_rows;
    const size_t o = ((size_t)lm_row_id(a, row0 + r, n_rows) * a.n_tiles + tile) * a.K;
#pragma unroll
    for (int k = 0; k < KT; ++k) {
      uint64_t best = head[0];
      int bw = 0;
#pragma unroll
      for (int j = 1; j < NW; ++j) {
        const bool up = head[j] > best;
        best = up ? head[j] : best;
        bw = up ? j : bw;
      }
      if (row_ok && k < a.K) a.cand_key[o + k] = best;
      if (k + 1 < KT) {
        // the winner's list moves on (lists are distinct ids, so the winner is unique unless all heads are empty)
        int np = 0;
#pragma unroll
        for (int j = 0; j < NW; ++j) {
          pos[j] += (j == bw) ? 1 : 0;
          np = (j == bw) ? pos[j] : np;
        }
        const uint64_t nh = np < KT ? L[bw * KT + np] : 0;
#pragma unroll
        for (int j = 0; j < NW; ++j) head[j] = (j == bw) ? nh : head[j];
      }
    }
  }
  }
}

// A block in LDS is hidden (32*NRT rows) followed by W (32*NW rows, each wave loading the 32 rows it
// owns); NBUF buffers, filled NBUF-1 blocks ahead; one extra operand read per MFMA round for W.  Every
// global load of the loop is hand-written, so the only wait is the one before a step's barrier.  NW = 4
// waves (tile of 128 ids, four buffers) or 8 (256 ids, two waves per SIMD, three buffers).  The 4*NRT
// hidden load slots are dealt to the waves in rounds; in a last, incomplete round the spare waves load
// a slot a second time (same bytes to the same place), which keeps the load count equal for all.
// WS: W is loaded with the streaming hint.  Right when the rows form one chunk, so that every line of W
// is wanted by exactly one workgroup (the pruning layer's 64 rows: 60 -> 53 us); with several row chunks
// the chunks of a vocabulary tile share W through the L2 and the hint undoes that.
template <int NRT, int KT, int NW, int NBUF, bool WS = false>
__global__ __launch_bounds__(64 * NW, 1) void lm_head_bf16_kernel(LmArgs a) {
  constexpr int ROWS = 32 * NRT;
  constexpr int TI = 32 * NW;
  constexpr int HB = ROWS * 128;     // bytes of one block of `hidden`
  constexpr int BB = HB + TI * 128;  // ... and of W behind it
  static_assert(NBUF * BB <= 160 * 1024, "buffers must fit 160 KB");
  static_assert(NBUF * BB >= ROWS * (2 * TI + 16) && NBUF * BB >= ROWS * NW * 64, "epilogue must fit the buffers");
  static_assert(KT != -2 || NBUF * BB >= ((NRT + 1) / 2) * 32 * (4 * TI + 16), "half of the fp32 tile must fit the buffers");
  constexpr int NH = (4 * NRT + NW - 1) / NW;  // hidden loads per wave and step
  constexpr int NLD = NH + 4;                  // global loads per wave and step
  extern __shared__ __attribute__((aligned(16))) unsigned char hbuf[];  // [NBUF][BB], reused by the epilogue
  const int tid = threadIdx.x, lane = tid & 63, ln = lane & 31, lh = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Workgroup -> (vocabulary tile, row chunk).  Workgroups are dealt to the eight XCDs in turn; the row
  // chunks of one vocabulary tile take consecutive turns of ONE XCD, so that they run together and
  // share that tile of W in its L2.
  // With a split feature dimension the n_ksplit slices of a (tile, chunk) are further workgroups of the same XCD.
  const int xcd = blockIdx.x & 7, turn = blockIdx.x >> 3;
  const int per_tile = a.n_chunks * a.n_ksplit;
  const int tile = (turn / per_tile) * 8 + xcd;
  if (tile >= a.n_tiles) return;
  const int v0 = tile * TI + 32 * w;
  const int n_rows = lm_rows(a);
  const int d = a.d, n_k = d / 64 / a.n_ksplit;                       // feature blocks of this workgroup
  const size_t k_off = (size_t)((turn % per_tile) / a.n_chunks) * n_k * 128;  // bytes to its first block in a row
  // Feature blocks are walked from a start that differs from tile to tile (by one block between neighbours,
  // when the host asks for it) and wrap around: workgroups that all read the same 128-byte column of W's rows
  // at the same time meet in few memory channels (a read-only probe of this pattern: 5.0 TB/s in step, 6.9 TB/s
  // with odd distances between the starts, less again with even ones).  Only the order of the sum changes.
  const int k_start = (tile * a.k_stagger) % n_k;
  auto blk = [&](int J) { const int p = J + k_start; return p >= n_k ? p - n_k : p; };

  // Row chunks of this workgroup: one, unless the launch was shaped for fewer rows than turn out to be computed
  // (the number of listed rows lives on the device); none if its chunk lies behind the last computed row.
  for (int row0 = ((turn % per_tile) % a.n_chunks) * ROWS; row0 < n_rows; row0 += a.n_chunks * ROWS) {
  // load slots of 8 rows x 128 bytes; lane -> (row lane/8 of the slot, chunk position lane%8, which
  // receives chunk (lane%8) ^ swizzle(row)).  hidden: wave w takes slots w, w+NW, ...; W: its own rows.
  uint32_t h_voff[NH], w_voff[4];
  int h_slot[NH];
#pragma unroll
  for (int i = 0; i < NH; ++i) {
    h_slot[i] = (w + NW * i) % (4 * NRT);
    const int r = 8 * h_slot[i] + (lane >> 3);
    h_voff[i] = ((uint32_t)lm_row_id(a, row0 + r, n_rows) * (uint32_t)d + (((lane & 7) ^ ((r >> 1) & 7)) * 8)) * 2;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 8 * i + (lane >> 3);  // row of this wave's 32
    w_voff[i] = ((uint32_t)min(v0 + r, a.V - 1) * (uint32_t)d + (((lane & 7) ^ ((r >> 1) & 7)) * 8)) * 2;
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)hbuf;
  // operand reads: row 32*rt + ln of hidden (row ln of this wave's W), logical chunk 2*c + lh
  int hrd[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) hrd[c] = ln * 128 + (((2 * c + lh) ^ ((ln >> 1) & 7)) * 16);
  const int w_rd = HB + w * (32 * 128);

  floatx16 acc[NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[rt][e] = 0.f;

  auto load_block = [&](int J, int buf) {
    const unsigned char* hb = (const unsigned char*)a.hidden + k_off + (size_t)J * 128;
    const unsigned char* wb = (const unsigned char*)a.W + k_off + (size_t)J * 128;
#pragma unroll
    for (int i = 0; i < NH; ++i) load_to_lds16(hb, h_voff[i], lds0 + buf * BB + h_slot[i] * 1024);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if constexpr (WS) load_to_lds16_stream(wb, w_voff[i], lds0 + buf * BB + HB + (4 * w + i) * 1024);
      else load_to_lds16(wb, w_voff[i], lds0 + buf * BB + HB + (4 * w + i) * 1024);
    }
  };
  constexpr int WAIT_ALL = 0x0F70;                                     // s_waitcnt vmcnt(0)
#pragma unroll
  for (int j = 0; j < NBUF - 1; ++j) load_block(blk(min(j, n_k - 1)), j);
  __builtin_amdgcn_s_waitcnt(WAIT_ALL);
  __syncthreads();

  bf16x8 hop[2][NRT], wop[2];  // operands of the current and of the next round
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt)
    hop[0][rt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(hbuf + hrd[0] + rt * (32 * 128)));
  wop[0] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(hbuf + w_rd + hrd[0]));
  // Step J (four MFMA rounds) computes from buffer J % NBUF and asks for block J + NBUF - 1, into the
  // buffer before its own.  Its one barrier stands before the last round: by then every load older than
  // the step's own and the NBUF - 3 blocks before them must have landed, which publishes block J+1; the
  // last round can therefore read the operands of step J+1's first round (no LDS latency is exposed
  // after a barrier), and no wave reads buffer J % NBUF after that barrier except from registers, so
  // step J+1 may overwrite it.  Past the end the last block is fetched again: no condition in the loop.
  constexpr int N012 = (3 * NLD) / 4;                 // loads a step issues before its barrier
  constexpr int PEND = (NBUF - 3) * NLD + N012;        // loads that may be in flight at the barrier
  constexpr int WAIT_MID = 0x0F70 | (PEND & 15) | ((PEND >> 4) << 14);
  static_assert(PEND < 64, "vmcnt is a 6-bit counter");
  int buf = 0;
  for (int J = 0; J < n_k; ++J) {
    const int buf_next = buf + 1 == NBUF ? 0 : buf + 1;
    const int buf_fill = buf == 0 ? NBUF - 1 : buf - 1;
    const unsigned char* cur = hbuf + buf * BB;
    const unsigned char* nxt = hbuf + buf_next * BB;
    const int Jn = blk(min(J + NBUF - 1, n_k - 1));
    const unsigned char* h_base = (const unsigned char*)a.hidden + k_off + (size_t)Jn * 128;
    const unsigned char* w_base = (const unsigned char*)a.W + k_off + (size_t)Jn * 128;
    const uint32_t dst = lds0 + buf_fill * BB;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (c == 3) {
        __builtin_amdgcn_s_waitcnt(WAIT_MID);
        __syncthreads();
      }
      const unsigned char* src = c < 3 ? cur + hrd[c + 1] : nxt + hrd[0];
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt)
        hop[(c + 1) & 1][rt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(src + rt * (32 * 128)));
      wop[(c + 1) & 1] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4*>(src + w_rd));
#pragma unroll
      for (int l = (c * NLD) / 4; l < ((c + 1) * NLD) / 4; ++l) {
        if (l < NH) load_to_lds16(h_base, h_voff[l], dst + h_slot[l] * 1024);
        else if constexpr (WS) load_to_lds16_stream(w_base, w_voff[l - NH], dst + HB + (4 * w + (l - NH)) * 1024);
        else load_to_lds16(w_base, w_voff[l - NH], dst + HB + (4 * w + (l - NH)) * 1024);
      }
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt)
        acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wop[c & 1], hop[c & 1][rt], acc[rt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    buf = buf_next;
  }
  __builtin_amdgcn_s_waitcnt(WAIT_ALL);  // the redundant tail loads, before LDS is reused
  __syncthreads();
  lm_epilogue<NRT, KT, NW>(a, acc, hbuf, tile, row0, n_rows, v0, w, tid);
  __syncthreads();  // the buffers are free for another row chunk
  }
}

// ------------------------------------------------------------------ merge of the parts' candidates
// One wavefront per row.  Every lane folds its share of the row's candidates into a K-entry list in
// one pass over memory; then K rounds of a wave-wide arg-max over the heads of the lists, the
// winning lane popping its head.  `emit(k, key)` is called on every lane with the k-th best key.
template <typename Emit>
SS_DEV void row_topk(const uint64_t* __restrict__ ck, int n, int K, int lane, Emit emit) {
  TopList<SS_MAX_K> top;
  top.clear();
  for (int e0 = lane; e0 < n; e0 += 256) {
    uint64_t c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) c[j] = e0 + 64 * j < n ? ck[e0 + 64 * j] : 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) top.insert(c[j]);
  }
  for (int k = 0; k < K; ++k) {
    uint64_t best = top.k[0];
    for (int off = 32; off > 0; off >>= 1) {
      const uint32_t lo = __shfl_xor((uint32_t)best, off, 64), hi = __shfl_xor((uint32_t)(best >> 32), off, 64);
      const uint64_t o = ((uint64_t)hi << 32) | lo;
      best = o > best ? o : best;
    }
    emit(k, best);
    if (best == top.k[0] && best != 0) {  // keys are unique (token ids are): this lane won, pop its head
#pragma unroll
      for (int j = 0; j + 1 < SS_MAX_K; ++j) top.k[j] = top.k[j + 1];
      top.k[SS_MAX_K - 1] = 0;
    }
  }
}

__global__ __launch_bounds__(64) void lm_head_reduce_kernel(LmArgs a) {
  const int lane = threadIdx.x;
  const int n_rows = lm_rows(a);
  if ((int)blockIdx.x >= n_rows) return;
  const int row = lm_row_id(a, blockIdx.x, n_rows);
  const int n = a.n_tiles * a.K;
  row_topk(a.cand_key + (size_t)row * n, n, a.K, lane, [&](int k, uint64_t best) {
    if (lane == 0) {
      a.idx[(size_t)row * a.K + k] = key_id(best);
      a.val[(size_t)row * a.K + k] = key_value(best);
    }
  });
}

// ------------------------------------------------------------------ fused tail: merge + verify + draft
// One workgroup of 16 wavefronts per sequence.  Only the rows the two tree steps read are merged: the
// arg-max of the T main rows (a wave per row), then, once the accepted path is known, the top-K of the
// gamma stream rows of its last node (a wave per stream).  Rows of a sequence: main row of node i at i,
// stream j of node i at T + i*gamma + (j-1).
struct TailArgs {
  const uint64_t* cand_key;  // [B*R][n_parts][K]
  int n_parts, K;
  const int32_t *tok, *parent;
  int T, gamma, max_depth, T2;
  const int32_t *tmpl_parent, *tmpl_rank;
  TemplateArg targ;
  int32_t *n_accept, *last, *bonus, *path, *out_tokens, *next_tok, *next_parent, *main_argmax;
};

__global__ __launch_bounds__(1024) void lm_tail_kernel(TailArgs t) {
  __shared__ VerifyLds vs;
  __shared__ int am[64];
  __shared__ int topk[SS_MAX_GAMMA * SS_MAX_K];
  __shared__ int dpar[64];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, b = blockIdx.x;
  const int R = t.T * (1 + t.gamma);
  const int n = t.n_parts * t.K;
  int p, my_tok;
  verify_load(tid, b, t.tok, t.parent, t.T, p, my_tok);  // in flight during the arg-max pass
  int tp, trank;
  draft_load(tid, t.tmpl_parent, t.tmpl_rank, t.targ, t.T2, tp, trank);
  for (int i = w; i < t.T; i += 16) {
    const uint64_t* ck = t.cand_key + ((size_t)b * R + i) * n;
    uint64_t best = 0;
    for (int e0 = lane; e0 < n; e0 += 512) {  // eight independent loads, then the compares
      uint64_t c[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) c[j] = e0 + 64 * j < n ? ck[e0 + 64 * j] : 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) best = c[j] > best ? c[j] : best;
    }
    for (int off = 32; off > 0; off >>= 1) {
      const uint32_t lo = __shfl_xor((uint32_t)best, off, 64), hi = __shfl_xor((uint32_t)(best >> 32), off, 64);
      const uint64_t o = ((uint64_t)hi << 32) | lo;
      best = o > best ? o : best;
    }
    if (lane == 0) {
      am[i] = key_id(best);
      if (t.main_argmax) t.main_argmax[(size_t)b * t.T + i] = key_id(best);
    }
  }
  __syncthreads();
  int node, bonus_tok;
  verify_sequence(tid, b, p, my_tok, am, 1, t.T, t.max_depth, t.n_accept, t.last, t.bonus, t.path, t.out_tokens, vs,
                  node, bonus_tok);
  if (w < t.gamma) {
    const uint64_t* ck = t.cand_key + ((size_t)b * R + t.T + (size_t)node * t.gamma + w) * n;
    row_topk(ck, n, t.K, lane, [&](int k, uint64_t best) {
      if (lane == 0) topk[w * t.K + k] = key_id(best);
    });
  }
  __syncthreads();
  draft_sequence(tid, b, tp, trank, topk, t.K, bonus_tok, t.gamma, t.T2, t.next_tok, t.next_parent, dpar);
}

// Tuning aids: a flavour (32-row tiles per workgroup, 8-wave kernel or not) that replaces the chosen one for
// the LM head or for the projections, and the stagger of the starting blocks.  Set through ss_lm_set_flavour /
// ss_lm_set_stagger; their initial values come from SS_LM_FLAVOUR / SS_LINEAR_FLAVOUR ("<row tiles>" or
// "<row tiles>w") and SS_LM_STAGGER, read once per process.
struct LmTuning {
  std::atomic<int> flavour[2];  // [LM head, projection]: row tiles | wide << 8, 0 = automatic
  std::atomic<int> stagger;     // feature blocks between neighbouring tiles' starts, -1 = automatic
  std::atomic<int> candidates_only;  // profiling aid: ss_lm_head_argmax_topk stops after the matrix kernel
};
static int flavour_code(long want, int wide) { return (want < 1 || want > (wide ? 5 : 6)) ? 0 : (int)want | (wide ? 256 : 0); }
static int flavour_from_env(const char* var) {
  const char* e = getenv(var);
  if (!e) return 0;
  char* end = nullptr;
  const long want = strtol(e, &end, 10);
  return flavour_code(want, end && *end == 'w');
}
static LmTuning& tuning() {
  static LmTuning t;
  static std::once_flag once;
  std::call_once(once, []() {
    t.flavour[0] = flavour_from_env("SS_LM_FLAVOUR");
    t.flavour[1] = flavour_from_env("SS_LINEAR_FLAVOUR");
    const char* e = getenv("SS_LM_STAGGER");
    const int v = e ? atoi(e) : -1;
    t.stagger = v < 0 ? -1 : (v > 1024 ? 1024 : v);
    t.candidates_only = 0;
  });
  return t;
}
struct LmFlavour {
  int nrt;   // 32-row tiles per workgroup
  int wide;  // 0: 4 waves, tile of 128 ids, nrt <= 6; 1: 8 waves, 256 ids, nrt <= 5; 2: 6 waves, 192 ids, nrt <= 5
             // (projections only: 22016 outputs are 115 such tiles x 2 row chunks = 230 workgroups, not 172)
};

// Log-sum-exp of a row from its tiles' (max, sum) pairs: one wavefront per row.
__global__ __launch_bounds__(64) void lm_head_lse_reduce_kernel(LmArgs a) {
  const int lane = threadIdx.x, row = blockIdx.x;
  const float2* pairs = reinterpret_cast<const float2*>(a.cand_key) + (size_t)row * a.n_tiles;
  float2 p = make_float2(-INFINITY, 0.f);
  for (int t = lane; t < a.n_tiles; t += 64) p = lse_merge(p, pairs[t]);
  for (int off = 32; off > 0; off >>= 1)
    p = lse_merge(p, make_float2(__shfl_xor(p.x, off, 64), __shfl_xor(p.y, off, 64)));
  if (lane == 0) a.lse[row] = p.x + logf(p.y);
}

template <int NRT, int KT, int WIDE>
static int launch_lm_bf16_rk(hipStream_t st, const LmArgs& a) {
  void (*kern)(LmArgs);
  size_t lds;
  int threads = 256;
  if constexpr (WIDE == 1) {
    kern = lm_head_bf16_kernel<NRT, KT, 8, 3>;
    lds = 3 * ((size_t)(32 * NRT) * 128 + 256 * 128);
    threads = 512;
  } else if constexpr (WIDE == 2) {
    kern = lm_head_bf16_kernel<NRT, KT, 6, 3>;
    lds = 3 * ((size_t)(32 * NRT) * 128 + 192 * 128);
    threads = 384;
  } else {
    kern = a.n_chunks == 1 ? lm_head_bf16_kernel<NRT, KT, 4, 4, true> : lm_head_bf16_kernel<NRT, KT, 4, 4, false>;
    lds = 4 * ((size_t)(32 * NRT) * 128 + 128 * 128);
  }
  // one attribute call per kernel instantiation (this function template has one pair of flags per <NRT, KT, WIDE>)
  static std::once_flag attr_once[2];  // [W streamed]
  static hipError_t attr_err[2] = {hipSuccess, hipSuccess};
  const int variant = (WIDE == 0 && a.n_chunks == 1) ? 1 : 0;
  std::call_once(attr_once[variant], [&]() {
    attr_err[variant] = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  });
  if (attr_err[variant] != hipSuccess)
    SS_FAIL(SS_ERR_HIP, "lm_head_bf16_kernel: hipFuncSetAttribute: %s", hipGetErrorString(attr_err[variant]));
  const dim3 grid(8 * a.n_chunks * a.n_ksplit * ceil_div(a.n_tiles, 8));
  hipLaunchKernelGGL(kern, grid, dim3(threads), lds, st, a);
  return check_launch("lm_head_bf16_kernel");
}
template <int NRT, int WIDE>
static int launch_lm_bf16_r(int KT, hipStream_t st, const LmArgs& a) {
  if constexpr (WIDE == 2) {  // six waves: the projections only
    if (KT == -2) return launch_lm_bf16_rk<NRT, -2, WIDE>(st, a);
    if (KT == 0) return launch_lm_bf16_rk<NRT, 0, WIDE>(st, a);
    SS_FAIL(SS_ERR_UNSUPPORTED, "lm_head_bf16_kernel: no six-wave kernel for epilogue %d", KT);
  } else {
    switch (KT) {
      case -2: return launch_lm_bf16_rk<NRT, -2, WIDE>(st, a);
      case -1: return launch_lm_bf16_rk<NRT, -1, WIDE>(st, a);
      case 0: return launch_lm_bf16_rk<NRT, 0, WIDE>(st, a);
      case 1: return launch_lm_bf16_rk<NRT, 1, WIDE>(st, a);
      case 4: return launch_lm_bf16_rk<NRT, 4, WIDE>(st, a);
      default: return launch_lm_bf16_rk<NRT, 8, WIDE>(st, a);
    }
  }
}
// Rows go to the workgroups in n_chunks chunks of 32*NRT rows; a.n_chunks and a.n_tiles must be set
// for the flavour (tiles of 256 ids if f.wide).
static int launch_lm_bf16(LmFlavour f, int KT, hipStream_t st, const LmArgs& args) {
  // Staggered starts when every part of W is wanted by one workgroup only (one row chunk): those launches are
  // bound by the stream of W (16..160 rows over a 262 MB W: 57..73 us in step, 45..66 us staggered).  With several
  // row chunks the chunks of a tile walk together either way and the gain is within the noise.
  LmArgs a = args;
  a.k_stagger = a.n_chunks == 1 ? 1 : 0;
  const int forced_stagger = tuning().stagger.load();
  if (forced_stagger >= 0) a.k_stagger = forced_stagger;
  if (f.wide == 2) {
    switch (f.nrt) {
      case 1: return launch_lm_bf16_r<1, 2>(KT, st, a);
      case 2: return launch_lm_bf16_r<2, 2>(KT, st, a);
      case 3: return launch_lm_bf16_r<3, 2>(KT, st, a);
      case 4: return launch_lm_bf16_r<4, 2>(KT, st, a);
      default: return launch_lm_bf16_r<5, 2>(KT, st, a);
    }
  }
  if (f.wide) {
    switch (f.nrt) {
      case 1: return launch_lm_bf16_r<1, 1>(KT, st, a);
      case 2: return launch_lm_bf16_r<2, 1>(KT, st, a);
      case 3: return launch_lm_bf16_r<3, 1>(KT, st, a);
      case 4: return launch_lm_bf16_r<4, 1>(KT, st, a);
      default: return launch_lm_bf16_r<5, 1>(KT, st, a);
    }
  }
  switch (f.nrt) {
    case 1: return launch_lm_bf16_r<1, 0>(KT, st, a);
    case 2: return launch_lm_bf16_r<2, 0>(KT, st, a);
    case 3: return launch_lm_bf16_r<3, 0>(KT, st, a);
    case 4: return launch_lm_bf16_r<4, 0>(KT, st, a);
    case 5: return launch_lm_bf16_r<5, 0>(KT, st, a);
    default: return launch_lm_bf16_r<6, 0>(KT, st, a);
  }
}

// Which MFMA kernel, how many rows per workgroup and how many row chunks.  A compute unit holds one workgroup
// (LDS) and sustains a fixed number of outstanding reads, so a launch takes about (rounds of 256 workgroups) x
// (bytes a workgroup loads) x (latency): the shape with the smallest rounds x (ids + rows) per tile wins; among
// equals the one with fewer workgroups, i.e. less traffic through the L2 in all (12288 outputs: 192 workgroups of
// 128 ids x 160 rows take 50 us, 256 workgroups of 192 ids x 96 rows 53 us).  Measured with weights that no cache holds, 320 rows: 32000 outputs ->
// 8 waves, 256 ids x 160 rows, 250 workgroups (4 waves x 128 ids would need two rounds); 22016 -> the same
// shape, 172 workgroups (projections: 6 waves, 192 ids x 160 rows, 230 workgroups, 68 us against 75); 12288 -> 4 waves, 128 ids x 160 rows, 192 workgroups (50 us; 256 ids x 64 rows in 240
// workgroups: 59 us); 4096 -> 4 waves, 128 ids x 64 rows.  Only balanced chunkings are considered (every
// chunk as many 32-row tiles as the largest needs).
static int flavour_ids(int wide) { return wide == 0 ? 128 : (wide == 1 ? 256 : 192); }
static LmFlavour lm_choose(int N, int V, LmArgs* a, bool six_waves_ok = false) {
  const int n32 = ceil_div(N < 1 ? 1 : N, 32);
  LmFlavour best{1, 0};
  long best_cost = -1, best_wgs = 0;
  for (int wide = 0; wide <= (six_waves_ok ? 2 : 1); ++wide) {
    const int ids = flavour_ids(wide), cap = wide ? 5 : 6;
    const long tiles = ceil_div(V, ids);
    for (int nrt = 1; nrt <= cap; ++nrt) {
      const int chunks = ceil_div(n32, nrt);
      if (ceil_div(n32, chunks) != nrt) continue;  // the same chunking with fewer tiles per chunk comes by itself
      const long wgs = tiles * chunks, rounds = (wgs + 255) / 256;
      const long cost = rounds * (ids + 32 * nrt);
      if (best_cost < 0 || cost < best_cost || (cost == best_cost && wgs < best_wgs)) {
        best_cost = cost;
        best_wgs = wgs;
        best = LmFlavour{nrt, wide};
      }
    }
  }
  a->n_tiles = ceil_div(V, flavour_ids(best.wide));
  a->n_chunks = ceil_div(n32, best.nrt);
  return best;
}

// Sum of the feature slices' fp32 partial products, in slice order, rounded once to bf16: four outputs per thread.
__global__ __launch_bounds__(256) void linear_ksplit_reduce_kernel(const float* __restrict__ part, uint16_t* __restrict__ y,
                                                                 size_t nv, int n_ksplit) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= nv) return;
  if (i + 4 <= nv && (nv & 3) == 0 && (((uintptr_t)part | (uintptr_t)y) & 15) == 0) {
    floatx4 sum = *reinterpret_cast<const floatx4*>(part + i);
    for (int sl = 1; sl < n_ksplit; ++sl) sum += *reinterpret_cast<const floatx4*>(part + (size_t)sl * nv + i);
    *reinterpret_cast<uintx2*>(y + i) = uintx2{pack_bf16x2(sum[0], sum[1]), pack_bf16x2(sum[2], sum[3])};
  } else {
    for (size_t j = i; j < nv && j < i + 4; ++j) {
      float sum = part[j];
      for (int sl = 1; sl < n_ksplit; ++sl) sum += part[(size_t)sl * nv + j];
      y[j] = (uint16_t)f32_to_bf16_bits(sum);
    }
  }
}

// Shape of a bf16 projection that may split the feature dimension between workgroups (the caller gave a
// workspace for the fp32 partial products).  Estimated time, by the reasoning of lm_choose: a workgroup loads
// (ids + rows) x (d / slices) x 2 bytes at about 16 KB per 0.3 us; with slices, the partial products are written
// and read back by a second kernel (5 us + their bytes at 3 TB/s).  Few outputs and many features (a layer's
// down and output maps: 4096 outputs fill 160 of 256 compute units with tiles of 128 ids x 64 rows) gain from
// four slices with tiles of 128 ids x 160 rows; maps with many outputs stay unsplit.
struct LinearPlan {
  LmFlavour f;
  int n_tiles, n_chunks, n_ksplit;
};
static LinearPlan linear_plan(int N, int d, int V) {
  const int n32 = ceil_div(N < 1 ? 1 : N, 32), blocks = d / 64;
  LinearPlan best{LmFlavour{1, 0}, 1, 1, 1};
  double best_us = -1.0;
  long best_wgs = 0;
  for (int ks = 1; ks <= 4; ks *= 2) {
    if (blocks % ks != 0 || blocks / ks < 2) continue;
    const double reduce_us = ks > 1 ? 5.0 + ((double)ks * N * V * 4 + (double)N * V * 2) / 3.0e6 : 0.0;
    for (int wide = 0; wide <= 2; ++wide) {
      const int ids = flavour_ids(wide), cap = wide ? 5 : 6;
      const long tiles = ceil_div(V, ids);
      for (int nrt = 1; nrt <= cap; ++nrt) {
        const int chunks = ceil_div(n32, nrt);
        if (ceil_div(n32, chunks) != nrt) continue;
        const long wgs = tiles * chunks * ks, rounds = (wgs + 255) / 256;
        // a cut map has to look a sixth better than the best uncut one before the second kernel is taken on
        const double us = ((double)rounds * (ids + 32 * nrt) * ((double)d / ks) * 2.0 * 0.30 / 16384.0 + reduce_us) * (ks > 1 ? 1.2 : 1.0);
        if (best_us < 0 || us < best_us - 1e-9 || (us < best_us + 1e-9 && wgs < best_wgs)) {
          best_us = us;
          best_wgs = wgs;
          best = LinearPlan{LmFlavour{nrt, wide}, (int)tiles, chunks, ks};
        }
      }
    }
  }
  return best;
}

static void lm_flavour_override(bool linear, int N, int V, LmFlavour* f, LmArgs* a) {
  const int code = tuning().flavour[linear ? 1 : 0].load();
  if (code == 0) return;
  const int want = code & 255, wide = code >> 8;
  const int n32 = ceil_div(N, 32);
  a->n_chunks = ceil_div(n32, want);
  f->nrt = ceil_div(n32, a->n_chunks);
  f->wide = wide;
  a->n_tiles = ceil_div(V, wide ? 256 : 128);
}

// Which rows a call computes: all N (rows == NULL), or the rows listed on the device; plan_rows is the number of
// rows the launch is shaped for (0 = N).
struct RowSel {
  const int32_t* rows;
  const int32_t* n;
  int plan_rows;
};
static int plan_n(const RowSel& sel, int N) { return (sel.rows && sel.plan_rows > 0 && sel.plan_rows < N) ? sel.plan_rows : N; }
static int check_sel(const char* fn, const RowSel& sel) {
  SS_REQUIRE((sel.rows == nullptr) == (sel.n == nullptr), SS_ERR_INVALID_ARG, "%s: live_rows and n_live must both be given", fn);
  SS_REQUIRE(sel.plan_rows >= 0, SS_ERR_INVALID_ARG, "%s: plan_rows=%d", fn, sel.plan_rows);
  return SS_OK;
}

// Candidate parts per row: one per vocabulary tile (64 ids in the fp32 kernel, 128 in the MFMA kernel).
static int lm_tiles(int V, int dtype) { return ceil_div(V, dtype == SS_BF16 ? 128 : 64); }

static int gemm_check(const char* fn, int N, int d, int V, int dtype);
static int lm_check(const char* fn, int N, int d, int V, int K, int dtype) {
  SS_REQUIRE(K >= 1 && K <= SS_MAX_K, SS_ERR_UNSUPPORTED, "%s: K=%d outside [1,%d]", fn, K, SS_MAX_K);
  SS_REQUIRE(K <= V || V < 1, SS_ERR_INVALID_ARG, "%s: K=%d exceeds V=%d", fn, K, V);
  return gemm_check(fn, N, d, V, dtype);
}
static int gemm_check(const char* fn, int N, int d, int V, int dtype) {
  SS_REQUIRE(N >= 0 && d >= 1 && V >= 1, SS_ERR_INVALID_ARG, "%s: N=%d d=%d V=%d", fn, N, d, V);
  SS_REQUIRE(dtype == SS_F32 || dtype == SS_BF16, SS_ERR_UNSUPPORTED, "%s: dtype %d", fn, dtype);
  SS_REQUIRE(dtype != SS_BF16 || d % 64 == 0, SS_ERR_UNSUPPORTED, "%s: bf16 path needs d %% 64 == 0 (d=%d)", fn, d);
  SS_REQUIRE(dtype != SS_BF16 || ((long)(N < 1 ? 1 : N) * d < (1L << 30) && (long)V * d < (1L << 30)), SS_ERR_UNSUPPORTED,
             "%s: hidden (%d x %d) or W (%d x %d) has 2^30 elements or more: too large for the bf16 path", fn, N, d, V, d);
  return SS_OK;
}

}  // namespace ss

extern "C" {

int ss_lm_set_flavour(int linear, int row_tiles, int wide) {
  return ss::tuning().flavour[linear ? 1 : 0].exchange(ss::flavour_code(row_tiles, wide != 0));
}

int ss_lm_set_stagger(int blocks) {
  return ss::tuning().stagger.exchange(blocks < 0 ? -1 : (blocks > 1024 ? 1024 : blocks));
}

int ss_lm_set_candidates_only(int on) { return ss::tuning().candidates_only.exchange(on ? 1 : 0); }

size_t ss_lm_head_workspace_bytes(int N, int d, int V, int K, int dtype) {
  ss::clear_error();
  if (ss::lm_check("ss_lm_head_workspace_bytes", N, d, V, K, dtype) != SS_OK) return 0;
  return (size_t)(N < 1 ? 1 : N) * ss::lm_tiles(V, dtype) * K * 8 + 512;
}

// The first kernel of a3: K candidates per (row, vocabulary tile) into the workspace.  Arguments are checked
// by the callers; fills *a for the kernel that merges the candidates.
static int lm_candidates(const char* fn, const void* hidden, const void* W, int N, int d, int V, int K, int dtype,
                         const ss::RowSel& sel, void* workspace, hipStream_t st, ss::LmArgs* out) {
  using namespace ss;
  LmArgs a;
  a.hidden = hidden; a.W = W; a.N = N; a.d = d; a.V = V; a.K = K;
  a.n_tiles = lm_tiles(V, dtype);
  a.n_chunks = 1;
  a.k_stagger = 0;
  char* ws = (char*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  a.cand_key = (uint64_t*)ws;
  a.idx = nullptr; a.val = nullptr;
  a.y = nullptr; a.lse = nullptr;
  a.live_rows = sel.rows; a.n_live = sel.n;
  a.n_ksplit = 1; a.part = nullptr;
  if (dtype == SS_F32) {
    dim3 grid(a.n_tiles, ceil_div(N, 32));
    SS_REQUIRE(grid.y <= 65535, SS_ERR_UNSUPPORTED, "%s: N too large", fn);
    hipLaunchKernelGGL(lm_head_f32_kernel<0>, grid, dim3(256), 0, st, a);
  } else {
    LmFlavour f = lm_choose(plan_n(sel, N), V, &a);
    lm_flavour_override(false, plan_n(sel, N), V, &f, &a);
    SS_REQUIRE((long)a.n_chunks * (a.n_tiles + 7) < (1L << 27), SS_ERR_UNSUPPORTED, "%s: N x V too large", fn);
    const int KT = K == 1 ? 1 : (K <= 4 ? 4 : 8);
    if (int rc = launch_lm_bf16(f, KT, st, a)) return rc;
  }
  *out = a;
  return check_launch(fn);
}

static int lm_topk_run(const char* fn, const void* hidden, const void* W, int N, int d, int V, int K, int dtype,
                       int32_t* idx, float* val, const ss::RowSel& sel, void* workspace, size_t workspace_bytes,
                       void* stream) {
  using namespace ss;
  if (int rc = lm_check(fn, N, d, V, K, dtype)) return rc;
  if (int rc = check_sel(fn, sel)) return rc;
  SS_REQUIRE(N == 0 || (hidden && W && idx && val), SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  const size_t need = ss_lm_head_workspace_bytes(N, d, V, K, dtype);
  SS_REQUIRE(N == 0 || (workspace != nullptr && workspace_bytes >= need), SS_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given",
             fn, need, workspace_bytes);
  if (N == 0) return SS_OK;
  hipStream_t st = (hipStream_t)stream;
  LmArgs a;
  if (int rc = lm_candidates(fn, hidden, W, N, d, V, K, dtype, sel, workspace, st, &a)) return rc;
  a.idx = idx; a.val = val;
  if (tuning().candidates_only.load()) return SS_OK;  // profiling aid: idx / val are not written
  hipLaunchKernelGGL(lm_head_reduce_kernel, dim3(N), dim3(64), 0, st, a);
  return check_launch(fn);
}

int ss_lm_head_argmax_topk(const void* hidden, const void* W, int N, int d, int V, int K, int dtype, int32_t* idx,
                           float* val, void* workspace, size_t workspace_bytes, void* stream) {
  ss::clear_error();
  return lm_topk_run("ss_lm_head_argmax_topk", hidden, W, N, d, V, K, dtype, idx, val, ss::RowSel{nullptr, nullptr, 0},
                     workspace, workspace_bytes, stream);
}

int ss_lm_head_argmax_topk_live(const void* hidden, const void* W, int N, int d, int V, int K, int dtype, int32_t* idx,
                                float* val, const int32_t* live_rows, const int32_t* n_live, int plan_rows,
                                void* workspace, size_t workspace_bytes, void* stream) {
  ss::clear_error();
  SS_REQUIRE(N == 0 || (live_rows && n_live), SS_ERR_INVALID_ARG, "ss_lm_head_argmax_topk_live: NULL row list");
  return lm_topk_run("ss_lm_head_argmax_topk_live", hidden, W, N, d, V, K, dtype, idx, val,
                     ss::RowSel{live_rows, n_live, plan_rows}, workspace, workspace_bytes, stream);
}

static int lm_tail_run(const char* fn, const void* hidden, const void* W, int d, int V, int K, int dtype, const int32_t* tok,
                       const int32_t* parent, int B, int T, int gamma, int max_depth, const int32_t* tmpl_parent,
                       const int32_t* tmpl_rank, const int32_t* branching, int T2, int32_t* n_accept,
                       int32_t* last, int32_t* bonus, int32_t* path, int32_t* out_tokens, int32_t* next_tok,
                       int32_t* next_parent, int32_t* main_argmax, const ss::RowSel& sel, void* workspace,
                       size_t workspace_bytes, void* stream) {
  using namespace ss;
  if (int rc = check_sel(fn, sel)) return rc;
  SS_REQUIRE(B >= 0 && B <= (1 << 20), SS_ERR_INVALID_ARG, "%s: B=%d", fn, B);
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T && T2 >= 1 && T2 <= SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: T=%d or T2=%d outside [1,%d]",
             fn, T, T2, SS_MAX_T);
  SS_REQUIRE(gamma >= 0 && gamma <= SS_MAX_GAMMA, SS_ERR_UNSUPPORTED, "%s: gamma=%d outside [0,%d]", fn, gamma,
             SS_MAX_GAMMA);
  SS_REQUIRE(max_depth >= 0 && max_depth < SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: max_depth=%d outside [0,%d)", fn, max_depth,
             SS_MAX_T);
  const long rows = (long)B * T * (1 + gamma);
  SS_REQUIRE(rows < (1L << 30), SS_ERR_UNSUPPORTED, "%s: %ld rows", fn, rows);
  const int N = (int)rows;
  if (int rc = lm_check(fn, N, d, V, K, dtype)) return rc;
  SS_REQUIRE(B == 0 || (hidden && W && tok && parent && n_accept && last && bonus && path && out_tokens && next_tok),
             SS_ERR_INVALID_ARG, "%s: NULL argument", fn);
  SS_REQUIRE((tmpl_parent == nullptr) == (tmpl_rank == nullptr), SS_ERR_INVALID_ARG,
             "%s: tmpl_parent and tmpl_rank must both be given or both be NULL", fn);
  TailArgs t;
  if (!tmpl_parent) {
    if (int rc = draft_template_from_branching(fn, branching, gamma, K, T2, &t.targ)) return rc;
  } else {
    for (int i = 0; i < SS_MAX_T; ++i) t.targ.parent[i] = t.targ.rank[i] = 0;
  }
  const size_t need = ss_lm_head_workspace_bytes(N, d, V, K, dtype);
  SS_REQUIRE(B == 0 || (workspace != nullptr && workspace_bytes >= need), SS_ERR_WORKSPACE,
             "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace_bytes);
  if (B == 0) return SS_OK;
  hipStream_t st = (hipStream_t)stream;
  LmArgs a;
  if (int rc = lm_candidates(fn, hidden, W, N, d, V, K, dtype, sel, workspace, st, &a)) return rc;
  t.cand_key = a.cand_key; t.n_parts = a.n_tiles; t.K = K;
  t.tok = tok; t.parent = parent;
  t.T = T; t.gamma = gamma; t.max_depth = max_depth; t.T2 = T2;
  t.tmpl_parent = tmpl_parent; t.tmpl_rank = tmpl_rank;
  t.n_accept = n_accept; t.last = last; t.bonus = bonus; t.path = path; t.out_tokens = out_tokens;
  t.next_tok = next_tok; t.next_parent = next_parent; t.main_argmax = main_argmax;
  hipLaunchKernelGGL(lm_tail_kernel, dim3(B), dim3(1024), 0, st, t);
  return check_launch(fn);
}

int ss_lm_head_verify_draft(const void* hidden, const void* W, int d, int V, int K, int dtype, const int32_t* tok,
                            const int32_t* parent, int B, int T, int gamma, int max_depth, const int32_t* tmpl_parent,
                            const int32_t* tmpl_rank, const int32_t* branching, int T2, int32_t* n_accept,
                            int32_t* last, int32_t* bonus, int32_t* path, int32_t* out_tokens, int32_t* next_tok,
                            int32_t* next_parent, int32_t* main_argmax, void* workspace, size_t workspace_bytes,
                            void* stream) {
  ss::clear_error();
  return lm_tail_run("ss_lm_head_verify_draft", hidden, W, d, V, K, dtype, tok, parent, B, T, gamma, max_depth, tmpl_parent,
                     tmpl_rank, branching, T2, n_accept, last, bonus, path, out_tokens, next_tok, next_parent, main_argmax,
                     ss::RowSel{nullptr, nullptr, 0}, workspace, workspace_bytes, stream);
}

int ss_lm_head_verify_draft_live(const void* hidden, const void* W, int d, int V, int K, int dtype, const int32_t* tok,
                                 const int32_t* parent, int B, int T, int gamma, int max_depth,
                                 const int32_t* tmpl_parent, const int32_t* tmpl_rank, const int32_t* branching, int T2,
                                 int32_t* n_accept, int32_t* last, int32_t* bonus, int32_t* path, int32_t* out_tokens,
                                 int32_t* next_tok, int32_t* next_parent, int32_t* main_argmax,
                                 const int32_t* live_rows, const int32_t* n_live, int plan_rows, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  ss::clear_error();
  SS_REQUIRE(B == 0 || (live_rows && n_live), SS_ERR_INVALID_ARG, "ss_lm_head_verify_draft_live: NULL row list");
  return lm_tail_run("ss_lm_head_verify_draft_live", hidden, W, d, V, K, dtype, tok, parent, B, T, gamma, max_depth,
                     tmpl_parent, tmpl_rank, branching, T2, n_accept, last, bonus, path, out_tokens, next_tok, next_parent,
                     main_argmax, ss::RowSel{live_rows, n_live, plan_rows}, workspace, workspace_bytes, stream);
}

int ss_lm_head_logsumexp(const void* hidden, const void* W, int N, int d, int V, int dtype, float* lse,
                         void* workspace, size_t workspace_bytes, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_lm_head_logsumexp";
  if (int rc = gemm_check(fn, N, d, V, dtype)) return rc;
  SS_REQUIRE(N == 0 || (hidden && W && lse), SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  const size_t need = ss_lm_head_workspace_bytes(N, d, V, 1, dtype);
  SS_REQUIRE(N == 0 || (workspace != nullptr && workspace_bytes >= need), SS_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given",
             fn, need, workspace_bytes);
  if (N == 0) return SS_OK;
  LmArgs a;
  a.hidden = hidden; a.W = W; a.N = N; a.d = d; a.V = V; a.K = 0;
  a.n_tiles = lm_tiles(V, dtype);
  a.n_chunks = 1;
  a.k_stagger = 0;
  a.cand_key = (uint64_t*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  a.idx = nullptr; a.val = nullptr; a.y = nullptr;
  a.lse = lse;
  a.live_rows = nullptr; a.n_live = nullptr;
  a.n_ksplit = 1; a.part = nullptr;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == SS_F32) {
    dim3 grid(a.n_tiles, ceil_div(N, 32));
    SS_REQUIRE(grid.y <= 65535, SS_ERR_UNSUPPORTED, "%s: N too large", fn);
    hipLaunchKernelGGL(lm_head_f32_kernel<2>, grid, dim3(256), 0, st, a);
  } else {
    LmFlavour f = lm_choose(N, V, &a);
    lm_flavour_override(false, N, V, &f, &a);
    SS_REQUIRE((long)a.n_chunks * (a.n_tiles + 7) < (1L << 27), SS_ERR_UNSUPPORTED, "%s: N x V too large", fn);
    if (int rc = launch_lm_bf16(f, -1, st, a)) return rc;
  }
  if (int rc = check_launch(fn)) return rc;
  hipLaunchKernelGGL(lm_head_lse_reduce_kernel, dim3(N), dim3(64), 0, st, a);
  return check_launch(fn);
}

static int linear_run(const char* fn, const void* x, const void* W, int N, int d, int V, int dtype, void* y,
                      const ss::RowSel& sel, void* stream) {
  using namespace ss;
  if (int rc = check_sel(fn, sel)) return rc;
  if (int rc = gemm_check(fn, N, d, V, dtype)) return rc;
  SS_REQUIRE(N == 0 || (x && W && y), SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  SS_REQUIRE((long)(N < 1 ? 1 : N) * V < (1L << 31), SS_ERR_UNSUPPORTED, "%s: y (%d x %d) has 2^31 elements or more", fn, N, V);
  if (N == 0) return SS_OK;
  LmArgs a;
  a.hidden = x; a.W = W; a.N = N; a.d = d; a.V = V; a.K = 0;
  a.n_tiles = lm_tiles(V, dtype);
  a.n_chunks = 1;
  a.k_stagger = 0;
  a.cand_key = nullptr; a.idx = nullptr; a.val = nullptr; a.lse = nullptr;
  a.live_rows = sel.rows; a.n_live = sel.n;
  a.n_ksplit = 1; a.part = nullptr;
  a.y = y;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == SS_F32) {
    dim3 grid(a.n_tiles, ceil_div(N, 32));
    SS_REQUIRE(grid.y <= 65535, SS_ERR_UNSUPPORTED, "%s: N too large", fn);
    hipLaunchKernelGGL(lm_head_f32_kernel<1>, grid, dim3(256), 0, st, a);
  } else {
    LmFlavour f = lm_choose(plan_n(sel, N), V, &a, true);
    lm_flavour_override(true, plan_n(sel, N), V, &f, &a);
    SS_REQUIRE((long)a.n_chunks * (a.n_tiles + 7) < (1L << 27), SS_ERR_UNSUPPORTED, "%s: N x V too large", fn);
    if (int rc = launch_lm_bf16(f, 0, st, a)) return rc;
  }
  return check_launch(fn);
}


int ss_linear_rows(const void* x, const void* W, int N, int d, int V, int dtype, void* y, void* stream) {
  ss::clear_error();
  return linear_run("ss_linear_rows", x, W, N, d, V, dtype, y, ss::RowSel{nullptr, nullptr, 0}, stream);
}

int ss_linear_rows_live(const void* x, const void* W, int N, int d, int V, int dtype, void* y, const int32_t* live_rows,
                        const int32_t* n_live, int plan_rows, void* stream) {
  ss::clear_error();
  SS_REQUIRE(N == 0 || (live_rows && n_live), SS_ERR_INVALID_ARG, "ss_linear_rows_live: NULL row list");
  return linear_run("ss_linear_rows_live", x, W, N, d, V, dtype, y, ss::RowSel{live_rows, n_live, plan_rows}, stream);
}

size_t ss_linear_rows_workspace_bytes(int N, int d, int V, int dtype) {
  ss::clear_error();
  if (ss::gemm_check("ss_linear_rows_workspace_bytes", N, d, V, dtype) != SS_OK) return 0;
  if (dtype != SS_BF16 || N == 0) return 256;
  const ss::LinearPlan p = ss::linear_plan(N, d, V);
  return p.n_ksplit > 1 ? (size_t)p.n_ksplit * N * V * sizeof(float) + 256 : 256;
}

int ss_linear_rows_splits(int N, int d, int V, int dtype) {
  ss::clear_error();
  if (ss::gemm_check("ss_linear_rows_splits", N, d, V, dtype) != SS_OK) return 0;
  return (dtype == SS_BF16 && N > 0) ? ss::linear_plan(N, d, V).n_ksplit : 1;
}

int ss_linear_rows_ws(const void* x, const void* W, int N, int d, int V, int dtype, void* y, void* workspace,
                      size_t workspace_bytes, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_linear_rows_ws";
  if (int rc = gemm_check(fn, N, d, V, dtype)) return rc;
  const LinearPlan p = (dtype == SS_BF16 && N > 0) ? linear_plan(N, d, V) : LinearPlan{LmFlavour{1, 0}, 1, 1, 1};
  if (p.n_ksplit == 1) return linear_run(fn, x, W, N, d, V, dtype, y, RowSel{nullptr, nullptr, 0}, stream);
  SS_REQUIRE(x && W && y, SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  SS_REQUIRE((long)N * V < (1L << 31), SS_ERR_UNSUPPORTED, "%s: y (%d x %d) has 2^31 elements or more", fn, N, V);
  const size_t need = (size_t)p.n_ksplit * N * V * sizeof(float) + 256;
  SS_REQUIRE(workspace != nullptr && workspace_bytes >= need, SS_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn,
             need, workspace_bytes);
  LmArgs a;
  a.hidden = x; a.W = W; a.N = N; a.d = d; a.V = V; a.K = 0;
  a.n_tiles = p.n_tiles; a.n_chunks = p.n_chunks;
  a.k_stagger = 0;
  a.cand_key = nullptr; a.idx = nullptr; a.val = nullptr; a.lse = nullptr; a.y = nullptr;
  a.live_rows = nullptr; a.n_live = nullptr;
  a.n_ksplit = p.n_ksplit;
  a.part = (float*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  SS_REQUIRE((long)a.n_chunks * a.n_ksplit * (a.n_tiles + 7) < (1L << 27), SS_ERR_UNSUPPORTED, "%s: N x V too large", fn);
  hipStream_t st = (hipStream_t)stream;
  if (int rc = launch_lm_bf16(p.f, -2, st, a)) return rc;
  const size_t nv = (size_t)N * V;
  hipLaunchKernelGGL(linear_ksplit_reduce_kernel, dim3((unsigned)((nv / 4 + 256) / 256)), dim3(256), 0, st, a.part, (uint16_t*)y, nv,
                     a.n_ksplit);
  return check_launch(fn);
}

}  // extern "C"
