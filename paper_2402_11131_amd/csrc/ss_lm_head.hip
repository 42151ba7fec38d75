// a3: LM head with fused arg-max / top-K (Sec. 3.2.1, 3.2.2).  logits = hidden . W^T
// are produced tile by tile in registers and reduced to K candidates per (row,
// vocabulary tile) in the same kernel; a second, tiny kernel merges the
// candidates of all tiles.  The logits themselves never reach memory.
//
// Order everywhere: larger logit first, equal logits -> lower token id first.
#include <limits.h>
#include <math.h>

#include "ss_common.h"

namespace ss {

struct LmArgs {
  const void* hidden;  // [N,d]
  const void* W;       // [V,d]
  int N, d, V, K;
  int n_tiles;         // vocabulary tiles
  float* cand_val;     // [N, n_tiles, K]
  int32_t* cand_idx;   // [N, n_tiles, K]
  int32_t* idx;        // [N,K]
  float* val;          // [N,K]
};

SS_DEV bool cand_better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }
SS_DEV bool cand_after(float v, int i, float pv, int pi) { return v < pv || (v == pv && i > pi); }

// ------------------------------------------------------------------ fp32 kernel (small problems)
//
// Workgroup tile 32 rows x 64 vocabulary columns, feature chunks of 32 through
// LDS; thread (wave w, lane c) accumulates rows w, w+4, ... of column c.
__global__ __launch_bounds__(256) void lm_head_f32_kernel(LmArgs a) {
  constexpr int BM = 32, BN = 64, BK = 32;
  __shared__ float As[BM][BK + 1];
  __shared__ float Ws[BN][BK + 1];
  __shared__ float Z[BM][BN + 1];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int v0 = blockIdx.x * BN, r0 = blockIdx.y * BM;
  const float* hidden = (const float*)a.hidden;
  const float* W = (const float*)a.W;
  float acc[BM / 4];
#pragma unroll
  for (int i = 0; i < BM / 4; ++i) acc[i] = 0.f;
  for (int k0 = 0; k0 < a.d; k0 += BK) {
    __syncthreads();
    for (int e = tid; e < BM * BK; e += 256) {
      const int r = e / BK, kk = e % BK;
      As[r][kk] = (r0 + r < a.N && k0 + kk < a.d) ? hidden[(size_t)(r0 + r) * a.d + k0 + kk] : 0.f;
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
#pragma unroll
  for (int i = 0; i < BM / 4; ++i) Z[w + 4 * i][lane] = acc[i];
  __syncthreads();
  // wave w selects for rows w, w+4, ...: K rounds of a wave-wide arg-max over the 64 columns
  for (int rr = w; rr < BM; rr += 4) {
    const int row = r0 + rr;
    if (row >= a.N) break;
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
        a.cand_val[o] = bv;
        a.cand_idx[o] = bi;
      }
      pv = bv;
      pi = bi;
    }
  }
}

// ------------------------------------------------------------------ bf16 MFMA kernel
//
// Workgroup = 4 waves; tile = (64*MT rows) x 128 vocabulary columns; wave w owns
// rows [16*MT*w, 16*MT*(w+1)) and all 128 columns, so the W tile is shared by the
// waves (through LDS, 16-byte chunks XOR-swizzled against bank conflicts) while
// each wave streams its own rows of `hidden` straight into MFMA A operands.
// With N <= 320 a workgroup covers all rows: W is read from HBM exactly once.
// v_mfma_f32_16x16x32_bf16: A = 16 rows x 32 features, B = 32 features x 16
// columns; inside a 64-feature stage, step s and lane group g use the 8-feature
// chunk 4*s + g for both operands.
template <int MT>
__global__ __launch_bounds__(256, 1) void lm_head_bf16_kernel(LmArgs a) {
  constexpr int BN = 128, BK = 64, NT = BN / 16, NS = 3;
  __shared__ __attribute__((aligned(16))) uint16_t Ws[NS][BN * BK];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, lq = lane & 15, lg = lane >> 4;
  const int v0 = blockIdx.x * BN;
  const int row0 = blockIdx.y * (64 * MT) + w * (16 * MT);
  const uint16_t* hidden = (const uint16_t*)a.hidden;
  const uint16_t* W = (const uint16_t*)a.W;
  const int d = a.d, n_k = d / BK;

  // W tile loader: 4 passes, thread -> (row = tid/8 + 32*pass, 16-byte chunk tid%8)
  const uint16_t* wsrc[4];
  int wdst[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int vr = (tid >> 3) + 32 * p, ch = tid & 7;
    wsrc[p] = W + (size_t)min(v0 + vr, a.V - 1) * d + ch * 8;
    wdst[p] = vr * BK + ((ch ^ (vr & 7)) * 8);
  }
  // A rows of this wave (clamped; rows >= N are computed and dropped)
  const uint16_t* asrc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) asrc[mt] = hidden + (size_t)min(row0 + 16 * mt + lq, a.N - 1) * d + lg * 8;

  typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 v8bf;
  floatx4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};

  uintx4 wg[2][4];     // W tiles in flight: loaded two stages ahead of their use
  uintx4 an[MT][2];    // next stage's A operands
  uintx4 ac[MT][2];    // current stage's A operands

  auto gload_w = [&](int kt, uintx4 (&dst)[4]) {
#pragma unroll
    for (int p = 0; p < 4; ++p) dst[p] = *reinterpret_cast<const uintx4*>(wsrc[p] + (size_t)kt * BK);
  };
  auto store_w = [&](int stage, const uintx4 (&src)[4]) {
#pragma unroll
    for (int p = 0; p < 4; ++p) *reinterpret_cast<uintx4*>(&Ws[stage][wdst[p]]) = src[p];
  };
  auto gload_a = [&](int kt, uintx4 (&dst)[MT][2]) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
        dst[mt][s2] = *reinterpret_cast<const uintx4*>(asrc[mt] + (size_t)kt * BK + 32 * s2);
  };

  // prologue: stage 0 in LDS, stage 1 in registers
  gload_w(0, wg[0]);
  if (n_k > 1) gload_w(1, wg[1]);
  gload_a(0, ac);
  store_w(0, wg[0]);
  __syncthreads();

  for (int kt = 0; kt < n_k; ++kt) {
    const int stage = kt % NS;
    // wg[kt&1] is free (its tile went to LDS at the end of the last iteration): start W(kt+2).
    // W(kt+1), in the other half, is stored after this stage's MFMAs, two iterations after its load.
    if (kt + 2 < n_k) {
      if (kt & 1) gload_w(kt + 2, wg[1]);
      else gload_w(kt + 2, wg[0]);
    }
    if (kt + 1 < n_k) gload_a(kt + 1, an);
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      v8bf bop[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        bop[nt] = __builtin_bit_cast(
            v8bf, *reinterpret_cast<const uintx4*>(&Ws[stage][(16 * nt + lq) * BK + (((4 * s2 + lg) ^ (lq & 7)) * 8)]));
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const v8bf aop = __builtin_bit_cast(v8bf, ac[mt][s2]);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bop[nt], acc[mt][nt], 0, 0, 0);
      }
    }
    if (kt + 1 < n_k) {
      if (kt & 1) store_w((kt + 1) % NS, wg[0]);
      else store_w((kt + 1) % NS, wg[1]);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      ac[mt][0] = an[mt][0];
      ac[mt][1] = an[mt][1];
    }
    __syncthreads();
  }

  // epilogue: acc[mt][nt][i] is the logit of row row0+16*mt+4*lg+i, column v0+16*nt+lq.
  // K rounds per row: lane-local best that comes after the previous winner, then a
  // butterfly over the 16 lanes that share the row.
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = row0 + 16 * mt + 4 * lg + i;
      float pv = INFINITY;
      int pi = -1;
      for (int k = 0; k < a.K; ++k) {
        float bv = -INFINITY;
        int bi = INT_MAX;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const float v = acc[mt][nt][i];
          const int col = v0 + 16 * nt + lq;
          if (col < a.V && cand_after(v, col, pv, pi) && v > bv) {
            bv = v;
            bi = col;
          }
        }
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
          const float ov = __shfl_xor(bv, off, 64);
          const int oi = __shfl_xor(bi, off, 64);
          if (cand_better(ov, oi, bv, bi)) {
            bv = ov;
            bi = oi;
          }
        }
        if (lq == 0 && row < a.N) {
          const size_t o = ((size_t)row * a.n_tiles + blockIdx.x) * a.K + k;
          a.cand_val[o] = bv;
          a.cand_idx[o] = bi;
        }
        pv = bv;
        pi = bi;
      }
    }
  }
}

// ------------------------------------------------------------------ merge of the tiles' candidates
// One wavefront per row; K rounds of "best candidate that comes after the previous winner".
__global__ __launch_bounds__(256) void lm_head_reduce_kernel(LmArgs a) {
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + w;
  if (row >= a.N) return;
  const int n = a.n_tiles * a.K;
  const float* cv = a.cand_val + (size_t)row * n;
  const int32_t* ci = a.cand_idx + (size_t)row * n;
  float pv = INFINITY;
  int pi = -1;
  for (int k = 0; k < a.K; ++k) {
    float bv = -INFINITY;
    int bi = INT_MAX;
    for (int e = lane; e < n; e += 64) {
      const float v = cv[e];
      const int i = ci[e];
      if (cand_after(v, i, pv, pi) && cand_better(v, i, bv, bi)) {
        bv = v;
        bi = i;
      }
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
      a.idx[(size_t)row * a.K + k] = bi;
      a.val[(size_t)row * a.K + k] = bv;
    }
    pv = bv;
    pi = bi;
  }
}

static int lm_tiles(int V, int dtype) { return ceil_div(V, dtype == SS_BF16 ? 128 : 64); }

static int lm_check(const char* fn, int N, int d, int V, int K, int dtype) {
  SS_REQUIRE(N >= 0 && d >= 1 && V >= 1, SS_ERR_INVALID_ARG, "%s: N=%d d=%d V=%d", fn, N, d, V);
  SS_REQUIRE(K >= 1 && K <= SS_MAX_K, SS_ERR_UNSUPPORTED, "%s: K=%d outside [1,%d]", fn, K, SS_MAX_K);
  SS_REQUIRE(K <= V, SS_ERR_INVALID_ARG, "%s: K=%d exceeds V=%d", fn, K, V);
  SS_REQUIRE(dtype == SS_F32 || dtype == SS_BF16, SS_ERR_UNSUPPORTED, "%s: dtype %d", fn, dtype);
  SS_REQUIRE(dtype != SS_BF16 || d % 64 == 0, SS_ERR_UNSUPPORTED, "%s: bf16 path needs d %% 64 == 0 (d=%d)", fn, d);
  return SS_OK;
}

}  // namespace ss

extern "C" {

size_t ss_lm_head_workspace_bytes(int N, int d, int V, int K, int dtype) {
  ss::clear_error();
  if (ss::lm_check("ss_lm_head_workspace_bytes", N, d, V, K, dtype) != SS_OK) return 0;
  return (size_t)(N < 1 ? 1 : N) * ss::lm_tiles(V, dtype) * K * 8 + 512;
}

int ss_lm_head_argmax_topk(const void* hidden, const void* W, int N, int d, int V, int K, int dtype, int32_t* idx,
                           float* val, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_lm_head_argmax_topk";
  if (int rc = lm_check(fn, N, d, V, K, dtype)) return rc;
  SS_REQUIRE(N == 0 || (hidden && W && idx && val), SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  const size_t need = ss_lm_head_workspace_bytes(N, d, V, K, dtype);
  SS_REQUIRE(N == 0 || (workspace != nullptr && workspace_bytes >= need), SS_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given",
             fn, need, workspace_bytes);
  if (N == 0) return SS_OK;
  LmArgs a;
  a.hidden = hidden; a.W = W; a.N = N; a.d = d; a.V = V; a.K = K;
  a.n_tiles = lm_tiles(V, dtype);
  char* ws = (char*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  a.cand_val = (float*)ws;
  a.cand_idx = (int32_t*)(ws + (size_t)N * a.n_tiles * K * 4);
  a.idx = idx; a.val = val;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == SS_F32) {
    dim3 grid(a.n_tiles, ceil_div(N, 32));
    SS_REQUIRE(grid.y <= 65535, SS_ERR_UNSUPPORTED, "%s: N too large", fn);
    hipLaunchKernelGGL(lm_head_f32_kernel, grid, dim3(256), 0, st, a);
  } else {
    int MT = ceil_div(N, 64);
    if (MT > 5) MT = 5;
    dim3 grid(a.n_tiles, ceil_div(N, 64 * MT));
    SS_REQUIRE(grid.y <= 65535, SS_ERR_UNSUPPORTED, "%s: N too large", fn);
    switch (MT) {
      case 1: hipLaunchKernelGGL(lm_head_bf16_kernel<1>, grid, dim3(256), 0, st, a); break;
      case 2: hipLaunchKernelGGL(lm_head_bf16_kernel<2>, grid, dim3(256), 0, st, a); break;
      case 3: hipLaunchKernelGGL(lm_head_bf16_kernel<3>, grid, dim3(256), 0, st, a); break;
      case 4: hipLaunchKernelGGL(lm_head_bf16_kernel<4>, grid, dim3(256), 0, st, a); break;
      default: hipLaunchKernelGGL(lm_head_bf16_kernel<5>, grid, dim3(256), 0, st, a); break;
    }
  }
  if (int rc = check_launch(fn)) return rc;
  hipLaunchKernelGGL(lm_head_reduce_kernel, dim3(ceil_div(N, 4)), dim3(256), 0, st, a);
  return check_launch(fn);
}

}  // extern "C"
