// Shared host/device helpers of libss (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "ss.h"

namespace ss {

// ---------------------------------------------------------------- errors (host)
void set_error(const char* fmt, ...);
void clear_error();

#define SS_FAIL(code, ...)        \
  do {                            \
    ::ss::set_error(__VA_ARGS__); \
    return (code);                \
  } while (0)

#define SS_REQUIRE(cond, code, ...)        \
  do {                                     \
    if (!(cond)) SS_FAIL(code, __VA_ARGS__); \
  } while (0)

// Checks the launch that was just issued.
inline int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) SS_FAIL(SS_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return SS_OK;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------- vector types
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t uintx4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t uintx2;

// ---------------------------------------------------------------- device helpers
#define SS_DEV __device__ __forceinline__

// fp32 -> bf16 bits, round to nearest even (inputs are finite here).
SS_DEV uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
SS_DEV uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}
SS_DEV float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// One step of merging per-split attention results (both the merge kernel and the in-kernel merge use it, so
// that they agree bit for bit): acc <- acc*keep + v*w with the roundings fixed.
SS_DEV floatx4 merge_step(floatx4 acc, float keep, floatx4 v, float w) {
  floatx4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = __builtin_fmaf(v[i], w, acc[i] * keep);
  return r;
}

// Node 0 is the root; for i > 0 a parent outside [0,i) counts as 0 (documented clamp).
SS_DEV int clamp_parent(int p, int i) { return (i == 0) ? -1 : ((p < 0 || p >= i) ? 0 : p); }

// Tree row r of a sequence with T nodes and gamma streams -> (node, stream); stream 0 = main row.
SS_DEV void row_split(int r, int T, int gamma, int& node, int& strm) {
  if (r < T) {
    node = r;
    strm = 0;
  } else {
    node = (r - T) / gamma;
    strm = (r - T) % gamma + 1;
  }
}

// What one query row needs to decide which of the step's own keys it may attend
// (Eq. 1 / Eq. 2 with the tree mask): main key c < T is visible iff bit c of anc;
// stream key c >= T is visible iff lo <= c < hi.
struct RowVis {
  uint64_t anc;
  int lo, hi;
};
// Both alternatives are evaluated and then selected (no control flow per score).
SS_DEV bool row_sees(const RowVis& v, int c, int T) {
  const bool as_main = ((v.anc >> (c & 63)) & 1ull) != 0;
  const bool as_stream = (c >= v.lo) & (c < v.hi);
  return (c < T) ? as_main : as_stream;
}
SS_DEV RowVis make_row_vis(int r, int T, int gamma, const uint64_t* anc_of_node, bool exclude_self) {
  int node, strm;
  row_split(r, T, gamma, node, strm);
  RowVis v;
  v.anc = anc_of_node[node];
  v.lo = T + node * gamma;
  v.hi = v.lo + (strm == 0 ? 0 : (exclude_self ? strm - 1 : strm));
  return v;
}

// Ancestor-or-self bit sets of all T <= 64 nodes into anc_out[T] (LDS), computed
// by the first T threads of the block, each walking up from its node.  par_lds[T]
// must hold the clamped parents.  Callers synchronise before and after.
SS_DEV void compute_anc(const int* par_lds, int T, uint64_t* anc_out, int tid) {
  if (tid < T) {
    uint64_t bits = 0;
    int n = tid;
    for (int step = 0; step < 64 && n >= 0; ++step) {
      bits |= 1ull << n;
      n = par_lds[n];
    }
    anc_out[tid] = bits;
  }
}

}  // namespace ss
