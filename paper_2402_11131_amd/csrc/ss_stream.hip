// n4: stream insertion (Eq. 3).  The rows of a step enter the first multi-stream layer as: main row of
// node i = M_i, stream j of node i = f(M_i) + P_j.  Elementwise and tiny (B*R*d elements): one workgroup
// per output row, 16-byte pieces where the row length allows.  Sums are formed in fp32 and rounded once.
#include <math.h>

#include "ss_common.h"

namespace ss {

struct StreamArgs {
  const void* M;   // [B,T,d]
  const void* fM;  // [B,T,d] or NULL (identity)
  const void* P;   // [gamma,d]
  void* X;         // [B,R,d]
  int B, T, gamma, d;
};

template <bool BF16>
__global__ __launch_bounds__(256) void stream_insert_kernel(StreamArgs a) {
  constexpr int ES = BF16 ? 2 : 4;   // bytes per element
  constexpr int PER = 16 / ES;       // elements per 16-byte piece
  const int R = a.T * (1 + a.gamma);
  const int b = blockIdx.x / R, r = blockIdx.x % R;
  int node, strm;
  row_split(r, a.T, a.gamma, node, strm);
  const size_t src_row = ((size_t)b * a.T + node) * a.d;
  const unsigned char* m = (const unsigned char*)(strm == 0 || a.fM == nullptr ? a.M : a.fM) + src_row * ES;
  const unsigned char* p = (const unsigned char*)a.P + (size_t)(strm > 0 ? strm - 1 : 0) * a.d * ES;
  unsigned char* x = (unsigned char*)a.X + ((size_t)b * R + r) * a.d * ES;
  const bool vec = (a.d % PER) == 0 && ((((uintptr_t)a.M | (uintptr_t)a.fM | (uintptr_t)a.P | (uintptr_t)a.X) & 15) == 0);
  if (vec) {
    for (int c = threadIdx.x; c < a.d / PER; c += 256) {
      uintx4 mv = *reinterpret_cast<const uintx4*>(m + (size_t)c * 16);
      if (strm > 0) {
        const uintx4 pv = *reinterpret_cast<const uintx4*>(p + (size_t)c * 16);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if constexpr (BF16) {
            const float lo = bf16_bits_to_f32(mv[q] & 0xffffu) + bf16_bits_to_f32(pv[q] & 0xffffu);
            const float hi = bf16_bits_to_f32(mv[q] >> 16) + bf16_bits_to_f32(pv[q] >> 16);
            mv[q] = pack_bf16x2(lo, hi);
          } else {
            mv[q] = __float_as_uint(__uint_as_float(mv[q]) + __uint_as_float(pv[q]));
          }
        }
      }
      *reinterpret_cast<uintx4*>(x + (size_t)c * 16) = mv;
    }
  } else {
    for (int e = threadIdx.x; e < a.d; e += 256) {
      if constexpr (BF16) {
        const uint16_t mb = ((const uint16_t*)m)[e];
        ((uint16_t*)x)[e] = strm == 0 ? mb
                                      : (uint16_t)f32_to_bf16_bits(bf16_bits_to_f32(mb) + bf16_bits_to_f32(((const uint16_t*)p)[e]));
      } else {
        const float mf = ((const float*)m)[e];
        ((float*)x)[e] = strm == 0 ? mf : mf + ((const float*)p)[e];
      }
    }
  }
}

// Eq. 3 followed by a dense map, by linearity: (f(M_i) + P_j).W^T = f(M_i).W^T + P_j.W^T, so the map is applied
// to the B*T main-stream states (and to f(M) if it is not the identity) and to the gamma embeddings only, 1+gamma
// times fewer rows than the step has, and the step's rows are put together from the results.  pack_rows_kernel
// gathers [M; f(M); P] into one row block for a single pass over W; expand_rows_kernel writes
//   Y[b, i] = Z[b*T + i],   Y[b, T + i*gamma + j-1] = Zf[b*T + i] + Zp[j-1]   (sum in fp32, rounded once).
struct PackArgs {
  const void *M, *fM, *P;
  void* out;   // [2*BT or BT, then gamma][d]
  int BT, gamma, d;
};
template <bool BF16>
__global__ __launch_bounds__(256) void pack_rows_kernel(PackArgs a) {
  constexpr int ES = BF16 ? 2 : 4;
  const int n = blockIdx.x, nf = a.fM ? a.BT : 0;
  const unsigned char* src;
  if (n < a.BT) src = (const unsigned char*)a.M + (size_t)n * a.d * ES;
  else if (n < a.BT + nf) src = (const unsigned char*)a.fM + (size_t)(n - a.BT) * a.d * ES;
  else src = (const unsigned char*)a.P + (size_t)(n - a.BT - nf) * a.d * ES;
  unsigned char* dst = (unsigned char*)a.out + (size_t)n * a.d * ES;
  const size_t bytes = (size_t)a.d * ES;
  if ((bytes & 15) == 0 && ((((uintptr_t)src | (uintptr_t)dst)) & 15) == 0) {
    for (size_t c = threadIdx.x; c < bytes / 16; c += 256)
      reinterpret_cast<uintx4*>(dst)[c] = reinterpret_cast<const uintx4*>(src)[c];
  } else {
    for (size_t c = threadIdx.x; c < bytes; c += 256) dst[c] = src[c];
  }
}

struct ExpandArgs {
  const void* Z;  // [BT (+BT) + gamma][V]
  void* Y;        // [B,R,V]
  int T, gamma, V, BT, has_f;
};
template <bool BF16>
__global__ __launch_bounds__(256) void expand_rows_kernel(ExpandArgs a) {
  const int R = a.T * (1 + a.gamma);
  const int b = blockIdx.x / R, r = blockIdx.x % R;
  int node, strm;
  row_split(r, a.T, a.gamma, node, strm);
  const size_t zm = (size_t)b * a.T + node;
  const size_t zf = a.has_f ? a.BT + zm : zm, zp = (size_t)a.BT * (a.has_f ? 2 : 1) + (strm > 0 ? strm - 1 : 0);
  const size_t yo = ((size_t)b * R + r) * a.V;
  if constexpr (BF16) {
    const uint16_t* Z = (const uint16_t*)a.Z;
    uint16_t* Y = (uint16_t*)a.Y;
    if ((a.V & 7) == 0 && ((((uintptr_t)a.Z | (uintptr_t)a.Y)) & 15) == 0) {  // 16-byte pieces
      for (int c = threadIdx.x; c < a.V / 8; c += 256) {
        uintx4 m = *reinterpret_cast<const uintx4*>(Z + (strm == 0 ? zm : zf) * a.V + 8 * c);
        if (strm > 0) {
          const uintx4 p = *reinterpret_cast<const uintx4*>(Z + zp * a.V + 8 * c);
#pragma unroll
          for (int q = 0; q < 4; ++q)
            m[q] = pack_bf16x2(bf16_bits_to_f32(m[q] & 0xffffu) + bf16_bits_to_f32(p[q] & 0xffffu),
                               bf16_bits_to_f32(m[q] >> 16) + bf16_bits_to_f32(p[q] >> 16));
        }
        *reinterpret_cast<uintx4*>(Y + yo + 8 * c) = m;
      }
    } else {
      for (int v = threadIdx.x; v < a.V; v += 256)
        Y[yo + v] = strm == 0 ? Z[zm * a.V + v]
                              : (uint16_t)f32_to_bf16_bits(bf16_bits_to_f32(Z[zf * a.V + v]) + bf16_bits_to_f32(Z[zp * a.V + v]));
    }
  } else {
    const float* Z = (const float*)a.Z;
    for (int v = threadIdx.x; v < a.V; v += 256)
      ((float*)a.Y)[yo + v] = strm == 0 ? Z[zm * a.V + v] : Z[zf * a.V + v] + Z[zp * a.V + v];
  }
}

static size_t sil_rows(int B, int T, int gamma, bool has_f) { return (size_t)B * T * (has_f ? 2 : 1) + gamma; }

// Value rotation (appendix ablation): stream n of node i takes the node's main-row value times e^{i eps n}.
// Features (2m, 2m+1) are (Re, Im); cos and sin of eps*n come from the host in a table (gamma <= 8 angles).
// One workgroup per stream row; a thread turns one pair at a time (bf16: one 32-bit word).
struct RotateArgs {
  void* v;  // [B,R,Hkv,D]: main rows read, stream rows written
  int T, gamma, row;  // row = Hkv*D elements
  float c[SS_MAX_GAMMA], s[SS_MAX_GAMMA];
};

template <bool BF16>
__global__ __launch_bounds__(256) void value_rotate_kernel(RotateArgs a) {
  const int R = a.T * (1 + a.gamma);
  const int per_seq = a.T * a.gamma;
  const int b = blockIdx.x / per_seq, k = blockIdx.x % per_seq;
  const int node = k / a.gamma, n = k % a.gamma;  // stream n+1
  const float c = a.c[n], sn = a.s[n];
  const size_t src = ((size_t)b * R + node) * a.row, dst = ((size_t)b * R + a.T + k) * a.row;
  for (int m = threadIdx.x; m < a.row / 2; m += 256) {
    float re, im;
    if constexpr (BF16) {
      const uint32_t w = ((const uint32_t*)((const uint16_t*)a.v + src))[m];
      re = bf16_bits_to_f32(w & 0xffffu);
      im = bf16_bits_to_f32(w >> 16);
    } else {
      const float2 w = ((const float2*)((const float*)a.v + src))[m];
      re = w.x;
      im = w.y;
    }
    const float o_re = __builtin_fmaf(re, c, -(im * sn)), o_im = __builtin_fmaf(re, sn, im * c);
    if constexpr (BF16) ((uint32_t*)((uint16_t*)a.v + dst))[m] = pack_bf16x2(o_re, o_im);
    else ((float2*)((float*)a.v + dst))[m] = make_float2(o_re, o_im);
  }
}

}  // namespace ss

extern "C" int ss_value_rotate(void* v_new, int B, int T, int gamma, int Hkv, int D, float eps, int dtype,
                               void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_value_rotate";
  SS_REQUIRE(B >= 0 && Hkv >= 1 && D >= 2 && D % 2 == 0, SS_ERR_INVALID_ARG, "%s: B=%d Hkv=%d D=%d (D must be even)", fn,
             B, Hkv, D);
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: T=%d outside [1,%d]", fn, T, SS_MAX_T);
  SS_REQUIRE(gamma >= 0 && gamma <= SS_MAX_GAMMA, SS_ERR_UNSUPPORTED, "%s: gamma=%d outside [0,%d]", fn, gamma,
             SS_MAX_GAMMA);
  SS_REQUIRE(dtype == SS_F32 || dtype == SS_BF16, SS_ERR_UNSUPPORTED, "%s: dtype %d", fn, dtype);
  SS_REQUIRE(B == 0 || gamma == 0 || v_new, SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  SS_REQUIRE((long)Hkv * D <= 0x7fffffffL && (long)B * T * gamma <= 0x7fffffffL, SS_ERR_UNSUPPORTED, "%s: too large", fn);
  SS_REQUIRE(((uintptr_t)v_new & (dtype == SS_BF16 ? 3 : 7)) == 0, SS_ERR_INVALID_ARG, "%s: v_new is not aligned to a pair", fn);
  if (B == 0 || gamma == 0) return SS_OK;
  RotateArgs a;
  a.v = v_new; a.T = T; a.gamma = gamma; a.row = Hkv * D;
  for (int n = 0; n < SS_MAX_GAMMA; ++n) {
    a.c[n] = (float)cos((double)eps * (n + 1));
    a.s[n] = (float)sin((double)eps * (n + 1));
  }
  const dim3 grid((unsigned)(B * T * gamma));
  if (dtype == SS_F32) hipLaunchKernelGGL(value_rotate_kernel<false>, grid, dim3(256), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(value_rotate_kernel<true>, grid, dim3(256), 0, (hipStream_t)stream, a);
  return check_launch(fn);
}

extern "C" int ss_stream_insert(const void* M, const void* fM, const void* P, int B, int T, int gamma, int d,
                                int dtype, void* X, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_stream_insert";
  SS_REQUIRE(B >= 0 && d >= 1, SS_ERR_INVALID_ARG, "%s: B=%d d=%d", fn, B, d);
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: T=%d outside [1,%d]", fn, T, SS_MAX_T);
  SS_REQUIRE(gamma >= 0 && gamma <= SS_MAX_GAMMA, SS_ERR_UNSUPPORTED, "%s: gamma=%d outside [0,%d]", fn, gamma,
             SS_MAX_GAMMA);
  SS_REQUIRE(dtype == SS_F32 || dtype == SS_BF16, SS_ERR_UNSUPPORTED, "%s: dtype %d", fn, dtype);
  SS_REQUIRE(B == 0 || (M && X && (P || gamma == 0)), SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  SS_REQUIRE((long)B * T * (1 + gamma) <= 0x7fffffffL, SS_ERR_UNSUPPORTED, "%s: grid too large", fn);
  if (B == 0) return SS_OK;
  StreamArgs a;
  a.M = M; a.fM = fM; a.P = P ? P : M; a.X = X;  // P is never read when gamma == 0
  a.B = B; a.T = T; a.gamma = gamma; a.d = d;
  const dim3 grid((unsigned)(B * T * (1 + gamma)));
  if (dtype == SS_F32) hipLaunchKernelGGL(stream_insert_kernel<false>, grid, dim3(256), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(stream_insert_kernel<true>, grid, dim3(256), 0, (hipStream_t)stream, a);
  return check_launch(fn);
}

extern "C" size_t ss_stream_insert_linear_workspace_bytes(int B, int T, int gamma, int d, int V, int dtype, int with_f) {
  ss::clear_error();
  if (B < 0 || T < 1 || gamma < 0 || d < 1 || V < 1 || (dtype != SS_F32 && dtype != SS_BF16)) return 0;
  const size_t n = ss::sil_rows(B, T, gamma, with_f != 0), es = dtype == SS_BF16 ? 2 : 4;
  return ss::align_up(n * d * es, 256) + ss::align_up(n * V * es, 256) + 256;
}

extern "C" int ss_stream_insert_linear(const void* M, const void* fM, const void* P, const void* W, int B, int T,
                                       int gamma, int d, int V, int dtype, void* Y, void* workspace,
                                       size_t workspace_bytes, void* stream) {
  using namespace ss;
  clear_error();
  const char* fn = "ss_stream_insert_linear";
  SS_REQUIRE(B >= 0 && d >= 1 && V >= 1, SS_ERR_INVALID_ARG, "%s: B=%d d=%d V=%d", fn, B, d, V);
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "%s: T=%d outside [1,%d]", fn, T, SS_MAX_T);
  SS_REQUIRE(gamma >= 0 && gamma <= SS_MAX_GAMMA, SS_ERR_UNSUPPORTED, "%s: gamma=%d outside [0,%d]", fn, gamma,
             SS_MAX_GAMMA);
  SS_REQUIRE(dtype == SS_F32 || dtype == SS_BF16, SS_ERR_UNSUPPORTED, "%s: dtype %d", fn, dtype);
  SS_REQUIRE(dtype != SS_BF16 || d % 64 == 0, SS_ERR_UNSUPPORTED, "%s: bf16 path needs d %% 64 == 0 (d=%d)", fn, d);
  SS_REQUIRE(B == 0 || (M && W && Y && (P || gamma == 0)), SS_ERR_INVALID_ARG, "%s: NULL tensor argument", fn);
  SS_REQUIRE((long)B * T * (1 + gamma) <= 0x7fffffffL && (long)B * T * (1 + gamma) * (long)V < (1L << 31), SS_ERR_UNSUPPORTED,
             "%s: too large", fn);
  const size_t need = ss_stream_insert_linear_workspace_bytes(B, T, gamma, d, V, dtype, fM != nullptr);
  SS_REQUIRE(B == 0 || (workspace != nullptr && workspace_bytes >= need), SS_ERR_WORKSPACE,
             "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace_bytes);
  if (B == 0) return SS_OK;
  const bool has_f = fM != nullptr;
  const size_t n = sil_rows(B, T, gamma, has_f), es = dtype == SS_BF16 ? 2 : 4;
  char* ws = (char*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  void* zin = ws;
  void* z = ws + align_up(n * d * es, 256);
  hipStream_t st = (hipStream_t)stream;
  PackArgs p;
  p.M = M; p.fM = fM; p.P = P ? P : M; p.out = zin; p.BT = B * T; p.gamma = gamma; p.d = d;
  if (dtype == SS_F32) hipLaunchKernelGGL(pack_rows_kernel<false>, dim3((unsigned)n), dim3(256), 0, st, p);
  else hipLaunchKernelGGL(pack_rows_kernel<true>, dim3((unsigned)n), dim3(256), 0, st, p);
  if (int rc = check_launch(fn)) return rc;
  if (int rc = ss_linear_rows(zin, W, (int)n, d, V, dtype, z, stream)) return rc;
  ExpandArgs e;
  e.Z = z; e.Y = Y; e.T = T; e.gamma = gamma; e.V = V; e.BT = B * T; e.has_f = has_f ? 1 : 0;
  const dim3 grid((unsigned)(B * T * (1 + gamma)));
  if (dtype == SS_F32) hipLaunchKernelGGL(expand_rows_kernel<false>, grid, dim3(256), 0, st, e);
  else hipLaunchKernelGGL(expand_rows_kernel<true>, grid, dim3(256), 0, st, e);
  return check_launch(fn);
}
