// Host-side pieces of the C ABI: error text, version, host tree helpers.
#include <stdarg.h>
#include <string.h>

#include "ss_common.h"

namespace ss {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
void clear_error() { g_err[0] = 0; }

// Measurement aid: every wave reads its own contiguous slab in rounds of 16 loads of 1 KB (16 bytes per
// lane), all issued before any is used; 2048 waves, eight per compute unit (128 KB in flight each).  The sum
// is kept alive through a store that never happens for real data.
constexpr int kProbeWaves = 2048, kProbeLoads = 16;
template <bool STREAM>
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const uintx4* __restrict__ src, size_t per_wave16, int rounds,
                                                             uint32_t* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const uintx4* p = src + wave * per_wave16 + lane;
  uintx4 acc = uintx4{0u, 0u, 0u, 0u};
  for (int r = 0; r < rounds; ++r) {
    uintx4 v[kProbeLoads];
#pragma unroll
    for (int i = 0; i < kProbeLoads; ++i) {
      const uintx4* q = p + (size_t)(r * kProbeLoads + i) * 64;
      v[i] = STREAM ? __builtin_nontemporal_load(q) : *q;
    }
#pragma unroll
    for (int i = 0; i < kProbeLoads; ++i) acc ^= v[i];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u && acc[0] == 0x7f4a7c15u) sink[0] = acc[1];
}

// Measurement aid: matrix-core instructions on registers only, 2048 waves (two per SIMD), five independent
// accumulator tiles per wave as in the LM-head kernel: what the chip sustains when nothing has to be loaded.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 probe_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float probe_floatx16;
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float* __restrict__ sink) {
  probe_floatx16 acc[5];
#pragma unroll
  for (int i = 0; i < 5; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  // operands with random bits (random sign and mantissa, magnitudes in [1/8, 32)), different for every
  // instruction of a round: constant or
  // tiny operands would toggle few wires and flatter the clock
  probe_bf16x8 a[4], b[5];
  uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
  auto next = [&]() {
    h = h * 1664525u + 1013904223u;
    const uint32_t bits = h >> 16;
    return __builtin_bit_cast(__bf16, (uint16_t)((bits & 0x807fu) | (((bits >> 7) & 0x7u) + 124u) << 7));
  };
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int e = 0; e < 8; ++e) a[r][e] = next();
#pragma unroll
  for (int i = 0; i < 5; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) b[i][e] = next();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int i = 0; i < 5; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r], b[i], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 5; ++i) s += acc[i][0] + acc[i][15];
  if (s == 12345.678f) sink[0] = s;
}

}  // namespace ss

extern "C" {

int ss_version(void) { return 100; }

int ss_probe_mfma_bf16(int iters, double* flops, void* sink, void* stream) {
  ss::clear_error();
  SS_REQUIRE(iters >= 1 && iters <= (1 << 20) && sink != nullptr, SS_ERR_INVALID_ARG,
             "ss_probe_mfma_bf16: iters=%d outside [1, 2^20] or no sink", iters);
  hipLaunchKernelGGL(ss::mfma_probe_kernel, dim3(512), dim3(256), 0, (hipStream_t)stream, iters, (float*)sink);
  if (flops) *flops = 2048.0 * iters * 20.0 * (2.0 * 32 * 32 * 16);
  return ss::check_launch("ss_probe_mfma_bf16");
}

int ss_probe_hbm_read(const void* buf, size_t bytes, int streaming, void* sink, void* stream) {
  ss::clear_error();
  const size_t chunk = (size_t)ss::kProbeWaves * ss::kProbeLoads * 1024;  // bytes of one round of all waves
  SS_REQUIRE(buf != nullptr && sink != nullptr && bytes >= chunk && ((uintptr_t)buf & 15) == 0, SS_ERR_INVALID_ARG,
             "ss_probe_hbm_read: needs a 16-byte aligned buffer of at least %zu bytes and a sink", chunk);
  const size_t rounds = bytes / chunk;
  SS_REQUIRE(rounds <= 0x7fffffff, SS_ERR_UNSUPPORTED, "ss_probe_hbm_read: buffer too large");
  const size_t per_wave16 = rounds * ss::kProbeLoads * 64;
  if (streaming)
    hipLaunchKernelGGL(ss::hbm_read_probe_kernel<true>, dim3(ss::kProbeWaves / 4), dim3(256), 0, (hipStream_t)stream,
                       (const ss::uintx4*)buf, per_wave16, (int)rounds, (uint32_t*)sink);
  else
    hipLaunchKernelGGL(ss::hbm_read_probe_kernel<false>, dim3(ss::kProbeWaves / 4), dim3(256), 0, (hipStream_t)stream,
                       (const ss::uintx4*)buf, per_wave16, (int)rounds, (uint32_t*)sink);
  return ss::check_launch("ss_probe_hbm_read");
}

const char* ss_last_error(void) { return ss::g_err; }

int ss_check_tree_host(const int32_t* parent, int B, int T, int max_depth) {
  ss::clear_error();
  SS_REQUIRE(parent != nullptr && B >= 0 && T >= 1, SS_ERR_INVALID_ARG, "ss_check_tree_host: bad arguments");
  SS_REQUIRE(T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "ss_check_tree_host: T=%d exceeds %d", T, SS_MAX_T);
  for (int b = 0; b < B; ++b) {
    const int32_t* p = parent + (size_t)b * T;
    int depth[SS_MAX_T];
    if (p[0] != -1) SS_FAIL(SS_ERR_BAD_TREE, "tree %d: parent[0]=%d, expected -1", b, p[0]);
    depth[0] = 0;
    for (int i = 1; i < T; ++i) {
      if (p[i] < 0 || p[i] >= i)
        SS_FAIL(SS_ERR_BAD_TREE, "tree %d: parent[%d]=%d not in [0,%d)", b, i, p[i], i);
      depth[i] = depth[p[i]] + 1;
      if (max_depth >= 0 && depth[i] > max_depth)
        SS_FAIL(SS_ERR_BAD_TREE, "tree %d: node %d has depth %d > %d", b, i, depth[i], max_depth);
    }
  }
  return SS_OK;
}

int ss_full_tree_template_host(const int32_t* branching, int gamma, int capacity, int32_t* parent_out,
                               int32_t* rank_out, int32_t* depth_out) {
  ss::clear_error();
  if (branching == nullptr || gamma < 0 || gamma > SS_MAX_GAMMA || capacity < 1) {
    ss::set_error("ss_full_tree_template_host: bad arguments");
    return -1;
  }
  if (capacity > SS_MAX_T) capacity = SS_MAX_T;
  // Breadth first: the nodes of level j are the children, in rank order, of the
  // nodes of level j-1 in their own order.
  int count = 1, lvl_lo = 0, lvl_hi = 1;
  if (parent_out) parent_out[0] = -1;
  if (rank_out) rank_out[0] = 0;
  if (depth_out) depth_out[0] = 0;
  for (int level = 1; level <= gamma; ++level) {
    const int fan = branching[level - 1];
    if (fan < 0) {
      ss::set_error("ss_full_tree_template_host: negative branching");
      return -1;
    }
    for (int p = lvl_lo; p < lvl_hi; ++p)
      for (int r = 0; r < fan; ++r) {
        if (count >= capacity) {
          ss::set_error("ss_full_tree_template_host: tree exceeds %d nodes", capacity);
          return -1;
        }
        if (parent_out) parent_out[count] = p;
        if (rank_out) rank_out[count] = r;
        if (depth_out) depth_out[count] = level;
        ++count;
      }
    lvl_lo = lvl_hi;
    lvl_hi = count;
  }
  return count;
}

}  // extern "C"
