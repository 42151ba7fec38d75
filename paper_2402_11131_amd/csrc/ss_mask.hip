// a1: draft-tree + stream attention mask (Sec. 3.2.2 Eq. 4 as read with the
// appendix mask figure; Eq. 1 / Eq. 2 for the stream rows).
#include "ss_common.h"

namespace ss {

// One workgroup per sequence.  parent -> LDS, ancestor sets by T threads, then
// all threads fill the R x R byte matrix with coalesced stores.
__global__ __launch_bounds__(256) void build_mask_kernel(const int32_t* __restrict__ parent, int T, int gamma,
                                                         uint32_t flags, uint8_t* __restrict__ mask,
                                                         uint64_t* __restrict__ anc_out,
                                                         int32_t* __restrict__ depth_out) {
  __shared__ int par[SS_MAX_T];
  __shared__ uint64_t anc[SS_MAX_T];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int R = T * (1 + gamma);
  if (tid < T) par[tid] = clamp_parent(parent[(size_t)b * T + tid], tid);
  __syncthreads();
  compute_anc(par, T, anc, tid);
  __syncthreads();
  if (tid < T) {
    if (anc_out) anc_out[(size_t)b * T + tid] = anc[tid];
    if (depth_out) depth_out[(size_t)b * T + tid] = __popcll(anc[tid]) - 1;
  }
  if (!mask) return;
  const bool excl = (flags & SS_STREAM_EXCLUDE_SELF) != 0;
  uint8_t* m = mask + (size_t)b * R * R;
  for (int e = tid; e < R * R; e += blockDim.x) {
    const int r = e / R, c = e - r * R;
    const RowVis v = make_row_vis(r, T, gamma, anc, excl);
    m[e] = row_sees(v, c, T) ? 1 : 0;
  }
}

}  // namespace ss

extern "C" int ss_build_mask(const int32_t* parent, int B, int T, int gamma, uint32_t flags, uint8_t* mask,
                             uint64_t* anc, int32_t* depth, void* stream) {
  ss::clear_error();
  SS_REQUIRE(B >= 0, SS_ERR_INVALID_ARG, "ss_build_mask: B < 0");
  SS_REQUIRE(parent != nullptr || B == 0, SS_ERR_INVALID_ARG, "ss_build_mask: parent NULL");
  SS_REQUIRE(T >= 1 && T <= SS_MAX_T, SS_ERR_UNSUPPORTED, "ss_build_mask: T=%d outside [1,%d]", T, SS_MAX_T);
  SS_REQUIRE(gamma >= 0 && gamma <= SS_MAX_GAMMA, SS_ERR_UNSUPPORTED, "ss_build_mask: gamma=%d outside [0,%d]",
             gamma, SS_MAX_GAMMA);
  SS_REQUIRE((flags & ~SS_STREAM_EXCLUDE_SELF) == 0, SS_ERR_INVALID_ARG, "ss_build_mask: unknown flags 0x%x", flags);
  if (B == 0) return SS_OK;
  hipLaunchKernelGGL(ss::build_mask_kernel, dim3(B), dim3(256), 0, (hipStream_t)stream, parent, T, gamma, flags,
                     mask, anc, depth);
  return ss::check_launch("ss_build_mask");
}
