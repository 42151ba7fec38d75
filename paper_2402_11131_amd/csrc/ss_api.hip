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

}  // namespace ss

extern "C" {

int ss_version(void) { return 100; }

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
