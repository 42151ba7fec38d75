// Calls the host-side helpers of the C ABI (the functions that read HOST arrays) on heap blocks of exactly the
// size the call needs, valid and invalid trees and templates alike.  Built with the host pass under
// -fsanitize=address,undefined by tests/test_sanitizers.py; exits 0 if nothing was reported.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ss.h"

int main() {
  {
    const int B = 3, T = 7;
    int32_t* par = (int32_t*)malloc(sizeof(int32_t) * B * T);
    const int32_t good[7] = {-1, 0, 0, 1, 1, 2, 5};
    for (int b = 0; b < B; ++b) memcpy(par + b * T, good, sizeof(good));
    if (ss_check_tree_host(par, B, T, -1) != SS_OK) return 2;
    if (ss_check_tree_host(par, B, T, 2) != SS_ERR_BAD_TREE) return 3;   // node 6 has depth 3
    par[2 * T + 4] = 4;                                                 // parent not below the node
    if (ss_check_tree_host(par, B, T, -1) != SS_ERR_BAD_TREE) return 4;
    par[2 * T + 4] = -3;
    if (ss_check_tree_host(par, B, T, -1) != SS_ERR_BAD_TREE) return 5;
    if (ss_check_tree_host(par, B, SS_MAX_T + 1, -1) != SS_ERR_UNSUPPORTED) return 6;
    if (ss_check_tree_host(nullptr, B, T, -1) != SS_ERR_INVALID_ARG) return 7;
    if (strlen(ss_last_error()) == 0) return 8;
    free(par);
  }
  {
    int32_t* br = (int32_t*)malloc(sizeof(int32_t) * 3);
    br[0] = 4; br[1] = 2; br[2] = 1;
    const int n = ss_full_tree_template_host(br, 3, SS_MAX_T, nullptr, nullptr, nullptr);
    if (n != 1 + 4 + 8 + 8) return 9;
    int32_t* p = (int32_t*)malloc(sizeof(int32_t) * n);
    int32_t* r = (int32_t*)malloc(sizeof(int32_t) * n);
    int32_t* d = (int32_t*)malloc(sizeof(int32_t) * n);
    if (ss_full_tree_template_host(br, 3, n, p, r, d) != n) return 10;
    if (ss_full_tree_template_host(br, 3, n - 1, p, r, d) != -1) return 11;   // one node too many for the arrays
    br[1] = -2;
    if (ss_full_tree_template_host(br, 3, n, p, r, d) != -1) return 12;
    br[1] = 2;
    if (ss_full_tree_template_host(br, 0, 1, p, r, d) != 1) return 13;        // gamma 0: the root alone
    br[0] = 8; br[1] = 8; br[2] = 8;
    if (ss_full_tree_template_host(br, 3, SS_MAX_T, nullptr, nullptr, nullptr) != -1) return 14;  // 585 nodes
    free(br); free(p); free(r); free(d);
  }
  // workspace and plan queries are host-only too
  if (ss_msa_workspace_bytes(4, 16, 4, 32, 32, 128, 4096, SS_BF16) == 0) return 15;
  if (ss_msa_workspace_bytes(4, 16, 4, 32, 32, 96, 4096, SS_BF16) != 0) return 16;
  int ns = 0, nk = 0;
  if (ss_msa_plan(4, 16, 4, 32, 32, 128, 4096, SS_BF16, &ns, &nk) != SS_OK || ns < 1 || nk < 1) return 17;
  if (ss_lm_head_workspace_bytes(320, 4096, 32000, 4, SS_BF16) == 0) return 18;
  printf("host driver done\n");
  return 0;
}
