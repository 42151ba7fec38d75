/* Runs every function of the oracle once on small inputs whose arrays are exactly as large as the call
 * needs (heap blocks, so that AddressSanitizer sees any access past an end), including the edge cases the
 * kernels are tested on: an empty prefix, a ragged last page, gamma = 0, a one-node tree, parents that have
 * to be clamped, a commit cut by the table's capacity.  Built with -fsanitize=address,undefined by
 * tests/test_sanitizers.py; exits 0 if nothing was reported.  Values are not checked here (the pins do that). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void ora_build_mask(const int32_t*, int, int, int, uint32_t, uint8_t*, uint64_t*, int32_t*);
void ora_msa_attention(const float*, const float*, const float*, const float*, const float*, const int32_t*, int,
                       const int32_t*, const int32_t*, int, int, int, int, int, int, int, double, uint32_t, double*);
void ora_lm_head_topk(const float*, const float*, int, int, int, int, int32_t*, double*, double*);
void ora_linear_rows(const float*, const float*, int, int, int, double*);
void ora_stream_insert(const float*, const float*, const float*, int, int, int, int, double*);
void ora_value_rotate(const float*, int, int, int, int, int, double, double*);
void ora_tree_verify(const int32_t*, const int32_t*, const int32_t*, long, long, int, int, int, int32_t*, int32_t*,
                     int32_t*, int32_t*, int32_t*);
int ora_full_tree_template(const int32_t*, int, int, int32_t*, int32_t*, int32_t*);
void ora_tree_draft(const int32_t*, long, int, const int32_t*, const int32_t*, const int32_t*, const int32_t*, int, int,
                    int, int, int32_t*, int32_t*);
void ora_lm_head_lse(const float*, const float*, int, int, int, double*);
void ora_transition_probs(const float*, const float*, const int32_t*, const int32_t*, int, int, int, int, double*);
void ora_tree_prune(const int32_t*, const int32_t*, const float*, float, int, int, int32_t*, int32_t*, int32_t*,
                    int32_t*, int32_t*);
void ora_kv_commit(const float*, const float*, float*, float*, const int32_t*, int, const int32_t*, const int32_t*,
                   const int32_t*, int, int, int, int, int, int, int32_t*);

static uint32_t rng_state = 12345u;
static float frand(void) {
  rng_state = rng_state * 1664525u + 1013904223u;
  return (float)((rng_state >> 8) & 0xffff) / 32768.0f - 1.0f;
}
static float* fbuf(size_t n) {
  float* p = (float*)malloc((n ? n : 1) * sizeof(float));
  for (size_t i = 0; i < n; i++) p[i] = frand();
  return p;
}
static int32_t* ibuf(size_t n, int32_t v) {
  int32_t* p = (int32_t*)malloc((n ? n : 1) * sizeof(int32_t));
  for (size_t i = 0; i < n; i++) p[i] = v;
  return p;
}

static void attention_case(int B, int T, int gamma, int H, int Hkv, int D, int page, const int* lens, uint32_t flags,
                           int bad_parents) {
  const int R = T * (1 + gamma);
  int max_pages = 1, total_pages = 0;
  for (int b = 0; b < B; b++) {
    const int np = (lens[b] + page - 1) / page;
    if (np > max_pages) max_pages = np;
    total_pages += np;
  }
  if (total_pages < 1) total_pages = 1;
  float* q = fbuf((size_t)B * R * H * D);
  float* kn = fbuf((size_t)B * R * Hkv * D);
  float* vn = fbuf((size_t)B * R * Hkv * D);
  float* kc = fbuf((size_t)total_pages * Hkv * page * D);
  float* vc = fbuf((size_t)total_pages * Hkv * D * page);
  int32_t* table = ibuf((size_t)B * max_pages, 0);
  int32_t* sl = ibuf(B, 0);
  int32_t* parent = ibuf((size_t)B * T, 0);
  int next = 0;
  for (int b = 0; b < B; b++) {
    sl[b] = lens[b];
    for (int p = 0; p < (lens[b] + page - 1) / page; p++) table[b * max_pages + p] = next++;
    parent[b * T] = -1;
    for (int i = 1; i < T; i++) parent[b * T + i] = bad_parents ? (i % 3 == 0 ? i + 5 : -7) : (i - 1) / 2;
  }
  double* out = (double*)malloc((size_t)B * R * H * D * sizeof(double));
  ora_msa_attention(q, kn, vn, kc, vc, table, max_pages, sl, parent, B, T, gamma, H, Hkv, D, page, 0.125, flags, out);
  uint8_t* mask = (uint8_t*)malloc((size_t)B * R * R);
  uint64_t* anc = (uint64_t*)malloc((size_t)B * T * sizeof(uint64_t));
  int32_t* depth = ibuf((size_t)B * T, 0);
  ora_build_mask(parent, B, T, gamma, flags, mask, anc, depth);
  ora_build_mask(parent, B, T, gamma, flags, NULL, NULL, NULL);
  free(q); free(kn); free(vn); free(kc); free(vc); free(table); free(sl); free(parent); free(out);
  free(mask); free(anc); free(depth);
}

int main(void) {
  { const int lens[2] = {0, 37}; attention_case(2, 5, 2, 4, 2, 8, 16, lens, 0, 0); }
  { const int lens[1] = {16}; attention_case(1, 1, 0, 2, 2, 4, 16, lens, 1, 0); }
  { const int lens[3] = {1, 64, 33}; attention_case(3, 64, 1, 1, 1, 4, 32, lens, 1, 1); }

  /* LM head, projection, log-sum-exp */
  {
    const int N = 3, d = 5, V = 7, K = 7;
    float* h = fbuf((size_t)N * d);
    float* W = fbuf((size_t)V * d);
    int32_t* idx = ibuf((size_t)N * K, 0);
    double* val = (double*)malloc((size_t)N * K * sizeof(double));
    double* z = (double*)malloc((size_t)N * V * sizeof(double));
    ora_lm_head_topk(h, W, N, d, V, K, idx, val, z);
    ora_lm_head_topk(h, W, N, d, V, 1, idx, val, NULL);
    ora_linear_rows(h, W, N, d, V, z);
    double* lse = (double*)malloc(N * sizeof(double));
    ora_lm_head_lse(h, W, N, d, V, lse);
    free(h); free(W); free(idx); free(val); free(z); free(lse);
  }
  /* verify, draft, template, pruning, transition probabilities */
  {
    const int B = 2, T = 6, gamma = 3, K = 2, max_depth = 3, V = 11, d = 4;
    int32_t parent[12] = {-1, 0, 0, 1, 1, 3, -1, 9, -4, 0, 2, 2};
    int32_t* tok = ibuf((size_t)B * T, 3);
    int32_t* am = ibuf((size_t)B * T, 3);
    int32_t *na = ibuf(B, 0), *last = ibuf(B, 0), *bonus = ibuf(B, 0);
    int32_t *path = ibuf((size_t)B * (max_depth + 1), 0), *ot = ibuf((size_t)B * (max_depth + 1), 0);
    ora_tree_verify(tok, parent, am, T, 1, B, T, max_depth, na, last, bonus, path, ot);
    ora_tree_verify(tok, parent, am, T, 1, B, T, 0, na, last, bonus, path, ot);
    const int32_t branching[3] = {2, 2, 1};
    int32_t tp[64], tr[64], td[64];
    const int T2 = ora_full_tree_template(branching, gamma, 64, tp, tr, td);
    if (T2 != 11) return 2;
    if (ora_full_tree_template(branching, gamma, 5, NULL, NULL, NULL) != -1) return 3;
    int32_t* topk = ibuf((size_t)B * T * gamma * K, 5);
    int32_t* nt = ibuf((size_t)B * T2, 0);
    int32_t* np = ibuf(T2, 0);
    ora_tree_draft(topk, (long)T * gamma * K, K, last, bonus, tp, tr, B, T, gamma, T2, nt, np);
    float* h = fbuf((size_t)B * T * d);
    float* W = fbuf((size_t)V * d);
    tok[3] = -1; tok[4] = V + 3;   /* tokens outside the vocabulary */
    double* prob = (double*)malloc((size_t)B * T * sizeof(double));
    ora_transition_probs(h, W, tok, parent, B, T, d, V, prob);
    float* pf = fbuf((size_t)B * T);
    int32_t *keep = ibuf((size_t)B * T, 0), *ntok = ibuf((size_t)B * T, 0), *npar = ibuf((size_t)B * T, 0),
            *old = ibuf((size_t)B * T, 0), *nn = ibuf(B, 0);
    ora_tree_prune(tok, parent, pf, 0.2f, B, T, keep, ntok, npar, old, nn);
    free(tok); free(am); free(na); free(last); free(bonus); free(path); free(ot); free(topk); free(nt); free(np);
    free(h); free(W); free(prob); free(pf); free(keep); free(ntok); free(npar); free(old); free(nn);
  }
  /* stream insertion, value rotation */
  {
    const int B = 2, T = 3, gamma = 2, d = 6, Hkv = 2, D = 4, R = T * (1 + gamma);
    float *M = fbuf((size_t)B * T * d), *fM = fbuf((size_t)B * T * d), *P = fbuf((size_t)gamma * d);
    double* X = (double*)malloc((size_t)B * R * d * sizeof(double));
    ora_stream_insert(M, fM, P, B, T, gamma, d, X);
    ora_stream_insert(M, NULL, P, B, T, gamma, d, X);
    float* v = fbuf((size_t)B * R * Hkv * D);
    double* vo = (double*)malloc((size_t)B * R * Hkv * D * sizeof(double));
    ora_value_rotate(v, B, T, gamma, Hkv, D, 0.3, vo);
    free(M); free(fM); free(P); free(X); free(v); free(vo);
  }
  /* cache commit: one sequence whose appended rows are cut by the table's capacity */
  {
    const int B = 2, T = 4, gamma = 1, R = T * (1 + gamma), Hkv = 2, D = 4, page = 16, max_pages = 2, max_depth = 3;
    float *kn = fbuf((size_t)B * R * Hkv * D), *vn = fbuf((size_t)B * R * Hkv * D);
    float *kc = fbuf((size_t)4 * Hkv * page * D), *vc = fbuf((size_t)4 * Hkv * D * page);
    int32_t table[4] = {2, 0, 3, 1};
    int32_t sl[2] = {15, 30};
    int32_t path[8] = {0, 1, 3, -1, 0, 2, 3, 1};
    int32_t na[2] = {2, 3};
    int32_t nl[2];
    ora_kv_commit(kn, vn, kc, vc, table, max_pages, sl, path, na, B, R, Hkv, D, page, max_depth, nl);
    if (nl[0] != 18 || nl[1] != 32) return 4;
    free(kn); free(vn); free(kc); free(vc);
  }
  printf("oracle driver done\n");
  return 0;
}
