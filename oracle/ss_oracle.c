/*
 * ss_oracle.c — TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow CPU statement of what the verify-and-speculate step of
 * Speculative Streaming (arXiv 2402.11131) computes, written from the paper.
 * Floating point is done in double.  Nothing here is blocked, fused or
 * reordered: every function is the definition written out as loops, so that it
 * can be checked against the paper by eye.  It shares no code with the HIP
 * library and must only be used by the tests, by the smoke check and by the
 * CPU-baseline leg of the benchmark.
 *
 * Row order inside a sequence of T tree nodes with gamma streams
 * (R = T*(1+gamma) rows, the batch size of Sec. 3.2.3):
 *   main row of node i: r = i;  stream j (1..gamma) of node i: r = T+i*gamma+j-1.
 * Node 0 is the root, parent[0] = -1, parent[i] < i.
 *
 * Readings of the paper used here (each is pinned by a test):
 *  - Eq. 2 writes S_{t(<=j)}: stream j sees streams 1..j of ITS OWN node, itself
 *    included.  Flag ORA_EXCLUDE_SELF gives the strict reading 1..j-1.
 *  - Eq. 4 as printed only links adjacent levels; the appendix attention-mask
 *    figure says a node attends to all its predecessors from the root and to
 *    itself, and that tokens are replicated per path, so ancestry follows
 *    parent[] and siblings / other branches are invisible.
 *  - "time step t" of Eq. 1/2 for a tree is a tree NODE: the streams of node i
 *    see the main rows of i's ancestors-or-self and i's own streams only; main
 *    rows never see stream keys.
 *  - Verification (Appendix A.1, "hard" matching): root always accepted; a node
 *    is accepted iff its parent is and its token equals the main-stream argmax
 *    at the parent; the deepest accepted node wins, ties -> lowest index.
 *  - Drafting (Sec. 3.2.2, Appendix A.1): new root = argmax at the last accepted
 *    node; level j of the new tree = top-k tokens of stream j of that node.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORA_EXCLUDE_SELF 1u

/* ------------------------------------------------------------------ tree */

/* Parent of node i with the same clamping rule the ABI documents: node 0 is the
 * root; for i > 0 a parent outside [0,i) counts as 0. */
static int ora_parent(const int32_t* parent, int i) {
  if (i == 0) return -1;
  int p = parent[i];
  if (p < 0 || p >= i) return 0;
  return p;
}

/* depth = number of edges from the root (walk up). */
static int ora_depth(const int32_t* parent, int i) {
  int d = 0;
  while (i > 0) {
    i = ora_parent(parent, i);
    d++;
  }
  return d;
}

/* 1 iff a lies on the path root..i (a == i counts). */
static int ora_is_anc_or_self(const int32_t* parent, int a, int i) {
  while (i >= 0) {
    if (i == a) return 1;
    i = ora_parent(parent, i);
  }
  return 0;
}

/* row -> (node, stream); stream 0 = main row. */
static void ora_row_split(int r, int T, int gamma, int* node, int* strm) {
  if (r < T) {
    *node = r;
    *strm = 0;
  } else {
    *node = (r - T) / gamma;
    *strm = (r - T) % gamma + 1;
  }
}

/* May row (i,j) attend the step's own key (i2,j2)?  Eq. 1, Eq. 2, Eq. 4 with the
 * appendix figure's reading. */
static int ora_visible(const int32_t* parent, int i, int j, int i2, int j2, uint32_t flags) {
  if (j2 == 0) return ora_is_anc_or_self(parent, i2, i); /* main key: ancestors and self */
  if (j == 0) return 0;                                  /* main rows never see stream keys */
  if (i2 != i) return 0;                                 /* only the node's own streams */
  return (flags & ORA_EXCLUDE_SELF) ? (j2 < j) : (j2 <= j);
}

/* a1: depth, ancestor bit sets and the dense R x R boolean mask.  Any output may be NULL. */
void ora_build_mask(const int32_t* parent, int B, int T, int gamma, uint32_t flags, uint8_t* mask,
                    uint64_t* anc, int32_t* depth) {
  int R = T * (1 + gamma);
  for (int b = 0; b < B; b++) {
    const int32_t* par = parent + (size_t)b * T;
    for (int i = 0; i < T; i++) {
      if (depth) depth[(size_t)b * T + i] = ora_depth(par, i);
      if (anc) {
        uint64_t bits = 0;
        for (int a = 0; a < T; a++)
          if (ora_is_anc_or_self(par, a, i)) bits |= (uint64_t)1 << a;
        anc[(size_t)b * T + i] = bits;
      }
    }
    if (!mask) continue;
    for (int r = 0; r < R; r++) {
      int i, j;
      ora_row_split(r, T, gamma, &i, &j);
      for (int c = 0; c < R; c++) {
        int i2, j2;
        ora_row_split(c, T, gamma, &i2, &j2);
        mask[((size_t)b * R + r) * R + c] = (uint8_t)ora_visible(par, i, j, i2, j2, flags);
      }
    }
  }
}

/* ------------------------------------------------------------------ MSA */

/*
 * a2: multi-stream attention, Eq. 1 (main rows) and Eq. 2 (stream rows), one
 * layer.  Inputs are float arrays holding exactly the stored values (a bf16
 * tensor is passed up-cast); all arithmetic is double; out is double.
 * Layouts as in the ABI: q/out [B,R,H,D], k_new/v_new [B,R,Hkv,D], k_cache
 * [pages,Hkv,page,D], v_cache [pages,Hkv,D,page], block_table [B,max_pages].
 */
void ora_msa_attention(const float* q, const float* k_new, const float* v_new, const float* k_cache,
                       const float* v_cache, const int32_t* block_table, int max_pages,
                       const int32_t* seq_lens, const int32_t* parent, int B, int T, int gamma, int H,
                       int Hkv, int D, int page, double scale, uint32_t flags, double* out) {
  int R = T * (1 + gamma);
  int g = H / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < B; b++) {
    for (int h = 0; h < H; h++) {
      int hk = h / g;
      int L = seq_lens[b];
      if (L < 0) L = 0;
      if (L > max_pages * page) L = max_pages * page;
      const int32_t* par = parent + (size_t)b * T;
      int C = L + R; /* keys: L cached main-stream tokens, then the R new rows */
      double* s = (double*)malloc(sizeof(double) * (size_t)C);
      double* o = (double*)malloc(sizeof(double) * (size_t)D);
      for (int r = 0; r < R; r++) {
        int i, j;
        ora_row_split(r, T, gamma, &i, &j);
        const float* qv = q + (((size_t)b * R + r) * H + h) * D;
        /* scores; masked keys get -inf */
        for (int c = 0; c < C; c++) {
          double dot = 0.0;
          if (c < L) {
            size_t pg = (size_t)block_table[(size_t)b * max_pages + c / page];
            const float* kv = k_cache + ((pg * Hkv + hk) * page + (size_t)(c % page)) * D;
            for (int d = 0; d < D; d++) dot += (double)qv[d] * (double)kv[d];
            s[c] = scale * dot;
          } else {
            int i2, j2;
            ora_row_split(c - L, T, gamma, &i2, &j2);
            if (ora_visible(par, i, j, i2, j2, flags)) {
              const float* kv = k_new + (((size_t)b * R + (c - L)) * Hkv + hk) * D;
              for (int d = 0; d < D; d++) dot += (double)qv[d] * (double)kv[d];
              s[c] = scale * dot;
            } else {
              s[c] = -INFINITY;
            }
          }
        }
        /* softmax over all keys (the row's own key is always visible, so max is finite) */
        double mx = -INFINITY;
        for (int c = 0; c < C; c++)
          if (s[c] > mx) mx = s[c];
        double den = 0.0;
        for (int c = 0; c < C; c++) {
          s[c] = (s[c] == -INFINITY) ? 0.0 : exp(s[c] - mx);
          den += s[c];
        }
        /* weighted sum of values */
        for (int d = 0; d < D; d++) o[d] = 0.0;
        for (int c = 0; c < C; c++) {
          double p = s[c] / den;
          if (p == 0.0) continue;
          if (c < L) {
            size_t pg = (size_t)block_table[(size_t)b * max_pages + c / page];
            const float* vv = v_cache + (pg * Hkv + hk) * (size_t)D * page + (size_t)(c % page);
            for (int d = 0; d < D; d++) o[d] += p * (double)vv[(size_t)d * page];
          } else {
            const float* vv = v_new + (((size_t)b * R + (c - L)) * Hkv + hk) * D;
            for (int d = 0; d < D; d++) o[d] += p * (double)vv[d];
          }
        }
        double* ov = out + (((size_t)b * R + r) * H + h) * D;
        for (int d = 0; d < D; d++) ov[d] = o[d];
      }
      free(s);
      free(o);
    }
  }
}

/* ------------------------------------------------------------------ LM head */

typedef struct {
  double z;
  int32_t v;
} ora_cand;

/* larger logit first; equal logits -> lower token id first */
static int ora_cand_cmp(const void* a, const void* b) {
  const ora_cand* x = (const ora_cand*)a;
  const ora_cand* y = (const ora_cand*)b;
  if (x->z > y->z) return -1;
  if (x->z < y->z) return 1;
  return (x->v > y->v) - (x->v < y->v);
}

/*
 * a3: z[n,v] = sum_d hidden[n,d]*W[v,d] in double, then a full sort of every
 * row; idx/val get the first K entries.  If logits != NULL it receives all of
 * z ([N,V] doubles).
 */
void ora_lm_head_topk(const float* hidden, const float* W, int N, int d, int V, int K, int32_t* idx,
                      double* val, double* logits) {
#pragma omp parallel for schedule(dynamic)
  for (int n = 0; n < N; n++) {
    ora_cand* c = (ora_cand*)malloc(sizeof(ora_cand) * (size_t)V);
    for (int v = 0; v < V; v++) {
      double acc = 0.0;
      const float* hv = hidden + (size_t)n * d;
      const float* wv = W + (size_t)v * d;
      for (int e = 0; e < d; e++) acc += (double)hv[e] * (double)wv[e];
      c[v].z = acc;
      c[v].v = v;
      if (logits) logits[(size_t)n * V + v] = acc;
    }
    qsort(c, (size_t)V, sizeof(ora_cand), ora_cand_cmp);
    for (int k = 0; k < K; k++) {
      idx[(size_t)n * K + k] = c[k].v;
      val[(size_t)n * K + k] = c[k].z;
    }
    free(c);
  }
}

/*
 * n1: the dense projections around multi-stream attention (Sec. 3.1: queries,
 * keys and values are H.W^Q, H.W^K, H.W^V of the hidden states H, for main and
 * stream rows alike; the feed-forward maps are of the same form).  With the
 * weight stored one output feature per row, y[n,v] = sum_e x[n,e] * W[v,e],
 * accumulated in double in the order of e.
 */
void ora_linear_rows(const float* x, const float* W, int N, int d, int V, double* y) {
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; n++)
    for (int v = 0; v < V; v++) {
      double acc = 0.0;
      for (int e = 0; e < d; e++) acc += (double)x[(size_t)n * d + e] * (double)W[(size_t)v * d + e];
      y[(size_t)n * V + v] = acc;
    }
}

/*
 * n4: stream insertion (Eq. 3).  At the first multi-stream layer the rows of a
 * step are formed from the main-stream hidden states M [B,T,d] of the tree
 * nodes: the main row of node i is M_i itself, stream j of node i starts as
 * f(M_i) + P_j with P [gamma,d] the stream identifier embeddings.  fM holds
 * f(M) [B,T,d]; NULL means the identity, which the paper's experiments use
 * (Appendix, experimental setup).  X [B,R,d] in the row order stated above.
 */
void ora_stream_insert(const float* M, const float* fM, const float* P, int B, int T, int gamma,
                       int d, double* X) {
  const int R = T * (1 + gamma);
  const float* src = fM ? fM : M;
  for (int b = 0; b < B; b++)
    for (int i = 0; i < T; i++) {
      for (int e = 0; e < d; e++)
        X[((size_t)b * R + i) * d + e] = (double)M[((size_t)b * T + i) * d + e];
      for (int j = 1; j <= gamma; j++) {
        const int r = T + i * gamma + (j - 1);
        for (int e = 0; e < d; e++)
          X[((size_t)b * R + r) * d + e] =
              (double)src[((size_t)b * T + i) * d + e] + (double)P[(size_t)(j - 1) * d + e];
      }
    }
}

/*
 * Value rotation (appendix ablation "Value Rotation"): instead of stream
 * embeddings, the value projection of stream n of a node is the main stream's
 * value projection of that node times e^{i eps n}, n = 1..gamma.  The paper does
 * not say how real features form complex numbers; the reading used here is that
 * of rotary embeddings in the interleaved convention: features (2m, 2m+1) of a
 * head are (Re, Im) of one complex number, and all pairs turn by the same angle
 * (the equation has no per-pair frequency).  v [B,R,Hkv,D] in the row order
 * stated above: main rows are read, stream rows are written; out is the whole
 * tensor in double (main rows copied).
 */
void ora_value_rotate(const float* v, int B, int T, int gamma, int Hkv, int D, double eps, double* out) {
  const int R = T * (1 + gamma);
  const size_t row = (size_t)Hkv * D;
  for (int b = 0; b < B; b++)
    for (int i = 0; i < T; i++) {
      const float* main_row = v + ((size_t)b * R + i) * row;
      for (size_t e = 0; e < row; e++) out[((size_t)b * R + i) * row + e] = (double)main_row[e];
      for (int n = 1; n <= gamma; n++) {
        double* dst = out + ((size_t)b * R + T + (size_t)i * gamma + (n - 1)) * row;
        const double c = cos(eps * n), sn = sin(eps * n);
        for (size_t m = 0; m < row / 2; m++) {
          const double re = (double)main_row[2 * m], im = (double)main_row[2 * m + 1];
          dst[2 * m] = re * c - im * sn;      /* (re + i im)(c + i sn) */
          dst[2 * m + 1] = re * sn + im * c;
        }
      }
    }
}

/* ------------------------------------------------------------------ verify */

/*
 * a4: greedy longest-path verification.  a[i] = main-stream argmax token at
 * node i, read at main_argmax[b*batch_stride + i*node_stride].
 */
void ora_tree_verify(const int32_t* tok, const int32_t* parent, const int32_t* main_argmax,
                     long batch_stride, long node_stride, int B, int T, int max_depth,
                     int32_t* n_accept, int32_t* last, int32_t* bonus, int32_t* path,
                     int32_t* out_tokens) {
  for (int b = 0; b < B; b++) {
    const int32_t* par = parent + (size_t)b * T;
    const int32_t* tk = tok + (size_t)b * T;
    const int32_t* a = main_argmax + (size_t)b * batch_stride;
    int ok[64];
    int best = 0, best_depth = 0;
    ok[0] = 1;
    for (int i = 1; i < T; i++) {
      int p = ora_parent(par, i);
      int dep = ora_depth(par, i);
      ok[i] = ok[p] && tk[i] == a[(size_t)p * node_stride] && dep <= max_depth;
      if (ok[i] && dep > best_depth) {
        best = i;
        best_depth = dep;
      }
    }
    n_accept[b] = best_depth;
    last[b] = best;
    bonus[b] = a[(size_t)best * node_stride];
    int32_t* pth = path + (size_t)b * (max_depth + 1);
    int32_t* ot = out_tokens + (size_t)b * (max_depth + 1);
    for (int k = 0; k <= max_depth; k++) {
      pth[k] = -1;
      ot[k] = -1;
    }
    for (int n = best, k = best_depth; n >= 0; n = ora_parent(par, n), k--) pth[k] = n;
    for (int k = 1; k <= best_depth; k++) ot[k - 1] = tk[pth[k]];
    ot[best_depth] = bonus[b];
  }
}

/* ------------------------------------------------------------------ draft */

/*
 * Full tree with branching[j-1] children per node of level j-1: nodes numbered
 * level by level, inside a level by (parent, rank).  Returns the node count
 * (1 + sum_j prod_{m<=j} branching[m-1]; uniform k: 1 + sum_g k^g, Sec. 3.2.3)
 * or -1 if it exceeds capacity.  Outputs may be NULL.
 */
int ora_full_tree_template(const int32_t* branching, int gamma, int capacity, int32_t* parent_out,
                           int32_t* rank_out, int32_t* depth_out) {
  int n = 1, level_begin = 0, level_end = 1;
  if (capacity < 1) return -1;
  if (parent_out) parent_out[0] = -1;
  if (rank_out) rank_out[0] = 0;
  if (depth_out) depth_out[0] = 0;
  for (int j = 1; j <= gamma; j++) {
    int k = branching[j - 1];
    for (int p = level_begin; p < level_end; p++) {
      for (int r = 0; r < k; r++) {
        if (n >= capacity) return -1;
        if (parent_out) parent_out[n] = p;
        if (rank_out) rank_out[n] = r;
        if (depth_out) depth_out[n] = j;
        n++;
      }
    }
    level_begin = level_end;
    level_end = n;
  }
  return n;
}

/*
 * a5: next tree draft from a template.  stream_topk[b*batch_stride +
 * ((i*gamma)+(j-1))*K + rank] = rank-th token of stream j of node i.
 */
void ora_tree_draft(const int32_t* stream_topk, long batch_stride, int K, const int32_t* last,
                    const int32_t* bonus, const int32_t* tmpl_parent, const int32_t* tmpl_rank, int B,
                    int T, int gamma, int T2, int32_t* next_tok, int32_t* next_parent) {
  (void)T;
  for (int b = 0; b < B; b++) {
    const int32_t* tk = stream_topk + (size_t)b * batch_stride;
    int node = last[b];
    next_tok[(size_t)b * T2] = bonus[b];
    for (int i = 1; i < T2; i++) {
      int j = ora_depth(tmpl_parent, i); /* level j draws from stream j */
      int r = tmpl_rank[i];
      int32_t t = -1;
      if (j >= 1 && j <= gamma && r >= 0 && r < K) t = tk[((size_t)node * gamma + (j - 1)) * K + r];
      next_tok[(size_t)b * T2 + i] = t;
    }
  }
  if (next_parent)
    for (int i = 0; i < T2; i++) next_parent[i] = (i == 0) ? -1 : ora_parent(tmpl_parent, i);
}

/*
 * n2: parallel tree pruning (Sec. 3.2.3, Appendix A.1 and its generation-step figure).
 *
 * Early-exit logits of main row i are zt_i = H(o(M_i)): h [B,T,d] holds o(M), the main-stream hidden
 * states of the tree nodes after the low-rank map, W [V,d] is the LM head H.  Z_i = softmax(zt_i) are
 * the normalised early-exit logits, and the transition probability between a parent p and its child c
 * is Z_p at the child's token: prob[c] = exp(zt_p[tok_c]) / sum_v exp(zt_p[v]).  The root has no
 * parent: prob[0] = 1.  A token outside [0,V) has probability 0.
 */
void ora_lm_head_lse(const float* h, const float* W, int N, int d, int V, double* lse) {
#pragma omp parallel for schedule(dynamic)
  for (int n = 0; n < N; n++) {
    double* z = (double*)malloc(sizeof(double) * (size_t)V);
    double m = -INFINITY, s = 0.0;
    for (int v = 0; v < V; v++) {
      double acc = 0.0;
      for (int e = 0; e < d; e++) acc += (double)h[(size_t)n * d + e] * (double)W[(size_t)v * d + e];
      z[v] = acc;
      if (acc > m) m = acc;
    }
    for (int v = 0; v < V; v++) s += exp(z[v] - m);
    lse[n] = m + log(s);
    free(z);
  }
}

void ora_transition_probs(const float* h, const float* W, const int32_t* tok, const int32_t* parent, int B,
                          int T, int d, int V, double* prob) {
  for (int b = 0; b < B; b++) {
    prob[(size_t)b * T] = 1.0;
    for (int i = 1; i < T; i++) {
      const int p = ora_parent(parent + (size_t)b * T, i);
      const int c = tok[(size_t)b * T + i];
      const float* hp = h + ((size_t)b * T + p) * d;
      double m = -INFINITY, s = 0.0, zc = 0.0;
      double* z = (double*)malloc(sizeof(double) * (size_t)V);
      for (int v = 0; v < V; v++) {
        double acc = 0.0;
        for (int e = 0; e < d; e++) acc += (double)hp[e] * (double)W[(size_t)v * d + e];
        z[v] = acc;
        if (acc > m) m = acc;
      }
      for (int v = 0; v < V; v++) s += exp(z[v] - m);
      if (c >= 0 && c < V) zc = exp(z[c] - m) / s;
      prob[(size_t)b * T + i] = (c >= 0 && c < V) ? zc : 0.0;
      free(z);
    }
  }
}

/*
 * A child whose transition probability is below the threshold is pruned together with its sub-tree
 * (Appendix A.1: the sub-tree starting at the pruned token goes).  The kept nodes keep their order and
 * are renumbered 0..n-1; new_parent refers to the new numbers; old_index maps back.  Entries from n
 * on are padding: token -1 (matches no prediction, so verification never accepts it), parent 0,
 * old_index -1.  prob is what the pruning layer decides on, in single precision.
 */
void ora_tree_prune(const int32_t* tok, const int32_t* parent, const float* prob, float threshold, int B,
                    int T, int32_t* keep, int32_t* new_tok, int32_t* new_parent, int32_t* old_index,
                    int32_t* n_nodes) {
  for (int b = 0; b < B; b++) {
    const int32_t* par = parent + (size_t)b * T;
    int32_t* kp = keep + (size_t)b * T;
    int new_of[64];
    int n = 0;
    for (int i = 0; i < T; i++) {
      if (i == 0) kp[i] = 1;
      else kp[i] = kp[ora_parent(par, i)] && !(prob[(size_t)b * T + i] < threshold);
      new_of[i] = kp[i] ? n : -1;
      if (kp[i]) {
        new_tok[(size_t)b * T + n] = tok[(size_t)b * T + i];
        new_parent[(size_t)b * T + n] = (i == 0) ? -1 : new_of[ora_parent(par, i)];
        old_index[(size_t)b * T + n] = i;
        n++;
      }
    }
    n_nodes[b] = n;
    for (int i = n; i < T; i++) {
      new_tok[(size_t)b * T + i] = -1;
      new_parent[(size_t)b * T + i] = 0;
      old_index[(size_t)b * T + i] = -1;
    }
  }
}

/*
 * n3: KV-cache commit.  Main-stream keys/values are cached, those of the speculative streams never
 * are (Sec. 3.2.1), and the cache is trimmed back to what was accepted after each generation step
 * (Appendix A.1): of the step's own rows only the main rows of the accepted path stay, appended in
 * path order behind the L cached tokens.  Caches are updated in place; new_len = L + n_accept + 1.
 * Layouts as in a2: k_cache [P][Hkv][page][D], v_cache [P][Hkv][D][page], k_new/v_new [B][R][Hkv][D].
 * A position past the block table's capacity is dropped; n_accept[b] < 0 means that nothing of sequence b is
 * appended (what ora_kv_alloc_pages reports when not even the first row has a page).
 */
void ora_kv_commit(const float* k_new, const float* v_new, float* k_cache, float* v_cache,
                   const int32_t* block_table, int max_pages, const int32_t* seq_lens, const int32_t* path,
                   const int32_t* n_accept, int B, int R, int Hkv, int D, int page, int max_depth,
                   int32_t* new_lens) {
  for (int b = 0; b < B; b++) {
    int L = seq_lens[b];
    int kept = 0;
    for (int j = 0; j <= n_accept[b] && j <= max_depth; j++) {
      int node = path[(size_t)b * (max_depth + 1) + j];
      int pos = L + j;
      if (pos >= max_pages * page) break;
      int pg = block_table[(size_t)b * max_pages + pos / page], slot = pos % page;
      for (int h = 0; h < Hkv; h++)
        for (int d = 0; d < D; d++) {
          size_t src = (((size_t)b * R + node) * Hkv + h) * D + d;
          k_cache[(((size_t)pg * Hkv + h) * page + slot) * D + d] = k_new[src];
          v_cache[(((size_t)pg * Hkv + h) * D + d) * page + slot] = v_new[src];
        }
      kept++;
    }
    if (new_lens) new_lens[b] = L + kept;
  }
}


/*
 * n3, page allocation (Appendix A.1: the cache grows by the accepted tokens after every generation step;
 * Sec. 3.2.1: only main-stream keys/values are cached).  Sequence b holds L = seq_lens[b] tokens in its
 * first ceil(L/page) logical pages; the accepted path adds the positions L .. L + n_accept[b].  Logical
 * pages those positions need beyond the mapped ones are taken from the top of a stack of free physical
 * pages, sequence after sequence in batch order, page after page in logical order, and written into the
 * block table.  A sequence stops growing at the table's capacity (max_pages*page tokens) or when the stack
 * is empty; n_commit[b] is then n_accept[b] clipped to the rows that have a page (-1: none).  *free_count
 * is lowered by the pages handed out.
 */
void ora_kv_alloc_pages(int32_t* block_table, int max_pages, const int32_t* seq_lens, const int32_t* n_accept,
                        int B, int page, int max_depth, const int32_t* free_pages, int32_t* free_count,
                        int32_t* n_commit) {
  int left = *free_count;
  for (int b = 0; b < B; b++) {
    int L = seq_lens[b];
    int acc = n_accept[b] > max_depth ? max_depth : n_accept[b];
    int mapped = (L + page - 1) / page; /* logical pages in use */
    int fit = -1;                       /* last path position that has a page */
    for (int j = 0; j <= acc; j++) {
      int lp = (L + j) / page;
      if (lp >= max_pages) break;
      if (lp >= mapped) {
        if (left == 0) break;
        block_table[(size_t)b * max_pages + lp] = free_pages[--left];
        mapped = lp + 1;
      }
      fit = j;
    }
    n_commit[b] = fit;
  }
  *free_count = left;
}

/*
 * n4 + n1 as one operation: the rows of Eq. 3 entering a dense map of the first multi-stream layer
 * (Sec. 3.1: queries, keys and values are H.W^Q, H.W^K, H.W^V of the rows' hidden states H).
 *   Y[b, r, v] = sum_e X[b, r, e] * W[v, e]   with X the rows of Eq. 3 (ora_stream_insert), never rounded:
 * the sum of Eq. 3 and the products are formed in double from the stored M, f(M), P and W.
 * Y [B,R,V] in the row order stated above.
 */
void ora_stream_insert_linear(const float* M, const float* fM, const float* P, const float* W, int B, int T,
                              int gamma, int d, int V, double* Y) {
  const int R = T * (1 + gamma);
  const float* src = fM ? fM : M;
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < B; b++)
    for (int r = 0; r < R; r++) {
      int i = r, j = 0; /* node, stream (0 = main row) */
      if (r >= T) {
        i = (r - T) / gamma;
        j = (r - T) % gamma + 1;
      }
      const float* m = (j == 0 ? M : src) + ((size_t)b * T + i) * d;
      for (int v = 0; v < V; v++) {
        double acc = 0.0;
        for (int e = 0; e < d; e++) {
          double x = (double)m[e];
          if (j > 0) x += (double)P[(size_t)(j - 1) * d + e];
          acc += x * (double)W[(size_t)v * d + e];
        }
        Y[((size_t)b * R + r) * V + v] = acc;
      }
    }
}
