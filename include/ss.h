/*
 * ss.h — C ABI of libss: the verify-and-speculate decode step of Speculative
 * Streaming (arXiv 2402.11131) on one AMD MI355X (gfx950).
 *
 * One decode step, as the paper states it (Sec. 3.2.2 and Appendix A.1): the
 * tree draft of the previous step is flattened into T main-stream rows, every
 * node carries gamma speculative-stream rows, the top N_s layers run
 * multi-stream attention (Eq. 1 for main rows, Eq. 2 for stream rows, tree mask
 * of Eq. 4 / the attention-mask figure of the appendix), the LM head turns the
 * last hidden states into logits, the longest draft path the main stream agrees
 * with is accepted, and the streams of the last accepted node give the next
 * tree draft.  The calls a1..a5 below are those pieces; n1..n4 are the rows
 * around them: the dense projections of a layer, the parallel tree-pruning layer
 * (Sec. 3.2.3), the commit of the accepted path to the KV cache (Appendix A.1)
 * and the insertion of the stream rows (Eq. 3).
 *
 * Conventions (all calls)
 *  - extern "C", plain pointers and sizes.  Unless a parameter says "host",
 *    every array is DEVICE memory owned by the caller; the library never frees
 *    or keeps it.  Outputs must not alias inputs.
 *  - Every call only enqueues work on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream).  No call synchronises with the device or reads
 *    device memory on the host, so the whole step can be chained on one stream.
 *  - Return value: SS_OK or an error code; ss_last_error() gives a thread-local
 *    message for the last failing call of the calling thread.  Argument, limit
 *    and workspace errors are found before anything is enqueued; SS_ERR_HIP
 *    reports a failed launch, and a call that consists of several kernels may
 *    then have enqueued the earlier ones.
 *  - Errors that only the device could see (a malformed parent array, a
 *    seq_len beyond the block table) cannot be reported by an asynchronous
 *    call; every kernel clamps such values so that all accesses stay in bounds
 *    and the result for that sequence is then unspecified but finite-time.
 *    ss_check_tree_host() validates a host copy of a tree.
 *
 * Row order inside one sequence (T tree nodes, gamma streams, R = T*(1+gamma)
 * rows; Sec. 3.2.3 gives the same count):
 *    main row of node i           r = i                          0 <= i < T
 *    stream j (1..gamma) of node i r = T + i*gamma + (j-1)
 * Node 0 is the root (the correction token of the previous step), parent[0] =
 * -1 and parent[i] < i.  Queries, the step's new keys/values and the LM-head
 * rows all use this order.
 */
#ifndef SS_H_
#define SS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define SS_OK 0
#define SS_ERR_INVALID_ARG 1 /* NULL pointer, non-positive size, bad stride     */
#define SS_ERR_UNSUPPORTED 2 /* dtype / head_dim / T / gamma / K outside limits */
#define SS_ERR_BAD_TREE 3    /* only from ss_check_tree_host                    */
#define SS_ERR_WORKSPACE 4   /* workspace NULL or smaller than *_workspace_bytes */
#define SS_ERR_HIP 5         /* a HIP runtime call failed at launch             */

/* element types of the floating-point tensors */
#define SS_F32 0
#define SS_BF16 1

/* limits */
#define SS_MAX_T 64     /* tree nodes per sequence (ancestor sets are 64-bit) */
#define SS_MAX_GAMMA 8  /* speculative streams per node                       */
#define SS_MAX_K 8      /* top-k width                                        */

/* flags of ss_build_mask / ss_msa_attention.
 * Eq. 2 lets stream j attend to streams 1..j of its own node (itself
 * included); with SS_STREAM_EXCLUDE_SELF it sees streams 1..j-1 only. */
#define SS_STREAM_EXCLUDE_SELF 1u
/* ss_msa_attention only, for profiling: run the attention kernel but not the
 * kernel that merges the KV splits; `out` is then left unwritten whenever the
 * problem is split (the per-split partial results stay in the workspace). */
#define SS_MSA_PARTIALS_ONLY 2u
/* ... and its counterpart: run only the kernel that merges the KV splits, on the
 * partial results a call with SS_MSA_PARTIALS_ONLY left in the same workspace
 * (same arguments).  A no-op when the problem is not split.  The two flags
 * together make one full call in two steps, so that a profiler or a pair of
 * events can bracket the attention kernel alone inside a real step. */
#define SS_MSA_MERGE_ONLY 4u

/* Library version (major*100 + minor). */
int ss_version(void);

/* Message of the last error on the calling thread ("" if none). */
const char* ss_last_error(void);

/*
 * Measurement aid (no part of the method): one pass of plain 16-byte loads
 * over DEVICE memory at `buf` (16-byte aligned), `bytes` rounded down to a
 * multiple of 32 MiB (at least that much is required), with the streaming
 * (non-temporal) hint if `streaming` is non-zero; nothing is written (`sink`,
 * 4 bytes of device memory, only keeps the loads alive).
 * Timed over a buffer larger than the last-level cache it gives the read rate
 * this GPU reaches, the practical ceiling next to the published HBM peak.
 */
int ss_probe_hbm_read(const void* buf, size_t bytes, int streaming, void* sink, void* stream);

/*
 * Measurement aid (no part of the method): 2048 wavefronts (two per SIMD of a
 * 256-unit GPU) each issue 20*iters bf16 matrix-core instructions of shape
 * 32x32x16 on registers only, five independent accumulator tiles per wave;
 * nothing is loaded or stored (`sink`, 4 bytes of device memory, only keeps
 * the results alive).  *flops (HOST, may be NULL) receives the floating-point
 * operations of the launch.  Timed, it gives the matrix-core rate the GPU
 * sustains at the clock it grants, next to the published peak.
 */
int ss_probe_mfma_bf16(int iters, double* flops, void* sink, void* stream);

/*
 * Host-side check of B trees: parent[b*T+0] == -1, 0 <= parent[b*T+i] < i, and
 * (if max_depth >= 0) depth <= max_depth.  `parent` is HOST memory.
 * Returns SS_OK or SS_ERR_BAD_TREE (message names the first offending entry).
 */
int ss_check_tree_host(const int32_t* parent, int B, int T, int max_depth);

/*
 * a1. Mask construction (Sec. 3.2.2 Eq. 4 with the reading of the appendix
 * attention-mask figure: a node attends to every predecessor from the root and
 * to itself; Eq. 1/Eq. 2 for which stream sees which).
 *
 * For each of B sequences with parent[b, 0..T): depth[i] (root 0), anc[i] = bit
 * set of the nodes on the root->i path (bit i included), and the boolean mask
 * over the step's own R x R block: row (i,j) may attend key (i',j') iff
 *    j' == 0 and i' is an ancestor-or-self of i                (main keys)
 * or j  > 0 and j' > 0 and i' == i and j' <= j                 (own streams;
 *                                    j' < j with SS_STREAM_EXCLUDE_SELF)
 * (j = 0 is the main row).  Prefix keys in the KV cache are visible to every
 * row and are not part of this matrix.
 *
 *  parent [B,T] int32 in;  mask [B,R,R] uint8 out (1 = may attend), may be NULL;
 *  anc [B,T] uint64 out or NULL;  depth [B,T] int32 out or NULL.
 * Limits: 1 <= T <= SS_MAX_T, 0 <= gamma <= SS_MAX_GAMMA.
 * Node 0 is always taken as the root; for i > 0 an entry parent[i] outside
 * [0, i) is treated as 0 (see "Conventions").  All calls that read a parent
 * array apply this rule.
 */
int ss_build_mask(const int32_t* parent, int B, int T, int gamma, uint32_t flags,
                  uint8_t* mask, uint64_t* anc, int32_t* depth, void* stream);

/*
 * a2. Multi-stream attention for one MSA layer (Eq. 1, Eq. 2, mask as in a1):
 * for every sequence b, row r and query head h (KV head h / (H/Hkv)),
 *    out[b,r,h,:] = softmax_c( scale * <q[b,r,h,:], K_c> + mask[r,c] ) . V_c
 * over the keys c = the first seq_lens[b] cached main-stream tokens of the
 * sequence (all visible) followed by the step's R new rows (masked as in a1).
 * Stream keys/values are never cached (Sec. 3.2.1): they exist only in
 * k_new / v_new.
 *
 *  q      [B,R,H,D]      k_new, v_new [B,R,Hkv,D]      out [B,R,H,D]
 *  k_cache [num_pages, Hkv, page_size, D]   token-major pages
 *  v_cache [num_pages, Hkv, D, page_size]   feature-major pages: the value of
 *          token s of a page, feature d, sits at [page, hkv, d, s]
 *  block_table [B, max_pages_per_seq] int32: physical page of logical page p,
 *          in [0, num_pages); entries outside that range are clamped on device
 *          (num_pages = first extent of k_cache / v_cache; bf16: each cache at
 *          most 1 TiB, else SS_ERR_UNSUPPORTED)
 *  seq_lens [B] int32: cached tokens per sequence, 0 <= seq_lens[b] <=
 *          max_pages_per_seq*page_size (larger values are clamped on device)
 *  parent [B,T] int32 as in a1.
 * dtype: SS_F32 (all of q,k,v,out fp32) or SS_BF16 (bf16 storage, fp32 scores,
 * softmax and accumulation; the probabilities are rounded to bf16 where they
 * enter the product with V, and the softmax denominator is the fp32 sum of
 * those rounded probabilities).  Limits: D in {64,128}, page_size in {16,32,64}, H % Hkv
 * == 0, T <= SS_MAX_T, gamma <= SS_MAX_GAMMA.  scale is the factor applied to
 * the dot products (1/sqrt(D) in the paper's MHA).
 * workspace: device scratch of at least ss_msa_workspace_bytes(...) bytes with
 * max_seq_len = max_pages_per_seq*page_size.  It holds the per-split partial
 * results and, when two splits are merged inside the attention kernel (see
 * ss_msa_set_merge_in_kernel), their arrival counters.  The counters must be
 * ZERO when a call is enqueued and every call leaves them zero: fill a new
 * workspace with zeros once (ss_msa_workspace_init, or any memset) and it can
 * be used for any number of calls of any shape it is large enough for.  A
 * workspace that was never zeroed gives wrong results for split problems, with
 * no error.  Calls that may run at the same time (different streams, graphs
 * replayed on different streams) need a workspace each; calls that follow each
 * other on one stream can share one.  The library keeps nothing between calls.
 */
size_t ss_msa_workspace_bytes(int B, int T, int gamma, int H, int Hkv, int D, int max_seq_len,
                              int dtype);
/* Fills `workspace_bytes` bytes of device memory at `workspace` with zeros by a
 * kernel on `stream` (safe inside a stream capture). */
int ss_msa_workspace_init(void* workspace, size_t workspace_bytes, void* stream);
int ss_msa_attention(const void* q, const void* k_new, const void* v_new, const void* k_cache,
                     const void* v_cache, const int32_t* block_table, int max_pages_per_seq,
                     int num_pages, const int32_t* seq_lens, const int32_t* parent, int B, int T,
                     int gamma, int H, int Hkv, int D, int page_size, float scale, int dtype,
                     uint32_t flags, void* out, void* workspace, size_t workspace_bytes,
                     void* stream);

/*
 * a2 for callers that cannot allocate device memory (code under HIP graph
 * capture that owns no buffers, tight serving loops, harnesses that forbid
 * hipMalloc): ss_msa_attention without the workspace arguments.  The partial
 * results and arrival counters live in an array of
 * ss_msa_static_scratch_bytes() = 32 MiB that is part of the library's device
 * code; every GPU the library is used on holds its own copy until the process
 * ends.  The call allocates and frees nothing.  The first call on a device
 * looks the array's address up (the device that is current in the calling
 * thread must be the one `stream` belongs to).  The counters are cleared by a
 * small kernel at the start of every call; the rest of the array keeps what the
 * last call left there.  All calls on one GPU share the array: calls that
 * overlap in time (different streams, graph replays on different streams) RACE
 * and give wrong results; enqueue them on one stream or use ss_msa_attention.
 * Results are those of ss_msa_attention, bit for bit.
 * Errors: those of ss_msa_attention; SS_ERR_UNSUPPORTED if the shape needs more
 * than the array holds (ss_msa_workspace_bytes tells the need), nothing is
 * enqueued then.
 */
size_t ss_msa_static_scratch_bytes(void);
int ss_msa_attention_static(const void* q, const void* k_new, const void* v_new,
                            const void* k_cache, const void* v_cache, const int32_t* block_table,
                            int max_pages_per_seq, int num_pages, const int32_t* seq_lens,
                            const int32_t* parent, int B, int T, int gamma, int H, int Hkv, int D,
                            int page_size, float scale, int dtype, uint32_t flags, void* out,
                            void* stream);

/*
 * What a full call of a2 with this shape will launch, as currently tuned:
 * *n_splits = number of splits of the cached prefix (1 = unsplit, no workspace
 * needed), *n_kernels = 1 if the call is a single kernel (unsplit, or two
 * splits merged inside the attention kernel), 2 if a merge kernel follows.
 * Either pointer may be NULL.  Host-only, no GPU work.  Returns SS_OK or the
 * error ss_msa_attention would return for the shape.
 */
int ss_msa_plan(int B, int T, int gamma, int H, int Hkv, int D, int max_seq_len, int dtype,
                int* n_splits, int* n_kernels);

/*
 * Tuning knob for a2: number of cached tokens one workgroup scans (the KV
 * split length).  0 = choose from the problem shape (default).  Values below
 * 64 count as 64, and values are rounded up to a multiple of 32 (SS_BF16) or
 * 64 (SS_F32).  The result of a2 does not depend on it
 * beyond floating-point rounding.  Returns the previous setting.
 */
int ss_msa_set_split_keys(int split_keys);

/*
 * Tuning knob for a2 (MFMA path, problems split in two): merge the two splits
 * inside the attention kernel instead of in a second kernel (default: on).  The
 * split that finishes second adds the other's partial rows to its own and writes
 * `out`; the arithmetic is that of the merge kernel, so the result is the same
 * bit for bit and does not depend on which split finishes first.  The splits
 * find each other through arrival counters at the end of the call's workspace
 * (see a2 for the zero-fill rule).  Returns the previous setting.
 */
int ss_msa_set_merge_in_kernel(int on);

/*
 * a3. LM head with fused argmax / top-K (Sec. 3.2.1: the last layer's main row
 * predicts y_t, stream j predicts y_{t+j}; Sec. 3.2.2: top-k tokens per stream).
 *    z[n,v] = sum_d hidden[n,d] * W[v,d]          (never written to memory)
 *    idx[n,0..K) = the K largest z[n,:] in decreasing order, ties -> lower v;
 *    val[n,0..K) = those logits (fp32).  The SS_BF16 path selects on the fp32
 *    logits with their five lowest mantissa bits set aside (2^-18 of a logit's
 *    magnitude): logits closer than that are ordered by token id, and val
 *    carries those five bits cleared.
 *  hidden [N,d], W [V,d] (dtype SS_F32 or SS_BF16), idx [N,K] int32, val [N,K] f32.
 * Limits: 1 <= K <= SS_MAX_K, K <= V, d % 64 == 0 for SS_BF16.
 * workspace: at least ss_lm_head_workspace_bytes(...) bytes.
 */
size_t ss_lm_head_workspace_bytes(int N, int d, int V, int K, int dtype);
int ss_lm_head_argmax_topk(const void* hidden, const void* W, int N, int d, int V, int K, int dtype,
                           int32_t* idx, float* val, void* workspace, size_t workspace_bytes,
                           void* stream);

/*
 * Tuning knobs for a3 / n1 / n2 (bf16 path), never needed for normal use; results
 * do not depend on them beyond floating-point summation order.
 * ss_lm_set_flavour: the kernel shape of the LM head and log-sum-exp (linear ==
 *  0) or of ss_linear_rows (linear != 0): row_tiles tiles of 32 rows per workgroup
 *  with the 4-wave kernel (wide == 0, 1..6 tiles) or the 8-wave kernel (wide != 0,
 *  1..5 tiles); row_tiles outside that range = choose from the shape (default).
 * ss_lm_set_stagger: feature blocks between the starting blocks of neighbouring
 *  vocabulary tiles, 0..1024; negative = automatic (default).
 * Both return the previous setting.  Initial values can be given by the
 * environment variables SS_LM_FLAVOUR / SS_LINEAR_FLAVOUR ("3" or "3w") and
 * SS_LM_STAGGER, which are read once per process.
 * ss_lm_set_candidates_only: a profiling aid like SS_MSA_PARTIALS_ONLY.  While
 *  it is on, ss_lm_head_argmax_topk (and its _live form) stops after the matrix
 *  kernel that leaves K candidates per row and vocabulary tile in the workspace:
 *  idx and val are NOT written.  Returns the previous setting; off by default.
 */
int ss_lm_set_flavour(int linear, int row_tiles, int wide);
int ss_lm_set_stagger(int blocks);
int ss_lm_set_candidates_only(int on);

/*
 * n1. Dense projection of the step's rows (Sec. 3.1: queries, keys and values
 * are H.W^Q, H.W^K, H.W^V of the hidden states H of main and stream rows; the
 * output projection and the feed-forward maps of a layer have the same form):
 *    y[n,v] = sum_e x[n,e] * W[v,e]
 *  x [N,d], W [V,d] (one output feature per row), y [N,V]; all device memory of
 *  type dtype (SS_F32 or SS_BF16), row-major, contiguous.  Products are
 *  accumulated in fp32; a bf16 result is rounded to nearest even once.
 *  It runs the main loop of a3 with a store in place of the search, so the same
 *  limits hold: d % 64 == 0 for SS_BF16, x and W below 2^30 elements; rows of y
 *  leave in 16-byte pieces when V % 8 == 0 (any V is accepted).
 * y must not overlap x or W.  N == 0 is a no-op.  No workspace.
 */
int ss_linear_rows(const void* x, const void* W, int N, int d, int V, int dtype, void* y,
                   void* stream);

/*
 * n1 with a workspace.  The same map as ss_linear_rows; with scratch memory at
 * hand a bf16 map with few outputs and many features (a layer's down and output
 * maps) is cut along the feature dimension: ss_linear_rows_splits(...) slices of
 * d run as workgroups of their own, leave fp32 partial products [slices,N,V] in
 * the workspace, and a second kernel adds them in slice order and rounds once.
 * The result differs from ss_linear_rows only by the order of the fp32 sum.
 *  workspace: device scratch of at least ss_linear_rows_workspace_bytes(...)
 *  bytes (any contents; 256 when the shape is not cut, and then it is not used).
 * Errors as ss_linear_rows, and SS_ERR_WORKSPACE.  SS_F32 runs ss_linear_rows.
 */
size_t ss_linear_rows_workspace_bytes(int N, int d, int V, int dtype);
int ss_linear_rows_splits(int N, int d, int V, int dtype);
int ss_linear_rows_ws(const void* x, const void* W, int N, int d, int V, int dtype, void* y,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * n4. Stream insertion (Eq. 3): the rows of a step as they enter the first
 * multi-stream layer, from the main-stream hidden states of the tree nodes.
 *    X[b, i]                 = M[b,i]                 main row of node i
 *    X[b, T + i*gamma + j-1] = f(M)[b,i] + P[j-1]     stream j = 1..gamma of node i
 *  M [B,T,d]; fM [B,T,d] = f(M), or NULL for the identity (the paper's
 *  experiments; a rank-eta f is two ss_linear_rows calls); P [gamma,d] stream
 *  identifier embeddings; X [B,R,d] with R = T*(1+gamma) in the row order of this
 *  header.  All device memory of type dtype, contiguous.  Sums are formed in
 *  fp32 and rounded once.  X must not overlap the inputs.  B == 0 is a no-op;
 *  with gamma == 0 P may be NULL.
 */
int ss_stream_insert(const void* M, const void* fM, const void* P, int B, int T, int gamma, int d,
                     int dtype, void* X, void* stream);

/*
 * n4 + n1 as one call: the rows of Eq. 3 through a dense map of the first
 * multi-stream layer (Sec. 3.1: queries, keys and values are H.W^Q, H.W^K, H.W^V
 * of the rows' hidden states), without ever forming the rows:
 *    Y[b, i]                 = M[b,i] . W^T
 *    Y[b, T + i*gamma + j-1] = (f(M)[b,i] + P[j-1]) . W^T = f(M)[b,i].W^T + P[j-1].W^T
 * The map is linear, so it is applied to the B*T main-stream states (twice if
 * fM is given) and the gamma embeddings in ONE pass over W, 1+gamma times fewer
 * rows than the step has, and the step's rows are sums of those results.
 *  M, fM (or NULL = identity), P as for ss_stream_insert; W [V,d]; Y [B,R,V];
 *  all of type dtype.  Limits of ss_linear_rows (d % 64 == 0 for SS_BF16).
 *  The three partial results are rounded to dtype before they are added (bf16:
 *  at most three roundings of 2^-9 per element instead of the one of
 *  ss_stream_insert + ss_linear_rows, which rounds the rows instead).
 *  workspace: at least ss_stream_insert_linear_workspace_bytes(...) bytes
 *  (with_f != 0 if fM is given).  Three kernels on `stream`.
 */
size_t ss_stream_insert_linear_workspace_bytes(int B, int T, int gamma, int d, int V, int dtype,
                                               int with_f);
int ss_stream_insert_linear(const void* M, const void* fM, const void* P, const void* W, int B, int T,
                            int gamma, int d, int V, int dtype, void* Y, void* workspace,
                            size_t workspace_bytes, void* stream);

/*
 * Value rotation, the appendix's alternative to stream embeddings (ablation
 * "Value Rotation"): streams start from the main-stream state (ss_stream_insert
 * with P = 0) and, in every multi-stream layer, the value projection of stream n
 * of a node is the main stream's value projection of that node times
 * e^{i*eps*n}, n = 1..gamma.  Features (2m, 2m+1) of a head are taken as (Re, Im)
 * of one complex number and every pair turns by the same angle eps*n:
 *    v[b, T + i*gamma + n-1, h, 2m  ] = re*cos(eps n) - im*sin(eps n)
 *    v[b, T + i*gamma + n-1, h, 2m+1] = re*sin(eps n) + im*cos(eps n)
 *  with (re, im) = v[b, i, h, 2m], v[b, i, h, 2m+1] (main row of node i).
 *  v_new [B,R,Hkv,D] of type dtype, the value block of the step handed to
 *  ss_msa_attention, updated IN PLACE: main rows are read, stream rows written
 *  (what they held is ignored).  eps: 0 <= eps <= pi/(2N) in the paper, any
 *  value accepted; cos and sin are taken in double on the host.  Products in
 *  fp32, a bf16 result rounded once.  D must be even.  B == 0 or gamma == 0 is
 *  a no-op.
 */
int ss_value_rotate(void* v_new, int B, int T, int gamma, int Hkv, int D, float eps, int dtype,
                    void* stream);

/*
 * n2. Parallel tree pruning (Sec. 3.2.3; Appendix A.1 and its generation-step
 * figure).  Early-exit logits of node i are zt_i = H(o(M_i)): the LM head H = W
 * applied to the main-stream hidden state after the low-rank map o (two
 * ss_linear_rows calls).  The transition probability between a parent p and its
 * child c is the softmax of zt_p at the child's token; a child below the
 * threshold is pruned with its sub-tree.  Three calls:
 *
 * ss_lm_head_logsumexp: lse[n] = log sum_v exp(sum_e hidden[n,e]*W[v,e]); the
 *  logits never reach memory (a3's loop with another epilogue; same limits and
 *  the workspace of ss_lm_head_workspace_bytes(N, d, V, 1, dtype)).
 *  hidden [N,d], W [V,d] of type dtype; lse [N] f32.
 *
 * ss_transition_probs: prob[b,0] = 1; for i > 0, with p = parent[b,i] (clamped
 *  as everywhere) and c = tok[b,i]:
 *     prob[b,i] = exp(sum_e h[b,p,e]*W[c,e] - lse[b*T + p]),  0 if c is outside [0,V).
 *  h [B,T,d] = o(M) of the tree nodes (the rows ss_lm_head_logsumexp was given,
 *  N = B*T), W [V,d], tok/parent [B,T] int32, lse [B*T] f32, prob [B,T] f32.
 *
 * ss_tree_prune: keep[b,0] = 1, keep[b,i] = keep[b,p] and not (prob[b,i] <
 *  threshold), compared in single precision.  Kept nodes keep their order and are
 *  renumbered 0..n-1: new_tok, new_parent (in new numbers, -1 for the root),
 *  old_index (the node's number before).  Entries n..T-1 are padding: new_tok -1
 *  (it matches no prediction, so ss_tree_verify never accepts it), new_parent 0,
 *  old_index -1.  n_nodes[b] = n.  All arrays [B,T] int32 except n_nodes [B];
 *  outputs must not alias inputs.  The padded tree is a valid input of every
 *  other call of this header: rows of padding nodes are computed and ignored.
 * All pointers are device memory.  B == 0 / N == 0 are no-ops.
 */
int ss_lm_head_logsumexp(const void* hidden, const void* W, int N, int d, int V, int dtype, float* lse,
                         void* workspace, size_t workspace_bytes, void* stream);
int ss_transition_probs(const void* h, const void* W, const int32_t* tok, const int32_t* parent,
                        const float* lse, int B, int T, int d, int V, int dtype, float* prob,
                        void* stream);
int ss_tree_prune(const int32_t* tok, const int32_t* parent, const float* prob, float threshold, int B,
                  int T, int32_t* keep, int32_t* new_tok, int32_t* new_parent, int32_t* old_index,
                  int32_t* n_nodes, void* stream);

/*
 * a4. Greedy ("hard matching") tree verification (Sec. 3.2.2, Appendix A.1):
 * the root is always accepted; node i is accepted iff its parent is accepted
 * and tok[i] equals the main-stream argmax token at its parent.  `last` is the
 * accepted node of greatest depth (ties -> lowest node index), n_accept its
 * depth (the number of accepted draft tokens, 0..max_depth), bonus the argmax
 * token at `last` (the correction token, next step's root).
 *
 *  tok, parent [B,T] int32 in.
 *  main_argmax: argmax token of main row i of sequence b at element
 *          main_argmax[b*argmax_batch_stride + i*argmax_node_stride]
 *          (so idx of a3 can be passed with strides R*K and K).
 *  n_accept, last, bonus [B] int32 out.
 *  path       [B, max_depth+1] int32 out: node ids root..last, then -1.
 *  out_tokens [B, max_depth+1] int32 out: tok of path[1..n_accept], then
 *          bonus, then -1: the n_accept+1 tokens this step emits.
 * Nodes deeper than max_depth are never accepted.  0 <= max_depth < SS_MAX_T.
 */
int ss_tree_verify(const int32_t* tok, const int32_t* parent, const int32_t* main_argmax,
                   long argmax_batch_stride, long argmax_node_stride, int B, int T, int max_depth,
                   int32_t* n_accept, int32_t* last, int32_t* bonus, int32_t* path,
                   int32_t* out_tokens, void* stream);

/*
 * a5. Top-k tree drafting (Sec. 3.2.2; Appendix A.1): the next tree has a
 * static shape (the template), only its tokens change.  Template node 0 is the
 * root; node i > 0 has parent tmpl_parent[i] < i, depth dep(i) in 1..gamma and
 * rank tmpl_rank[i] in [0,K):
 *    next_tok[b,0] = bonus[b]
 *    next_tok[b,i] = stream_topk[b, last[b], dep(i)-1, tmpl_rank[i]]
 * i.e. level j of the tree holds top-k tokens of stream j of the last accepted
 * node, and tokens of stream j are predecessors of those of stream j+1.
 *
 *  stream_topk: top-K token ids of stream j (1..gamma) of node i of sequence b
 *          at stream_topk[b*topk_batch_stride + ((i*gamma)+(j-1))*K + rank]
 *          (idx of a3 offset by T*K elements, batch stride R*K).
 *  last, bonus [B] int32 (outputs of a4).
 *  Template, one of:
 *    tmpl_parent, tmpl_rank [T2] int32 DEVICE arrays, or
 *    both NULL and branching [gamma] int32 HOST array: the full tree with
 *    branching[j-1] children per level-(j-1) node, nodes numbered level by
 *    level, within a level by (parent, rank); then T2 must equal
 *    1 + sum_j prod_{m<=j} branching[m-1]  (uniform k: 1 + sum_g k^g, Sec. 3.2.3).
 *  next_tok [B,T2] int32 out;  next_parent [T2] int32 out or NULL (the template's
 *  parent array, the `parent` input of the next step).
 * A template entry with depth > gamma or rank outside [0,K) yields token -1.
 * Limits: 1 <= T2 <= SS_MAX_T, gamma <= SS_MAX_GAMMA, K <= SS_MAX_K.
 */
int ss_tree_draft(const int32_t* stream_topk, long topk_batch_stride, int K, const int32_t* last,
                  const int32_t* bonus, const int32_t* tmpl_parent, const int32_t* tmpl_rank,
                  const int32_t* branching, int B, int T, int gamma, int T2, int32_t* next_tok,
                  int32_t* next_parent, void* stream);

/*
 * a3 + a4 + a5 in one call: the tail of a decode step (Sec. 3.2.1, 3.2.2,
 * Appendix A.1) in two kernels instead of four.  `hidden` holds the last
 * layer's rows of B sequences, R = T*(1+gamma) rows each: the main row of node
 * i at row i, stream j (1..gamma) of node i at row T + i*gamma + (j-1).  The
 * result equals ss_lm_head_argmax_topk on all B*R rows, then ss_tree_verify
 * on the main rows' arg-max, then ss_tree_draft on the stream rows' top-K;
 * the merge of the per-tile candidates is done only for the rows those two
 * steps read (the T main rows; the gamma stream rows of the last accepted
 * node), inside the kernel that verifies and drafts.
 *  hidden [B*R,d], W [V,d], dtype, K: as for a3 (K = width of the draft).
 *  tok, parent [B,T]; max_depth; n_accept, last, bonus [B]; path, out_tokens
 *  [B,max_depth+1]: as for a4.
 *  tmpl_parent, tmpl_rank (DEVICE) or branching (HOST), T2, next_tok [B,T2],
 *  next_parent [T2] or NULL: as for a5.
 *  main_argmax [B,T] int32 out or NULL: the main rows' arg-max tokens.
 *  workspace: at least ss_lm_head_workspace_bytes(B*R, d, V, K, dtype) bytes.
 * Limits and errors: those of a3, a4 and a5.
 */
int ss_lm_head_verify_draft(const void* hidden, const void* W, int d, int V, int K, int dtype,
                            const int32_t* tok, const int32_t* parent, int B, int T, int gamma,
                            int max_depth, const int32_t* tmpl_parent, const int32_t* tmpl_rank,
                            const int32_t* branching, int T2, int32_t* n_accept, int32_t* last,
                            int32_t* bonus, int32_t* path, int32_t* out_tokens, int32_t* next_tok,
                            int32_t* next_parent, int32_t* main_argmax, void* workspace,
                            size_t workspace_bytes, void* stream);

/*
 * Host helper for a5: writes the full-tree template described above into HOST
 * arrays parent_out/rank_out/depth_out (each [T2] or NULL) and returns the node
 * count, or -1 if it would exceed `capacity` or SS_MAX_T.  All pointers HOST.
 */
int ss_full_tree_template_host(const int32_t* branching, int gamma, int capacity,
                               int32_t* parent_out, int32_t* rank_out, int32_t* depth_out);

/*
 * n3. KV-cache commit after verification (Sec. 3.2.1: main-stream keys/values
 * are cached, those of the speculative streams never are; Appendix A.1: the
 * cache is backtracked lazily after each generation step).  Of the step's own
 * rows only the main rows of the accepted path stay: the key/value row of node
 * path[b][j], j = 0..n_accept[b], is appended at position seq_lens[b] + j of
 * sequence b's paged cache; everything else of k_new/v_new is dropped.  One call
 * per layer (each layer has its own caches and its own k_new/v_new).
 *
 *  k_new, v_new [B,R,Hkv,D] in (row order as above, R = T*(1+gamma)).
 *  k_cache [num_pages,Hkv,page_size,D], v_cache [num_pages,Hkv,D,page_size]
 *          in/out, layouts as in a2.
 *  block_table [B,max_pages_per_seq], seq_lens [B] in.  The table must map the
 *          positions that are written; a position at or past
 *          max_pages_per_seq*page_size is dropped (with all that follow it).
 *  path [B,max_depth+1], n_accept [B] in: as ss_tree_verify returns them.
 *  new_seq_lens [B] int32 out, or NULL: seq_lens[b] + number of rows appended
 *          (n_accept[b] + 1 unless the table's capacity cut it).  Must not be
 *          the seq_lens array itself.
 * Node ids outside [0,T) and page ids outside [0,num_pages) are clamped into
 * range, n_accept above max_depth counts as max_depth, and a negative n_accept
 * means that nothing of that sequence is appended (new_seq_lens[b] =
 * seq_lens[b]): what ss_kv_alloc_pages reports for a sequence without a page.
 */
int ss_kv_commit(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                 const int32_t* block_table, int max_pages_per_seq, int num_pages,
                 const int32_t* seq_lens, const int32_t* path, const int32_t* n_accept, int B, int T,
                 int gamma, int Hkv, int D, int page_size, int max_depth, int dtype,
                 int32_t* new_seq_lens, void* stream);

/*
 * n2, making pruning pay (Sec. 3.2.3: pruning exists to keep the step from
 * becoming compute-bound).  After ss_tree_prune sequence b keeps the nodes
 * 0 .. n_nodes[b]-1 of its compacted tree and the arrays are padded back to T
 * nodes; the calls below take n_nodes (or the list of kept rows made from it)
 * and do not compute the rows of padding nodes.  Everything stays on the device:
 * no call needs the counts on the host.
 *
 * ss_live_rows: live_rows[0 .. *n_live) = the rows b*R + r, ascending, of the
 *  kept nodes (main row r = i, stream rows r = T + i*gamma + j-1 for i <
 *  n_nodes[b], clamped to [1,T]); live_rows [B*R] int32, n_live [1] int32.
 *
 * ss_msa_attention_pruned: ss_msa_attention with n_nodes [B]: the rows of
 *  padding nodes are neither computed nor written (`out` keeps what it held
 *  there); the kept rows are packed into the first row chunks of a launch, so
 *  that whole workgroups leave at once; kept rows are those of
 *  ss_msa_attention up to floating-point summation order (padding nodes hang
 *  off the root, so no kept row attends to them).
 *
 * ss_linear_rows_live, ss_lm_head_argmax_topk_live, ss_lm_head_verify_draft_live:
 *  the calls without the suffix, computing only the rows listed in live_rows
 *  (device, ascending, *n_live of them) and leaving every other row of their
 *  outputs untouched.  plan_rows (HOST) is the number of rows the launch is
 *  shaped for: 0 = all N; a smaller number, e.g. what a serving loop expects to
 *  survive pruning, lets fewer, fuller workgroups do the work; if more rows turn
 *  out to be listed than planned for, workgroups take several row chunks in turn
 *  (slower, never wrong).
 */
int ss_live_rows(const int32_t* n_nodes, int B, int T, int gamma, int32_t* live_rows, int32_t* n_live,
                 void* stream);
int ss_msa_attention_pruned(const void* q, const void* k_new, const void* v_new, const void* k_cache,
                            const void* v_cache, const int32_t* block_table, int max_pages_per_seq,
                            int num_pages, const int32_t* seq_lens, const int32_t* parent,
                            const int32_t* n_nodes, int B, int T, int gamma, int H, int Hkv, int D,
                            int page_size, float scale, int dtype, uint32_t flags, void* out,
                            void* workspace, size_t workspace_bytes, void* stream);
int ss_linear_rows_live(const void* x, const void* W, int N, int d, int V, int dtype, void* y,
                        const int32_t* live_rows, const int32_t* n_live, int plan_rows, void* stream);
int ss_lm_head_argmax_topk_live(const void* hidden, const void* W, int N, int d, int V, int K, int dtype,
                                int32_t* idx, float* val, const int32_t* live_rows,
                                const int32_t* n_live, int plan_rows, void* workspace,
                                size_t workspace_bytes, void* stream);
int ss_lm_head_verify_draft_live(const void* hidden, const void* W, int d, int V, int K, int dtype,
                                 const int32_t* tok, const int32_t* parent, int B, int T, int gamma,
                                 int max_depth, const int32_t* tmpl_parent, const int32_t* tmpl_rank,
                                 const int32_t* branching, int T2, int32_t* n_accept, int32_t* last,
                                 int32_t* bonus, int32_t* path, int32_t* out_tokens, int32_t* next_tok,
                                 int32_t* next_parent, int32_t* main_argmax, const int32_t* live_rows,
                                 const int32_t* n_live, int plan_rows, void* workspace,
                                 size_t workspace_bytes, void* stream);

/*
 * n3, page allocation (Appendix A.1: the cache grows by the accepted tokens
 * after every generation step).  Sequence b uses the first
 * ceil(seq_lens[b]/page_size) entries of its block-table row; its accepted path
 * adds the positions seq_lens[b] .. seq_lens[b] + n_accept[b].  The logical
 * pages those positions need beyond the ones in use are taken from the top of a
 * stack of free physical pages and written into block_table: sequences are
 * served in batch order, pages in logical order, so the result is that of a
 * sequential allocator and does not depend on scheduling.  One call per step
 * serves all layers when they share one table (each layer's caches are indexed
 * by the same page ids); ss_kv_commit per layer follows with n_commit in place
 * of n_accept.
 *
 *  block_table [B,max_pages_per_seq] int32 in/out.
 *  seq_lens, n_accept [B] int32 in (n_accept as ss_tree_verify returns it;
 *          values above max_depth count as max_depth, negative = no rows).
 *  free_pages [*free_count ..] int32 in: the stack, top at index *free_count-1.
 *  free_count [1] int32 in/out (DEVICE): lowered by the pages handed out.
 *  n_commit [B] int32 out: n_accept[b] clipped to the path rows that have a
 *          page; smaller than n_accept[b] when the table's capacity
 *          (max_pages_per_seq*page_size tokens) or an empty stack stopped the
 *          sequence; -1 when not even the first row has one.
 * One small kernel on `stream`; B == 0 is a no-op.  Calls that share a stack must
 * follow each other on one stream.
 */
int ss_kv_alloc_pages(int32_t* block_table, int max_pages_per_seq, const int32_t* seq_lens,
                      const int32_t* n_accept, int B, int page_size, int max_depth,
                      const int32_t* free_pages, int32_t* free_count, int32_t* n_commit,
                      void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SS_H_ */
