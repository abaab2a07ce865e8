/*
 * medusa.h -- C ABI of the MI355X (gfx950) hot path of one Medusa verification step
 * (Cai et al., "Medusa: Simple LLM Inference Acceleration Framework with Multiple
 * Decoding Heads", arXiv 2401.10774).
 *
 * One decoding step (Sec. 2, opening paragraph; Fig. 1) is
 *   (1) candidate generation : medusa_heads, medusa_topk_tree      (Sec. 2.1.1, 2.1.2)
 *   (2) candidate processing : tree_attention (+ medusa_heads with w1 == NULL for the
 *                              original model's logits at every tree token)  (Sec. 2.1.2)
 *   (3) candidate acceptance : medusa_accept                        (Sec. 2.3.1)
 *   carry-over               : kv_commit                            (Fig. 1 caption)
 *
 * Conventions shared by every call
 *   - Every tensor pointer is DEVICE memory owned by the caller, dense, innermost
 *     dimension contiguous, in the layout written next to the argument.  The library
 *     never allocates, frees or retains caller memory.  The only object it owns is
 *     medusa_tree_t (small host + device tables).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue their kernels on it and return without synchronising.
 *   - Return value: MEDUSA_OK (0) or a negative medusa_status_t.  Arguments are checked
 *     on the host before anything is launched; on error nothing is enqueued.  Contents of
 *     device arrays (e.g. prefix_len) cannot be checked on the host: the kernels clamp
 *     every index they derive from device data, so bad contents give wrong rows, never an
 *     out-of-bounds access.
 *   - medusa_topk_tree, the medusa_accept family, kv_commit and the split reductions of tree_linear
 *     elect the last workgroup of a launch with ticket counters in device memory of the library (they
 *     return to zero when a launch completes).  The library keeps 16 sets of them and gives every
 *     stream it sees a set of its own, in order of first use: calls on different streams may overlap;
 *     from the 17th distinct stream of a process on, streams share the last set and calls of the same
 *     entry point on those must not overlap.  Batch size B <= 4096 for these calls.
 *   - dtype is the storage type of activations, weights and KV: MEDUSA_F32 or
 *     MEDUSA_BF16.  Accumulation is always fp32; logits are always fp32.
 *   - Ties in arg-max / top-k: larger value first, then lower token id.  NaN logits are
 *     outside the contract.
 */
#ifndef MEDUSA_H_
#define MEDUSA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MEDUSA_OK = 0,
  MEDUSA_EINVAL = -1,        /* null pointer, non-positive size, inconsistent arguments */
  MEDUSA_EUNSUPPORTED = -2,  /* a size outside the supported range (see each call)      */
  MEDUSA_EWORKSPACE = -3,    /* workspace missing or too small                           */
  MEDUSA_EHIP = -4,          /* a HIP runtime call failed                                */
  MEDUSA_ESCRATCH = -5       /* the shape needs more scratch than the library's built-in array holds */
} medusa_status_t;

/* Values of the `dtype` and `mode` arguments.  The arguments themselves are plain ints, so that any
 * value a caller passes is looked at by the argument checks (and refused with MEDUSA_EINVAL) rather
 * than being an out-of-range enumeration value. */
typedef enum { MEDUSA_F32 = 0, MEDUSA_BF16 = 1 } medusa_dtype_t;
typedef enum { MEDUSA_GREEDY = 0, MEDUSA_TYPICAL = 1 } medusa_accept_mode_t;

#define MEDUSA_MAX_TREE_TOKENS 128 /* T = candidates + root                              */
#define MEDUSA_MAX_HEADS 8         /* K = tree depth                                     */
#define MEDUSA_MAX_TOPK 16         /* S_k = 1 + largest rank used at level k             */

typedef struct medusa_tree medusa_tree_t;
typedef void* medusa_stream_t; /* a hipStream_t */

/* Static text for a status code; never freed. */
const char* medusa_status_string(int status);

/* ----------------------------------------------------------------------------------
 * Candidate tree (Sec. 2.1.2, Fig. 2; sparse trees of Sec. 2.3.3 via explicit nodes).
 *
 * A node is the tuple of ranks (i_1..i_k): the i_j-th best prediction of Medusa head j
 * at level j.  Node 0 is the root (the original LM head's own next token); the other
 * nodes are numbered depth-major and, inside a depth, lexicographically by rank tuple.
 * T = 1 + number of candidate nodes.  Limits: T <= 128, K <= 8, every rank < 16.
 *
 * medusa_tree_create_cartesian: level k has ranks 0..branching[k-1]-1 under every
 *   level-(k-1) node, i.e. sum_k prod_{i<=k} s_i candidate nodes (Sec. 2.1.2).
 * medusa_tree_create_nodes: `ranks` is a host array [n_nodes][K] of rank tuples padded
 *   with -1; the set must be prefix-closed (every node's parent is present) and free of
 *   duplicates.  K is the padded tuple width and must equal the deepest tuple's length.
 * Both build the tables on the host, upload a device copy, and return a handle in *out.
 * The handle is immutable and may be used from any stream; destroy it only after all
 * work that uses it has completed.  A tree belongs to the device that was current when
 * it was created.
 * -------------------------------------------------------------------------------- */
int medusa_tree_create_cartesian(const int32_t* branching /* host [K] */, int K, medusa_tree_t** out);
int medusa_tree_create_nodes(const int32_t* ranks /* host [n_nodes][K] */, int n_nodes, int K,
                             medusa_tree_t** out);
/* medusa_tree_create_optimized (Sec. 2.3.3, appendix on the optimized tree): `accuracy` is a
 *   host array [K][S]; accuracy[k-1][i] estimates how often the i-th best prediction of head k is
 *   the right token (values in [0,1]).  A node (i_1..i_k) is estimated correct with probability
 *   prod_j accuracy[j-1][i_j], which is also its contribution to the expected acceptance length;
 *   the tree of n_nodes candidates maximising the sum is grown greedily from the root by always
 *   adding the best child of an included node (ties: shallower, then lexicographically smaller).
 *   K <= 8, S <= 16, n_nodes <= 127 and <= the number of nodes that exist.  If
 *   expected_accept_len is not NULL it receives 1 + the sum of the chosen nodes' estimates. */
int medusa_tree_create_optimized(const double* accuracy /* host [K][S] */, int K, int S, int n_nodes,
                                 medusa_tree_t** out, double* expected_accept_len);
int medusa_tree_destroy(medusa_tree_t* tree);

/* Sizes: T tokens, K levels, n_leaves candidates (root-to-leaf paths), S = max_k S_k,
 * topk_per_head[k-1] = S_k (host array [K], may be NULL).  Any out pointer may be NULL. */
int medusa_tree_query(const medusa_tree_t* tree, int32_t* T, int32_t* K, int32_t* n_leaves,
                      int32_t* S, int32_t* topk_per_head);

/* Copies the host tables into caller HOST arrays (any may be NULL):
 *   parent[T] (-1 for the root), depth[T] (root 0), rank[T] (-1 for the root),
 *   token_src[T]: index into the per-sequence list [root, top-S_1 of head 1, top-S_2 of
 *                 head 2, ...] that supplies the node's token,
 *   anc_mask[T][2]: bit u of the 128-bit row t (word u/64, bit u%64) is set iff u is an
 *                 ancestor of t or u == t  -- the tree part of the attention mask,
 *   paths[n_leaves][K+1]: root-to-leaf node lists in lexicographic order of the leaves'
 *                 rank tuples, -1 padded. */
int medusa_tree_tables(const medusa_tree_t* tree, int32_t* parent, int32_t* depth, int32_t* rank,
                       int32_t* token_src, uint64_t* anc_mask, int32_t* paths);

/* ----------------------------------------------------------------------------------
 * medusa_heads (Sec. 2.1.1):  logits[m,k,:] = W2_k . ( SiLU(W1_k . h_m) + h_m )
 *   hidden  [M, d]        dtype   rows h_m
 *   w1      [K, d, d]     dtype   out x in; NULL => no residual block: logits = W2_k . h_m
 *                                 (K = 1 with w2 = the LM head gives the original model's
 *                                  logits, used for the M = B*T tree tokens in step (2))
 *   w2      [K, V, d]     dtype   out x in
 *   resid   [M, K, d]     dtype   workspace written by the call: SiLU(W1 h) + h rounded
 *                                 once to dtype; may be NULL iff w1 == NULL
 *   logits  [M, K, V]     fp32    output
 * Limits: 1 <= M <= 16384, 1 <= K <= 8, d a multiple of 8 (bf16: of 64), d <= 16384, V >= 1.
 * -------------------------------------------------------------------------------- */
int medusa_heads(const void* hidden, const void* w1, const void* w2, void* resid, float* logits,
                 int M, int d, int V, int K, int dtype, medusa_stream_t stream);

/* ----------------------------------------------------------------------------------
 * medusa_topk_tree (Sec. 2.1.2): per sequence, the top-S_k tokens of head k (sorted, best
 * first) and the root token = arg-max of the LM head (Sec. 2.3.1: the first token is
 * greedy), gathered into the tree:  tree_tokens[b,t] = list_b[token_src[t]],
 * position_ids[b,t] = prefix_len[b] + depth[t]  (Fig. 2 caption).
 *   medusa_logits [B, K_heads, V] fp32   K_heads >= tree K; heads beyond the tree's depth unused
 *   lm_logits     [B, V]          fp32
 *   prefix_len    [B]             int32
 *   topk_ids      [B, K, S]       int32  out, entries beyond S_k are -1
 *   tree_tokens   [B, T]          int32  out
 *   position_ids  [B, T]          int32  out
 *   workspace: medusa_topk_tree_workspace_bytes(B, K) bytes of device scratch (per-chunk
 *   candidate lists); contents undefined before and after.  8-byte aligned.
 * Limits: V >= S (every S_k <= V), B >= 1.
 * -------------------------------------------------------------------------------- */
size_t medusa_topk_tree_workspace_bytes(int B, int K);
int medusa_topk_tree(const float* medusa_logits, const float* lm_logits, const medusa_tree_t* tree,
                     const int32_t* prefix_len, int B, int V, int K_heads, int32_t* topk_ids,
                     int32_t* tree_tokens, int32_t* position_ids, void* workspace, size_t workspace_bytes,
                     medusa_stream_t stream);

/* ----------------------------------------------------------------------------------
 * tree_attention (Sec. 2.1.2): for every sequence b, query head g, tree token t
 *   out[b,g,t,:] = softmax_j( scale * q[b,g,t,:] . key_j ) . value_j
 * over the keys  { cache rows j < prefix_len[b] }  U  { tree rows u : bit u of
 * anc_mask[t] }: a tree token sees the whole prefix and, of the tree, only its own
 * continuation (ancestors and itself).  Query head g reads KV head g / (Hq/Hkv).
 *   q               [B, Hq, T, D]      dtype
 *   k_tree, v_tree  [B, Hkv, T, D]     dtype   this layer's K/V of the tree tokens
 *   k_cache,v_cache [B, Hkv, Lcap, D]  dtype   one layer of the cache (never written here)
 *   prefix_len      [B] int32                  values are clamped to [0, Lcap]
 *   out             [B, Hq, T, D]      dtype
 *   workspace: tree_attention_workspace_bytes(...) bytes of device scratch (split
 *   partials); contents undefined before and after.  Must be 256-byte aligned.
 * Limits: D in {64, 128}; Hq a multiple of Hkv; T from the tree (<= 128).
 * -------------------------------------------------------------------------------- */
size_t tree_attention_workspace_bytes(int B, int Hq, int Hkv, int T, int D, int Lcap);
int tree_attention(const void* q, const void* k_tree, const void* v_tree, const void* k_cache,
                   const void* v_cache, const int32_t* prefix_len, const medusa_tree_t* tree, void* out,
                   int B, int Hq, int Hkv, int D, int Lcap, float scale, int dtype,
                   void* workspace, size_t workspace_bytes, medusa_stream_t stream);

/* tree_attention_static: tree_attention for callers that cannot allocate device memory or keep a
 * workspace -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and kernels as tree_attention, but the split partials go to an array
 * built into the library's device image (tree_attention_static_scratch_bytes() = 8 MiB per GPU, held
 * until the process ends) instead of a caller workspace.  The call allocates nothing: no hipMalloc,
 * no hipFree, no allocating library routine; the first call on a device looks the array's address
 * up once.  Shapes whose tree_attention_workspace_bytes() exceeds the array are refused with
 * MEDUSA_ESCRATCH and nothing is enqueued (the 7B shapes at batch 1, any prefix length, need 4.4 MB).
 * All calls on one GPU share the array, which keeps the last call's partials (nothing in it has to
 * start at zero: every partial that is read was written by the same call): calls that overlap on
 * one GPU -- two streams, two threads -- race; order them. */
size_t tree_attention_static_scratch_bytes(void);
int tree_attention_static(const void* q, const void* k_tree, const void* v_tree, const void* k_cache,
                          const void* v_cache, const int32_t* prefix_len, const medusa_tree_t* tree, void* out,
                          int B, int Hq, int Hkv, int D, int Lcap, float scale, int dtype,
                          medusa_stream_t stream);

/* ----------------------------------------------------------------------------------
 * medusa_accept (Sec. 2.3.1): node t (t >= 1) passes its test on the original model's
 * row of its parent:
 *   greedy : tree_tokens[b,t] == argmax logits[b,parent[t],:]
 *   typical: p = softmax(logits[b,parent[t],:] / temperature), H = -sum p ln p,
 *            p[tree_tokens[b,t]] > min(eps, delta * exp(-H))            (strict)
 * The root always passes.  A node is accepted iff it and all its ancestors pass.  The
 * result is the accepted node of greatest depth (first in candidate order on ties, which
 * is the lowest node index at that depth); its root path is the accepted prefix.
 *   logits          [B, T, V] fp32    original-model logits at every tree token
 *   tree_tokens     [B, T]    int32
 *   accept_len      [B]       int32 out: 1..K+1 (root included)
 *   best_node       [B]       int32 out: last accepted node (row to gather the next hidden state from)
 *   path_nodes      [B, K+1]  int32 out: accepted nodes in depth order, -1 padded
 *   accepted_tokens [B, K+1]  int32 out: their tokens, -1 padded
 *   next_root       [B]       int32 out: argmax logits[b,best_node,:], the next step's root
 *   workspace: medusa_accept_workspace_bytes(B, T, V) bytes of device scratch.
 * temperature > 0 is required in typical mode and ignored in greedy mode.
 * -------------------------------------------------------------------------------- */
size_t medusa_accept_workspace_bytes(int B, int T, int V);
int medusa_accept(const float* logits, const int32_t* tree_tokens, const medusa_tree_t* tree, int B, int V,
                  int mode, float temperature, float eps, float delta,
                  int32_t* accept_len, int32_t* best_node, int32_t* path_nodes, int32_t* accepted_tokens,
                  int32_t* next_root, void* workspace, size_t workspace_bytes, medusa_stream_t stream);

/* ----------------------------------------------------------------------------------
 * medusa_verify_logits + medusa_accept_fused: steps (2) and (3) of Sec. 2 with the acceptance step's
 * pass over the logits folded into the projection that produces them (Sec. 2.3.1 needs, per row of
 * the original model's logits, the arg-max and -- for typical acceptance -- max, sum exp and
 * sum z exp of z = logit / temperature; medusa_accept reads all B*T*V logits again to get them).
 *
 * medusa_verify_logits = medusa_heads(hidden_tree, NULL, w_lm, NULL, logits, M, d, V, 1, dtype) --
 * the same logits, bit for bit -- whose kernel also leaves, per row and 128-column piece of its
 * output tiles, (arg-max key, max, sum, weighted sum) in `stats`.  medusa_accept_fused then gives
 * medusa_accept's results from those partials and the few logits it looks up (the candidates' own),
 * in a kernel that reads a few KB per row.  The arg-max, and with it greedy acceptance and next_root,
 * is exact; the typical-acceptance statistics are summed in another order than medusa_accept's
 * (fp32), so a probability within rounding of its threshold may fall on either side.
 *   stats: medusa_verify_stats_bytes(M, V) bytes of device scratch, 256-byte aligned, written by
 *   medusa_verify_logits and read and partly rewritten by medusa_accept_fused; one such pair of calls
 *   per buffer at a time.  mode, temperature: the same values in both calls (medusa_accept_fused
 *   reports accept_len[b] = -1 for statistics that were produced for another mode or temperature).
 * The fused epilogue exists in the large-tile kernel only (many tree rows: batches of trees);
 * medusa_verify_fused_available(M, d, V, dtype) says whether a shape gets it (1) or
 * medusa_verify_logits returns MEDUSA_EUNSUPPORTED and the caller stays with medusa_heads +
 * medusa_accept (0).  Other limits and the ticket counters: as for medusa_heads / medusa_accept.
 * -------------------------------------------------------------------------------- */
size_t medusa_verify_stats_bytes(int M, int V);
int medusa_verify_fused_available(int M, int d, int V, int dtype);
int medusa_verify_logits(const void* hidden_tree, const void* w_lm, float* logits, void* stats, size_t stats_bytes, int M,
                         int d, int V, int dtype, int mode, float temperature, medusa_stream_t stream);
int medusa_accept_fused(const float* logits, const void* stats, const int32_t* tree_tokens, const medusa_tree_t* tree, int B,
                        int V, int mode, float temperature, float eps, float delta, int32_t* accept_len, int32_t* best_node,
                        int32_t* path_nodes, int32_t* accepted_tokens, int32_t* next_root, medusa_stream_t stream);

/* ----------------------------------------------------------------------------------
 * medusa_accept_sampled: acceptance by rejection sampling, the alternative to typical acceptance
 * that Sec. 2 (opening paragraph) and Sec. 2.3.1 (first paragraph) name -- "the rejection sampling
 * scheme as used in speculative decoding" -- and that keeps the original model's distribution.
 * The paper does not define the rule; this library's reading: the candidates under a node are a
 * deterministic list, i.e. drafts whose proposal is a point mass on their token, so with
 * p = softmax(logits[b,node,:] / temperature) child i of an accepted node (in rank order) is accepted
 * iff all earlier children were rejected and
 *     uniforms[b, child_i] < p(x_i) / (1 - sum_{j<i} p(x_j)),      x_j = tree_tokens[b, child_j],
 * which is speculative rejection sampling against the residual distribution left by the rejected
 * children.  The root is always accepted; the walk follows the accepted child while there is one.
 * At the node where it ends, next_token is drawn from p without that node's children's tokens
 * (renormalised; p itself at a leaf) by inversion in token-id order with uniforms[b, 0]: the
 * smallest token whose cumulative mass exceeds uniforms[b,0] * total.  The tokens a step emits
 * (accepted candidates, then next_token) are then distributed as the original model's own samples.
 *   logits       [B, T, V] fp32, tree_tokens [B, T] int32 (as for medusa_accept)
 *   uniforms     [B, T] fp32 in [0, 1), caller-supplied (the library draws no random numbers)
 *   accept_len, best_node, path_nodes, accepted_tokens: as for medusa_accept
 *   next_token   [B] int32 out: the sampled token that follows the accepted prefix
 *   workspace: medusa_accept_workspace_bytes(B, T, V) bytes of device scratch.
 * temperature > 0.  Comparisons are made in fp32 (sums in a fixed order): a uniform within rounding
 * of its boundary may fall on either side.  Same limits and the same ticket counters as
 * medusa_accept (the two must not overlap on one GPU either).
 * -------------------------------------------------------------------------------- */
int medusa_accept_sampled(const float* logits, const int32_t* tree_tokens, const medusa_tree_t* tree,
                          const float* uniforms, int B, int V, float temperature, int32_t* accept_len,
                          int32_t* best_node, int32_t* path_nodes, int32_t* accepted_tokens, int32_t* next_token,
                          void* workspace, size_t workspace_bytes, medusa_stream_t stream);

/* ----------------------------------------------------------------------------------
 * kv_commit (Fig. 1 caption: the accepted prefix is the context of the next step): for
 * every layer l, KV head h and j < accept_len[b]
 *   cache[l,b,h,prefix_len[b]+j,:] = tree[l,b,h,path_nodes[b,j],:]      (K and V)
 * then prefix_len[b] += accept_len[b].  Rows that would fall at or beyond Lcap are
 * dropped (and prefix_len saturates at Lcap): capacity is the caller's contract.
 *   k_cache, v_cache [NL, B, Hkv, Lcap, D] dtype  in/out
 *   k_tree, v_tree   [NL, B, Hkv, T, D]    dtype
 *   path_nodes       [B, path_stride] int32, accept_len [B] int32 (from medusa_accept)
 *   prefix_len       [B] int32 in (in/out when prefix_len_out is NULL)
 *   prefix_len_out   [B] int32 out, or NULL to update prefix_len in place; a caller that keeps
 *                    the lengths of consecutive steps in two arrays passes the other one here
 * Limits: D * sizeof(dtype) a multiple of 16.
 * -------------------------------------------------------------------------------- */
int kv_commit(void* k_cache, void* v_cache, const void* k_tree, const void* v_tree,
              const int32_t* path_nodes, int path_stride, const int32_t* accept_len, int32_t* prefix_len,
              int32_t* prefix_len_out, int NL, int B, int Hkv, int T, int D, int Lcap, int dtype,
              medusa_stream_t stream);

/* ----------------------------------------------------------------------------------
 * medusa_carry_over (Sec. 2, opening paragraph; Fig. 1 caption): the activations the next decoding
 * step starts from.  Its Medusa heads read the hidden state of the last accepted token, and its root
 * token is the original model's prediction there, whose logits step (2) has already produced:
 *   h_next[b,:]  = hidden_tree[b, best_node[b], :]
 *   lm_next[b,:] = verify_logits[b, best_node[b], :]
 *   hidden_tree   [B, T, d] dtype    the backbone's last hidden states of the tree tokens
 *   verify_logits [B, T, V] fp32     the logits medusa_heads(w1 == NULL) wrote for them
 *   best_node     [B] int32          from medusa_accept (values are clamped to [0, T-1])
 *   h_next        [B, d] dtype out;  lm_next [B, V] fp32 out (the lm_logits of the next medusa_topk_tree)
 * Either (input, output) pair may be NULL together to skip it.  Outputs must not alias the inputs.
 * Raw row copies: bit-exact.  Limits: B <= 65535; bf16: d even.
 * -------------------------------------------------------------------------------- */
int medusa_carry_over(const void* hidden_tree, const float* verify_logits, const int32_t* best_node, void* h_next,
                      float* lm_next, int B, int T, int d, int V, int dtype, medusa_stream_t stream);

/* ----------------------------------------------------------------------------------
 * Backbone operators on the tree tokens (App. G: operator table, "Parallel decoding" rows
 * X W_Q, X W_K, X W_V, X W_u, X W_g, X W_d; Sec. 2.1.2 for the positional indices).  Together
 * with tree_attention they make up the simplified decoder block whose latency App. G models.
 *
 * tree_linear:  y = x . w^T,  or  y = SiLU(x . w^T) * mul  when mul != NULL (gate projection
 * combined with the up projection), accumulated in fp32 and rounded once to dtype.
 *   x    token-major [B*T, d_in] (x_heads == 0) or head-major [B, x_heads, T, d_in/x_heads]
 *        (the layout tree_attention writes), dtype
 *   w    [d_out, d_in] dtype, out x in
 *   mul  [B*T, d_out] token-major dtype, or NULL
 *   y    token-major [B*T, d_out] (y_heads == 0) or head-major [B, y_heads, T, d_out/y_heads]
 *        (the layout tree_attention and tree_rope read), dtype; must not alias x or mul
 *   workspace  device scratch of at least tree_linear_workspace_bytes(...) bytes (may be 0: then
 *        NULL is fine), caller-owned, contents irrelevant before and after.  It holds the fp32
 *        partial tiles when the reduction over d_in is split across workgroups, which the library
 *        does for few tree tokens and small d_out so that the whole chip streams the weights; with
 *        NULL or too small a workspace the call still works, unsplit and slower.  Calls that use
 *        the workspace must not overlap on one GPU (the workspace is theirs alone while they run).
 * Limits: B*T <= 16384; d_in (and d_in/x_heads) a multiple of 8 (bf16: of 64); d_out a multiple
 * of y_heads.  All pointers are device pointers; returns MEDUSA_EINVAL / MEDUSA_EUNSUPPORTED
 * without launching anything when a limit is violated.
 * -------------------------------------------------------------------------------- */
size_t tree_linear_workspace_bytes(int B, int T, int d_in, int d_out, int dtype);
int tree_linear(const void* x, const void* w, const void* mul, void* y, int B, int T, int d_in, int d_out,
                int x_heads, int y_heads, int dtype, void* workspace, size_t workspace_bytes,
                medusa_stream_t stream);

/* tree_linear with the head-major output cut into y_segments tensors (App. G: X W_Q, X W_K and X W_V
 * read the same X, so one call over the stacked weight rows [W_Q; W_K; W_V] streams X once and
 * launches once): segment s takes the consecutive d_out / y_segments output columns
 * s * d_out / y_segments .. and is a head-major tensor [B, y_heads, T, d_out / (y_segments * y_heads)]
 * that starts y_segment_stride elements after segment s - 1 (y = start of segment 0).
 *   y_heads          heads PER SEGMENT (> 0 when y_segments > 1)
 *   y_segment_stride elements (not bytes) between segment starts, >= B * T * d_out / y_segments
 * y_segments == 1 is tree_linear.  Everything else as for tree_linear; workspace size from
 * tree_linear_workspace_bytes with the total d_out.  MEDUSA_EINVAL when d_out does not divide into
 * y_segments x y_heads whole heads or the segments would overlap.
 */
int tree_linear_segments(const void* x, const void* w, const void* mul, void* y, int B, int T, int d_in, int d_out,
                         int x_heads, int y_heads, int y_segments, size_t y_segment_stride, int dtype,
                         void* workspace, size_t workspace_bytes, medusa_stream_t stream);

/* tree_rope: rotary position embedding, in place, of q [B, Hq, T, D] and k [B, Hkv, T, D] (dtype)
 * at position_ids [B, T] (int32, device; the table medusa_topk_tree writes: prefix length +
 * depth of the node).  Element j < D/2 is paired with element j + D/2; the pair is rotated by
 * position * theta^(-2j/D).  D must be even. */
int tree_rope(void* q, void* k, const int32_t* position_ids, int B, int Hq, int Hkv, int T, int D, float theta,
              int dtype, medusa_stream_t stream);

/* Gate and up projections of the gated feed-forward in one pass (App. G, operator table, rows
 * X W_g and X W_u): y = SiLU(x w_g^T) * (x w_u^T), rounded once, with no intermediate in memory.
 *   x     [B*T, d_in] token-major, or head-major [B, x_heads, T, d_in/x_heads] when x_heads > 0
 *   w_gu  [2*d_out, d_in]: the rows of w_g and w_u interleaved in blocks of 16 -- rows 32b..32b+15
 *         are rows 16b..16b+15 of w_g, rows 32b+16..32b+31 the same rows of w_u (a layout the caller
 *         prepares once per weight pair)
 *   y     [B*T, d_out] token-major, or head-major [B, y_heads, T, d_out/y_heads] when y_heads > 0
 * All device pointers, caller-owned.  bf16 only (MEDUSA_EUNSUPPORTED for fp32: two tree_linear calls
 * do the same there); d_in a multiple of 64, d_out a multiple of 16, B*T <= 16384.  Tuned for up to
 * 192 rows (the tree tokens of one or two sequences) and for batches of trees large enough for the large-tile
 * kernel (medusa_gemm_plan(B*T, 2*d_out, d_in, 1, 0) says kind 3); correct, but not measured against two
 * tree_linear calls, for row counts in between. */
int tree_linear_swiglu(const void* x, const void* w_gu, void* y, int B, int T, int d_in, int d_out, int x_heads,
                       int y_heads, int dtype, medusa_stream_t stream);

/* The weight layout tree_linear_swiglu reads, made from the two matrices (a one-time copy per weight
 * pair; no counterpart in the paper):
 *   w_gate, w_up [d_out, d_in] dtype;  w_gu [2*d_out, d_in] dtype out, laid out as described above.
 * All device pointers, 16-byte aligned, caller-owned, not overlapping.  d_out a multiple of 16, rows a
 * multiple of 16 bytes (else MEDUSA_EUNSUPPORTED). */
int tree_interleave_gate_up(const void* w_gate, const void* w_up, void* w_gu, int d_out, int d_in, int dtype,
                            medusa_stream_t stream);

/* ----------------------------------------------------------------------------------
 * Diagnostic (no counterpart in the paper; host only, touches no GPU): which kernel arrangement
 * the library would launch for a bf16 product of M activation rows with K weight matrices of
 * N rows x d columns (medusa_heads, tree_linear), with or without a workspace.
 * plan6 (host, 6 ints, written): [0] kind: 0 wave-per-row GEMV, 1 skinny MFMA tiles, 2 128 x 128
 * tiles, 3 large tiles;  [1] kind 1: weight rows per workgroup (32..128), kind 3: activation rows per
 * tile (128 or 192), else 0;  [2] kind 1: the kernel for weights that come from HBM (1 KB runs per
 * weight row, straight into an LDS ring);  [3] kind 1/2: groups of 16 activation rows per row block
 * (1..8);  [4] row blocks;  [5] workgroups that share one tile's reduction (1 = unsplit; > 1 only
 * with a workspace).
 * Returns MEDUSA_EINVAL for a null pointer or a non-positive size.
 * -------------------------------------------------------------------------------- */
int medusa_gemm_plan(int M, int N, int d, int K, int have_workspace, int* plan6);

/* ----------------------------------------------------------------------------------
 * Profiling entry (no counterpart in the paper): medusa_heads with three caller-owned hipEvent_t
 * handles recorded on the call's stream -- ev_begin before the residual-block kernel (the W1
 * stream), ev_between after it and before the vocabulary projection (the W2 stream, the largest
 * single read of a step), ev_end after that -- so that a benchmark can time the two kernels
 * inside a running step.  With w1 == NULL ev_begin and ev_between are recorded back to back.
 * Everything else is medusa_heads; MEDUSA_EINVAL if an event is NULL.
 * -------------------------------------------------------------------------------- */
int medusa_heads_timed(const void* hidden, const void* w1, const void* w2, void* resid, float* logits, int M, int d,
                       int V, int K, int dtype, medusa_stream_t stream, void* ev_begin, void* ev_between,
                       void* ev_end);

#ifdef __cplusplus
}
#endif
#endif /* MEDUSA_H_ */
