/*
 * dream.h - C ABI of the MI355X (gfx950) hot path of DREAM's speculative decode step.
 *
 * Four operations, one call each:
 *   dream_tree_verify_attn  target-side attention of all drafted tree nodes against the KV cache
 *                           under the draft-tree mask (Section 3.1, tree-masking paragraph: the
 *                           tree mask built while drafting is reused for verification).
 *   dream_draft_xattn       the attention core of the draft's cross-attention block,
 *                           softmax(Q K^T / sqrt(z)) V  (Section 3.1, Eq. 1), keys/values being the
 *                           cached target features followed by the draft's own features of nodes
 *                           drafted earlier (Section 3.1, paragraph after Eq. 1).
 *   dream_visual_compress   importance score of every visual token = the attention weight it
 *                           receives, summed over rows and heads of the last-layer attention
 *                           matrix; keep the top-scoring ones by ratio; subsample (Section 3.3).
 *   dream_accept_path       greedy (temperature 0) form of the acceptance rule of Section 2.1 over
 *                           the verified tree plus the bonus target token (Section 4).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name ends in _host.  The caller owns every
 *     buffer.  The library allocates nothing, never synchronises, and enqueues all work on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream).  Results are valid
 *     once the caller has synchronised the stream.
 *   - Inputs are never written; outputs are fully overwritten; the workspace is scratch whose
 *     content means nothing between calls (no initialisation is needed).  A *_workspace() query
 *     never returns less than DREAM_WORKSPACE_MIN_BYTES.  Calls that share a workspace must be
 *     ordered on one stream.
 *   - Tensors are dense, C order.  bf16 means the upper 16 bits of an IEEE float32.
 *   - Every function returns a dream_status (0 = ok, negative = error) and never throws or
 *     aborts.  Argument errors are detected on the host before anything is launched; the text of
 *     the last error of the calling thread is available from dream_last_error().
 *   - Device-resident metadata (prefix_len, parent, q_node, token, q_pos) is trusted to be
 *     meaningful; dream_tree_validate_host() is the host-side check for a parent array.  The
 *     kernels still never follow it out of bounds or into a loop: a prefix length is clamped to
 *     [0, s_max - n_tree], a node index to [0, n_tree), and a parent that does not precede its
 *     node is treated as "no parent" (results for such input are unspecified, not a fault).
 *
 * Tree convention: node 0 is the root (the target's last emitted token, depth 0, always
 * accepted); parent[0] = -1 and 0 <= parent[i] < i for i > 0.  The K/V rows of the n_tree tree
 * nodes of sequence b sit at cache rows [prefix_len[b], prefix_len[b] + n_tree).
 */
#ifndef DREAM_H
#define DREAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DREAM_F32 = 0, DREAM_BF16 = 1 } dream_dtype;

typedef enum {
    DREAM_OK = 0,
    DREAM_ERR_INVALID_ARG = -1, /* null required pointer, inconsistent sizes                   */
    DREAM_ERR_UNSUPPORTED = -2, /* shape outside what the kernels are built for                */
    DREAM_ERR_WORKSPACE = -3,   /* workspace_bytes smaller than the matching *_workspace()     */
    DREAM_ERR_HIP = -4          /* a HIP launch reported an error                              */
} dream_status;

#define DREAM_WORKSPACE_MIN_BYTES 256
#define DREAM_MAX_TREE 256      /* tree nodes per sequence handled by the attention calls      */
#define DREAM_MAX_TREE_ACCEPT 1024 /* tree nodes per sequence handled by dream_accept_path     */
#define DREAM_MAX_TREE_WIDTH 16     /* children per node / frontier rows of one tree-expansion level */
#define DREAM_MAX_POOL 1024         /* candidates (root included) dream_tree_finalize ranks */
#define DREAM_MAX_VISUAL 16384  /* visual tokens per sequence handled by dream_visual_compress */

/* Attention geometry shared by the three attention-shaped calls. */
typedef struct {
    int32_t batch;      /* B                                                                   */
    int32_t n_q_heads;  /* Hq                                                                  */
    int32_t n_kv_heads; /* Hkv; Hq % Hkv == 0; query head h reads KV head h / (Hq/Hkv)         */
    int32_t head_dim;   /* D in {64, 128, 256}                                                 */
    int32_t dtype;      /* dream_dtype of q, k, v and out                                      */
    float scale;        /* multiplies q.k before the softmax; 0 selects 1/sqrt(D) (Eq. 1)      */
    int64_t s_max;      /* row capacity of every [B, Hkv, s_max, D] cache                      */
} dream_attn_desc;

/* ---------------------------------------------------------------------------------------------
 * Tree-masked verification attention (Section 3.1; Eq. 1 gives the attention form).
 *   q          [B, n_tree, Hq, D]   queries of the tree nodes
 *   k_cache    [B, Hkv, s_max, D]   rows [0, P_b) prefix (visual + text), [P_b, P_b+n_tree) tree
 *   v_cache    [B, Hkv, s_max, D]
 *   prefix_len [B] int32            P_b
 *   parent     [B, n_tree] int32
 *   tree_mask  nullable, [B, n_tree, W] uint64 with W = ceil(n_tree / 64) words per node: bit (a % 64)
 *              of word a / 64 of node i set iff tree node a is visible to node i.  When given it
 *              replaces the mask derived from `parent` (node i sees itself and its ancestors).
 *   max_kv_len host-known upper bound of P_b + n_tree over the batch (<= s_max); only used to
 *              choose the launch shape, pass s_max if unknown.
 *   out        [B, n_tree, Hq, D]   same dtype as q
 *   lse        nullable, [B, Hq, n_tree] float32: natural-log sum of exp of the scaled scores.
 * Node i attends keys {0..P_b-1} and {P_b + a : a visible to i}.  n_tree in [1, DREAM_MAX_TREE].
 * ------------------------------------------------------------------------------------------- */
size_t dream_tree_verify_attn_workspace(const dream_attn_desc *desc, int32_t n_tree, int64_t max_kv_len);
int dream_tree_verify_attn(const dream_attn_desc *desc, const void *q, const void *k_cache,
                           const void *v_cache, const int32_t *prefix_len, int32_t n_tree,
                           const int32_t *parent, const uint64_t *tree_mask, int64_t max_kv_len,
                           void *out, float *lse, void *workspace, size_t workspace_bytes,
                           void *stream);

/* ---------------------------------------------------------------------------------------------
 * Draft cross-attention core (Section 3.1, Eq. 1 and the paragraph after it).
 *   q          [B, n_q, Hq, D]      projected draft features of the nodes being expanded
 *   kx_cache   [B, Hkv, s_max, D]   rows [0, n_b): projected target features S^L W_K;
 *   vx_cache                        rows [n_b, n_b+n_tree): projected draft features of tree nodes
 *   prefix_len [B] int32            n_b
 *   parent     [B, n_tree] int32
 *   q_node     nullable, [B, n_q] int32: tree node of each query row (NULL: row r is node r,
 *              which needs n_q <= n_tree)
 *   out        [B, n_q, Hq, D]
 * Query of node i attends rows {0..n_b-1} and {n_b + a : a a STRICT ancestor of i}; a query with
 * no visible key yields a zero row.  n_q in [1, DREAM_MAX_TREE], n_tree in [1, DREAM_MAX_TREE].
 * ------------------------------------------------------------------------------------------- */
size_t dream_draft_xattn_workspace(const dream_attn_desc *desc, int32_t n_q, int64_t max_kv_len);
int dream_draft_xattn(const dream_attn_desc *desc, const void *q, const void *kx_cache,
                      const void *vx_cache, const int32_t *prefix_len, int32_t n_tree,
                      const int32_t *parent, int32_t n_q, const int32_t *q_node,
                      int64_t max_kv_len, void *out, void *workspace, size_t workspace_bytes,
                      void *stream);

/* ---------------------------------------------------------------------------------------------
 * Visual-token compression (Section 3.3; kept count per Section 3: round(v / r)).
 * Stage A (skipped when scores_in != NULL): row r of q sits at position pos_r (q_pos[b,r], or r
 * when q_pos is NULL) and attends keys 0..pos_r causally;
 *   score[b, j] = sum over heads and rows with pos_r >= j of softmax_row_r(scale q k^T)[j]
 * for j in [vis_start, vis_start + vis_len).
 * Stage B: k = (vis_len*keep_num + keep_den/2) / keep_den (round half up, integer division); the
 * k highest scores win, equal scores resolved toward the lower index; kept_idx receives their
 * absolute positions in ascending order.  Optional gather: gather_dst[b,t,:] =
 * gather_src[b, kept_idx[b,t], :].
 *   q          [B, n_q, Hq, D] (dtype of desc; bf16 only for stage A), q_pos nullable [B, n_q]
 *   k_cache    [B, Hkv, s_max, D]; n_keys = live key rows, every pos_r < n_keys <= s_max
 *   scores_in  nullable [B, vis_len] float32 (skips stage A); scores_out nullable [B, vis_len] float32
 *   row_lse_in nullable [B, Hq, n_q] float32: natural-log sum of exp of the scaled scores of every row over its causal
 *              keys, -inf for a row without keys.  Section 3.3 takes the scores from the attention matrix the target's
 *              last layer has just computed: an attention kernel that leaves a log-sum-exp per row (as
 *              dream_tree_verify_attn does) already holds the normaliser of every row, and stage A then needs one pass
 *              over q k^T instead of two.  Ignored when scores_in is given.
 *   kept_idx   [B, k] int32;  n_kept_host nullable, HOST int32 receiving k
 *   gather_src nullable [B, n_rows_src, row_elems] of desc->dtype, gather_dst [B, k, row_elems];
 *              n_rows_src is the row capacity per sequence (kept positions are < n_rows_src)
 * desc->head_dim, heads and s_max are ignored when scores_in is given.
 * ------------------------------------------------------------------------------------------- */
size_t dream_visual_compress_workspace(const dream_attn_desc *desc, int32_t n_q, int32_t vis_len);
int dream_visual_compress(const dream_attn_desc *desc, const void *q, const int32_t *q_pos,
                          int32_t n_q, const void *k_cache, int32_t n_keys, int32_t vis_start,
                          int32_t vis_len, int32_t keep_num, int32_t keep_den,
                          const float *scores_in, const float *row_lse_in, float *scores_out, int32_t *kept_idx,
                          int32_t *n_kept_host, const void *gather_src, int64_t n_rows_src,
                          void *gather_dst, int64_t row_elems, void *workspace,
                          size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Per-node arg-max and greedy accepted path (Section 2.1 rule at temperature 0; Section 4).
 *   logits      [B, n_tree, vocab] float32 or bf16 (finite values)
 *   token       [B, n_tree] int32   drafted token of each node (token[b,0] is not examined)
 *   parent      [B, n_tree] int32
 *   node_argmax [B, n_tree] int32   lowest index of the row maximum
 *   accept_len  [B] int32           depth of the deepest accepted node (root excluded)
 *   accept_path [B, max_depth+1]    root ... deepest accepted node, then -1
 *   bonus_token [B] int32           node_argmax of the deepest accepted node
 * Node i > 0 is accepted iff its parent is accepted, token[i] == node_argmax[parent[i]] and its
 * depth <= max_depth.  Among equally deep accepted nodes the lowest node index wins.
 * n_tree in [1, DREAM_MAX_TREE_ACCEPT].
 * ------------------------------------------------------------------------------------------- */
size_t dream_accept_path_workspace(int32_t batch, int32_t n_tree, int32_t vocab);
int dream_accept_path(const void *logits, int32_t logits_dtype, int32_t batch, int32_t n_tree,
                      int32_t vocab, const int32_t *token, const int32_t *parent,
                      int32_t max_depth, int32_t *node_argmax, int32_t *accept_len,
                      int32_t *accept_path, int32_t *bonus_token, void *workspace,
                      size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * dream_accept_path for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * dream_accept_path without the workspace: the per-chunk partial results live in a scratch array inside the
 * library (DREAM_ACCEPT_STATIC_SCRATCH_BYTES of device memory per GPU, held until the process ends).  The
 * call allocates nothing and frees nothing.
 *   Limit: batch * n_tree * ceil(vocab / 8192) partial results of 8 bytes (two arrays, each rounded up to
 *   256 bytes) must fit the scratch: up to 131040 of them, e.g. 32 sequences x 60 nodes at a vocabulary
 *   of 524288; larger problems return DREAM_ERR_UNSUPPORTED (use dream_accept_path).
 *   Every call on a GPU shares that GPU's scratch: calls that overlap on one GPU (two streams, two host
 *   threads) race; calls ordered on one stream do not.  Nothing in the scratch has to start at zero.
 * dream_accept_static_init() looks up the scratch address for the CURRENT device (once per device; the first
 * dream_accept_path_static call on a device does it otherwise).  Call it at set-up, outside any capture.
 * ------------------------------------------------------------------------------------------- */
#define DREAM_ACCEPT_STATIC_SCRATCH_BYTES (1 << 20)
int dream_accept_static_init(void);
int dream_accept_path_static(const void *logits, int32_t logits_dtype, int32_t batch, int32_t n_tree,
                             int32_t vocab, const int32_t *token, const int32_t *parent,
                             int32_t max_depth, int32_t *node_argmax, int32_t *accept_len,
                             int32_t *accept_path, int32_t *bonus_token, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Attention entropy of a layer, Eq. 2 (Section 3.2): row r of q sits at position pos_r (q_pos[b,r],
 * or r when q_pos is NULL) and attends keys 0..pos_r with A = softmax_row(scale q k^T);
 *   row_entropy[b, h, r] = - sum_j A_j log A_j   (natural logarithm; nullable output)
 *   ae[b]                = mean of row_entropy over heads and rows   ([B] float32)
 * q [B, n_q, Hq, D] and k_cache [B, Hkv, s_max, D] of desc->dtype, n_keys live key rows.  The
 * attention matrix is never stored: one streaming pass keeps a running (max, sum, score-weighted sum)
 * per row, as the log-sum-exp pass of dream_visual_compress does.
 * ------------------------------------------------------------------------------------------- */
size_t dream_attention_entropy_workspace(const dream_attn_desc *desc, int32_t n_q);
int dream_attention_entropy(const dream_attn_desc *desc, const void *q, const int32_t *q_pos, int32_t n_q,
                            const void *k_cache, int32_t n_keys, float *row_entropy, float *ae,
                            void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * KV-cache commit of the accepted path (Section 2.1: the tokens after the first rejected one are
 * discarded and decoding continues from the accepted prefix; Section 4: KV caching).
 *   caches_host    HOST array of n_caches DEVICE pointers, each a cache [B, Hkv, s_max, D] of
 *                  desc->dtype (K and V of every layer, the draft's feature caches, ...),
 *                  16-byte aligned, modified in place
 *   prefix_len     [B] int32   the tree rows of sequence b sit at [prefix_len[b], +n_tree)
 *   accept_path    [B, path_stride] int32   root first (as dream_accept_path writes it)
 *   accept_len     [B] int32   number of accepted nodes below the root, < min(path_stride, n_tree)
 *   prefix_len_out nullable [B] int32, must not alias prefix_len
 * In every cache, for every KV head: row prefix_len[b] + j receives the old content of row
 * prefix_len[b] + accept_path[b][j] for j = 0 .. accept_len[b]; all other rows keep their content.
 * prefix_len_out[b] = prefix_len[b] + accept_len[b] + 1 (prefix, root and accepted nodes; the bonus
 * token's row is written by the next round).  Uses desc->batch, n_kv_heads, head_dim, dtype, s_max.
 * The call needs no workspace; the pointers are read on the host before it returns.
 * DREAM_ERR_UNSUPPORTED if min(path_stride, n_tree) rows exceed 64 KB or a row is not a multiple
 * of 16 bytes.  Device metadata is trusted but clamped to the tree rows.
 * ------------------------------------------------------------------------------------------- */
int dream_kv_commit(const dream_attn_desc *desc, void *const *caches_host, int32_t n_caches,
                    const int32_t *prefix_len, int32_t n_tree, const int32_t *accept_path,
                    int32_t path_stride, const int32_t *accept_len, int32_t *prefix_len_out,
                    void *stream);

/* ---------------------------------------------------------------------------------------------
 * Draft-tree construction (Section 3.1, last paragraph: width-k tree expansion with the top-k
 * reordering of EAGLE-2; Section 4: k children per node, a depth, a budget of drafted tokens).
 * The draft model runs between the levels, so a level is one call:
 *   logits        [B, F, V] draft logits of the F <= DREAM_MAX_TREE_WIDTH frontier nodes (f32 or bf16)
 *   cum_in        [B, F] float32   score (log-probability of the whole path) of each frontier node
 *   k             children per node, 1 <= k <= min(DREAM_MAX_TREE_WIDTH, V)
 *   cand_token    [B, F, k] int32  the k most probable tokens of each row, most probable first;
 *                                  equal logits resolve toward the lower token (the logits themselves
 *                                  are compared, so this is exact)
 *   cand_score    [B, F, k] float32  cum_in + logit - logsumexp(row)
 *   next_frontier [B, min(k, F*k)] int32  flat indices f*k + j of the best candidates of the level by
 *                                  cand_score (float32), best first, equal scores toward the lower index
 * dream_tree_finalize ranks a pool of candidates gathered over all levels:
 *   pool_score/pool_parent/pool_token [B, n_pool]; entry 0 is the root (its score is ignored), entry
 *   i > 0 has parent pool_parent[b,i] < i; n_pool <= DREAM_MAX_POOL
 *   keeps the root and the min(budget, n_pool-1) best other entries (score descending, equal scores
 *   toward the lower index) and lists them in pool order, so a parent precedes its children:
 *   tree_parent [B, T] (-1 for the root; -2 if the parent of a kept entry was dropped, which cannot
 *   happen when scores do not increase along a path), tree_token [B, T], tree_pool_index [B, T],
 *   T = 1 + min(budget, n_pool-1), also written to *n_tree_host (nullable, HOST).
 * ------------------------------------------------------------------------------------------- */
size_t dream_tree_expand_workspace(int32_t batch, int32_t n_frontier, int32_t vocab, int32_t k);
int dream_tree_expand_level(const void *logits, int32_t logits_dtype, int32_t batch, int32_t n_frontier,
                            int32_t vocab, const float *cum_in, int32_t k, int32_t *cand_token,
                            float *cand_score, int32_t *next_frontier, void *workspace,
                            size_t workspace_bytes, void *stream);
int dream_tree_finalize(const float *pool_score, const int32_t *pool_parent, const int32_t *pool_token,
                        int32_t batch, int32_t n_pool, int32_t budget, int32_t *tree_parent,
                        int32_t *tree_token, int32_t *tree_pool_index, int32_t *n_tree_host,
                        void *stream);

/* ---------------------------------------------------------------------------------------------
 * Acceptance at a sampling temperature (Section 2.1: accept a drafted token d with probability
 * min(1, P_target(d) / P_draft(d)); Section 4 evaluates at temperature 1).  Over a tree the children
 * of the current node (root first) are tried in node order; after a rejected child the target
 * distribution becomes the normalised positive part of (target - draft) and the rejected token
 * leaves the draft distribution; the first accepted child becomes the current node.  With no
 * accepted child (or none within max_depth) the next token is drawn from the current target
 * distribution by inverting its cumulative sum in token order.
 *   target_logits [B, n_tree, V]   target logits at every node (f32 or bf16)
 *   draft_logits  [B, n_tree, V]   draft logits at every node: row i is the distribution node i's
 *                                  children were proposed from (rows of leaves are not read)
 *   batch * n_tree <= 65535
 *   token, parent [B, n_tree] int32;  u_accept [B, n_tree] float32 in [0,1): the random number of
 *   node i's test;  u_bonus [B] float32 in [0,1): the random number of the final draw
 *   temperature > 0: both logit rows are divided by it
 *   accept_len [B], accept_path [B, max_depth+1] (root first, then -1), bonus_token [B] int32
 * Probabilities are float32 with fixed-order reductions (reproducible run to run).
 * ------------------------------------------------------------------------------------------- */
size_t dream_spec_accept_workspace(int32_t batch, int32_t n_tree, int32_t vocab);
int dream_spec_accept(const void *target_logits, const void *draft_logits, int32_t logits_dtype,
                      int32_t batch, int32_t n_tree, int32_t vocab, const int32_t *token,
                      const int32_t *parent, const float *u_accept, const float *u_bonus,
                      int32_t max_depth, float temperature, int32_t *accept_len, int32_t *accept_path,
                      int32_t *bonus_token, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * The linear maps of Eq. 1 (Section 3.1: Q = E W_Q, K = S W_K, V = S W_V) for the rows a decode step
 * adds, written where attention reads them:
 *   y[b, r, h, :] = x[b, r, :] . w[h*D .. h*D+D-1, :]^T       (float32 accumulation, bf16 result)
 *   x          [B, n_rows, hidden] bf16     feature rows (draft features E, target features S^L)
 *   w          [n_heads*D, hidden] bf16     row n holds the weights of output feature n
 *   row_base   nullable [B] int32; row_index nullable [B, n_rows] int32 (needs row_base)
 *   out        row_base == NULL: dense [B, n_rows, n_heads, D] (queries);
 *              otherwise a cache [B, n_heads, s_max, D]: row r of sequence b lands at cache row
 *              row_base[b] + (row_index ? row_index[b, r] : r) of every head (cache append; the rest
 *              of the cache keeps its content).  Uses desc->batch, head_dim (D), dtype (bf16 only),
 *              s_max.  hidden must be a multiple of 256, D of 16; x, w, out 16-byte aligned.
 *              A destination row outside [0, s_max) is dropped (nothing is written for it).
 * dream_project_rows_multi runs up to DREAM_MAX_PROJ_JOBS such maps over the same B, n_rows and
 * hidden in ONE launch (a draft level's W_Q, W_K and W_V: together they fill the chip where the
 * narrow K/V maps of a grouped-query model alone would not).  `jobs` is a host array read during
 * the call; jobs must not write overlapping memory.
 * ------------------------------------------------------------------------------------------- */
#define DREAM_MAX_PROJ_JOBS 4
typedef struct dream_proj_job {
    const void *x;             /* device */
    const void *w;             /* device */
    int32_t n_heads;
    const int32_t *row_base;   /* device, nullable */
    const int32_t *row_index;  /* device, nullable */
    void *out;                 /* device */
} dream_proj_job;
int dream_project_rows(const dream_attn_desc *desc, const void *x, int32_t n_rows, int32_t hidden,
                       const void *w, int32_t n_heads, const int32_t *row_base,
                       const int32_t *row_index, void *out, void *stream);
int dream_project_rows_multi(const dream_attn_desc *desc, const dream_proj_job *jobs, int32_t n_jobs,
                             int32_t n_rows, int32_t hidden, void *stream);

/* Host-side check of one parent array: parent_host[0] == -1 and 0 <= parent_host[i] < i.
 * Writes the maximum depth to *max_depth_out (nullable).  DREAM_OK or DREAM_ERR_INVALID_ARG. */
int dream_tree_validate_host(const int32_t *parent_host, int32_t n_tree, int32_t *max_depth_out);

/* Text of the calling thread's last error ("" if none); static storage, never NULL. */
const char *dream_last_error(void);

/* Host-only: writes a short description of the launch plan the attention calls would use for n_q query
 * rows per sequence and keys up to max_kv_len (kernel and its template arguments, workgroups, key splits,
 * whether a merge launch follows) into buf (NUL-terminated, truncated to buf_bytes).  Needs no GPU.
 * More than 64 query rows are taken as a verification call over a tree of n_q nodes (the plan of a tree above 64
 * nodes differs: four mask words per node, see DREAM_MAX_TREE).
 * DREAM_OK, or DREAM_ERR_INVALID_ARG / DREAM_ERR_UNSUPPORTED for a descriptor the attention calls reject. */
int dream_attn_plan_describe(const dream_attn_desc *desc, int32_t n_q, int64_t max_kv_len, char *buf,
                             size_t buf_bytes);

/* Measurement aid, not a step of the method: reads `bytes` (rounded down to 16) from the device pointer src
 * once with 16-byte loads and writes nothing (sink: 4 device bytes, almost never stored to).  The time of
 * this call is the floor for any kernel that has to read that many bytes in one launch.  src 16-byte aligned. */
int dream_stream_read(const void *src, size_t bytes, void *sink, void *stream);

/* One-time set-up for the CURRENT device, optional: raises the dynamic-LDS limit of every kernel that needs
 * it and looks up the static scratch of dream_accept_path_static, so that no later call has to (each call
 * otherwise does this itself the first time it needs it).  Call it outside any stream capture.  DREAM_OK,
 * or DREAM_ERR_HIP when no GPU is usable. */
int dream_init(void);

#ifdef __cplusplus
}
#endif
#endif /* DREAM_H */
