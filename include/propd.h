/*
 * propd.h - C ABI of the MI355X token-tree verification library.
 *
 * The library implements the verification step of ProPD's parallel decoding
 * (arXiv 2402.13485): tree-masked attention, the early-pruning pass and greedy
 * acceptance, as HIP kernels for gfx950.  Plain C99: pointers and sizes only.
 *
 * Common rules for every entry point
 *   - Pointers named in a parameter list are DEVICE pointers unless the comment
 *     says "host".  The caller owns every buffer, before and after the call; the
 *     library allocates nothing, frees nothing and keeps no pointer.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream).  No entry point synchronises with the host or copies
 *     between host and device; outputs are valid once the stream reaches the end
 *     of the enqueued work.  `workspace` is scratch for the duration of that work
 *     and must not be shared by calls that may overlap on different streams.
 *   - Scalars are validated on the host: a bad scalar, a NULL required pointer or
 *     a short workspace returns an error code and enqueues nothing.  The content
 *     of device arrays is not validated: a tree whose parent array is not
 *     topological (parent[i] < i), or a mask that does not belong to the parent
 *     array, gives unspecified results, but never an out-of-bounds access
 *     (indices read from device arrays are range-checked in the kernels).
 *   - Tensors are dense and row-major with the innermost dimension contiguous;
 *     base pointers must be 16-byte aligned.
 *   - Trees: node 0 of every sequence is the root, i.e. the token the model has
 *     already fixed; it counts towards T, is never pruned and is always accepted.
 *     Nodes are stored in a topological (for instance breadth-first) order.
 *     Per-sequence slots have T_max entries; entries at or beyond n_nodes[b] are
 *     padding: never read as data, and written only where a comment says so.
 */
#ifndef PROPD_H
#define PROPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Entry points are the only symbols the shared library exports. */
#if defined(__GNUC__)
#define PROPD_API __attribute__((visibility("default")))
#else
#define PROPD_API
#endif

typedef enum {
  PROPD_OK = 0,
  PROPD_ERR_INVALID_ARG = 1, /* a scalar out of range or a required pointer is NULL */
  PROPD_ERR_UNSUPPORTED = 2, /* a legal request this build has no kernel for        */
  PROPD_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than propd_workspace_bytes */
  PROPD_ERR_DEVICE = 4       /* the HIP runtime refused a launch                    */
} propd_status;

typedef enum { PROPD_F32 = 0, PROPD_BF16 = 1 } propd_dtype;

/* Largest tree, root included.  A node's ancestor set is a 128-bit set, two
 * uint64 words, word 0 holding nodes 0..63. */
#define PROPD_MAX_TREE 128

/* A batch of token trees (Section 2: candidates organised as a tree that shares
 * common prefixes; node = one candidate token at one future position). */
typedef struct propd_tree {
  int32_t B;               /* sequences, >= 1                                         */
  int32_t T_max;           /* slot size, 1..PROPD_MAX_TREE                            */
  const int32_t *n_nodes;  /* [B]          T_b in 1..T_max                            */
  const int32_t *parent;   /* [B,T_max]    parent[0] = -1, 0 <= parent[i] < i         */
  const int32_t *token;    /* [B,T_max]    candidate token id of each node            */
  const int32_t *depth;    /* [B,T_max]    edges to the root, depth[0] = 0            */
  const uint64_t *anc;     /* [B,T_max,2]  ancestor-or-self set: the cached tree mask */
} propd_tree;

/* Same fields, writable: where a call produces a tree. */
typedef struct propd_tree_out {
  int32_t *n_nodes;
  int32_t *parent;
  int32_t *token;
  int32_t *depth;
  uint64_t *anc;
} propd_tree_out;

/* A per-node row tensor that continues past the pruning point and has to be
 * narrowed to the surviving nodes.  It is viewed as [B, outer, T_max] rows of
 * row_bytes bytes; hidden states [B,T_max,Hd] have outer = 1, tree K or V
 * [B,H,T_max,d] have outer = H.  Strides are in bytes and apply to src and dst. */
typedef struct propd_payload {
  const void *src;         /* device                                                  */
  void *dst;               /* device, must not overlap src                            */
  size_t row_bytes;
  int64_t outer;
  int64_t stride_b, stride_outer, stride_t;
} propd_payload;

/*
 * Build the cached tree mask from parent pointers (Section 2, "Verification";
 * Section 4.1, "Implementation Optimization": the mask lives on the GPU).
 *   anc[b,i]  = set of nodes on the root path of i, i included
 *   depth[b,i] = number of edges from i to the root
 * Padding slots get anc = 0 and depth = -1.  depth may be NULL.
 */
PROPD_API propd_status propd_tree_mask(int32_t B, int32_t T_max, const int32_t *n_nodes,
                             const int32_t *parent, int32_t *depth, uint64_t *anc,
                             void *hip_stream);

/*
 * Debug check of a tree (the other entry points trust the content of the tree arrays, see the
 * common rules above; Section 2 defines the tree, its root and the mask).  Enqueues one small
 * kernel that writes, for every sequence, a word of PROPD_TREE_* flags, 0 for a consistent tree:
 *   PROPD_TREE_BAD_SIZE    n_nodes[b] outside [1, T_max]
 *   PROPD_TREE_BAD_PARENT  parent[0] != -1, or some parent[i] outside [0, i)
 *   PROPD_TREE_BAD_DEPTH   depth[i] is not the number of edges to the root (skipped if depth is NULL)
 *   PROPD_TREE_BAD_MASK    anc[i] is not the set of nodes on the root path of i (skipped if anc is NULL)
 * flags is a device array [B]; like every call it does not synchronise: read it after the stream
 * has reached this point.  token is not looked at.
 */
enum {
  PROPD_TREE_BAD_SIZE = 1,
  PROPD_TREE_BAD_PARENT = 2,
  PROPD_TREE_BAD_DEPTH = 4,
  PROPD_TREE_BAD_MASK = 8
};
PROPD_API propd_status propd_validate_tree(const propd_tree *tree, int32_t *flags, void *hip_stream);

/*
 * Tree-masked attention (Section 2, "Verification"; Figure 2(b,c)).  For every
 * sequence b, head h and tree node i < T_b:
 *     out[b,h,i,:] = softmax_j( scale * <q[b,h,i,:], k_j> ) . v_j
 * where j runs over all L_b = seq_lens[b] cached prefix tokens and over the tree
 * nodes in anc[b,i] (the node's own candidate sequence, itself included).
 *
 *   dt        PROPD_BF16: tensors are bf16, d in {64, 128}; scores, softmax and
 *             the output accumulation are fp32, the result is rounded to bf16.
 *             (d = 128, the head size of every model of Section 5.1, runs the tiled
 *             matrix-core kernel and needs 16-byte aligned tensors and workspace;
 *             d = 64 runs a plain one-wave-per-query kernel, without workspace.)
 *             PROPD_F32: tensors are fp32, d in {64, 128}, fp32 throughout.
 *   q, k_tree, v_tree, out   [B,H,T_max,d]
 *   k_cache, v_cache         [B,H,L_max,d]; rows >= L_b are never used
 *   seq_lens  [B], 0 <= L_b <= L_max
 *   scale     softmax scale, must be > 0 (1/sqrt(d) in every workload here)
 *   tree      n_nodes and anc are read (token, parent, depth may be NULL)
 *   out       rows i >= T_b are left untouched
 *   workspace propd_workspace_bytes(PROPD_WS_TREE_ATTENTION, ...) bytes
 */
PROPD_API propd_status propd_tree_attention(const propd_tree *tree, propd_dtype dt, int32_t H, int32_t d,
                                  float scale, const void *q, const void *k_cache,
                                  const void *v_cache, const void *k_tree, const void *v_tree,
                                  const int32_t *seq_lens, int32_t L_max, void *out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Early pruning (Section 4.1, "Pruning Process" and "Implementation
 * Optimization").
 *   1. Early head: for every node p that has children, scores over the vocabulary
 *      z_p = head_weight . hidden_states[b,p,:]  (fp32 accumulation).
 *   2. Top-k test: child c of p fails unless its token is among the top_k best
 *      scores of z_p.  Membership is decided by counting,
 *      rank_c = #{v : z_p[v] > z_p[tok_c]} + #{v < tok_c : z_p[v] == z_p[tok_c]},
 *      fail_c = rank_c >= top_k.  top_k >= vocab prunes nothing.
 *   3. Branch elimination: a node survives iff no node of its root path failed.
 *   4. Survivors are compacted in order; the cached mask is subsampled to the
 *      surviving rows and columns; the listed row payloads are gathered.
 *
 *   hidden_states [B,T_max,hidden]  layer-n hidden state of every tree token
 *   head_weight   [vocab,hidden]    weight of the bias-free early head, one row
 *                                   per vocabulary entry (nn.Linear layout)
 *   dt            PROPD_BF16 (hidden must be a multiple of 32) or PROPD_F32
 *   tree          all five arrays are read; token ids outside [0, vocab) fail
 * Outputs (each fully written, padding included; any may NOT alias an input):
 *   keep_bits  [B,2]      bit i set iff node i survives
 *   new_index  [B,T_max]  position of node i among survivors, -1 if pruned/padding
 *   orig_index [B,T_max]  old index of survivor j, -1 for j >= n_kept[b]
 *   n_kept     [B]        number of survivors (also written to tree_out->n_nodes)
 *   cu_nodes   [B+1]      exclusive prefix sum of n_kept (ragged offsets)
 *   tree_out   compacted tree in the same padded layout, survivors first:
 *              parent re-indexed, token and depth copied, anc subsampled;
 *              slots >= n_kept[b] hold -1 (anc: 0)
 *   rank_out   [B,T_max] or NULL: rank_c as counted (root 0, padding -1, vocab for a token
 *              id outside the vocabulary); ranks of near-equal scores may differ from a
 *              higher-precision evaluation
 *   payloads   host array of n_payloads descriptors (0..PROPD_MAX_PAYLOADS, read
 *              during the call only).  Row (b,o,orig_index[b,j]) of src is copied
 *              to row (b,o,j) of dst for j < n_kept[b]; other dst rows are untouched.
 *   workspace  propd_workspace_bytes(PROPD_WS_EARLY_PRUNE, ...) bytes, 16-byte aligned.  The
 *              scores themselves are never stored: the scratch holds per-node tables and,
 *              for the probability criterion, two floats per score row and 64 columns.
 * hidden_states and head_weight must be 16-byte aligned for PROPD_BF16
 * (PROPD_ERR_INVALID_ARG otherwise).
 * The bf16 scoring kernel chooses between two tile shapes on the device, from the number of
 * score rows.  The environment variable PROPD_HEAD_PLAN (read once per process; for tuning and
 * tests) overrides the choice: 1 = 256-row tiles, 2 = 352-row tiles; which nodes survive does
 * not depend on it beyond the order of rounding noted for rank_out.
 */
#define PROPD_MAX_PAYLOADS 8
PROPD_API propd_status propd_early_prune(const propd_tree *tree, propd_dtype dt, int32_t hidden,
                               int32_t vocab, int32_t top_k, const void *hidden_states,
                               const void *head_weight, uint64_t *keep_bits, int32_t *new_index,
                               int32_t *orig_index, int32_t *n_kept, int32_t *cu_nodes,
                               const propd_tree_out *tree_out, int32_t *rank_out,
                               int32_t n_payloads, const propd_payload *payloads,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Greedy acceptance (Section 3, "acceptance length"; Section 5.1: greedy
 * decoding, so the output equals the large model's own).  With
 * g_i = argmax_v logits[b,i,v] (lowest id among equal maxima), a child is
 * accepted iff its token equals g at its parent and its parent is accepted; the
 * root is always accepted.  The result is the deepest accepted node (lowest
 * index among equally deep ones).
 *
 *   logits      [B,T_max,vocab], dt = PROPD_BF16 or PROPD_F32; rows >= T_b unused
 *   tree        n_nodes, parent, token, anc are read
 *   accept_len  [B]              nodes on the accepted path, root included (>= 1)
 *   accept_path [B,path_stride]  node indices (of the tree passed in) root first,
 *                                -1 padded; entries beyond path_stride are dropped
 *   next_token  [B]              g at the last accepted node
 *   workspace   propd_workspace_bytes(PROPD_WS_ACCEPT_PATH, ...) bytes
 */
PROPD_API propd_status propd_accept_path(const propd_tree *tree, propd_dtype dt, int32_t vocab,
                               const void *logits, int32_t *accept_len, int32_t *accept_path,
                               int32_t path_stride, int32_t *next_token, void *workspace,
                               size_t workspace_bytes, void *hip_stream);

/*
 * propd_accept_path for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, serving loops and harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as propd_accept_path, minus the workspace: the partial
 * arg-max records go to a fixed array in device memory that belongs to the library (one
 * copy per GPU, PROPD_STATIC_ACCEPT_MAX_NODES * 64 bytes = 512 KB, held until the process
 * ends).  The call allocates nothing and frees nothing.
 *   - B * T_max must not exceed PROPD_STATIC_ACCEPT_MAX_NODES: PROPD_ERR_UNSUPPORTED otherwise.
 *   - hip_stream must belong to the device that is current when the call is made.
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap on one GPU
 *     (different streams, different threads) race.  Nothing in it has to be cleared
 *     between calls: a call reads only records it has written itself.
 */
#define PROPD_STATIC_ACCEPT_MAX_NODES 8192
PROPD_API propd_status propd_accept_path_static(const propd_tree *tree, propd_dtype dt, int32_t vocab,
                               const void *logits, int32_t *accept_len, int32_t *accept_path,
                               int32_t path_stride, int32_t *next_token, void *hip_stream);

/*
 * Early pruning by the probability-based criterion (Section 4.1, "Pruning Criterion", the
 * second of the two criteria; the paper sets it aside because its implementation moved the
 * probabilities to the host - here everything stays on the device).  The early head's scores
 * of a node become probabilities, q_c = softmax(z_p)[tok_c] for a child c of p, and the
 * candidate sequence that ends in node i gets the marginal probability of its tokens,
 * m_i = product of q over the root path of i (root excluded, m_root = 1).  Then either
 *   PROPD_PROB_THRESHOLD  node i goes when m_i < threshold (0 <= threshold <= 1), or
 *   PROPD_PROB_RANK       node i goes when keep_count or more nodes of its tree have a larger
 *                         marginal (equal marginals: the lower node index counts as larger),
 *                         i.e. the keep_count most probable sequences stay (keep_count >= 1).
 * Marginals never grow along a path, so both rules remove whole branches; the root always
 * stays; a token id outside [0,vocab) has probability 0 and always goes.  What follows the
 * decision - compaction, mask subsampling, payload rows, every output - is exactly as in
 * propd_early_prune, with the same arguments, layouts and workspace size.
 *
 *   log_marginal  [B,T_max] fp32 or NULL: log m_i of every node of the INPUT tree (0 for the
 *                 root and for padding), fully written
 * Scores are accumulated in fp32 and the marginals are summed in fp32 as logarithms: a
 * decision can differ from an exact evaluation where log m_i is within about 1e-3 of the
 * boundary.
 */
typedef enum { PROPD_PROB_THRESHOLD = 0, PROPD_PROB_RANK = 1 } propd_prob_mode;
PROPD_API propd_status propd_early_prune_prob(const propd_tree *tree, propd_dtype dt, int32_t hidden, int32_t vocab,
                               propd_prob_mode mode, float threshold, int32_t keep_count,
                               const void *hidden_states, const void *head_weight,
                               uint64_t *keep_bits, int32_t *new_index, int32_t *orig_index,
                               int32_t *n_kept, int32_t *cu_nodes, const propd_tree_out *tree_out,
                               float *log_marginal, int32_t n_payloads,
                               const propd_payload *payloads, void *workspace,
                               size_t workspace_bytes, void *hip_stream);

/*
 * Commit of the accepted path: what a decoding loop does between acceptance and the next
 * step (Section 2, "Verification": the longest verified sequence is kept; Section 5.1:
 * greedy decoding).  With a = accept_len[b] and L = seq_lens[b]:
 *   - the K/V rows of the accepted nodes accept_path[b,0..a-1] (root first) are copied from
 *     k_tree / v_tree to rows L..L+a-1 of k_cache / v_cache, for every head;
 *   - seq_lens[b] becomes L + a;
 *   - out_tokens[b,0..a-2] are the tokens of the accepted candidates (the path without its
 *     root, which was emitted by the step before), out_tokens[b,a-1] = next_token[b], the
 *     rest of the row is -1: the a tokens this step adds to the output, the last of which
 *     is the next step's root.
 * If the cache has room for fewer than a rows, only those that fit are copied and
 * seq_lens[b] stops at L_max; the tokens are still all written.
 *
 *   tree        B, T_max, n_nodes and (for out_tokens) token are read
 *   k_tree,v_tree   [B,H,T_max,d]   dt = PROPD_BF16 or PROPD_F32, d*sizeof a multiple of 16
 *   k_cache,v_cache [B,H,L_max,d]   in/out; rows outside L..L+a-1 are untouched
 *   seq_lens    [B]  in/out
 *   accept_len, accept_path, next_token   as written by propd_accept_path, same path_stride
 *   out_tokens  [B,out_stride] or NULL; entries beyond out_stride are dropped
 * Values read from device memory are made safe rather than reported: seq_lens is clamped to
 * [0, L_max], accept_len to [0, path_stride], and a path entry outside [0, n_nodes[b]) copies
 * no row (its cache row keeps its contents) and gives token -1.
 * No workspace.  Data pointers must be 16-byte aligned (PROPD_ERR_INVALID_ARG otherwise).
 * Must not overlap with a call that reads the same cache or seq_lens.
 */
PROPD_API propd_status propd_commit_path(const propd_tree *tree, propd_dtype dt, int32_t H, int32_t d,
                               const int32_t *accept_len, const int32_t *accept_path,
                               int32_t path_stride, const int32_t *next_token, const void *k_tree,
                               const void *v_tree, void *k_cache, void *v_cache, int32_t L_max,
                               int32_t *seq_lens, int32_t *out_tokens, int32_t out_stride,
                               void *hip_stream);

/*
 * Dynamic token-tree generation (Section 4.2): the controller that picks the tree size from
 * measured iteration times and measured head accuracies.  HOST code: every pointer below is
 * a host pointer, nothing is enqueued on a stream, no device is touched.  It is meant to run
 * now and then between decoding steps (Section 4.2.3), not every step.
 *
 * State lives in caller-owned host memory of propd_controller_bytes() bytes, 8-byte aligned,
 * set up once by propd_controller_init(); a state that was not initialised is rejected with
 * PROPD_ERR_INVALID_ARG.  Calls on one state must not overlap.
 *
 *   sizes        [n_sizes] the candidate tree sizes S (root included), strictly rising,
 *                1 <= size <= PROPD_MAX_TREE
 *   n_heads      number of prediction heads; head i proposes the token i+1 places after the root
 *   k_max        candidates per head that the statistics cover
 *   alpha        weight of a new sample in every running mean, 0 < alpha <= 1
 *   lambda       decay of the regression weight with the age of a mean, W = exp(-lambda * age),
 *                in units of 1/`now`
 *   hit_rate_init [n_heads*k_max] or NULL: starting values of P_i^k (frequency of "the true token
 *                is within the top-k of head i", k = 1..k_max), rising in k, within [0,1];
 *                NULL = zeros
 *
 * observe_time   Section 4.2.1: T_perf^size <- (1-alpha) T_perf^size + alpha t (the first
 *                sample of a size starts its mean), and its age restarts at `now`.  `size`
 *                must be one of S.  `now` is the caller's clock in any unit (steps, seconds).
 * observe_hit    Section 4.2.2: P_head^k <- (1-alpha) P_head^k + alpha [rank < k] for every k;
 *                `rank` is the 0-based position of the token that was finally decoded in
 *                that head's candidate list, negative (or >= k_max) when it was not in it.
 * fit            Section 4.2.1: beta0, beta1 minimising sum_i W_i (T_perf^i - beta0 - beta1 i)^2
 *                over the sizes seen so far, closed form.  One size seen: beta1 = 0.  None:
 *                PROPD_ERR_UNSUPPORTED.
 * build_tree     Section 4.2.2: the tree of `size` nodes with the largest estimated acceptance
 *                length, root first, every parent before its children:
 *                  parent[i]  index of the parent (-1 for the root)
 *                  depth[i]   0 for the root; a node at depth d comes from head d-1
 *                  choice[i]  0-based rank of the node's token in its head's list (-1 root)
 *                  node_value[i]  product of the accuracies p_j^(k_j) along its path (root 1)
 *                  *expected_len  sum of the node values
 *                  *n_built   nodes written: `size`, or fewer when the heads have no more
 *                             candidates (n_heads levels of k_max each)
 *                Output arrays hold `size` entries; any of them may be NULL except n_built.
 *                Equal values: the shallower node first, then the earlier parent, then the
 *                lower rank.
 * best_size      Section 4.2.3: speed[j] = l(sizes[j]) / T_est^(sizes[j]) for every candidate
 *                size (0 where the estimated time is not positive), *best_size = the size
 *                with the largest speed (the smaller one on a tie); speed, beta0, beta1 may
 *                be NULL.
 */
PROPD_API size_t propd_controller_bytes(int32_t n_sizes, int32_t n_heads, int32_t k_max);
PROPD_API propd_status propd_controller_init(void *state, size_t state_bytes, const int32_t *sizes,
                               int32_t n_sizes, int32_t n_heads, int32_t k_max, double alpha,
                               double lambda, const double *hit_rate_init);
PROPD_API propd_status propd_controller_observe_time(void *state, int32_t size, double t, double now);
PROPD_API propd_status propd_controller_observe_hit(void *state, int32_t head, int32_t rank);
PROPD_API propd_status propd_controller_fit(const void *state, double now, double *beta0, double *beta1);
PROPD_API propd_status propd_controller_build_tree(const void *state, int32_t size, int32_t *n_built,
                               int32_t *parent, int32_t *depth, int32_t *choice,
                               double *node_value, double *expected_len);
PROPD_API propd_status propd_controller_best_size(const void *state, double now, int32_t *best_size,
                               double *speed, double *beta0, double *beta1);

/* Workspace size in bytes for one call with these dimensions (arguments a call
 * does not have are ignored).  Pure host arithmetic: no device is queried, so the size is
 * the same on every machine and a size asked for before a call is accepted by that call.
 * Returns 0 for a bad `which`. */
typedef enum {
  PROPD_WS_TREE_ATTENTION = 0,
  PROPD_WS_EARLY_PRUNE = 1,
  PROPD_WS_ACCEPT_PATH = 2
} propd_ws_kind;
PROPD_API size_t propd_workspace_bytes(propd_ws_kind which, int32_t B, int32_t T_max, int32_t H, int32_t d,
                             int32_t L_max, int32_t hidden, int32_t vocab);

/* Static, NUL-terminated description of a status code. */
PROPD_API const char *propd_status_string(propd_status status);

#ifdef __cplusplus
}
#endif
#endif /* PROPD_H */
