/*
 * CPU oracle for the token-tree verification step of ProPD.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP sources, and nothing in the product path may call it.
 *
 * Every function states the passage of the paper it follows.  Floating point
 * is carried in double precision on the exact input bits (bf16 inputs are
 * widened exactly).  Trees are given by parent pointers only; ancestor sets are
 * found by walking them, never by bit tricks, so that the mask the GPU caches
 * is checked against an independent construction.
 *
 * Pins (see tests/test_oracle_*.py, all CPU-only):
 *   tree_mask        brute-force reachability, chain/star closed forms, bit counts
 *   tree_attention   library scaled-dot-product attention (causal special case,
 *                    explicit-mask general case, per-path linear sequences),
 *                    closed forms (q = 0, v = const)
 *   early_head_rank  membership in a stable descending sort, k = V, planted chain
 *   prune_compact    exhaustive fail patterns on small trees against a set-based
 *                    restatement; mask regenerated from compacted parents
 *   accept_path      simulated greedy autoregressive decoding, brute force over paths
 *   commit_path      library attention over the committed cache, many-step greedy
 *                    decoding against plain autoregressive decoding
 *
 * Return value of every function: 0 on success, a positive code on bad input.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_TREE 128
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static double load_value(const void *base, int dtype, int64_t idx) {
  if (dtype == ORACLE_F32) return (double)((const float *)base)[idx];
  uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

static int check_tree(int32_t T, const int32_t *parent) {
  if (T < 1 || T > ORACLE_MAX_TREE) return 1;
  if (parent[0] != -1) return 2;
  for (int32_t i = 1; i < T; ++i)
    if (parent[i] < 0 || parent[i] >= i) return 3;
  return 0;
}

/* Root path of node i, root first.  Returns its length (depth + 1). */
static int root_path(const int32_t *parent, int32_t i, int32_t *path) {
  int32_t tmp[ORACLE_MAX_TREE];
  int n = 0;
  for (int32_t x = i; x >= 0; x = parent[x]) tmp[n++] = x;
  for (int a = 0; a < n; ++a) path[a] = tmp[n - 1 - a];
  return n;
}

/*
 * Token-tree attention mask (Section 2, "Verification"; Figure 2(c)): a tree
 * token may look at exactly the tokens of its own candidate sequence, that is
 * the nodes on its root path, itself included.  anc[b,i] is that set as a
 * 128-bit set (word 0 = nodes 0..63), depth[b,i] the number of edges to the root.
 * Slots i >= n_nodes[b] get anc = 0, depth = -1.
 */
int propd_oracle_tree_mask(int32_t B, int32_t T_max, const int32_t *n_nodes,
                           const int32_t *parent, int32_t *depth, uint64_t *anc) {
  if (T_max < 1 || T_max > ORACLE_MAX_TREE) return 1;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t *par = parent + (int64_t)b * T_max;
    int32_t T = n_nodes[b];
    if (T > T_max) return 1;
    int rc = check_tree(T, par);
    if (rc) return rc;
    for (int32_t i = 0; i < T_max; ++i) {
      uint64_t *a = anc + ((int64_t)b * T_max + i) * 2;
      a[0] = a[1] = 0;
      depth[(int64_t)b * T_max + i] = -1;
      if (i >= T) continue;
      int32_t steps = -1;
      for (int32_t x = i; x >= 0; x = par[x]) {
        a[x >> 6] |= (uint64_t)1 << (x & 63);
        ++steps;
      }
      depth[(int64_t)b * T_max + i] = steps;
    }
  }
  return 0;
}

/*
 * Tree attention for a list of (b, h, i) rows (Section 2, "Verification").
 * Node i attends to every one of the L_b cached prefix tokens (the prefix is
 * computed once and shared) and to the tree tokens on its own root path:
 *   s_j = scale * <q_i, k_j>,  w_j = exp(s_j - max s),  o = sum w_j v_j / sum w_j.
 * Layouts: q, k_tree, v_tree [B,H,T_max,d]; k_cache, v_cache [B,H,L_max,d];
 * out [n_rows, d] in double, not rounded.
 */
int propd_oracle_tree_attention_rows(int32_t B, int32_t H, int32_t T_max, int32_t d,
                                     int32_t L_max, int dtype, double scale,
                                     const int32_t *n_nodes, const int32_t *parent,
                                     const int32_t *seq_lens, const void *q,
                                     const void *k_cache, const void *v_cache,
                                     const void *k_tree, const void *v_tree,
                                     int64_t n_rows, const int32_t *rows, double *out) {
  if (T_max < 1 || T_max > ORACLE_MAX_TREE || d < 1) return 1;
  for (int32_t b = 0; b < B; ++b) {
    if (n_nodes[b] > T_max || seq_lens[b] < 0 || seq_lens[b] > L_max) return 1;
    int rc = check_tree(n_nodes[b], parent + (int64_t)b * T_max);
    if (rc) return rc;
  }
  for (int64_t r = 0; r < n_rows; ++r) {
    int32_t b = rows[3 * r], h = rows[3 * r + 1], i = rows[3 * r + 2];
    if (b < 0 || b >= B || h < 0 || h >= H || i < 0 || i >= n_nodes[b]) return 4;
  }
  int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t r = 0; r < n_rows; ++r) {
    int32_t b = rows[3 * r], h = rows[3 * r + 1], i = rows[3 * r + 2];
    int32_t L = seq_lens[b];
    int32_t path[ORACLE_MAX_TREE];
    int np = root_path(parent + (int64_t)b * T_max, i, path);
    int64_t n = (int64_t)L + np;
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    if (!s) {
      failed = 1;
      continue;
    }
    int64_t q_off = (((int64_t)b * H + h) * T_max + i) * d;
    int64_t cache_off = ((int64_t)b * H + h) * (int64_t)L_max * d;
    int64_t tree_off = ((int64_t)b * H + h) * (int64_t)T_max * d;
    double m = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
      const void *kb = j < L ? k_cache : k_tree;
      int64_t k_off = j < L ? cache_off + j * d : tree_off + (int64_t)path[j - L] * d;
      double acc = 0.0;
      for (int32_t x = 0; x < d; ++x)
        acc += load_value(q, dtype, q_off + x) * load_value(kb, dtype, k_off + x);
      s[j] = scale * acc;
      if (s[j] > m) m = s[j];
    }
    double denom = 0.0;
    double *o = out + r * d;
    for (int32_t x = 0; x < d; ++x) o[x] = 0.0;
    for (int64_t j = 0; j < n; ++j) {
      double w = exp(s[j] - m);
      denom += w;
      const void *vb = j < L ? v_cache : v_tree;
      int64_t v_off = j < L ? cache_off + j * d : tree_off + (int64_t)path[j - L] * d;
      for (int32_t x = 0; x < d; ++x) o[x] += w * load_value(vb, dtype, v_off + x);
    }
    for (int32_t x = 0; x < d; ++x) o[x] /= denom;
    free(s);
  }
  return failed ? 5 : 0;
}

/* All rows (b, h, i < n_nodes[b]); out [B,H,T_max,d] double, other rows untouched. */
int propd_oracle_tree_attention(int32_t B, int32_t H, int32_t T_max, int32_t d, int32_t L_max,
                                int dtype, double scale, const int32_t *n_nodes,
                                const int32_t *parent, const int32_t *seq_lens, const void *q,
                                const void *k_cache, const void *v_cache, const void *k_tree,
                                const void *v_tree, double *out) {
  int64_t total = 0;
  for (int32_t b = 0; b < B; ++b) {
    if (n_nodes[b] < 1 || n_nodes[b] > T_max) return 1;
    total += (int64_t)H * n_nodes[b];
  }
  int32_t *rows = (int32_t *)calloc(3 * (size_t)total, sizeof(int32_t));
  double *tmp = (double *)malloc(sizeof(double) * (size_t)total * d);
  if (!rows || !tmp) {
    free(rows);
    free(tmp);
    return 5;
  }
  int64_t r = 0;
  for (int32_t b = 0; b < B; ++b)
    for (int32_t h = 0; h < H; ++h)
      for (int32_t i = 0; i < n_nodes[b]; ++i) {
        rows[3 * r] = b;
        rows[3 * r + 1] = h;
        rows[3 * r + 2] = i;
        ++r;
      }
  int rc = propd_oracle_tree_attention_rows(B, H, T_max, d, L_max, dtype, scale, n_nodes, parent,
                                            seq_lens, q, k_cache, v_cache, k_tree, v_tree, total,
                                            rows, tmp);
  if (!rc)
    for (r = 0; r < total; ++r) {
      int64_t off = (((int64_t)rows[3 * r] * H + rows[3 * r + 1]) * T_max + rows[3 * r + 2]) * d;
      memcpy(out + off, tmp + r * d, sizeof(double) * (size_t)d);
    }
  free(rows);
  free(tmp);
  return rc;
}

static int cmp_desc(const void *a, const void *b) {
  double x = *(const double *)a, y = *(const double *)b;
  return (x < y) - (x > y);
}

/*
 * Early prediction head and the top-k test (Section 4.1, "Pruning Process",
 * first two steps).  After the early layers every tree token x_i is mapped by
 * the head to scores over the vocabulary, z_p = W h_p with W stored [V, Hd];
 * TopK(x_i) is the k best-scoring ids.  A child c of p belongs to it exactly
 * when fewer than k ids beat its own token, counting an equal score as a win
 * for the lower id:
 *   rank_c = #{v : z_p[v] > z_p[tok_c]} + #{v < tok_c : z_p[v] == z_p[tok_c]}.
 * rank [B,T_max]: 0 for the root, -1 for padding.
 * margin [B,T_max]: distance of z_p[tok_c] to the far side of the k boundary
 * (to the (k+1)-th best score if the child passes, to the k-th best if it
 * fails); +inf for the root, when k >= V, and for padding.
 */
int propd_oracle_early_head_rank(int32_t B, int32_t T_max, int32_t hidden, int32_t vocab,
                                 int dtype, int32_t top_k, const int32_t *n_nodes,
                                 const int32_t *parent, const int32_t *token,
                                 const void *hidden_states, const void *head_weight,
                                 int32_t *rank, double *margin) {
  if (T_max < 1 || T_max > ORACLE_MAX_TREE || top_k < 1 || vocab < 1 || hidden < 1) return 1;
  for (int32_t b = 0; b < B; ++b) {
    if (n_nodes[b] > T_max) return 1;
    int rc = check_tree(n_nodes[b], parent + (int64_t)b * T_max);
    if (rc) return rc;
    for (int32_t c = 1; c < n_nodes[b]; ++c) {
      int32_t t = token[(int64_t)b * T_max + c];
      if (t < 0 || t >= vocab) return 6;
    }
  }
  for (int64_t x = 0; x < (int64_t)B * T_max; ++x) {
    rank[x] = -1;
    margin[x] = INFINITY;
  }
  int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t bp = 0; bp < (int64_t)B * T_max; ++bp) {
    int32_t b = (int32_t)(bp / T_max), p = (int32_t)(bp % T_max);
    int32_t T = n_nodes[b];
    if (p >= T) continue;
    const int32_t *par = parent + (int64_t)b * T_max;
    if (p == 0) rank[bp] = 0;
    int has_child = 0;
    for (int32_t c = p + 1; c < T; ++c) has_child |= (par[c] == p);
    if (!has_child) continue;
    double *z = (double *)malloc(sizeof(double) * 2 * (size_t)vocab);
    if (!z) {
      failed = 1;
      continue;
    }
    double *zs = z + vocab;
    for (int32_t v = 0; v < vocab; ++v) {
      double acc = 0.0;
      for (int32_t x = 0; x < hidden; ++x)
        acc += load_value(hidden_states, dtype, bp * hidden + x) *
               load_value(head_weight, dtype, (int64_t)v * hidden + x);
      z[v] = acc;
    }
    memcpy(zs, z, sizeof(double) * (size_t)vocab);
    qsort(zs, (size_t)vocab, sizeof(double), cmp_desc);
    for (int32_t c = p + 1; c < T; ++c) {
      if (par[c] != p) continue;
      int32_t tok = token[(int64_t)b * T_max + c];
      int32_t r = 0;
      for (int32_t v = 0; v < vocab; ++v)
        r += (z[v] > z[tok]) || (z[v] == z[tok] && v < tok);
      rank[(int64_t)b * T_max + c] = r;
      double mg = INFINITY;
      if (top_k < vocab) mg = (r < top_k) ? z[tok] - zs[top_k] : zs[top_k - 1] - z[tok];
      margin[(int64_t)b * T_max + c] = mg;
    }
    free(z);
  }
  return failed ? 5 : 0;
}

/*
 * Probability-based selection (Section 4.1, "Pruning Criterion", the second criterion): the
 * early head's scores are turned into predicted probabilities, q_c = softmax(z_p)[tok_c] for
 * a child c of p, and a candidate sequence gets the marginal probability of its tokens, the
 * product of q along its root path.  In logarithms:
 *   logq[c]   = z_p[tok_c] - log sum_v exp(z_p[v])        (0 for the root)
 *   logm[c]   = logm[parent(c)] + logq[c]                  (0 for the root)
 * Both [B,T_max]; padding entries are set to 0 and carry no meaning.
 * The decisions themselves (threshold or rank over logm) are taken by the caller.
 */
int propd_oracle_early_head_logprob(int32_t B, int32_t T_max, int32_t hidden, int32_t vocab,
                                    int dtype, const int32_t *n_nodes, const int32_t *parent,
                                    const int32_t *token, const void *hidden_states,
                                    const void *head_weight, double *logq, double *logm) {
  if (T_max < 1 || T_max > ORACLE_MAX_TREE || vocab < 1 || hidden < 1) return 1;
  for (int32_t b = 0; b < B; ++b) {
    if (n_nodes[b] > T_max) return 1;
    int rc = check_tree(n_nodes[b], parent + (int64_t)b * T_max);
    if (rc) return rc;
    for (int32_t c = 1; c < n_nodes[b]; ++c) {
      int32_t t = token[(int64_t)b * T_max + c];
      if (t < 0 || t >= vocab) return 6;
    }
  }
  for (int64_t x = 0; x < (int64_t)B * T_max; ++x) logq[x] = logm[x] = 0.0;
  int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t bp = 0; bp < (int64_t)B * T_max; ++bp) {
    int32_t b = (int32_t)(bp / T_max), p = (int32_t)(bp % T_max);
    int32_t T = n_nodes[b];
    if (p >= T) continue;
    const int32_t *par = parent + (int64_t)b * T_max;
    int has_child = 0;
    for (int32_t c = p + 1; c < T; ++c) has_child |= (par[c] == p);
    if (!has_child) continue;
    double *z = (double *)malloc(sizeof(double) * (size_t)vocab);
    if (!z) {
      failed = 1;
      continue;
    }
    double zmax = -INFINITY;
    for (int32_t v = 0; v < vocab; ++v) {
      double acc = 0.0;
      for (int32_t x = 0; x < hidden; ++x)
        acc += load_value(hidden_states, dtype, bp * hidden + x) *
               load_value(head_weight, dtype, (int64_t)v * hidden + x);
      z[v] = acc;
      if (acc > zmax) zmax = acc;
    }
    double sum = 0.0;
    for (int32_t v = 0; v < vocab; ++v) sum += exp(z[v] - zmax);
    double lse = zmax + log(sum);
    for (int32_t c = p + 1; c < T; ++c)
      if (par[c] == p) logq[(int64_t)b * T_max + c] = z[token[(int64_t)b * T_max + c]] - lse;
    free(z);
  }
  if (failed) return 5;
  for (int32_t b = 0; b < B; ++b)
    for (int32_t c = 1; c < n_nodes[b]; ++c) {
      int64_t o = (int64_t)b * T_max;
      logm[o + c] = logm[o + parent[o + c]] + logq[o + c];
    }
  return 0;
}

/*
 * Branch elimination, compaction and mask subsampling (Section 4.1, third
 * step of "Pruning Process" and "Implementation Optimization").  A token
 * fails when its rank is not below k; every candidate sequence that contains a
 * failed token goes, i.e. a node survives only if it passes and its parent
 * survives; the root (the token the model has already fixed) always stays.
 * Survivors keep their relative order.  The new mask is the old mask restricted
 * to surviving rows and columns.
 *
 * Outputs, all fully written:
 *   keep_bits [B,2]     bit i set iff node i survives
 *   new_index [B,T_max] position of node i among survivors, -1 if pruned/padding
 *   orig_index[B,T_max] old index of survivor j, -1 for j >= n_kept[b]
 *   n_kept [B], cu_nodes [B+1] (exclusive prefix sum of n_kept)
 *   parent_out/token_out/depth_out [B,T_max]  survivors first, -1 beyond
 *   anc_out [B,T_max,2]  restricted mask, 0 beyond
 */
int propd_oracle_prune_compact(int32_t B, int32_t T_max, int32_t top_k, const int32_t *n_nodes,
                               const int32_t *parent, const int32_t *token, const int32_t *rank,
                               uint64_t *keep_bits, int32_t *new_index, int32_t *orig_index,
                               int32_t *n_kept, int32_t *cu_nodes, int32_t *parent_out,
                               int32_t *token_out, int32_t *depth_out, uint64_t *anc_out) {
  if (T_max < 1 || T_max > ORACLE_MAX_TREE || top_k < 1) return 1;
  cu_nodes[0] = 0;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t *par = parent + (int64_t)b * T_max;
    const int32_t *tok = token + (int64_t)b * T_max;
    const int32_t *rk = rank + (int64_t)b * T_max;
    int32_t T = n_nodes[b];
    if (T > T_max) return 1;
    int rc = check_tree(T, par);
    if (rc) return rc;
    unsigned char keep[ORACLE_MAX_TREE];
    unsigned char mask[ORACLE_MAX_TREE][ORACLE_MAX_TREE];
    int32_t dep[ORACLE_MAX_TREE];
    memset(mask, 0, sizeof mask);
    for (int32_t i = 0; i < T; ++i) {
      keep[i] = (i == 0) ? 1 : (keep[par[i]] && rk[i] < top_k);
      dep[i] = -1;
      for (int32_t x = i; x >= 0; x = par[x]) {
        mask[i][x] = 1;
        ++dep[i];
      }
    }
    int32_t *ni = new_index + (int64_t)b * T_max, *oi = orig_index + (int64_t)b * T_max;
    int32_t *po = parent_out + (int64_t)b * T_max, *to = token_out + (int64_t)b * T_max;
    int32_t *dn = depth_out + (int64_t)b * T_max;
    uint64_t *ao = anc_out + (int64_t)b * T_max * 2;
    keep_bits[2 * b] = keep_bits[2 * b + 1] = 0;
    for (int32_t i = 0; i < T_max; ++i) {
      ni[i] = oi[i] = po[i] = to[i] = dn[i] = -1;
      ao[2 * i] = ao[2 * i + 1] = 0;
    }
    int32_t cnt = 0;
    for (int32_t i = 0; i < T; ++i)
      if (keep[i]) {
        keep_bits[2 * b + (i >> 6)] |= (uint64_t)1 << (i & 63);
        ni[i] = cnt;
        oi[cnt] = i;
        ++cnt;
      }
    n_kept[b] = cnt;
    cu_nodes[b + 1] = cu_nodes[b] + cnt;
    for (int32_t j = 0; j < cnt; ++j) {
      int32_t i = oi[j];
      po[j] = (i == 0) ? -1 : ni[par[i]];
      to[j] = tok[i];
      dn[j] = dep[i];
      for (int32_t j2 = 0; j2 < cnt; ++j2)
        if (mask[i][oi[j2]]) ao[2 * j + (j2 >> 6)] |= (uint64_t)1 << (j2 & 63);
    }
  }
  return 0;
}

/*
 * Row payloads that continue past the pruning point (hidden states, tree K/V
 * rows) are narrowed to the survivors, which is what "reduces the computation in
 * subsequent layers" (Section 3, Observation 1; Section 4.1).  A tensor is seen
 * as [B, outer, T_max] rows of row_bytes bytes with byte strides; survivor row
 * (b, o, orig_index[b,j]) of src is copied to (b, o, j) of dst for j < n_kept[b].
 */
int propd_oracle_gather_rows(int32_t B, int64_t outer, int32_t T_max, int64_t row_bytes,
                             int64_t stride_b, int64_t stride_outer, int64_t stride_t,
                             const int32_t *orig_index, const int32_t *n_kept,
                             const unsigned char *src, unsigned char *dst) {
  for (int32_t b = 0; b < B; ++b)
    for (int64_t o = 0; o < outer; ++o)
      for (int32_t j = 0; j < n_kept[b]; ++j) {
        int32_t i = orig_index[(int64_t)b * T_max + j];
        if (i < 0 || i >= T_max) return 7;
        memcpy(dst + b * stride_b + o * stride_outer + (int64_t)j * stride_t,
               src + b * stride_b + o * stride_outer + (int64_t)i * stride_t, (size_t)row_bytes);
      }
  return 0;
}

/*
 * Greedy acceptance (Section 3, "acceptance length"; Section 5.1: greedy
 * decoding so that the output equals the large model's own).  g_i is the
 * model's greedy choice after node i (lowest id among equal maxima).  A child
 * is accepted when its token equals its parent's greedy choice and its parent
 * is accepted; the root is the already-fixed token and is always accepted.
 * The result is the deepest accepted node (lowest index among equals), its
 * root path, the path's node count, and the greedy choice at its end.
 *   accept_path [B,path_stride]  node indices root first, -1 padded
 */
int propd_oracle_accept_path(int32_t B, int32_t T_max, int32_t vocab, int dtype,
                             const int32_t *n_nodes, const int32_t *parent, const int32_t *token,
                             const void *logits, int32_t *accept_len, int32_t *accept_path,
                             int32_t path_stride, int32_t *next_token) {
  if (T_max < 1 || T_max > ORACLE_MAX_TREE || vocab < 1 || path_stride < 1) return 1;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t *par = parent + (int64_t)b * T_max;
    const int32_t *tok = token + (int64_t)b * T_max;
    int32_t T = n_nodes[b];
    if (T > T_max) return 1;
    int rc = check_tree(T, par);
    if (rc) return rc;
    int32_t g[ORACLE_MAX_TREE];
    for (int32_t i = 0; i < T; ++i) {
      int64_t off = ((int64_t)b * T_max + i) * vocab;
      int32_t best = 0;
      double bv = load_value(logits, dtype, off);
      for (int32_t v = 1; v < vocab; ++v) {
        double x = load_value(logits, dtype, off + v);
        if (x > bv) {
          bv = x;
          best = v;
        }
      }
      g[i] = best;
    }
    int32_t best_node = 0, best_len = 1;
    for (int32_t i = 0; i < T; ++i) {
      int32_t path[ORACLE_MAX_TREE];
      int np = root_path(par, i, path);
      int ok = 1;
      for (int a = 1; a < np; ++a) ok &= (tok[path[a]] == g[path[a - 1]]);
      if (ok && np > best_len) {
        best_len = np;
        best_node = i;
      }
    }
    if (best_len > path_stride) return 8;
    int32_t path[ORACLE_MAX_TREE];
    int np = root_path(par, best_node, path);
    for (int32_t a = 0; a < path_stride; ++a)
      accept_path[(int64_t)b * path_stride + a] = a < np ? path[a] : -1;
    accept_len[b] = np;
    next_token[b] = g[best_node];
  }
  return 0;
}

/*
 * Commit of the accepted path (Section 2, "Verification": the longest verified
 * sequence is kept; Section 5.1: greedy decoding).  For every sequence, with
 * a = accept_len and L = seq_lens: the K/V rows of the a accepted nodes (root
 * first) become rows L..L+a-1 of the cache of every head, the length becomes
 * L + a, and the step's a tokens are the tokens of the accepted candidates (the
 * path without the root) followed by next_token.  Rows that do not fit under
 * L_max are dropped and the length stops there.
 *   elem_bytes  bytes of one K/V element (2 or 4); rows are copied as bytes
 *   out_tokens  [B,out_stride], -1 padded, or NULL
 */
int propd_oracle_commit_path(int32_t B, int32_t H, int32_t d, int32_t T_max, int32_t L_max,
                             int32_t elem_bytes, const int32_t *n_nodes, const int32_t *token,
                             const int32_t *accept_len, const int32_t *accept_path,
                             int32_t path_stride, const int32_t *next_token,
                             const unsigned char *k_tree, const unsigned char *v_tree,
                             unsigned char *k_cache, unsigned char *v_cache, int32_t *seq_lens,
                             int32_t *out_tokens, int32_t out_stride) {
  if (B < 1 || H < 1 || d < 1 || T_max < 1 || L_max < 1 || path_stride < 1) return 1;
  const int64_t row = (int64_t)d * elem_bytes;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t a = accept_len[b], L = seq_lens[b], T = n_nodes[b];
    if (a < 1 || a > path_stride || L < 0 || L > L_max || T < 1 || T > T_max) return 2;
    for (int32_t j = 0; j < a; ++j) {
      const int32_t node = accept_path[(int64_t)b * path_stride + j];
      if (node < 0 || node >= T) return 3;
      if (L + j >= L_max) continue; /* no room: dropped */
      for (int32_t h = 0; h < H; ++h) {
        const int64_t unit = (int64_t)b * H + h;
        const int64_t src = (unit * T_max + node) * row, dst = (unit * L_max + L + j) * row;
        memcpy(k_cache + dst, k_tree + src, (size_t)row);
        memcpy(v_cache + dst, v_tree + src, (size_t)row);
      }
    }
    seq_lens[b] = L + a > L_max ? L_max : L + a;
    if (out_tokens) {
      for (int32_t j = 0; j < out_stride; ++j) {
        int32_t v = -1;
        if (j + 1 < a) v = token[(int64_t)b * T_max + accept_path[(int64_t)b * path_stride + j + 1]];
        else if (j + 1 == a) v = next_token[b];
        out_tokens[(int64_t)b * out_stride + j] = v;
      }
    }
  }
  return 0;
}

/* Number of OpenMP threads the parallel loops above will use (1 without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int propd_oracle_threads(void) { return omp_get_max_threads(); }
void propd_oracle_set_threads(int n) { omp_set_num_threads(n); }
#else
int propd_oracle_threads(void) { return 1; }
void propd_oracle_set_threads(int n) { (void)n; }
#endif
