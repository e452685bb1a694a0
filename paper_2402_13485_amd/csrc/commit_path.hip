// Commit of the accepted path: the step that follows acceptance in a decoding loop
// (Section 2, "Verification": the longest verified sequence is kept; Section 5.1: greedy
// decoding).  The K/V rows of the accepted nodes move from the tree tensors to the end of
// the cache, the sequence grows by the acceptance length, and the step's tokens (the
// accepted candidates, then the model's own choice after the last of them) are written out.
#include "common.h"

namespace propd {

constexpr int kCommitThreads = 256;

// One workgroup per (sequence, head): 16 lanes move the 16-byte pieces of one row.  Indices
// read from device arrays are range-checked; rows that would pass the end of the cache are
// dropped.
__global__ __launch_bounds__(kCommitThreads) void commit_rows_kernel(
    int H, int T_max, int L_max, int row_bytes, const int32_t *__restrict__ n_nodes,
    const int32_t *__restrict__ accept_len, const int32_t *__restrict__ accept_path,
    int path_stride, const int32_t *__restrict__ seq_lens, const unsigned char *__restrict__ k_tree,
    const unsigned char *__restrict__ v_tree, unsigned char *__restrict__ k_cache,
    unsigned char *__restrict__ v_cache) {
  const int unit = blockIdx.x, b = unit / H;
  int T = n_nodes[b];
  T = T < 1 ? 1 : (T > T_max ? T_max : T);
  int L = seq_lens[b];
  L = L < 0 ? 0 : (L > L_max ? L_max : L);
  int a = accept_len[b];
  a = a < 0 ? 0 : (a > path_stride ? path_stride : a);
  a = a > L_max - L ? L_max - L : a;
  const int pieces = row_bytes / 16;
  const size_t tree_base = (size_t)unit * T_max * row_bytes, cache_base = (size_t)unit * L_max * row_bytes;
  for (int item = threadIdx.x; item < a * pieces; item += kCommitThreads) {
    const int j = item / pieces, c = item - j * pieces;
    const int node = accept_path[(size_t)b * path_stride + j];
    if (node < 0 || node >= T) continue;
    const size_t src = tree_base + (size_t)node * row_bytes + 16 * c;
    const size_t dst = cache_base + (size_t)(L + j) * row_bytes + 16 * c;
    *reinterpret_cast<u32x4 *>(k_cache + dst) = *reinterpret_cast<const u32x4 *>(k_tree + src);
    *reinterpret_cast<u32x4 *>(v_cache + dst) = *reinterpret_cast<const u32x4 *>(v_tree + src);
  }
}

// One lane per sequence: the new length and the step's tokens.  Runs after the row copy,
// which reads the old lengths.
__global__ __launch_bounds__(kCommitThreads) void commit_tokens_kernel(
    int B, int T_max, int L_max, const int32_t *__restrict__ n_nodes,
    const int32_t *__restrict__ token, const int32_t *__restrict__ accept_len,
    const int32_t *__restrict__ accept_path, int path_stride,
    const int32_t *__restrict__ next_token, int32_t *__restrict__ seq_lens,
    int32_t *__restrict__ out_tokens, int out_stride) {
  const int b = blockIdx.x * kCommitThreads + threadIdx.x;
  if (b >= B) return;
  int T = n_nodes[b];
  T = T < 1 ? 1 : (T > T_max ? T_max : T);
  int L = seq_lens[b];
  L = L < 0 ? 0 : (L > L_max ? L_max : L);
  int a = accept_len[b];
  a = a < 0 ? 0 : (a > path_stride ? path_stride : a);
  const int kept = a > L_max - L ? L_max - L : a;
  seq_lens[b] = L + kept;
  if (out_tokens) {
    for (int j = 0; j < out_stride; ++j) {
      int v = -1;
      if (j + 1 < a) {
        const int node = accept_path[(size_t)b * path_stride + j + 1];
        if (node >= 0 && node < T) v = token[(size_t)b * T_max + node];
      } else if (j + 1 == a) {
        v = next_token[b];
      }
      out_tokens[(size_t)b * out_stride + j] = v;
    }
  }
}

}  // namespace propd

extern "C" propd_status propd_commit_path(const propd_tree *tree, propd_dtype dt, int32_t H,
                                          int32_t d, const int32_t *accept_len,
                                          const int32_t *accept_path, int32_t path_stride,
                                          const int32_t *next_token, const void *k_tree,
                                          const void *v_tree, void *k_cache, void *v_cache,
                                          int32_t L_max, int32_t *seq_lens, int32_t *out_tokens,
                                          int32_t out_stride, void *hip_stream) {
  using namespace propd;
  if (!tree || tree->B < 1 || tree->T_max < 1 || tree->T_max > PROPD_MAX_TREE || H < 1 || d < 1 ||
      L_max < 1 || path_stride < 1 || !tree->n_nodes || !accept_len || !accept_path || !k_tree ||
      !v_tree || !k_cache || !v_cache || !seq_lens)
    return PROPD_ERR_INVALID_ARG;
  if (dt != PROPD_BF16 && dt != PROPD_F32) return PROPD_ERR_INVALID_ARG;
  if (out_tokens && (out_stride < 1 || !tree->token || !next_token)) return PROPD_ERR_INVALID_ARG;
  const long long row_bytes = (long long)d * (dt == PROPD_BF16 ? 2 : 4);
  if (row_bytes % 16 != 0 || row_bytes > (1 << 20)) return PROPD_ERR_UNSUPPORTED;
  for (const void *ptr : {k_tree, v_tree, (const void *)k_cache, (const void *)v_cache})
    if (reinterpret_cast<uintptr_t>(ptr) % 16 != 0) return PROPD_ERR_INVALID_ARG;
  const long long units = (long long)tree->B * H;
  if (units > (1ll << 30)) return PROPD_ERR_UNSUPPORTED;
  hipStream_t st = as_stream(hip_stream);
  hipLaunchKernelGGL(commit_rows_kernel, dim3((unsigned)units), dim3(kCommitThreads), 0, st, H,
                     tree->T_max, L_max, (int)row_bytes, tree->n_nodes, accept_len, accept_path,
                     path_stride, seq_lens, reinterpret_cast<const unsigned char *>(k_tree),
                     reinterpret_cast<const unsigned char *>(v_tree),
                     reinterpret_cast<unsigned char *>(k_cache),
                     reinterpret_cast<unsigned char *>(v_cache));
  if (!launch_ok()) return PROPD_ERR_DEVICE;
  hipLaunchKernelGGL(commit_tokens_kernel, dim3((unsigned)((tree->B + kCommitThreads - 1) / kCommitThreads)),
                     dim3(kCommitThreads), 0, st, tree->B, tree->T_max, L_max, tree->n_nodes,
                     tree->token, accept_len, accept_path, path_stride, next_token, seq_lens,
                     out_tokens, out_stride);
  return launch_ok() ? PROPD_OK : PROPD_ERR_DEVICE;
}
