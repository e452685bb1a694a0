// Cached token-tree mask: ancestor-or-self sets built on the GPU from parent
// pointers (Section 2, "Verification"; Section 4.1, "Implementation
// Optimization": the mask is kept on the GPU and later subsampled, never rebuilt
// on the host).
#include "common.h"

namespace propd {

// One workgroup per sequence, one lane per node.  Each lane climbs its own root
// path; the climb is bounded by T steps and every index is range-checked, so a
// malformed parent array cannot loop or read out of bounds.
__global__ __launch_bounds__(PROPD_MAX_TREE) void tree_mask_kernel(
    int T_max, const int32_t *__restrict__ n_nodes, const int32_t *__restrict__ parent,
    int32_t *__restrict__ depth, uint64_t *__restrict__ anc) {
  const int b = blockIdx.x;
  const int i = threadIdx.x;
  if (i >= T_max) return;
  int T = n_nodes[b];
  T = T < 0 ? 0 : (T > T_max ? T_max : T);
  const int32_t *par = parent + (size_t)b * T_max;
  uint64_t lo = 0, hi = 0;
  int steps = -1;
  if (i < T) {
    int x = i;
    for (int guard = 0; guard < T && x >= 0 && x < T; ++guard) {
      if (x < 64) lo |= 1ull << x; else hi |= 1ull << (x - 64);
      ++steps;
      x = par[x];
    }
  }
  anc[((size_t)b * T_max + i) * 2 + 0] = lo;
  anc[((size_t)b * T_max + i) * 2 + 1] = hi;
  if (depth) depth[(size_t)b * T_max + i] = steps;
}

// Debug check of the tree arrays (the fast entry points trust them): one workgroup per
// sequence, one lane per node; every lane recomputes its own root path from the parent
// pointers (bounded climb, indices range-checked) and compares with what the arrays say.
__global__ __launch_bounds__(PROPD_MAX_TREE) void validate_tree_kernel(
    int T_max, const int32_t *__restrict__ n_nodes, const int32_t *__restrict__ parent,
    const int32_t *__restrict__ depth, const uint64_t *__restrict__ anc,
    int32_t *__restrict__ flags) {
  const int b = blockIdx.x, i = threadIdx.x;
  const int T_raw = n_nodes[b];
  const int T = T_raw < 1 ? 1 : (T_raw > T_max ? T_max : T_raw);
  const int32_t *par = parent + (size_t)b * T_max;
  int bad = (T_raw < 1 || T_raw > T_max) ? PROPD_TREE_BAD_SIZE : 0;
  if (i < T) {
    const int p = par[i];
    const bool topo = i == 0 ? p == -1 : (p >= 0 && p < i);
    if (!topo) bad |= PROPD_TREE_BAD_PARENT;
    uint64_t lo = 0, hi = 0;
    int steps = -1, x = i;
    for (int guard = 0; guard < T && x >= 0 && x < T; ++guard) {
      if (x < 64) lo |= 1ull << x; else hi |= 1ull << (x - 64);
      ++steps;
      const int up = par[x];
      x = up < x ? up : -1;  // a pointer that does not go towards the root ends the climb
    }
    if (depth && depth[(size_t)b * T_max + i] != steps) bad |= PROPD_TREE_BAD_DEPTH;
    if (anc && (anc[((size_t)b * T_max + i) * 2] != lo || anc[((size_t)b * T_max + i) * 2 + 1] != hi))
      bad |= PROPD_TREE_BAD_MASK;
  }
  __shared__ int s_bad;
  if (i == 0) s_bad = 0;
  __syncthreads();
  if (bad) atomicOr(&s_bad, bad);
  __syncthreads();
  if (i == 0) flags[b] = s_bad;
}

}  // namespace propd

extern "C" propd_status propd_validate_tree(const propd_tree *tree, int32_t *flags, void *hip_stream) {
  if (!tree || tree->B < 1 || tree->T_max < 1 || tree->T_max > PROPD_MAX_TREE || !tree->n_nodes ||
      !tree->parent || !flags)
    return PROPD_ERR_INVALID_ARG;
  hipLaunchKernelGGL(propd::validate_tree_kernel, dim3(tree->B), dim3(PROPD_MAX_TREE), 0,
                     propd::as_stream(hip_stream), tree->T_max, tree->n_nodes, tree->parent,
                     tree->depth, tree->anc, flags);
  return propd::launch_ok() ? PROPD_OK : PROPD_ERR_DEVICE;
}

extern "C" propd_status propd_tree_mask(int32_t B, int32_t T_max, const int32_t *n_nodes,
                                        const int32_t *parent, int32_t *depth, uint64_t *anc,
                                        void *hip_stream) {
  if (B < 1 || T_max < 1 || T_max > PROPD_MAX_TREE || !n_nodes || !parent || !anc)
    return PROPD_ERR_INVALID_ARG;
  hipLaunchKernelGGL(propd::tree_mask_kernel, dim3(B), dim3(PROPD_MAX_TREE), 0,
                     propd::as_stream(hip_stream), T_max, n_nodes, parent, depth, anc);
  return propd::launch_ok() ? PROPD_OK : PROPD_ERR_DEVICE;
}

extern "C" const char *propd_status_string(propd_status status) {
  switch (status) {
    case PROPD_OK: return "ok";
    case PROPD_ERR_INVALID_ARG: return "invalid argument";
    case PROPD_ERR_UNSUPPORTED: return "unsupported configuration";
    case PROPD_ERR_WORKSPACE: return "workspace missing or too small";
    case PROPD_ERR_DEVICE: return "HIP launch failed";
  }
  return "unknown status";
}
