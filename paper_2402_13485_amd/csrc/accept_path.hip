// Greedy longest-accepted-path selection (Section 3, "acceptance length";
// Section 5.1: greedy decoding so that the output equals the large model's).
//
// Two kernels:
//   row_argmax_kernel   g_i = argmax over the vocabulary of every tree node's
//                       logits row; one workgroup streams one row with 16-byte
//                       loads (HBM-bound: T_b * V * sizeof(dtype) bytes per sequence)
//   accept_path_kernel  one workgroup per sequence; token/g match bits by wave
//                       ballot, acceptance by testing the cached ancestor bitset
//                       against the match bits, deepest accepted node by a
//                       workgroup arg-max, path read off the winner's bitset.
#include "common.h"

namespace propd {

constexpr int kArgmaxThreads = 256;

__device__ __forceinline__ void argmax_take(float x, int idx, float &bv, int &bi) {
  if (x > bv || (x == bv && idx < bi)) {
    bv = x;
    bi = idx;
  }
}

// The same for a lane's own elements, which it visits in rising index order: a strictly larger
// value replaces the best, so the first of equal values stays.  Branch-free.
__device__ __forceinline__ void argmax_next(float x, int idx, float &bv, int &bi) {
  const bool take = x > bv;
  bv = take ? x : bv;
  bi = take ? idx : bi;
}

template <bool kBf16>
__global__ __launch_bounds__(kArgmaxThreads) void row_argmax_kernel(
    int T_max, int vocab, const int32_t *__restrict__ n_nodes, const void *__restrict__ logits,
    int32_t *__restrict__ greedy) {
  const int b = blockIdx.x / T_max, i = blockIdx.x - b * T_max;
  if (i >= n_nodes[b]) return;
  const size_t row = (size_t)b * T_max + i;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  const int tid = threadIdx.x;
  if (kBf16) {
    const uint16_t *p = reinterpret_cast<const uint16_t *>(logits) + row * (size_t)vocab;
    // peel to a 16-byte boundary, then 8 values per load
    int head = (int)(((16 - (reinterpret_cast<uintptr_t>(p) & 15)) & 15) >> 1);
    head = head < vocab ? head : vocab;
    if (tid < head) argmax_next(bf16_bits_to_f32(p[tid]), tid, bv, bi);
    const int nvec = (vocab - head) >> 3;
    const u32x4 *pv = reinterpret_cast<const u32x4 *>(p + head);
    // eight independent loads in flight per lane before any of them is used
    constexpr int kInFlight = 8;
    for (int c0 = tid; c0 < nvec; c0 += kInFlight * kArgmaxThreads) {
      u32x4 u[kInFlight];
#pragma unroll
      for (int k = 0; k < kInFlight; ++k) {
        const int c = c0 + k * kArgmaxThreads;
        u[k] = __builtin_nontemporal_load(pv + (c < nvec ? c : c0));
      }
#pragma unroll
      for (int k = 0; k < kInFlight; ++k) {
        const int c = c0 + k * kArgmaxThreads;
        if (c >= nvec) break;
        const int base = head + (c << 3);
        const uint32_t w[4] = {u[k].x, u[k].y, u[k].z, u[k].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          argmax_next(__uint_as_float(w[e] << 16), base + 2 * e, bv, bi);
          argmax_next(__uint_as_float(w[e] & 0xffff0000u), base + 2 * e + 1, bv, bi);
        }
      }
    }
    for (int v = head + (nvec << 3) + tid; v < vocab; v += kArgmaxThreads)
      argmax_next(bf16_bits_to_f32(p[v]), v, bv, bi);
  } else {
    const float *p = reinterpret_cast<const float *>(logits) + row * (size_t)vocab;
    int head = (int)(((16 - (reinterpret_cast<uintptr_t>(p) & 15)) & 15) >> 2);
    head = head < vocab ? head : vocab;
    if (tid < head) argmax_next(p[tid], tid, bv, bi);
    const int nvec = (vocab - head) >> 2;
    const f32x4 *pv = reinterpret_cast<const f32x4 *>(p + head);
    for (int c = tid; c < nvec; c += kArgmaxThreads) {
      f32x4 u = __builtin_nontemporal_load(pv + c);
      const int base = head + (c << 2);
      argmax_next(u.x, base, bv, bi);
      argmax_next(u.y, base + 1, bv, bi);
      argmax_next(u.z, base + 2, bv, bi);
      argmax_next(u.w, base + 3, bv, bi);
    }
    for (int v = head + (nvec << 2) + tid; v < vocab; v += kArgmaxThreads)
      argmax_next(p[v], v, bv, bi);
  }
  // wave reduction, then across the four waves
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(bv, o, kWave);
    int oi = __shfl_xor(bi, o, kWave);
    argmax_take(ov, oi, bv, bi);
  }
  __shared__ float sv[kArgmaxThreads / kWave];
  __shared__ int si[kArgmaxThreads / kWave];
  if ((tid & 63) == 0) {
    sv[tid >> 6] = bv;
    si[tid >> 6] = bi;
  }
  __syncthreads();
  if (tid == 0) {
#pragma unroll
    for (int w = 1; w < kArgmaxThreads / kWave; ++w) argmax_take(sv[w], si[w], bv, bi);
    greedy[row] = bi == 0x7fffffff ? 0 : bi;
  }
}

__global__ __launch_bounds__(PROPD_MAX_TREE) void accept_path_kernel(
    int T_max, int vocab, const int32_t *__restrict__ n_nodes, const int32_t *__restrict__ parent,
    const int32_t *__restrict__ token, const uint64_t *__restrict__ anc,
    const int32_t *__restrict__ greedy, int32_t *__restrict__ accept_len,
    int32_t *__restrict__ accept_path, int path_stride, int32_t *__restrict__ next_token) {
  const int b = blockIdx.x, i = threadIdx.x;
  int T = n_nodes[b];
  T = T < 1 ? 1 : (T > T_max ? T_max : T);
  const size_t base = (size_t)b * T_max;
  const bool valid = i < T;
  __shared__ uint64_t s_match[2];
  __shared__ int s_key[2];

  // does this node carry the model's own choice at its parent?
  bool match = false;
  uint64_t a_lo = 0, a_hi = 0;
  if (valid) {
    a_lo = anc[(base + i) * 2];
    a_hi = anc[(base + i) * 2 + 1];
    if (i == 0) {
      match = true;
    } else {
      const int p = parent[base + i];
      match = p >= 0 && p < T && token[base + i] == greedy[base + p];
    }
  }
  const uint64_t mb = __ballot(match);
  if ((i & 63) == 0) s_match[i >> 6] = mb;
  __syncthreads();
  // accepted iff every node of the root path matched; key orders by depth, then
  // by lower node index
  const bool acc = valid && ((a_lo & ~s_match[0]) | (a_hi & ~s_match[1])) == 0;
  const int nbits = __popcll(a_lo) + __popcll(a_hi);
  int key = acc ? (nbits << 8) | (255 - i) : -1;
  key = wave_reduce_max(key);
  __syncthreads();
  if ((i & 63) == 0) s_key[i >> 6] = key;
  __syncthreads();
  key = s_key[0] > s_key[1] ? s_key[0] : s_key[1];
  int best = key >= 0 ? 255 - (key & 255) : 0;  // the root is always accepted
  const uint64_t w_lo = anc[(base + best) * 2], w_hi = anc[(base + best) * 2 + 1];
  const int len = __popcll(w_lo) + __popcll(w_hi);
  if (valid && test_bit128(w_lo, w_hi, i)) {
    const int pos = popc128_below(w_lo, w_hi, i);
    if (pos < path_stride) accept_path[(size_t)b * path_stride + pos] = i;
  }
  for (int a = len + i; a < path_stride; a += PROPD_MAX_TREE)
    accept_path[(size_t)b * path_stride + a] = -1;
  if (i == 0) {
    accept_len[b] = len;
    next_token[b] = greedy[base + best];
  }
}

}  // namespace propd

extern "C" propd_status propd_accept_path(const propd_tree *tree, propd_dtype dt, int32_t vocab,
                                          const void *logits, int32_t *accept_len,
                                          int32_t *accept_path, int32_t path_stride,
                                          int32_t *next_token, void *workspace,
                                          size_t workspace_bytes, void *hip_stream) {
  using namespace propd;
  if (!tree || tree->B < 1 || tree->T_max < 1 || tree->T_max > PROPD_MAX_TREE || vocab < 1 ||
      path_stride < 1 || !tree->n_nodes || !tree->parent || !tree->token || !tree->anc ||
      !logits || !accept_len || !accept_path || !next_token)
    return PROPD_ERR_INVALID_ARG;
  if (dt != PROPD_BF16 && dt != PROPD_F32) return PROPD_ERR_INVALID_ARG;
  const size_t need =
      propd_workspace_bytes(PROPD_WS_ACCEPT_PATH, tree->B, tree->T_max, 0, 0, 0, 0, vocab);
  if (!workspace || workspace_bytes < need) return PROPD_ERR_WORKSPACE;
  int32_t *greedy = reinterpret_cast<int32_t *>(workspace);
  hipStream_t st = as_stream(hip_stream);
  if ((long long)tree->B * tree->T_max > (1ll << 30)) return PROPD_ERR_UNSUPPORTED;
  dim3 grid((unsigned)(tree->T_max * tree->B));
  if (dt == PROPD_BF16)
    hipLaunchKernelGGL(row_argmax_kernel<true>, grid, dim3(kArgmaxThreads), 0, st, tree->T_max,
                       vocab, tree->n_nodes, logits, greedy);
  else
    hipLaunchKernelGGL(row_argmax_kernel<false>, grid, dim3(kArgmaxThreads), 0, st, tree->T_max,
                       vocab, tree->n_nodes, logits, greedy);
  if (!launch_ok()) return PROPD_ERR_DEVICE;
  hipLaunchKernelGGL(accept_path_kernel, dim3(tree->B), dim3(PROPD_MAX_TREE), 0, st, tree->T_max,
                     vocab, tree->n_nodes, tree->parent, tree->token, tree->anc, greedy,
                     accept_len, accept_path, path_stride, next_token);
  return launch_ok() ? PROPD_OK : PROPD_ERR_DEVICE;
}
