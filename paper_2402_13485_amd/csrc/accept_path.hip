// Greedy longest-accepted-path selection (Section 3, "acceptance length";
// Section 5.1: greedy decoding so that the output equals the large model's).
//
// Two kernels:
//   row_argmax_kernel   partial arg-max of every tree node's logits row.  A row is cut into
//                       up to kMaxSlices slices of about 16 KB; a persistent grid walks the
//                       (row, slice) items of the rows that exist (their number is device
//                       data), 16-byte loads, all loads of an item in flight before the first
//                       is used (HBM-bound: T_b * V * sizeof(dtype) bytes per sequence)
//   accept_path_kernel  one workgroup per sequence; merges the slices of every row into
//                       g_i = argmax (lowest id among equal maxima), token/g match bits by
//                       wave ballot, acceptance by testing the cached ancestor bitset
//                       against the match bits, deepest accepted node by a workgroup
//                       arg-max, path read off the winner's bitset.
#include <mutex>

#include "common.h"

namespace propd {

constexpr int kArgmaxThreads = 256;
constexpr int kMaxSlices = 8;        // slices of a logits row, at most
constexpr int kSliceBytes = 16384;   // aimed-at size of a slice
constexpr int kArgmaxMaxGrid = 2048;  // eight resident workgroups per compute unit

struct RowPart {  // arg-max of one slice of one row
  float v;
  int32_t i;
};

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

// Arg-max over elements [lo, hi) of one row, spread over the workgroup's threads; every thread
// visits its elements in rising index order.
template <bool kBf16>
__device__ __forceinline__ void argmax_slice(const void *row_ptr, int lo, int hi, int tid, float &bv,
                                             int &bi) {
  constexpr int kInFlight = 4;  // independent 16-byte loads of a lane before any is used
  if (kBf16) {
    const uint16_t *p = reinterpret_cast<const uint16_t *>(row_ptr);
    // peel to a 16-byte boundary, then 8 values per load
    int head = (int)(((16 - (reinterpret_cast<uintptr_t>(p + lo) & 15)) & 15) >> 1);
    head = head < hi - lo ? head : hi - lo;
    if (tid < head) argmax_next(bf16_bits_to_f32(p[lo + tid]), lo + tid, bv, bi);
    const int first = lo + head, nvec = (hi - first) >> 3;
    const u32x4 *pv = reinterpret_cast<const u32x4 *>(p + first);
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
        const int base = first + (c << 3);
        const uint32_t w[4] = {u[k].x, u[k].y, u[k].z, u[k].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          argmax_next(__uint_as_float(w[e] << 16), base + 2 * e, bv, bi);
          argmax_next(__uint_as_float(w[e] & 0xffff0000u), base + 2 * e + 1, bv, bi);
        }
      }
    }
    for (int v = first + (nvec << 3) + tid; v < hi; v += kArgmaxThreads)
      argmax_next(bf16_bits_to_f32(p[v]), v, bv, bi);
  } else {
    const float *p = reinterpret_cast<const float *>(row_ptr);
    int head = (int)(((16 - (reinterpret_cast<uintptr_t>(p + lo) & 15)) & 15) >> 2);
    head = head < hi - lo ? head : hi - lo;
    if (tid < head) argmax_next(p[lo + tid], lo + tid, bv, bi);
    const int first = lo + head, nvec = (hi - first) >> 2;
    const f32x4 *pv = reinterpret_cast<const f32x4 *>(p + first);
    for (int c0 = tid; c0 < nvec; c0 += kInFlight * kArgmaxThreads) {
      f32x4 u[kInFlight];
#pragma unroll
      for (int k = 0; k < kInFlight; ++k) {
        const int c = c0 + k * kArgmaxThreads;
        u[k] = __builtin_nontemporal_load(pv + (c < nvec ? c : c0));
      }
#pragma unroll
      for (int k = 0; k < kInFlight; ++k) {
        const int c = c0 + k * kArgmaxThreads;
        if (c >= nvec) break;
        const int base = first + (c << 2);
        argmax_next(u[k].x, base, bv, bi);
        argmax_next(u[k].y, base + 1, bv, bi);
        argmax_next(u[k].z, base + 2, bv, bi);
        argmax_next(u[k].w, base + 3, bv, bi);
      }
    }
    for (int v = first + (nvec << 2) + tid; v < hi; v += kArgmaxThreads) argmax_next(p[v], v, bv, bi);
  }
}

__device__ __forceinline__ int clamp_nodes(int T, int T_max) { return T < 1 ? 1 : (T > T_max ? T_max : T); }

// Tree sizes of 64 sequences, one per lane, with their inclusive prefix sums over the lanes.
struct SeqSizes {
  int mine, incl, total;
};
__device__ __forceinline__ SeqSizes load_seq_sizes(int b0, int B, int T_max,
                                                   const int32_t *__restrict__ n_nodes) {
  const int lane = threadIdx.x & 63;
  SeqSizes z;
  z.mine = b0 + lane < B ? clamp_nodes(n_nodes[b0 + lane], T_max) : 0;
  z.incl = z.mine;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(z.incl, o, kWave);
    if (lane >= o) z.incl += up;
  }
  z.total = __shfl(z.incl, 63, kWave);
  return z;
}

// Items are (row, slice) pairs of the rows that exist, rows counted sequence by sequence.
// Every wave finds the sequence of a row by itself from the prefix sums (no LDS, no workgroup
// barrier); `first` holds the sizes of sequences 0..63, loaded once.
__device__ __forceinline__ void locate_row(int r, int B, int T_max, const int32_t *__restrict__ n_nodes,
                                           const SeqSizes &first, int &b_out, int &i_out) {
  int base = 0, b_found = -1, i_found = 0;
  for (int b0 = 0; b0 < B && b_found < 0; b0 += 64) {
    const SeqSizes z = b0 == 0 ? first : load_seq_sizes(b0, B, T_max, n_nodes);
    if (r < base + z.total) {
      // the holder is the first sequence whose inclusive count passes r
      const int src = __popcll(__ballot(base + z.incl <= r));
      b_found = b0 + src;
      i_found = r - (base + __shfl(z.incl - z.mine, src, kWave));
    }
    base += z.total;
  }
  b_out = b_found;
  i_out = i_found;
}

template <bool kBf16>
__global__ __launch_bounds__(kArgmaxThreads) void row_argmax_kernel(
    int B, int T_max, int vocab, int slices, int per, const int32_t *__restrict__ n_nodes,
    const void *__restrict__ logits, RowPart *__restrict__ part) {
  const int tid = threadIdx.x, lane = tid & 63;
  const SeqSizes first = load_seq_sizes(0, B, T_max, n_nodes);
  int rows = first.total;
  for (int b0 = 64; b0 < B; b0 += 64) rows += load_seq_sizes(b0, B, T_max, n_nodes).total;
  const long long items = (long long)rows * slices;
  __shared__ float sv[kArgmaxThreads / kWave];
  __shared__ int si[kArgmaxThreads / kWave];
  for (long long w = blockIdx.x; w < items; w += gridDim.x) {
    const int r = (int)(w / slices), s = (int)(w - (long long)r * slices);
    int b, i;
    locate_row(r, B, T_max, n_nodes, first, b, i);
    if (b < 0) break;  // cannot happen: r < rows
    const size_t row = (size_t)b * T_max + i;
    const int lo = s * per < vocab ? s * per : vocab, hi = lo + per < vocab ? lo + per : vocab;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    const char *row_ptr = reinterpret_cast<const char *>(logits) + row * (size_t)vocab * (kBf16 ? 2 : 4);
    argmax_slice<kBf16>(row_ptr, lo, hi, tid, bv, bi);
    // wave reduction, then across the four waves
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      float ov = __shfl_xor(bv, o, kWave);
      int oi = __shfl_xor(bi, o, kWave);
      argmax_take(ov, oi, bv, bi);
    }
    if (lane == 0) {
      sv[tid >> 6] = bv;
      si[tid >> 6] = bi;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
      for (int wv = 1; wv < kArgmaxThreads / kWave; ++wv) argmax_take(sv[wv], si[wv], bv, bi);
      RowPart out;
      out.v = bv;
      out.i = bi;
      part[row * kMaxSlices + s] = out;
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(PROPD_MAX_TREE) void accept_path_kernel(
    int T_max, int slices, const int32_t *__restrict__ n_nodes, const int32_t *__restrict__ parent,
    const int32_t *__restrict__ token, const uint64_t *__restrict__ anc,
    const RowPart *__restrict__ part, int32_t *__restrict__ accept_len,
    int32_t *__restrict__ accept_path, int path_stride, int32_t *__restrict__ next_token) {
  const int b = blockIdx.x, i = threadIdx.x;
  const int T = clamp_nodes(n_nodes[b], T_max);
  const size_t base = (size_t)b * T_max;
  const bool valid = i < T;
  __shared__ uint64_t s_match[2];
  __shared__ int s_key[2];
  __shared__ int s_greedy[PROPD_MAX_TREE];

  // g_i: the slices of row i, merged (lowest id among equal maxima)
  uint64_t a_lo = 0, a_hi = 0;
  if (valid) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int s = 0; s < slices; ++s) {
      const RowPart q = part[(base + i) * kMaxSlices + s];
      argmax_take(q.v, q.i, bv, bi);
    }
    s_greedy[i] = bi == 0x7fffffff ? 0 : bi;
    a_lo = anc[(base + i) * 2];
    a_hi = anc[(base + i) * 2 + 1];
  }
  __syncthreads();
  // does this node carry the model's own choice at its parent?
  bool match = false;
  if (valid) {
    if (i == 0) {
      match = true;
    } else {
      const int p = parent[base + i];
      match = p >= 0 && p < T && token[base + i] == s_greedy[p];
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
  if ((i & 63) == 0) s_key[i >> 6] = key;
  __syncthreads();
  key = s_key[0] > s_key[1] ? s_key[0] : s_key[1];
  const int best = key >= 0 ? 255 - (key & 255) : 0;  // the root is always accepted
  const uint64_t w_lo = anc[(base + best) * 2], w_hi = anc[(base + best) * 2 + 1];
  const int full = __popcll(w_lo) + __popcll(w_hi);
  // A path buffer shorter than the accepted path keeps the path's first path_stride nodes:
  // they are accepted themselves, and the model's choice after the last of them (the token
  // of the next node of the path) continues the same greedy output.
  const int len = full < path_stride ? full : path_stride;
  if (valid && test_bit128(w_lo, w_hi, i)) {
    const int pos = popc128_below(w_lo, w_hi, i);
    if (pos < path_stride) accept_path[(size_t)b * path_stride + pos] = i;
    if (pos == len - 1) {
      accept_len[b] = len;
      next_token[b] = s_greedy[i];
    }
  }
  for (int a = len + i; a < path_stride; a += PROPD_MAX_TREE)
    accept_path[(size_t)b * path_stride + a] = -1;
}

}  // namespace propd

namespace {

using namespace propd;

// How a row of `vocab` elements is cut: slices of whole 16-byte groups, about kSliceBytes each.
void slice_plan(int vocab, int elem_bytes, int &slices, int &per) {
  const long long bytes = (long long)vocab * elem_bytes;
  long long n = (bytes + kSliceBytes - 1) / kSliceBytes;
  n = n < 1 ? 1 : (n > kMaxSlices ? kMaxSlices : n);
  long long p = (vocab + n - 1) / n;
  p = (p + 15) / 16 * 16;
  slices = (int)((vocab + p - 1) / p);
  per = (int)p;
}

propd_status accept_impl(const propd_tree *tree, propd_dtype dt, int32_t vocab, const void *logits,
                         int32_t *accept_len, int32_t *accept_path, int32_t path_stride,
                         int32_t *next_token, void *scratch, hipStream_t st) {
  int slices, per;
  slice_plan(vocab, dt == PROPD_BF16 ? 2 : 4, slices, per);
  RowPart *part = reinterpret_cast<RowPart *>(scratch);
  long long grid = (long long)tree->B * tree->T_max * slices;
  grid = grid > kArgmaxMaxGrid ? kArgmaxMaxGrid : grid;
  if (dt == PROPD_BF16)
    hipLaunchKernelGGL(row_argmax_kernel<true>, dim3((unsigned)grid), dim3(kArgmaxThreads), 0, st,
                       tree->B, tree->T_max, vocab, slices, per, tree->n_nodes, logits, part);
  else
    hipLaunchKernelGGL(row_argmax_kernel<false>, dim3((unsigned)grid), dim3(kArgmaxThreads), 0, st,
                       tree->B, tree->T_max, vocab, slices, per, tree->n_nodes, logits, part);
  if (!launch_ok()) return PROPD_ERR_DEVICE;
  hipLaunchKernelGGL(accept_path_kernel, dim3(tree->B), dim3(PROPD_MAX_TREE), 0, st, tree->T_max,
                     slices, tree->n_nodes, tree->parent, tree->token, tree->anc, part, accept_len,
                     accept_path, path_stride, next_token);
  return launch_ok() ? PROPD_OK : PROPD_ERR_DEVICE;
}

propd_status accept_check(const propd_tree *tree, propd_dtype dt, int32_t vocab, const void *logits,
                          const int32_t *accept_len, const int32_t *accept_path,
                          int32_t path_stride, const int32_t *next_token) {
  if (!tree || tree->B < 1 || tree->T_max < 1 || tree->T_max > PROPD_MAX_TREE || vocab < 1 ||
      path_stride < 1 || !tree->n_nodes || !tree->parent || !tree->token || !tree->anc ||
      !logits || !accept_len || !accept_path || !next_token)
    return PROPD_ERR_INVALID_ARG;
  if (dt != PROPD_BF16 && dt != PROPD_F32) return PROPD_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(logits) % (dt == PROPD_BF16 ? 2 : 4) != 0) return PROPD_ERR_INVALID_ARG;
  if ((long long)tree->B * tree->T_max > (1ll << 27)) return PROPD_ERR_UNSUPPORTED;
  return PROPD_OK;
}

}  // namespace

namespace propd {
size_t accept_path_workspace_bytes(int B, int T_max) {
  return align_up((size_t)B * T_max * kMaxSlices * sizeof(RowPart), 256);
}
}  // namespace propd

extern "C" propd_status propd_accept_path(const propd_tree *tree, propd_dtype dt, int32_t vocab,
                                          const void *logits, int32_t *accept_len,
                                          int32_t *accept_path, int32_t path_stride,
                                          int32_t *next_token, void *workspace,
                                          size_t workspace_bytes, void *hip_stream) {
  const propd_status ok = accept_check(tree, dt, vocab, logits, accept_len, accept_path, path_stride, next_token);
  if (ok != PROPD_OK) return ok;
  const size_t need = propd::accept_path_workspace_bytes(tree->B, tree->T_max);
  if (!workspace || workspace_bytes < need) return PROPD_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 8 != 0) return PROPD_ERR_INVALID_ARG;
  return accept_impl(tree, dt, vocab, logits, accept_len, accept_path, path_stride, next_token,
                     workspace, as_stream(hip_stream));
}

// ------------------------------------------------------------------------------------
// The same call for callers that cannot allocate (code under graph capture, serving loops
// that forbid hipMalloc): the partial arg-max records live in a fixed array in device
// memory that belongs to the library, one copy per GPU.
// ------------------------------------------------------------------------------------
namespace {

constexpr size_t kStaticNodes = PROPD_STATIC_ACCEPT_MAX_NODES;
static __device__ __align__(256) unsigned char scratch[kStaticNodes * propd::kMaxSlices * sizeof(propd::RowPart)];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, once known

// Device address of this GPU's copy of `scratch` (in host code the array's name is only a
// handle for the runtime): looked up once per device, with that device current.
void *static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" propd_status propd_accept_path_static(const propd_tree *tree, propd_dtype dt, int32_t vocab,
                                                 const void *logits, int32_t *accept_len,
                                                 int32_t *accept_path, int32_t path_stride,
                                                 int32_t *next_token, void *hip_stream) {
  const propd_status ok = accept_check(tree, dt, vocab, logits, accept_len, accept_path, path_stride, next_token);
  if (ok != PROPD_OK) return ok;
  if ((size_t)tree->B * (size_t)tree->T_max > kStaticNodes) return PROPD_ERR_UNSUPPORTED;
  void *ptr = static_scratch();
  if (!ptr) return PROPD_ERR_DEVICE;
  return accept_impl(tree, dt, vocab, logits, accept_len, accept_path, path_stride, next_token, ptr,
                     as_stream(hip_stream));
}
