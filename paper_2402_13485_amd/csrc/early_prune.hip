// Early pruning of the token tree (Section 4.1: "Pruning Process", "Pruning Criterion" and
// "Implementation Optimization").
//
// Kernel chain, all on the caller's stream, no host round trip:
//   prune_prepare_kernel  one launch, two kinds of workgroups.  Workgroup 0: which nodes have
//                         children (only those need early-head scores), the table of score
//                         rows, and every node's children grouped by parent.  The others:
//                         each child's OWN score z_p[tok_c], 8 children per workgroup, by the
//                         same chain of matrix instructions that the scoring kernel runs for
//                         that element, so the two values are the same bits
//   early_head_bf16_kernel  scores z = hidden[parent rows] . head_weight^T as a bf16 MFMA
//                         GEMM with fp32 accumulation (M = parent rows, N = vocabulary,
//                         K = hidden).  The scores never leave the registers: the epilogue
//                         compares every score of a row with the own scores of that row's
//                         children and leaves, per child and column tile, the count of scores
//                         that beat it (the top-k membership test; plain stores, every slot
//                         written exactly once, so the sums do not depend on any order), or, for the
//                         probability criterion, leaves (max, sum of exponentials) per row
//                         and column tile
//   early_head_f32_kernel plain fp32 variant with the same epilogue
//   row_lse_kernel        probability criterion: log-sum-exp of every row from the tile
//                         partials, log-probability of every child's token
//   prune_compact_kernel  per sequence: the criterion's decision per node (rank against k, or
//                         path marginal against the threshold / the keep count), fail bits by
//                         ballot, branch elimination by testing the cached ancestor bitset
//                         against the fail bits, order-preserving compaction by prefix
//                         popcount, mask subsampling by bit extraction
//   cu_nodes_kernel       exclusive prefix sum of survivor counts (when there are payloads
//                         it rides along as one extra block of the gather launch)
//   gather_rows_kernel    survivor rows of the listed payload tensors
#include <cstdlib>
#include <type_traits>
#include <utility>

#include "common.h"

namespace propd {

// ------------------------------------------------------------------------------------
// scratch layout
// ------------------------------------------------------------------------------------
struct PruneScratch {
  int32_t *row_src;     // [B*T_max]  score row -> b*T_max + node
  int32_t *row_base;    // [B+1]      score rows of the sequences before b; [B] = total rows
  int32_t *row_info;    // [B*T_max][2] score row -> (first position in child_list, children)
  int32_t *child_list;  // [B*T_max]  b*T_max + child, grouped by parent, per sequence slot
  float *own;           // [B*T_max]  z_parent[token] of every non-root node
  float *logq;          // [B*T_max]  probability criterion: log q of every node's token
  float *lse_part;      // [row_cap * parts][2]  probability criterion: (max, sum exp) per tile
  int32_t *cnt_part;    // [vocab / 128][B*T_max]  top-k criterion: per column tile, the scores of the
                        //                       parent's row that beat the node's token
  size_t row_cap, parts, total_bytes;
};

static PruneScratch carve_scratch(void *base, int B, int T_max, int vocab) {
  PruneScratch s;
  char *p = reinterpret_cast<char *>(base);
  size_t off = 0;
  const size_t nt = (size_t)B * T_max;
  auto take = [&](size_t bytes) {
    char *q = p ? p + off : nullptr;
    off += align_up(bytes, 256);
    return q;
  };
  s.row_src = reinterpret_cast<int32_t *>(take(nt * 4));
  s.row_base = reinterpret_cast<int32_t *>(take((size_t)(B + 1) * 4));
  s.row_info = reinterpret_cast<int32_t *>(take(nt * 8));
  s.child_list = reinterpret_cast<int32_t *>(take(nt * 4));
  s.own = reinterpret_cast<float *>(take(nt * 4));
  s.logq = reinterpret_cast<float *>(take(nt * 4));
  s.row_cap = (size_t)B * (T_max > 1 ? T_max - 1 : 1);  // a node with children is not a leaf
  // column parts of a row: one per wave column of a tile, at most four per 256 columns (two
  // per 128-wide tile, four per 256-wide tile; the fp32 kernel has one per 256-wide slice)
  s.parts = 4 * (((size_t)vocab + 255) / 256);
  s.lse_part = reinterpret_cast<float *>(take(s.row_cap * s.parts * 8));
  s.cnt_part = reinterpret_cast<int32_t *>(take((((size_t)vocab + 127) / 128) * nt * 4));
  s.total_bytes = off;
  return s;
}

size_t early_prune_workspace_bytes(int B, int T_max, int vocab) {
  return carve_scratch(nullptr, B, T_max, vocab).total_bytes;
}

__device__ __forceinline__ int clamp_tree(int T, int T_max) { return T < 1 ? 1 : (T > T_max ? T_max : T); }

constexpr int kScanThreads = 256;

// Exclusive prefix sum of in[0..n) into out[0..n], out[n] = total.  One workgroup.
__device__ void block_exclusive_scan(const int32_t *__restrict__ in, int32_t *__restrict__ out,
                                     int n) {
  const int tid = threadIdx.x;
  const int per = (n + kScanThreads - 1) / kScanThreads;
  const int lo = tid * per, hi = (lo + per < n) ? lo + per : n;
  int sum = 0;
  for (int x = lo; x < hi; ++x) sum += in[x];
  // exclusive scan of the per-thread sums: within each wave by shuffles, then across waves
  const int lane = tid & 63, wv = tid >> 6;
  int incl = sum;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(incl, o, kWave);
    if (lane >= o) incl += up;
  }
  __shared__ int s_wave[kScanThreads / kWave];
  if (lane == kWave - 1) s_wave[wv] = incl;
  __syncthreads();
  int before = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kScanThreads / kWave; ++w) {
    if (w < wv) before += s_wave[w];
    total += s_wave[w];
  }
  if (tid == 0) out[n] = total;
  int run = before + incl - sum;
  for (int x = lo; x < hi; ++x) {
    const int v = in[x];
    out[x] = run;
    run += v;
  }
}

__global__ __launch_bounds__(kScanThreads) void cu_nodes_kernel(int B,
                                                                const int32_t *__restrict__ n_kept,
                                                                int32_t *__restrict__ cu_nodes) {
  block_exclusive_scan(n_kept, cu_nodes, B);
}

// ------------------------------------------------------------------------------------
// preparation: tables (the first workgroups) and the children's own scores (the others)
// ------------------------------------------------------------------------------------
struct PrepareArgs {
  int B, T_max, hidden, vocab;
  const int32_t *n_nodes, *parent, *token;
  const void *hidden_states, *head_weight;
  int32_t *row_src, *row_base, *row_info, *child_list;
  float *own;
};

constexpr int kTableWaves = kScanThreads / kWave;  // sequences per table workgroup, one per wave

// Everything a wave needs from other lanes goes through a 128-entry array of its own in LDS,
// ordered by the wave's own program order (LDS operations of a wave complete in order).
__device__ __forceinline__ void wave_lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// The valid parent of node `nd` of a tree with T nodes as loaded (-1: none; a parent that is no
// earlier node makes no edge).
__device__ __forceinline__ int valid_parent(int nd, int T, int p) {
  return (nd > 0 && nd < T && p >= 0 && p < nd) ? p : -1;
}

// Table workgroup g, wave wv: the tables of sequence b = kTableWaves * g + wv, two nodes per lane
// (lane and lane + 64).  A sequence's score rows follow those of all sequences before it, so the
// wave needs the number of nodes with children of every earlier sequence: the waves of the
// workgroup count them together (sequence x by wave x % kTableWaves, a mark per parent in LDS,
// all loads of a wave's sequences in flight before the first is used) and exchange the counts
// through LDS.  No workgroup waits for another: each one counts for itself what it needs.
__device__ void prepare_tables(const PrepareArgs &a, int g) {
  constexpr int kBatch = 8;  // sequences a wave counts per round
  __shared__ int s_cnt[kTableWaves][PROPD_MAX_TREE];
  __shared__ int s_rows[kTableWaves];  // score rows before this workgroup's sequences, per counting wave
  __shared__ int s_own[kTableWaves];   // nodes with children of the workgroup's own sequences
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int *cnt = s_cnt[wv];
  const int b = kTableWaves * g + wv;
  const int node[2] = {lane, lane + 64};

  // ---- nodes with children of the earlier sequences this wave counts: x = wv, wv + 4, ... < 4 g
  int rows_before = 0;
  for (int x0 = wv; x0 < kTableWaves * g; x0 += kTableWaves * kBatch) {
    int Tx[kBatch], px[kBatch][2];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int x = x0 + kTableWaves * i;
      const bool in = x < kTableWaves * g;
      const size_t base = (size_t)(in ? x : 0) * a.T_max;
      Tx[i] = in ? clamp_tree(a.n_nodes[x], a.T_max) : 0;
#pragma unroll
      for (int h = 0; h < 2; ++h) px[i][h] = node[h] < a.T_max ? a.parent[base + node[h]] : -1;
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      if (x0 + kTableWaves * i >= kTableWaves * g) break;  // uniform
      cnt[node[0]] = 0;
      cnt[node[1]] = 0;
      wave_lds_fence();
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int p = valid_parent(node[h], Tx[i], px[i][h]);
        if (p >= 0) cnt[p] = 1;
      }
      wave_lds_fence();
      rows_before += __popcll(__ballot(cnt[node[0]] != 0)) + __popcll(__ballot(cnt[node[1]] != 0));
      wave_lds_fence();
    }
  }

  // ---- this wave's own sequence
  int T = 0, par[2] = {-1, -1}, slot[2] = {0, 0}, mine[2] = {0, 0}, incl[2] = {0, 0}, par_before[2] = {0, 0};
  int run_par = 0;
  const size_t base = (size_t)(b < a.B ? b : 0) * a.T_max;
  if (b < a.B) {  // uniform over the wave
    T = clamp_tree(a.n_nodes[b], a.T_max);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      par[h] = valid_parent(node[h], T, node[h] < a.T_max ? a.parent[base + node[h]] : -1);
      cnt[node[h]] = 0;
    }
    wave_lds_fence();
    // children per parent; the value before the addition numbers a child among its siblings
#pragma unroll
    for (int h = 0; h < 2; ++h) slot[h] = par[h] >= 0 ? atomicAdd(&cnt[par[h]], 1) : 0;
    wave_lds_fence();
    mine[0] = cnt[node[0]];
    mine[1] = cnt[node[1]];
    wave_lds_fence();
    // exclusive prefix of the child counts over the nodes, and of "has children"
    int run = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      incl[h] = mine[h];
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const int up = __shfl_up(incl[h], o, kWave);
        if (lane >= o) incl[h] += up;
      }
      const int total = __shfl(incl[h], 63, kWave);
      incl[h] += run;
      run += total;
      const uint64_t has = __ballot(mine[h] > 0);
      par_before[h] = run_par + __popcll(has & ((1ull << lane) - 1ull));
      run_par += __popcll(has);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) cnt[node[h]] = incl[h] - mine[h];  // first position of this node's children
    wave_lds_fence();
#pragma unroll
    for (int h = 0; h < 2; ++h)
      if (par[h] >= 0) a.child_list[base + cnt[par[h]] + slot[h]] = (int)base + node[h];
  }
  if (lane == 0) {
    s_rows[wv] = rows_before;
    s_own[wv] = run_par;
  }
  __syncthreads();
  if (b >= a.B) return;
  int first = 0;
#pragma unroll
  for (int w = 0; w < kTableWaves; ++w) first += s_rows[w] + (w < wv ? s_own[w] : 0);
  // positions are global: b*T_max + position in the sequence's slot
#pragma unroll
  for (int h = 0; h < 2; ++h)
    if (mine[h] > 0) {
      const int r = first + par_before[h];
      a.row_src[r] = (int)base + node[h];
      a.row_info[2 * r] = (int)base + incl[h] - mine[h];
      a.row_info[2 * r + 1] = mine[h];
    }
  if (lane == 0) {
    a.row_base[b] = first;
    if (b == a.B - 1) a.row_base[a.B] = first + run_par;
  }
}

// The children's own scores, bf16: workgroup (b, group) takes nodes 8*group .. +7 of
// sequence b (few nodes per workgroup: the rows are fetched once, from all over the weight
// matrix, and it is the number of workgroups that brings the bytes in flight).  Tile rows:
// A row j = hidden state of the parent of node j, B row j = weight row of node j's token; the
// diagonal of A . B^T holds the scores wanted (rows 8..15 of the 16-row tile repeat rows
// 0..7).  All four waves fetch (coalesced, eight 256-deep steps ahead, through registers into
// a padded double buffer in LDS); wave 0 runs the chain of 16x16x32 matrix instructions over
// K in rising order, starting from zero: the chain the 352-row tiles of the scoring kernel run
// for every element (the 32x32x16 chain of the 256-row tiles, two instructions per 32 of K,
// gives the same bits: measured, and held to it by the test of equal scores on both shapes).
constexpr int kOwnNodes = 8;                      // children per workgroup
constexpr int kOwnStep = 256;                     // K per fetch step
constexpr int kOwnRowBytes = kOwnStep * 2 + 16;   // padded: the 8 rows start 4 banks apart
constexpr int kOwnAhead = 8;

__device__ void own_scores_bf16(const PrepareArgs &a, int b, int group) {
  __shared__ __attribute__((aligned(16))) unsigned char s_tile[2][2][kOwnNodes * kOwnRowBytes];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int T = clamp_tree(a.n_nodes[b], a.T_max);
  if (kOwnNodes * group >= T) return;  // uniform over the workgroup
  const size_t base = (size_t)b * a.T_max;
  // loader: thread -> (row, 16-byte piece of the step's 512 bytes)
  const int ld_row = tid >> 5, ld_piece = tid & 31;
  int nd = kOwnNodes * group + ld_row;
  nd = nd < T ? nd : T - 1;
  int p = nd > 0 ? a.parent[base + nd] : 0;
  p = (p >= 0 && p < T) ? p : 0;
  int tk = a.token[base + nd];
  tk = (tk >= 0 && tk < a.vocab) ? tk : 0;
  const uint16_t *a_src = reinterpret_cast<const uint16_t *>(a.hidden_states) + (base + p) * (size_t)a.hidden + ld_piece * 8;
  const uint16_t *b_src = reinterpret_cast<const uint16_t *>(a.head_weight) + (size_t)tk * a.hidden + ld_piece * 8;
  const int n_steps = (a.hidden + kOwnStep - 1) / kOwnStep;
  const int n_k32 = a.hidden / 32;
  u32x4 ra[kOwnAhead], rb[kOwnAhead];
  auto fetch = [&](int slot, int step) {
    const bool in = step < n_steps && step * kOwnStep + ld_piece * 8 < a.hidden;
    const int off = in ? step * kOwnStep : 0;
    ra[slot] = *reinterpret_cast<const u32x4 *>(a_src + off);
    rb[slot] = *reinterpret_cast<const u32x4 *>(b_src + off);
  };
#pragma unroll
  for (int i = 0; i < kOwnAhead; ++i) fetch(i, i);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  // fragment of the 16x16x32 instruction: lane -> row lane % 16 (rows 8..15 repeat rows 0..7),
  // 8 consecutive k from 8 * (lane / 16)
  const int c16 = lane & 15, kq = lane >> 4;
  const int frag_off = (c16 & (kOwnNodes - 1)) * kOwnRowBytes + kq * 16;
  for (int s0 = 0; s0 < n_steps; s0 += kOwnAhead) {
#pragma unroll
    for (int i = 0; i < kOwnAhead; ++i) {
      const int step = s0 + i;
      if (step >= n_steps) break;  // uniform
      unsigned char *buf_a = s_tile[step & 1][0], *buf_b = s_tile[step & 1][1];
      *reinterpret_cast<u32x4 *>(buf_a + ld_row * kOwnRowBytes + ld_piece * 16) = ra[i];
      *reinterpret_cast<u32x4 *>(buf_b + ld_row * kOwnRowBytes + ld_piece * 16) = rb[i];
      fetch(i, step + kOwnAhead);
      __syncthreads();  // the step is in LDS; wave 0 is done with the other buffer
      if (wave == 0) {
        const int k32_left = n_k32 - step * (kOwnStep / 32);
        if (k32_left >= kOwnStep / 32) {
          // a whole step: no condition between the reads, so that all of them are in flight
          // before the first product needs its pair
#pragma unroll
          for (int ks = 0; ks < kOwnStep / 32; ++ks) {
            const bf16x8 fa = *reinterpret_cast<const bf16x8 *>(buf_a + frag_off + ks * 64);
            const bf16x8 fb = *reinterpret_cast<const bf16x8 *>(buf_b + frag_off + ks * 64);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, acc, 0, 0, 0);
          }
        } else {
#pragma unroll
          for (int ks = 0; ks < kOwnStep / 32; ++ks) {
            if (ks < k32_left) {
              const bf16x8 fa = *reinterpret_cast<const bf16x8 *>(buf_a + frag_off + ks * 64);
              const bf16x8 fb = *reinterpret_cast<const bf16x8 *>(buf_b + frag_off + ks * 64);
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, acc, 0, 0, 0);
            }
          }
        }
      }
    }
  }
  if (wave != 0) return;
  mfma_settle();
  // element (row, col) of the tile sits in lane col + 16 * (row / 4), register row % 4: the
  // diagonal element of column j < 8 is in the lane quarter j >> 2, register j & 3
  float diag = 0.f;
#pragma unroll
  for (int r = 0; r < 4; ++r)
    if (r == (c16 & 3)) diag = acc[r];
  const int my_node = kOwnNodes * group + c16;
  if (c16 < kOwnNodes && kq == (c16 >> 2) && my_node > 0 && my_node < T) a.own[base + my_node] = diag;
}

// fp32: one lane per node, the same sequential fused multiply-add chain as the scoring kernel
__device__ void own_scores_f32(const PrepareArgs &a, int b, int group) {
  const int T = clamp_tree(a.n_nodes[b], a.T_max);
  const int nd = kOwnNodes * group + (int)threadIdx.x;
  if (threadIdx.x >= kOwnNodes || nd < 1 || nd >= T) return;
  const size_t base = (size_t)b * a.T_max;
  int p = a.parent[base + nd];
  p = (p >= 0 && p < T) ? p : 0;
  int tk = a.token[base + nd];
  tk = (tk >= 0 && tk < a.vocab) ? tk : 0;
  const float *h = reinterpret_cast<const float *>(a.hidden_states) + (base + p) * (size_t)a.hidden;
  const float *w = reinterpret_cast<const float *>(a.head_weight) + (size_t)tk * a.hidden;
  float acc = 0.f;
  for (int x = 0; x < a.hidden; ++x) acc = fmaf(h[x], w[x], acc);
  a.own[base + nd] = acc;
}

template <bool kBf16>
__global__ __launch_bounds__(kScanThreads) void prune_prepare_kernel(PrepareArgs a) {
  const int table_groups = (a.B + kTableWaves - 1) / kTableWaves;
  if ((int)blockIdx.x < table_groups) {
    prepare_tables(a, blockIdx.x);
    return;
  }
  const int groups = (a.T_max + kOwnNodes - 1) / kOwnNodes;
  const int ob = blockIdx.x - table_groups;
  const int b = ob / groups, group = ob - b * groups;
  if (kBf16) own_scores_bf16(a, b, group);
  else own_scores_f32(a, b, group);
}

// What the scoring kernels need besides the operands.
struct HeadTables {
  const int32_t *row_src, *row_base, *row_info, *child_list, *token;
  const float *own;
  int32_t *cnt_part;  // [column tile][cnt_stride]
  int cnt_stride;     // B * T_max
  float *lse_part;
  int parts;  // column parts per row in lse_part
};

// children of a row taken per pass of the counting epilogue
constexpr int kEpiChildren = 16;

// ------------------------------------------------------------------------------------
// early head, bf16 MFMA
// ------------------------------------------------------------------------------------
// C[m][v] = sum_x A[m][x] * W[v][x].  Both operands are contiguous along x, which is
// the layout the 32x32x16 MFMA wants (8 consecutive x per lane), so tiles go
// global -> LDS -> MFMA operands without any transpose.
//   - workgroup tile 256 rows x 64*FN vocabulary entries with FN = 2, 3 or 4, eight waves
//     in a 4 x 2 arrangement, each owning 64 x 32*FN as 2 x FN MFMA tiles of 32 x 32.
//     Wider tiles move fewer operand bytes per FLOP (the kernel is bound by operand
//     delivery, not by the matrix cores); FN is the width with the fewest
//     rounds-of-workgroups x width on this chip, computed by every workgroup from the row
//     count on the device, so the host never needs that count;
//   - K advances 32 per step through a ring of LDS stages filled by direct global->LDS loads
//     (no staging registers, no LDS stores), up to three steps ahead of the math; one barrier
//     per K step.  A row of a stage is 64 bytes (4 chunks of 16); the lane that fills chunk c
//     of LDS row r fetches chunk c ^ key(r) of the global row, with key(r) = (r >> 2) & 3, so
//     that the 16 rows one quarter-wave reads for a chunk column fall into 16 different bank
//     groups;
//   - operand fragments are double-buffered in registers: the LDS reads of one half step
//     are issued before the MFMAs of the half step before it, and the barrier sits between
//     two MFMA groups whose operands are already in registers, so the matrix core has work
//     queued while waves meet;
//   - the A rows are gathered through the row table by the loads themselves; rows past
//     the last one and vocabulary entries past the last re-read the last valid one and
//     are left out by the epilogue;
//   - the scores stay in the accumulators: the epilogue turns them into rank counts (or
//     log-sum-exp partials) and nothing of size rows x vocabulary ever reaches memory;
//   - the grid is one-dimensional, persistent and XCD-aware.  Workgroups are handed to the 8
//     XCDs round-robin, each XCD has its own L2: tile id -> (xcd, slot), and an XCD walks
//     its own vocabulary tiles with all row tiles of one vocabulary tile adjacent in time,
//     so a weight tile is fetched from HBM once and hits in that XCD's L2 for the other
//     row tiles.
constexpr int kBK = 32;
constexpr int kGemmBM = 256;
constexpr int kGemmMinFN = 2, kGemmMaxFN = 4;
constexpr int kGemmThreads = 512;
// ring depth: five stages where they fit into the 160 KB of LDS, four for the widest tile
__host__ __device__ constexpr int gemm_stages(int fn) { return fn == 4 ? 4 : 5; }
__host__ __device__ constexpr int gemm_stage_bytes(int fn) { return (256 + 64 * fn) * 64; }
constexpr int kGemmRowBytes = kBK * 2;                                           // 64
constexpr int kGemmWOffset = kGemmBM * kGemmRowBytes;                            // W rows follow the A rows
constexpr int kGemmLdsBytes = 5 * gemm_stage_bytes(3);  // the largest ring: 140 KB (4 x 32 KB for FN = 4)
static_assert(gemm_stages(4) * gemm_stage_bytes(4) <= kGemmLdsBytes && gemm_stages(2) * gemm_stage_bytes(2) <= kGemmLdsBytes, "ring");
constexpr int kXcds = 8;

// Tile width (in units of 64 vocabulary entries) for m_tiles row tiles: the time of a
// launch goes as rounds of workgroups over the compute units times the width; ties go to
// the wider tile.
__host__ __device__ inline int gemm_pick_fn(int m_tiles, int vocab, int cus) {
  int best = kGemmMaxFN;
  long long best_cost = -1;
  for (int fn = kGemmMaxFN; fn >= kGemmMinFN; --fn) {
    const long long n_tiles = (vocab + 64 * fn - 1) / (64 * fn);
    const long long rounds = (n_tiles * m_tiles + cus - 1) / cus;
    const long long cost = rounds * fn;
    if (best_cost < 0 || cost < best_cost) {
      best = fn;
      best_cost = cost;
    }
  }
  return best;
}

template <int N>
__device__ __forceinline__ void gemm_wait_vmem() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int N>
__device__ __forceinline__ void gemm_wait_at_most(int n) {
  if constexpr (N == 0) {
    gemm_wait_vmem<0>();
  } else {
    if (n >= N) gemm_wait_vmem<N>();
    else gemm_wait_at_most<N - 1>(n);
  }
}
// Waits until at most n <= MAXN of this wave's loads are outstanding (n = whole steps of 1 to 4 loads).
template <int MAXN>
__device__ __forceinline__ void gemm_wait_outstanding(int n) { gemm_wait_at_most<MAXN>(n); }

// LDS read issued as inline assembly so that the wait for it can be placed by hand: the
// compiler's own placement waits for every outstanding LDS read, also the ones issued ahead
// for the next half step.  The result is valid only after gemm_wait_frag<>().
template <int OFFSET>
__device__ __forceinline__ u32x4 gemm_lds_read16(uint32_t addr) {
  u32x4 r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET));
  return r;
}

template <int FN>
struct GemmFrag {
  u32x4 a[2], b[FN];
};

// Waits until at most N LDS reads of this wave are outstanding (they return in order); the
// fragment named is the one waited for, so that its uses stay below the wait.
template <int N, int FN>
__device__ __forceinline__ void gemm_wait_frag(GemmFrag<FN> &f) {
  if constexpr (FN == 2)
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.b[0]), "+v"(f.b[1]) : "n"(N));
  else if constexpr (FN == 3)
    asm volatile("s_waitcnt lgkmcnt(%5)"
                 : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.b[0]), "+v"(f.b[1]), "+v"(f.b[2])
                 : "n"(N));
  else
    asm volatile("s_waitcnt lgkmcnt(%6)"
                 : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.b[0]), "+v"(f.b[1]), "+v"(f.b[2]), "+v"(f.b[3])
                 : "n"(N));
}

// ---- epilogues.  Accumulator layout of the 32x32 MFMA: lane -> column l32 (+ 32 y), register
//      r -> row 8*(r/4) + 4*g + r%4 (+ 32 x): a row of the tile lives in the 32 lanes of one
//      half of a wave, so a ballot over a comparison counts two rows at once.

// Top-k membership by counting (Section 4.1, "Pruning Criterion"): for every child c of the
// row's node, the scores of the row that beat the child's own score (a higher score, or the
// same score at a lower id) are counted; the count of this column tile goes to the child's
// slot of the tile in cnt_part, and the decision kernel adds the tiles up.
//
// The children of the tile's rows are staged in LDS (the ring is free by now), kEpiChildren
// per row and pass.  "Beats" is turned into one comparison per score: for the columns of a
// wave that all lie above the child's token the threshold is the own score (z > own), for
// columns that all lie below it the next smaller float (z > pred(own), i.e. z >= own); only
// the one wave whose columns contain the token compares per lane, on a side path marked by
// a NaN threshold, which the main comparison counts as nothing.  A lane walks its 32 rows
// with the thresholds of the next row already requested, four per LDS read, counts its own
// columns in a byte per child, and one cross-lane sum per row and four children (DPP)
// leaves the row's counts in the last lane of each half wave.
typedef __attribute__((ext_vector_type(4))) int i32x4;

// A loop whose index is a compile-time constant in every iteration: accumulator registers can
// only be named by constants, and an ordinary loop this large is not always unrolled.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// the largest float below x (x itself for -inf and NaN): z > float_pred(x)  <=>  z >= x
__device__ __forceinline__ float float_pred(float x) {
  const uint32_t u = __float_as_uint(x);
  if (x > 0.f) return __uint_as_float(u - 1u);
  if (x == 0.f) return __uint_as_float(0x80000001u);
  if (x < 0.f && x > -INFINITY) return __uint_as_float(u + 1u);
  return x;
}

// Sum over the 32 lanes of each half wave, left in lanes 31 and 63.
__device__ __forceinline__ int half_wave_sum_to_last(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);  // row_shr:8: lane 15 of a row = its sum
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
  return v;
}

template <int FN>
__device__ __forceinline__ void epilogue_count(f32x16 (&acc)[2][FN], int m0, int v0, int n_tile, int vocab,
                                               int tid_in, int my_pos, int my_cc,
                                               const HeadTables &tb, unsigned char *smem) {
  constexpr int BM = kGemmBM, WN = 32 * FN, E = kEpiChildren;
  static_assert(E % 4 == 0 && FN * 32 < 256 && kGemmThreads % E == 0, "four byte-sized counts per word");
  // Everything below is derived from this copy of the thread id, which the compiler cannot
  // see through: otherwise it computes the dozens of LDS addresses of this epilogue before the
  // K loop and keeps them in scratch memory across it.
  int tid = tid_in;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave >> 1, wn = wave & 1;
  int *s_max = reinterpret_cast<int *>(smem);
  int *s_cc = s_max + 64;                                // [BM] children of the row in this pass | flags << 8
  int *s_pos = s_cc + BM;                                // [BM] first position in child_list
  float *s_thr = reinterpret_cast<float *>(s_pos + BM);  // [2][BM][E] threshold per wave column
  float *s_own = s_thr + 2 * BM * E;                     // [BM][E]
  int *s_tok = reinterpret_cast<int *>(s_own + BM * E);  // [BM][E]
  int *s_node = s_tok + BM * E;                          // [BM][E]
  int *s_count = s_node + BM * E;                        // [2][BM][E/4] packed counts per wave column
  // columns past the vocabulary (last column tile only) can beat nothing
  if (v0 + 2 * WN > vocab) {
#pragma unroll
    for (int y = 0; y < FN; ++y) {
      const bool out = v0 + wn * WN + y * 32 + l32 >= vocab;
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[x][y][r] = out ? -INFINITY : acc[x][y][r];
    }
  }
  __syncthreads();  // every wave is done with the ring
  if (tid == 0) *s_max = 0;
  __syncthreads();
  {
    const int wave_max = wave_reduce_max(tid < BM ? my_cc : 0);
    if (lane == 0 && wave_max > 0) atomicMax(s_max, wave_max);
  }
  __syncthreads();
  const int max_cc = *s_max;
  // this lane's rows: row0 + a constant per (x, r)
  const int row0 = wm * 64 + 4 * g;
  const int *cc_base = s_cc + row0;
  const float *thr_base = s_thr + wn * BM * E + row0 * E;
  const float *own_base = s_own + row0 * E;
  const int *tok_base = s_tok + row0 * E;
  int *count_base = s_count + wn * BM * (E / 4) + row0 * (E / 4);
  // staging: this thread's slots are (row = tid / E + 32 j, child = tid % E)
  const int st_row = tid / E, st_e = tid % E;
  for (int e0 = 0; e0 < max_cc; e0 += E) {
    if (tid < BM) {
      int n = my_cc - e0;
      s_cc[tid] = n < 0 ? 0 : (n > E ? E : n);
      s_pos[tid] = my_pos + e0;
    }
    __syncthreads();
    {
      // all threads stage the (row, child) slots of the pass: the loads of a thread's slots
      // are in flight together, first the children's ids, then their tokens and own scores
      constexpr int kSlots = BM * E / kGemmThreads, kRowStep = kGemmThreads / E, kChunk = 4;
#pragma unroll
      for (int j0 = 0; j0 < kSlots; j0 += kChunk) {
        int c[kChunk], t[kChunk];
        float o[kChunk];
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
          const int row = st_row + kRowStep * (j0 + j);
          c[j] = st_e < (s_cc[row] & 255) ? tb.child_list[s_pos[row] + st_e] : -1;
        }
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
          t[j] = c[j] >= 0 ? tb.token[c[j]] : -1;
          o[j] = c[j] >= 0 ? tb.own[c[j]] : INFINITY;
        }
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
          const int row = st_row + kRowStep * (j0 + j), slot = row * E + st_e;
          // an id outside the vocabulary is beaten by nothing here (the decision kernel fails it)
          const bool ok = t[j] >= 0 && t[j] < vocab;
          s_own[slot] = ok ? o[j] : INFINITY;
          s_tok[slot] = ok ? t[j] : -1;
          s_node[slot] = c[j];
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const int c0 = v0 + half * WN;
            float thr = INFINITY;
            if (ok) {
              const bool inside = t[j] >= c0 && t[j] < c0 + WN;
              thr = t[j] < c0 ? o[j] : (inside ? __uint_as_float(0x7fc00000u) : float_pred(o[j]));
              if (inside) atomicOr(&s_cc[row], 256 << half);  // this row has a side-path entry
            }
            s_thr[(half * BM * E) + slot] = thr;
          }
        }
      }
    }
    __syncthreads();
    // this lane's 32 rows, in the order (x, r); the thresholds of the next row are requested
    // before the current row is counted
    auto row_off = [](int idx) { return (idx >> 4) * 32 + 8 * ((idx & 15) >> 2) + (idx & 3); };
    int meta_cur = cc_base[row_off(0)];  // children | side-path flags of the two wave columns << 8
    f32x4 thr_cur = *reinterpret_cast<const f32x4 *>(thr_base + row_off(0) * E);
    static_for<32>([&](auto idx_c) {
      constexpr int idx = decltype(idx_c)::value;
      constexpr int x = idx >> 4, r = idx & 15;
      constexpr int off = (idx >> 4) * 32 + 8 * ((idx & 15) >> 2) + (idx & 3);
      int meta_nxt = 0;
      f32x4 thr_nxt = {0.f, 0.f, 0.f, 0.f};
      if (idx + 1 < 32) {
        meta_nxt = cc_base[row_off(idx + 1)];
        thr_nxt = *reinterpret_cast<const f32x4 *>(thr_base + row_off(idx + 1) * E);
      }
      const int m_lo = __builtin_amdgcn_readlane(meta_cur, 0), m_hi = __builtin_amdgcn_readlane(meta_cur, 32);
      const int n_both = (m_lo & 255) > (m_hi & 255) ? (m_lo & 255) : (m_hi & 255);
      const bool side_path = (((m_lo | m_hi) >> (8 + wn)) & 1) != 0;  // rare: the token's own columns
      for (int e4 = 0; e4 < n_both; e4 += 4) {
        if (e4 > 0) thr_cur = *reinterpret_cast<const f32x4 *>(thr_base + off * E + e4);  // more than four children
        int packed = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float thr = thr_cur[j];
          int cnt = 0;
#pragma unroll
          for (int y = 0; y < FN; ++y) cnt += acc[x][y][r] > thr ? 1 : 0;
          if (side_path && thr != thr) {
            const float own = own_base[off * E + e4 + j];
            const int tok = tok_base[off * E + e4 + j];
#pragma unroll
            for (int y = 0; y < FN; ++y) {
              const int col = v0 + wn * WN + y * 32 + l32;
              const float z = acc[x][y][r];
              cnt += (col != tok && (z > own || (z == own && col < tok))) ? 1 : 0;
            }
          }
          packed += cnt << (8 * j);
        }
        packed = half_wave_sum_to_last(packed);
        if (l32 == 31) count_base[off * (E / 4) + (e4 >> 2)] = packed;
      }
      meta_cur = meta_nxt;
      thr_cur = thr_nxt;
    });
    __syncthreads();
    // every (child, column tile) slot is written by exactly one workgroup, zero counts too
#pragma unroll
    for (int j = 0; j < BM * E / kGemmThreads; ++j) {
      const int row = st_row + (kGemmThreads / E) * j, slot = row * E + st_e;
      const int c = s_node[slot];
      if (c >= 0) {
        const int word = slot >> 2, sh = 8 * (slot & 3);
        tb.cnt_part[(size_t)n_tile * tb.cnt_stride + c] =
            ((s_count[word] >> sh) & 255) + ((s_count[BM * (E / 4) + word] >> sh) & 255);
      }
    }
    __syncthreads();  // the next pass, or the next tile's loads, reuse this memory
  }
}

// (max, sum of exp(z - max)) of two parts of a row, merged
__device__ __forceinline__ void lse_merge(float &m, float &s, float m2, float s2) {
  const float mm = m > m2 ? m : m2;
  s = (m == -INFINITY ? 0.f : s * expf(m - mm)) + (m2 == -INFINITY ? 0.f : s2 * expf(m2 - mm));
  m = mm;
}

// Probability criterion: (max, sum of exponentials) of this wave's columns for every row of
// the tile, one pair per row and column part, merged later by row_lse_kernel.
template <int FN>
__device__ __forceinline__ void epilogue_lse(const f32x16 (&acc)[2][FN], int m0, int v0, int m_total,
                                             int vocab, int n_tile, int wm, int wn, int lane,
                                             const HeadTables &tb) {
  constexpr int WN = 32 * FN;
  const int l32 = lane & 31, g = lane >> 5;
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float mx = -INFINITY;
#pragma unroll
      for (int y = 0; y < FN; ++y)
        if (v0 + wn * WN + y * 32 + l32 < vocab) mx = fmaxf(mx, acc[x][y][r]);
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, kWave));
      float sum = 0.f;
#pragma unroll
      for (int y = 0; y < FN; ++y)
        if (v0 + wn * WN + y * 32 + l32 < vocab) sum += expf(acc[x][y][r] - mx);
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) sum += __shfl_xor(sum, o, kWave);
      const int m = m0 + wm * 64 + x * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
      if (l32 == 0 && m < m_total) {
        float *dst = tb.lse_part + ((size_t)m * tb.parts + 2 * n_tile + wn) * 2;
        dst[0] = mx;
        dst[1] = sum;
      }
    }
}

template <int FN, int KIND>
__device__ __forceinline__ void early_head_tile(
    int hidden, int vocab, int m_total, int m0, int v0, int n_tile,
    const uint16_t *__restrict__ hidden_states, const uint16_t *__restrict__ head_weight,
    const HeadTables &tb, unsigned char *gemm_smem) {
  constexpr int BM = kGemmBM, WN = 32 * FN;
  constexpr int kStages = gemm_stages(FN), kStageBytes = gemm_stage_bytes(FN);
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void global_void;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void *)gemm_smem;

  // The thread id is made opaque: what is derived from it (addresses, row and chunk numbers)
  // is then computed here, inside the loop over tiles, and not hoisted out of that loop into
  // registers that stay occupied while the other tile shapes run.
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, g = lane >> 5;
  // children of the tile's rows (thread t < 256 looks after row m0 + t), fetched early
  int my_pos = 0, my_cc = 0;
  if (KIND == 0 && tid < BM && m0 + tid < m_total) {
    my_pos = tb.row_info[2 * (m0 + tid)];
    my_cc = tb.row_info[2 * (m0 + tid) + 1];
  }

  // ---- loader: a load instruction fills 16 rows (1 KB).  A stage has 16 such groups of A
  //      rows and 4*FN of W rows; wave w takes groups w and w+8 of each (the second W group
  //      only where it exists).
  const int ld_row = lane >> 2;
  const int ld_chunk = ((lane & 3) ^ ((lane >> 4) & 3)) << 4;  // byte offset in the global row
  const bool second_w = FN == 4 ? true : (FN == 2 ? false : wave < 4);
  // Few score rows (a small batch): groups of 16 rows that lie wholly past the last row are
  // not fetched at all, and a wave whose 64 rows lie past it neither reads fragments nor
  // multiplies.  What such rows hold in LDS and in the accumulators is never looked at.
  const bool a_on[2] = {m0 + 16 * wave < m_total, m0 + 16 * (wave + 8) < m_total};
  const bool w_on = m0 + wm * 64 < m_total;
  const int per_step = (a_on[0] ? 1 : 0) + (a_on[1] ? 1 : 0) + (second_w ? 2 : 1);  // loads of this wave per K step
  const unsigned char *a_src[2], *b_src[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    int m = m0 + 16 * (wave + 8 * j) + ld_row;
    m = m < m_total ? m : m_total - 1;
    a_src[j] = reinterpret_cast<const unsigned char *>(hidden_states + (size_t)tb.row_src[m] * hidden) + ld_chunk;
    int v = v0 + 16 * (wave + 8 * j) + ld_row;
    v = v < vocab ? v : vocab - 1;
    b_src[j] = reinterpret_cast<const unsigned char *>(head_weight + (size_t)v * hidden) + ld_chunk;
  }
  auto issue = [&](int slot) {  // the next K step of every source pointer
    unsigned char *dst = gemm_smem + slot * kStageBytes + wave * 1024;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (a_on[j]) __builtin_amdgcn_global_load_lds((global_void *)a_src[j], (lds_void *)(dst + j * 8192), 16, 0, 0);
      a_src[j] += kGemmRowBytes;
    }
    __builtin_amdgcn_global_load_lds((global_void *)b_src[0], (lds_void *)(dst + kGemmWOffset), 16, 0, 0);
    b_src[0] += kGemmRowBytes;
    if (second_w) {
      __builtin_amdgcn_global_load_lds((global_void *)b_src[1], (lds_void *)(dst + kGemmWOffset + 8192), 16, 0, 0);
      b_src[1] += kGemmRowBytes;
    }
  };

  // ---- per-lane LDS read offsets: operand row l32 of a 32-row block, chunk 2*ks + g
  uint32_t a_rd[2], b_rd[2];
  {
    const int key = (l32 >> 2) & 3;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int off = l32 * kGemmRowBytes + (((2 * ks + g) ^ key) << 4);
      a_rd[ks] = smem_base + wm * 64 * kGemmRowBytes + off;
      b_rd[ks] = smem_base + kGemmWOffset + wn * WN * kGemmRowBytes + off;
    }
  }
  typedef GemmFrag<FN> Frag;
  auto read = [&](Frag &f, uint32_t so, int ks) {
    const uint32_t pa = a_rd[ks] + so, pb = b_rd[ks] + so;
    f.a[0] = gemm_lds_read16<0>(pa);
    f.a[1] = gemm_lds_read16<32 * kGemmRowBytes>(pa);
    f.b[0] = gemm_lds_read16<0>(pb);
    f.b[1] = gemm_lds_read16<32 * kGemmRowBytes>(pb);
    if constexpr (FN >= 3) f.b[2] = gemm_lds_read16<64 * kGemmRowBytes>(pb);
    if constexpr (FN >= 4) f.b[3] = gemm_lds_read16<96 * kGemmRowBytes>(pb);
  };

  f32x16 acc[2][FN];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < FN; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;
  auto mma = [&](const Frag &f) {
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < FN; ++y)
        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, f.a[x]), __builtin_bit_cast(bf16x8, f.b[y]), acc[x][y], 0, 0, 0);
  };

  const int n_steps = hidden / kBK;
  // The ring: the step being multiplied, the next one (already landed, its first fragments
  // are read before this step ends) and kStages-2 steps in flight; the slot of the step
  // being multiplied is handed back to the loads as soon as its last fragments are in
  // registers, half a step before the step ends.
  const int n_pro = n_steps < kStages ? n_steps : kStages;
  int slot_ld = 0;
  for (int i = 0; i < n_pro; ++i) {
    issue(slot_ld);
    slot_ld = slot_ld + 1 == kStages ? 0 : slot_ld + 1;
  }
  constexpr int kMaxOutstanding = (kStages - 1) * 4;
  gemm_wait_outstanding<kMaxOutstanding>((n_pro - 1) * per_step);
  __builtin_amdgcn_s_barrier();
  constexpr int kReads = 2 + FN;  // LDS reads of one half step
  Frag f0, f1;
  if (w_on) read(f0, 0, 0);
  uint32_t so = 0;  // byte offset of the stage being multiplied
  for (int step = 0; step + 1 < n_steps; ++step) {
    if (w_on) {
      read(f1, so, 1);
      gemm_wait_frag<kReads>(f0);  // the reads just issued fly while the MFMAs below run
      mma(f0);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (w_on) gemm_wait_frag<0>(f1);  // this wave is done with the slot of this step
    // the next step has landed once at most the steps after it (kStages-2 of them were
    // issued) are outstanding
    {
      const int issued_after = n_steps - 2 - step < kStages - 2 ? n_steps - 2 - step : kStages - 2;
      gemm_wait_outstanding<kMaxOutstanding>(issued_after * per_step);
    }
    __builtin_amdgcn_s_barrier();  // it is visible; every wave is done with this step's slot
    if (step + kStages < n_steps) {
      issue(slot_ld);  // into the slot of this step
      slot_ld = slot_ld + 1 == kStages ? 0 : slot_ld + 1;
    }
    so = so + kStageBytes == kStages * kStageBytes ? 0 : so + kStageBytes;
    if (w_on) {
      read(f0, so, 0);
      mma(f1);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  if (w_on) {
    read(f1, so, 1);
    gemm_wait_frag<kReads>(f0);
    mma(f0);
    gemm_wait_frag<0>(f1);
    mma(f1);
  }

  mfma_settle();
  if (KIND == 0)
    epilogue_count<FN>(acc, m0, v0, n_tile, vocab, tid, my_pos, my_cc, tb, gemm_smem);
  else
    epilogue_lse<FN>(acc, m0, v0, m_total, vocab, n_tile, wm, wn, lane, tb);
}



// ------------------------------------------------------------------------------------
// Few score rows (at most 128 in the whole batch: a small batch or small trees).  The
// scoring kernel is then a stream of the weight matrix through the compute units, and a step
// (a barrier, fragment reads whose latency a handful of matrix instructions cannot hide)
// costs more than its bytes.  This tile takes 64-deep steps: half as many steps for the same
// bytes, whole 128-byte lines from every row.  Same 128-wide column tile, wave layout, accumulator layout and epilogues as the
// 256 x 128 tile above, of which only the upper 128 rows exist; LDS rows are 128 bytes, their
// eight 16-byte chunks XOR-swizzled with key(row) = (row >> 1) & 7 (a fragment read takes rows
// r .. r + 15 of one chunk column in one pass: two rows share a 256-byte bank line, eight keys
// spread the eight pairs).
// ------------------------------------------------------------------------------------
constexpr int kSmallBM = 128, kSmallBK = 64, kSmallStages = 4;
constexpr int kSmallRowBytes = kSmallBK * 2;                          // 128
constexpr int kSmallWOffset = kSmallBM * kSmallRowBytes;              // 16 KB of score rows, then 16 KB of weight rows
constexpr int kSmallStageBytes = 2 * kSmallWOffset;                   // 32 KB
static_assert(kSmallStages * kSmallStageBytes <= kGemmLdsBytes, "ring");

template <int KIND>
__device__ __forceinline__ void early_head_small_tile(
    int hidden, int vocab, int m_total, int v0, int n_tile,
    const uint16_t *__restrict__ hidden_states, const uint16_t *__restrict__ head_weight,
    const HeadTables &tb, unsigned char *gemm_smem) {
  constexpr int FN = 2, BM = kGemmBM;
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void global_void;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void *)gemm_smem;
  // The thread id is made opaque: what is derived from it (addresses, row and chunk numbers)
  // is then computed here, inside the loop over tiles, and not hoisted out of that loop into
  // registers that stay occupied while the other tile shapes run.
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, g = lane >> 5;
  int my_pos = 0, my_cc = 0;
  if (KIND == 0 && tid < BM && tid < m_total) {
    my_pos = tb.row_info[2 * tid];
    my_cc = tb.row_info[2 * tid + 1];
  }

  // ---- loader: a load instruction fills 8 rows of 128 bytes (1 KB).  A stage has 16 such
  //      groups of score rows and 16 of weight rows; wave w takes groups 2w and 2w + 1 of each.
  //      Groups of score rows wholly past the last row are not fetched.
  const int ld_row = lane >> 3, ld_pos = lane & 7;
  const unsigned char *a_src[2], *b_src[2];
  bool a_on[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int r = 8 * (2 * wave + j) + ld_row;  // row of the tile = LDS row
    const int chunk = (ld_pos ^ ((r >> 1) & 7)) << 4;
    a_on[j] = 8 * (2 * wave + j) < m_total;
    const int m = r < m_total ? r : m_total - 1;
    a_src[j] = reinterpret_cast<const unsigned char *>(hidden_states + (size_t)tb.row_src[m] * hidden) + chunk;
    int v = v0 + r;
    v = v < vocab ? v : vocab - 1;
    b_src[j] = reinterpret_cast<const unsigned char *>(head_weight + (size_t)v * hidden) + chunk;
  }
  const int per_step = (a_on[0] ? 1 : 0) + (a_on[1] ? 1 : 0) + 2;  // loads of this wave per K step
  const bool w_on = wm * 64 < m_total;                             // this wave's 64 rows hold score rows
  auto issue = [&](int slot) {
    unsigned char *dst = gemm_smem + slot * kSmallStageBytes + wave * 2048;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (a_on[j]) __builtin_amdgcn_global_load_lds((global_void *)a_src[j], (lds_void *)(dst + j * 1024), 16, 0, 0);
      a_src[j] += kSmallRowBytes;
      __builtin_amdgcn_global_load_lds((global_void *)b_src[j], (lds_void *)(dst + kSmallWOffset + j * 1024), 16, 0, 0);
      b_src[j] += kSmallRowBytes;
    }
  };

  // ---- per-lane LDS read addresses: operand row l32 of a 32-row block (the key of row + 32 is
  //      the key of the row), chunk 2 * ks + g for the K sub-step ks of 16
  uint32_t a_rd[4], b_rd[4];
  {
    const int key = (l32 >> 1) & 7;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int off = l32 * kSmallRowBytes + (((2 * ks + g) ^ key) << 4);
      a_rd[ks] = smem_base + wm * 64 * kSmallRowBytes + off;
      b_rd[ks] = smem_base + kSmallWOffset + wn * 64 * kSmallRowBytes + off;
    }
  }
  typedef GemmFrag<FN> Frag;
  auto read = [&](Frag &f, uint32_t so, int ks) {
    const uint32_t pa = a_rd[ks] + so, pb = b_rd[ks] + so;
    f.a[0] = gemm_lds_read16<0>(pa);
    f.a[1] = gemm_lds_read16<32 * kSmallRowBytes>(pa);
    f.b[0] = gemm_lds_read16<0>(pb);
    f.b[1] = gemm_lds_read16<32 * kSmallRowBytes>(pb);
  };
  f32x16 acc[2][FN];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < FN; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;
  auto mma = [&](const Frag &f) {
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < FN; ++y)
        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, f.a[x]), __builtin_bit_cast(bf16x8, f.b[y]), acc[x][y], 0, 0, 0);
  };

  const int n_steps = hidden / kSmallBK;
  const int n_pro = n_steps < kSmallStages ? n_steps : kSmallStages;
  constexpr int kMaxOutstanding = (kSmallStages - 1) * 4;
  int slot_ld = 0;
  for (int i = 0; i < n_pro; ++i) {
    issue(slot_ld);
    slot_ld = slot_ld + 1 == kSmallStages ? 0 : slot_ld + 1;
  }
  gemm_wait_outstanding<kMaxOutstanding>((n_pro - 1) * per_step);
  __builtin_amdgcn_s_barrier();
  constexpr int kReads = 2 + FN;  // LDS reads of one K sub-step
  Frag f0, f1;
  if (w_on) read(f0, 0, 0);
  uint32_t so = 0;  // byte offset of the stage being multiplied
  for (int step = 0; step < n_steps; ++step) {
    if (w_on) {
      read(f1, so, 1);
      gemm_wait_frag<kReads>(f0);  // the reads just issued fly while the MFMAs below run
      mma(f0);
      read(f0, so, 2);
      gemm_wait_frag<kReads>(f1);
      mma(f1);
      read(f1, so, 3);
      gemm_wait_frag<kReads>(f0);
      mma(f0);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (w_on) gemm_wait_frag<0>(f1);  // this wave is done with the slot of this step
    if (step + 1 < n_steps) {
      const int issued_after = n_steps - 2 - step < kSmallStages - 2 ? n_steps - 2 - step : kSmallStages - 2;
      gemm_wait_outstanding<kMaxOutstanding>(issued_after * per_step);
      __builtin_amdgcn_s_barrier();  // it is visible; every wave is done with this step's slot
      if (step + kSmallStages < n_steps) {
        issue(slot_ld);  // into the slot of this step
        slot_ld = slot_ld + 1 == kSmallStages ? 0 : slot_ld + 1;
      }
      so = so + kSmallStageBytes == kSmallStages * kSmallStageBytes ? 0 : so + kSmallStageBytes;
      if (w_on) read(f0, so, 0);
    }
    if (w_on) mma(f1);
    __builtin_amdgcn_sched_barrier(0);
  }
  mfma_settle();
  if (KIND == 0)
    epilogue_count<FN>(acc, 0, v0, n_tile, vocab, tid, my_pos, my_cc, tb, gemm_smem);
  else
    epilogue_lse<FN>(acc, 0, v0, m_total, vocab, n_tile, wm, wn, lane, tb);
}

#include "early_head_tall.h"

// Which tile shape a call uses: decided on the device by every workgroup (and by the kernels
// that read the per-tile results) from the row count, which the host never sees.  The cost of
// a shape is rounds of workgroups over the compute units x tile area, the tall shape's area
// weighted by what it was measured to cost per output relative to the other.
struct HeadPlan {
  int tall;     // 1: 352 x 256 tiles, 0: 256 x 64*fn tiles
  int fn;
  int m_tiles, n_tiles;
  int n_parts;  // column parts per row that the epilogue writes
};
constexpr int kTallCostPercent = 85;

__host__ __device__ inline HeadPlan head_plan(int m_total, int vocab, int cus, int force) {
  HeadPlan pl;
  pl.tall = 0;
  pl.m_tiles = (m_total + kGemmBM - 1) / kGemmBM;
  pl.fn = gemm_pick_fn(pl.m_tiles > 0 ? pl.m_tiles : 1, vocab, cus);
  pl.n_tiles = (vocab + 64 * pl.fn - 1) / (64 * pl.fn);
  pl.n_parts = 2 * pl.n_tiles;
  if (m_total <= 0) return pl;
  const long long rounds = ((long long)pl.m_tiles * pl.n_tiles + cus - 1) / cus;
  const long long cost = rounds * kGemmBM * 64 * pl.fn * 100;
  const int mt = (m_total + kTallBM - 1) / kTallBM, nt = (vocab + kTallBN - 1) / kTallBN;
  const long long rounds_tall = ((long long)mt * nt + cus - 1) / cus;
  const long long cost_tall = rounds_tall * kTallBM * kTallBN * kTallCostPercent;
  if (force == 2 || (force == 0 && cost_tall < cost)) {
    pl.tall = 1;
    pl.m_tiles = mt;
    pl.n_tiles = nt;
    pl.n_parts = 4 * nt;
  }
  return pl;
}

constexpr int kHeadLdsBytes = kTallLdsBytes > kGemmLdsBytes ? kTallLdsBytes : kGemmLdsBytes;

// Persistent over the tiles: tile -> (xcd, slot) as described above, a workgroup takes tiles
// blockIdx.x, blockIdx.x + gridDim.x, ... (the grid is a multiple of the XCD count).
template <int KIND>
__global__ __launch_bounds__(kGemmThreads, 1) void early_head_bf16_kernel(
    int hidden, int vocab, int B, int cus, int force, const uint16_t *__restrict__ hidden_states,
    const uint16_t *__restrict__ head_weight, HeadTables tb) {
  const int m_total = tb.row_base[B];
  if (m_total <= 0) return;
  const HeadPlan pl = head_plan(m_total, vocab, cus, force);
  const int m_tiles = pl.m_tiles, n_tiles = pl.n_tiles;
  const long long total = (long long)kXcds * ((n_tiles + kXcds - 1) / kXcds) * m_tiles;
  extern __shared__ __attribute__((aligned(1024))) unsigned char gemm_smem[];
  for (long long tile = blockIdx.x; tile < total; tile += gridDim.x) {
    const int xcd = (int)(tile % kXcds);
    const long long slot = tile / kXcds;
    const int n_tile = (int)(slot / m_tiles) * kXcds + xcd;
    if (n_tile >= n_tiles) continue;
    const int m_tile = (int)(slot % m_tiles);
    if (pl.tall) {
      early_head_tall_tile<KIND>(hidden, vocab, m_total, m_tile * kTallBM, n_tile * kTallBN, n_tile,
                                 hidden_states, head_weight, tb, gemm_smem);
      continue;
    }
    const int m0 = m_tile * kGemmBM, v0 = n_tile * 64 * pl.fn;
    if (pl.fn == 2 && m_total <= kSmallBM && hidden % kSmallBK == 0)
      early_head_small_tile<KIND>(hidden, vocab, m_total, v0, n_tile, hidden_states, head_weight, tb, gemm_smem);
    else if (pl.fn == 2)
      early_head_tile<2, KIND>(hidden, vocab, m_total, m0, v0, n_tile, hidden_states, head_weight, tb, gemm_smem);
    else if (pl.fn == 3)
      early_head_tile<3, KIND>(hidden, vocab, m_total, m0, v0, n_tile, hidden_states, head_weight, tb, gemm_smem);
    else
      early_head_tile<4, KIND>(hidden, vocab, m_total, m0, v0, n_tile, hidden_states, head_weight, tb, gemm_smem);
  }
}

// fp32 variant: one score per thread, a plain sequential dot product, then the same two
// epilogues on a 256-wide slice of the row (column part = slice index).
template <int KIND>
__global__ __launch_bounds__(256) void early_head_f32_kernel(
    int hidden, int vocab, int B, const float *__restrict__ hidden_states,
    const float *__restrict__ head_weight, HeadTables tb) {
  const int m = blockIdx.x;
  if (m >= tb.row_base[B]) return;
  const int v = blockIdx.y * 256 + threadIdx.x;
  const bool in = v < vocab;
  const float *h = hidden_states + (size_t)tb.row_src[m] * hidden;
  const float *w = head_weight + (size_t)(in ? v : vocab - 1) * hidden;
  float z = 0.f;
  for (int x = 0; x < hidden; ++x) z = fmaf(h[x], w[x], z);
  const int lane = threadIdx.x & 63;
  if (KIND == 0) {
    __shared__ int s_cnt[4];
    const int pos = tb.row_info[2 * m], cc = tb.row_info[2 * m + 1];
    for (int e = 0; e < cc; ++e) {
      const int c = tb.child_list[pos + e];
      const int t = tb.token[c];
      const bool ok = t >= 0 && t < vocab;  // an id outside the vocabulary: the decision kernel fails it
      const float own = tb.own[c];
      const int cnt = __popcll(__ballot(ok && in && (z > own || (z == own && v < t))));
      if (lane == 0) s_cnt[threadIdx.x >> 6] = cnt;
      __syncthreads();
      if (threadIdx.x == 0)
        tb.cnt_part[(size_t)blockIdx.y * tb.cnt_stride + c] = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
      __syncthreads();
    }
  } else {
    float mx = in ? z : -INFINITY;
    mx = wave_reduce_max(mx);
    float sum = in ? expf(z - mx) : 0.f;
    sum = wave_reduce_sum(sum);
    __shared__ float s_m[4], s_s[4];
    if (lane == 0) {
      s_m[threadIdx.x >> 6] = mx;
      s_s[threadIdx.x >> 6] = sum;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int wv = 1; wv < 4; ++wv) lse_merge(mx, sum, s_m[wv], s_s[wv]);
      float *dst = tb.lse_part + ((size_t)m * tb.parts + blockIdx.y) * 2;
      dst[0] = mx;
      dst[1] = sum;
    }
  }
}

// ------------------------------------------------------------------------------------
// probability-based selection (Section 4.1, "Pruning Criterion", second criterion)
// ------------------------------------------------------------------------------------
// One wave per score row: log sum_v exp(z[v]) from the row's tile partials (the first
// n_parts of them were written), then logq = own score - that for every child of the
// row's node.  A token id outside the vocabulary has probability 0 (logq = -inf).
__global__ __launch_bounds__(kWave) void row_lse_kernel(int B, int vocab, int cus, int force, int bf16,
                                                        HeadTables tb, float *__restrict__ logq) {
  const int m = blockIdx.x;
  const int m_total = tb.row_base[B];
  if (m >= m_total) return;
  int n_parts;
  if (bf16) {
    n_parts = head_plan(m_total, vocab, cus, force).n_parts;
  } else {
    n_parts = (vocab + 255) / 256;
  }
  const int lane = threadIdx.x;
  float mx = -INFINITY, sum = 0.f;
  const float *part = tb.lse_part + (size_t)m * tb.parts * 2;
  for (int i = lane; i < n_parts; i += kWave) lse_merge(mx, sum, part[2 * i], part[2 * i + 1]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float m2 = __shfl_xor(mx, o, kWave), s2 = __shfl_xor(sum, o, kWave);
    lse_merge(mx, sum, m2, s2);
  }
  const float lse = mx + logf(sum);
  const int pos = tb.row_info[2 * m], cc = tb.row_info[2 * m + 1];
  for (int e = lane; e < cc; e += kWave) {
    const int c = tb.child_list[pos + e];
    const int t = tb.token[c];
    logq[c] = (t >= 0 && t < vocab) ? tb.own[c] - lse : -INFINITY;
  }
}

// which criterion decides (Section 4.1, "Pruning Criterion")
struct Criterion {
  int kind;             // 0 top-k, 1 probability threshold, 2 probability rank
  int top_k;            // kind 0
  float log_threshold;  // kind 1
  int keep_count;       // kind 2
  float *log_marginal;  // kinds 1, 2: optional output
};

// ------------------------------------------------------------------------------------
// the decision, branch elimination, compaction, mask subsampling
// ------------------------------------------------------------------------------------
// One workgroup per sequence, one lane per node.
//   top-k: a node fails when `top_k` or more scores of its parent's row beat its token's, or
//     its token id lies outside the vocabulary.
//   probability: the log marginal of a node's sequence is the sum of logq over its root path
//     (the cached ancestor set, root excluded, in root-to-node order); it fails when the
//     marginal is below the threshold, or when `keep_count` or more sequences of the tree are
//     more probable (equal marginals: the lower node index counts as more probable); a
//     marginal of zero probability always fails.
constexpr int kCompactSplit = 4;  // threads that add up one node's per-tile counts

__global__ __launch_bounds__(PROPD_MAX_TREE * kCompactSplit) void prune_compact_kernel(
    int B, int T_max, int vocab, int cus, int force, int bf16, Criterion crit, const int32_t *__restrict__ n_nodes,
    const int32_t *__restrict__ parent, const int32_t *__restrict__ token,
    const int32_t *__restrict__ depth, const uint64_t *__restrict__ anc,
    const int32_t *__restrict__ row_base, const int32_t *__restrict__ cnt_part,
    const float *__restrict__ logq, uint64_t *__restrict__ keep_bits,
    int32_t *__restrict__ new_index, int32_t *__restrict__ orig_index, int32_t *__restrict__ n_kept,
    int32_t *__restrict__ out_n_nodes, int32_t *__restrict__ out_parent,
    int32_t *__restrict__ out_token, int32_t *__restrict__ out_depth,
    uint64_t *__restrict__ out_anc, int32_t *__restrict__ rank_out) {
  const int b = blockIdx.x, i = threadIdx.x & (PROPD_MAX_TREE - 1), q = threadIdx.x / PROPD_MAX_TREE;
  const size_t base = (size_t)b * T_max;
  // Everything this thread reads is requested before the first value is used: the tree size,
  // the tile count and the node's own words do not wait for each other.  Slots past the tree
  // are read too (they exist) and dropped.
  const bool slot = i < T_max, worker = q == 0;
  const int T_raw = n_nodes[b];
  uint64_t a_lo = 0, a_hi = 0;
  int my_token = -1;
  if (worker && slot) {
    a_lo = anc[(base + i) * 2];
    a_hi = anc[(base + i) * 2 + 1];
    my_token = token[base + i];
  }
  __shared__ uint64_t s_fail[2], s_keep[2];
  __shared__ float s_q[PROPD_MAX_TREE], s_lm[PROPD_MAX_TREE];
  __shared__ int s_sum[kCompactSplit][PROPD_MAX_TREE];

  if (crit.kind == 0) {
    // rank = the counts of all column tiles (row_base == NULL: nothing was scored)
    int n_tiles = 0;
    if (row_base) {
      const int m_total = row_base[B];
      if (bf16) {
        if (m_total > 0) n_tiles = head_plan(m_total, vocab, cus, force).n_tiles;
      } else if (m_total > 0) {
        n_tiles = (vocab + 255) / 256;
      }
    }
    int sum = 0;
    if (slot && i > 0) {
      const int32_t *src = cnt_part + base + i;
      const size_t stride = (size_t)B * T_max;
      constexpr int kInFlight = 32;
      for (int t0 = q; t0 < n_tiles; t0 += kCompactSplit * kInFlight) {
        int v[kInFlight];
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
          const int t = t0 + kCompactSplit * k;
          v[k] = t < n_tiles ? src[(size_t)t * stride] : 0;
        }
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) sum += v[k];
      }
    }
    s_sum[q][i] = sum;
  }
  const int T = clamp_tree(T_raw, T_max);
  const bool valid = i < T;
  if (!valid) {
    a_lo = a_hi = 0;
    my_token = -1;
  }
  __syncthreads();
  // from here on one thread per node does the work; the others only meet it at the barriers
  bool fail = false;
  if (crit.kind == 0) {
    if (worker) {
      int my_rank = -1;
      if (valid) {
        my_rank = 0;
#pragma unroll
        for (int k = 0; k < kCompactSplit; ++k) my_rank += s_sum[k][i];
        // a token id outside the vocabulary can be in no top-k list
        if (i > 0 && (my_token < 0 || my_token >= vocab)) my_rank = vocab;
      }
      if (rank_out && i < T_max) rank_out[base + i] = my_rank;
      fail = valid && i > 0 && my_rank >= crit.top_k;
    }
  } else {
    if (worker) s_q[i] = (valid && i > 0) ? logq[base + i] : 0.f;
    __syncthreads();
    float lm = 0.f;
    if (worker && valid && i > 0) {
      uint64_t lo = a_lo & ~1ull, hi = a_hi;
      while (lo) {
        lm += s_q[__ffsll((long long)lo) - 1];
        lo &= lo - 1;
      }
      while (hi) {
        lm += s_q[64 + __ffsll((long long)hi) - 1];
        hi &= hi - 1;
      }
    }
    if (worker) s_lm[i] = valid ? lm : -INFINITY;
    __syncthreads();
    if (worker && valid && i > 0) {
      if (crit.kind == 1) {
        fail = !(lm >= crit.log_threshold);
      } else {
        int ahead = 0;
        for (int j = 0; j < T; ++j) ahead += (s_lm[j] > lm) || (s_lm[j] == lm && j < i);
        fail = ahead >= crit.keep_count;
      }
      fail = fail || !(lm > -INFINITY);
    }
    if (worker && crit.log_marginal && i < T_max) crit.log_marginal[base + i] = valid ? lm : 0.f;
  }
  if (!worker) {  // the two barriers below
    __syncthreads();
    __syncthreads();
    return;
  }
  const uint64_t fb = __ballot(fail);
  if ((i & 63) == 0) s_fail[i >> 6] = fb;
  __syncthreads();
  // a node goes as soon as any node of its root path failed
  const bool keep = valid && ((a_lo & s_fail[0]) | (a_hi & s_fail[1])) == 0;
  const uint64_t kb = __ballot(keep);
  if ((i & 63) == 0) s_keep[i >> 6] = kb;
  __syncthreads();
  const uint64_t k_lo = s_keep[0], k_hi = s_keep[1];
  const int kept = __popcll(k_lo) + __popcll(k_hi);
  const int ni = keep ? popc128_below(k_lo, k_hi, i) : -1;
  if (i < T_max) new_index[base + i] = ni;
  if (keep) {
    orig_index[base + ni] = i;
    out_token[base + ni] = my_token;
    out_depth[base + ni] = depth[base + i];
    int p = i == 0 ? -1 : parent[base + i];
    out_parent[base + ni] = (p >= 0 && p < T) ? popc128_below(k_lo, k_hi, p) : -1;
    // subsample the cached mask: keep the columns of survivors, renumbered
    uint64_t r_lo = 0, r_hi = 0;
    uint64_t w = a_lo & k_lo;
    while (w) {
      const int j = __ffsll((long long)w) - 1;
      w &= w - 1;
      const int pos = popc128_below(k_lo, k_hi, j);
      if (pos < 64) r_lo |= 1ull << pos; else r_hi |= 1ull << (pos - 64);
    }
    w = a_hi & k_hi;
    while (w) {
      const int j = 64 + __ffsll((long long)w) - 1;
      w &= w - 1;
      const int pos = popc128_below(k_lo, k_hi, j);
      if (pos < 64) r_lo |= 1ull << pos; else r_hi |= 1ull << (pos - 64);
    }
    out_anc[(base + ni) * 2] = r_lo;
    out_anc[(base + ni) * 2 + 1] = r_hi;
  }
  if (i >= kept && i < T_max) {
    orig_index[base + i] = -1;
    out_token[base + i] = -1;
    out_depth[base + i] = -1;
    out_parent[base + i] = -1;
    out_anc[(base + i) * 2] = 0;
    out_anc[(base + i) * 2 + 1] = 0;
  }
  if (i == 0) {
    keep_bits[2 * b] = k_lo;
    keep_bits[2 * b + 1] = k_hi;
    n_kept[b] = kept;
    if (out_n_nodes) out_n_nodes[b] = kept;
  }
}

// ------------------------------------------------------------------------------------
// payload rows of survivors
// ------------------------------------------------------------------------------------
struct PayloadArgs {
  const char *src[PROPD_MAX_PAYLOADS];
  char *dst[PROPD_MAX_PAYLOADS];
  unsigned long long row_bytes[PROPD_MAX_PAYLOADS];
  long long outer[PROPD_MAX_PAYLOADS];
  long long stride_b[PROPD_MAX_PAYLOADS], stride_outer[PROPD_MAX_PAYLOADS],
      stride_t[PROPD_MAX_PAYLOADS];
  int vec16[PROPD_MAX_PAYLOADS];  // rows, strides and bases are all 16-byte multiples
  long long block_end[PROPD_MAX_PAYLOADS];  // flattened grid: blocks of payloads 0..p end here
  int slices[PROPD_MAX_PAYLOADS];           // item slices per (b, o) slot
  int n;
};

constexpr int kGatherThreads = 256;

// Work items are (survivor row j, 16-byte piece c) pairs of one (b, o) slot of one payload.
// The grid is flat: a block finds its payload from the per-payload block counts, then its
// (b, o) slot and its slice of that slot's item list.  Every
// thread moves up to kGatherItems independent pieces, so the copies of a long row (hidden
// states) and of many short rows (tree K/V) are equally spread over the chip.
constexpr int kGatherItems = 8;

__global__ __launch_bounds__(kGatherThreads) void gather_rows_kernel(
    PayloadArgs args, int B, int T_max, const int32_t *__restrict__ orig_index,
    const int32_t *__restrict__ n_kept, int32_t *__restrict__ cu_nodes) {
  static_assert(kGatherThreads == kScanThreads, "the extra block runs the workgroup scan");
  if ((long long)blockIdx.x == args.block_end[args.n - 1]) {
    // one block past the payload blocks: the prefix sum of the survivor counts rides along
    // with this launch instead of taking one of its own
    block_exclusive_scan(n_kept, cu_nodes, B);
    return;
  }
  int pl = 0;
  while (pl < args.n - 1 && (long long)blockIdx.x >= args.block_end[pl]) ++pl;
  const long long local = (long long)blockIdx.x - (pl > 0 ? args.block_end[pl - 1] : 0);
  const long long outer = args.outer[pl];
  const long long bo = local / args.slices[pl];
  const unsigned slice = (unsigned)(local - bo * args.slices[pl]);
  if (bo >= (long long)B * outer) return;
  const long long o = bo % outer;
  const int b = (int)(bo / outer);
  int kept = n_kept[b];
  kept = kept > T_max ? T_max : kept;
  const unsigned long long unit = args.vec16[pl] ? 16 : 1;  // bytes per piece
  const unsigned long long per_row = args.row_bytes[pl] / unit;
  const unsigned long long items = (unsigned long long)kept * per_row;
  const char *sbase = args.src[pl] + b * args.stride_b[pl] + o * args.stride_outer[pl];
  char *dbase = args.dst[pl] + b * args.stride_b[pl] + o * args.stride_outer[pl];
  const unsigned long long first =
      ((unsigned long long)slice * kGatherItems) * kGatherThreads + threadIdx.x;
  if (args.vec16[pl] && (unsigned long long)T_max * per_row < (1ull << 31)) {
    // the common case: 16-byte pieces, 32-bit index arithmetic, all loads of the thread's
    // pieces in flight before the first store (items past the end re-read piece 0)
    const unsigned per32 = (unsigned)per_row, items32 = (unsigned)items, first32 = (unsigned)first;
    u32x4 v[kGatherItems];
    char *dptr[kGatherItems];
    bool ok[kGatherItems];
#pragma unroll
    for (int k = 0; k < kGatherItems; ++k) {
      unsigned item = first32 + (unsigned)k * kGatherThreads;
      ok[k] = item < items32;
      item = ok[k] ? item : 0u;
      const unsigned j = item / per32, c = item - j * per32;
      int i = kept > 0 ? orig_index[(size_t)b * T_max + j] : 0;
      ok[k] = ok[k] && i >= 0 && i < T_max;
      i = ok[k] ? i : 0;
      v[k] = *reinterpret_cast<const u32x4 *>(sbase + (long long)i * args.stride_t[pl] + c * 16u);
      dptr[k] = dbase + (long long)j * args.stride_t[pl] + c * 16u;
    }
#pragma unroll
    for (int k = 0; k < kGatherItems; ++k)
      if (ok[k]) *reinterpret_cast<u32x4 *>(dptr[k]) = v[k];
    return;
  }
#pragma unroll
  for (int k = 0; k < kGatherItems; ++k) {
    const unsigned long long item = first + (unsigned long long)k * kGatherThreads;
    if (item >= items) break;
    const int j = (int)(item / per_row);
    const unsigned long long c = item - (unsigned long long)j * per_row;
    const int i = orig_index[(size_t)b * T_max + j];
    if (i < 0 || i >= T_max) continue;
    const char *s = sbase + (long long)i * args.stride_t[pl] + c * unit;
    char *d = dbase + (long long)j * args.stride_t[pl] + c * unit;
    if (args.vec16[pl])
      *reinterpret_cast<u32x4 *>(d) = *reinterpret_cast<const u32x4 *>(s);
    else
      *d = *s;
  }
}

}  // namespace propd

static int prune_compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      cus = prop.multiProcessorCount;
    if (cus <= 0) cus = 256;
  }
  return cus;
}

static propd_status prune_impl(
    const propd::Criterion &crit, const propd_tree *tree, propd_dtype dt, int32_t hidden, int32_t vocab,
    const void *hidden_states, const void *head_weight, uint64_t *keep_bits, int32_t *new_index,
    int32_t *orig_index, int32_t *n_kept, int32_t *cu_nodes, const propd_tree_out *tree_out,
    int32_t *rank_out, int32_t n_payloads, const propd_payload *payloads, void *workspace,
    size_t workspace_bytes, void *hip_stream) {
  using namespace propd;
  if (!tree || tree->B < 1 || tree->T_max < 1 || tree->T_max > PROPD_MAX_TREE || hidden < 1 ||
      vocab < 1 || (crit.kind == 0 && crit.top_k < 1))
    return PROPD_ERR_INVALID_ARG;
  if (!tree->n_nodes || !tree->parent || !tree->token || !tree->depth || !tree->anc ||
      !hidden_states || !head_weight || !keep_bits || !new_index || !orig_index || !n_kept ||
      !cu_nodes || !tree_out || !tree_out->parent || !tree_out->token || !tree_out->depth ||
      !tree_out->anc)
    return PROPD_ERR_INVALID_ARG;
  if (dt != PROPD_BF16 && dt != PROPD_F32) return PROPD_ERR_INVALID_ARG;
  if (n_payloads < 0 || n_payloads > PROPD_MAX_PAYLOADS || (n_payloads > 0 && !payloads))
    return PROPD_ERR_INVALID_ARG;
  if (dt == PROPD_BF16 && hidden % kBK != 0) return PROPD_ERR_UNSUPPORTED;
  // operand rows are fetched 16 bytes per lane (bf16) or 4 (fp32); the scratch holds 8-byte records
  const uintptr_t op_align = dt == PROPD_BF16 ? 16 : 4;
  if (reinterpret_cast<uintptr_t>(hidden_states) % op_align != 0 ||
      reinterpret_cast<uintptr_t>(head_weight) % op_align != 0 ||
      reinterpret_cast<uintptr_t>(workspace) % 16 != 0 || reinterpret_cast<uintptr_t>(tree->anc) % 8 != 0)
    return PROPD_ERR_INVALID_ARG;
  const int B = tree->B, T_max = tree->T_max;
  if ((long long)B * T_max > (1ll << 24)) return PROPD_ERR_UNSUPPORTED;
  long long max_rows = 0, total_blocks = 0;
  PayloadArgs pa = {};
  for (int p = 0; p < n_payloads; ++p) {
    const propd_payload &pl = payloads[p];
    if (!pl.src || !pl.dst || pl.outer < 1 || pl.row_bytes == 0 || pl.stride_t < 0 ||
        pl.stride_b < 0 || pl.stride_outer < 0 || pl.src == pl.dst)
      return PROPD_ERR_INVALID_ARG;
    pa.src[p] = reinterpret_cast<const char *>(pl.src);
    pa.dst[p] = reinterpret_cast<char *>(pl.dst);
    pa.row_bytes[p] = pl.row_bytes;
    pa.outer[p] = pl.outer;
    pa.stride_b[p] = pl.stride_b;
    pa.stride_outer[p] = pl.stride_outer;
    pa.stride_t[p] = pl.stride_t;
    const uintptr_t any = reinterpret_cast<uintptr_t>(pl.src) | reinterpret_cast<uintptr_t>(pl.dst) |
                          (uintptr_t)pl.row_bytes | (uintptr_t)pl.stride_b |
                          (uintptr_t)pl.stride_outer | (uintptr_t)pl.stride_t;
    pa.vec16[p] = (any & 15) == 0;
    const long long rows = (long long)B * pl.outer;  // grid.x: one slot per (b, o)
    if (rows > (1ll << 31) - 1) return PROPD_ERR_UNSUPPORTED;
    max_rows = rows > max_rows ? rows : max_rows;
    const long long pieces = (long long)T_max * (long long)(pl.row_bytes / (pa.vec16[p] ? 16 : 1));
    const long long slices = (pieces + kGatherThreads * kGatherItems - 1) /
                             (kGatherThreads * kGatherItems);
    if (slices > (1 << 24)) return PROPD_ERR_UNSUPPORTED;
    pa.slices[p] = (int)slices;
    total_blocks += rows * slices;
    pa.block_end[p] = total_blocks;
    if (total_blocks > (1ll << 31) - 2) return PROPD_ERR_UNSUPPORTED;
  }
  const size_t need = early_prune_workspace_bytes(B, T_max, vocab);
  if (!workspace || workspace_bytes < need) return PROPD_ERR_WORKSPACE;
  PruneScratch ws = carve_scratch(workspace, B, T_max, vocab);
  hipStream_t st = as_stream(hip_stream);

  static const int force = [] {  // tile-shape override for tuning runs: 1 = 256-row tiles, 2 = 352-row tiles
    const char *e = getenv("PROPD_HEAD_PLAN");
    return e ? atoi(e) : 0;
  }();
  const bool scored = !(crit.kind == 0 && crit.top_k >= vocab);
  // top_k >= vocab: every id of the vocabulary is inside the list, no scores are needed (ids
  // outside the vocabulary still fail, in the decision kernel)
  const int cus = prune_compute_units();
  if (scored) {
    PrepareArgs pr;
    pr.B = B;
    pr.T_max = T_max;
    pr.hidden = hidden;
    pr.vocab = vocab;
    pr.n_nodes = tree->n_nodes;
    pr.parent = tree->parent;
    pr.token = tree->token;
    pr.hidden_states = hidden_states;
    pr.head_weight = head_weight;
    pr.row_src = ws.row_src;
    pr.row_base = ws.row_base;
    pr.row_info = ws.row_info;
    pr.child_list = ws.child_list;
    pr.own = ws.own;
    const unsigned prep_grid = (unsigned)((B + kTableWaves - 1) / kTableWaves) +
                               (unsigned)B * (unsigned)((T_max + kOwnNodes - 1) / kOwnNodes);
    if (dt == PROPD_BF16)
      hipLaunchKernelGGL(prune_prepare_kernel<true>, dim3(prep_grid), dim3(kScanThreads), 0, st, pr);
    else
      hipLaunchKernelGGL(prune_prepare_kernel<false>, dim3(prep_grid), dim3(kScanThreads), 0, st, pr);
    if (!launch_ok()) return PROPD_ERR_DEVICE;
    HeadTables tb;
    tb.row_src = ws.row_src;
    tb.row_base = ws.row_base;
    tb.row_info = ws.row_info;
    tb.child_list = ws.child_list;
    tb.token = tree->token;
    tb.own = ws.own;
    tb.cnt_part = ws.cnt_part;
    tb.cnt_stride = B * T_max;
    tb.lse_part = ws.lse_part;
    tb.parts = (int)ws.parts;
    if (dt == PROPD_BF16) {
      constexpr int BM = kGemmBM, BN = 64 * kGemmMinFN;  // the tile count is largest for the narrowest tiles
      static bool attr_set = false;
      if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&early_head_bf16_kernel<0>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kHeadLdsBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(&early_head_bf16_kernel<1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kHeadLdsBytes) != hipSuccess)
          return PROPD_ERR_DEVICE;
        attr_set = true;
      }
      // one workgroup per compute unit and round, two rounds resident in the queue; fewer when
      // even the largest row count has fewer tiles
      const long long m_tiles_cap = (ws.row_cap + BM - 1) / BM;
      const long long n_groups = ((vocab + BN - 1) / BN + kXcds - 1) / kXcds;
      long long grid = kXcds * n_groups * m_tiles_cap;
      const long long persistent = (2ll * cus + kXcds - 1) / kXcds * kXcds;
      grid = grid < persistent ? grid : persistent;
      if (crit.kind == 0)
        hipLaunchKernelGGL(early_head_bf16_kernel<0>, dim3((unsigned)grid), dim3(kGemmThreads), kHeadLdsBytes, st,
                           hidden, vocab, B, cus, force, reinterpret_cast<const uint16_t *>(hidden_states),
                           reinterpret_cast<const uint16_t *>(head_weight), tb);
      else
        hipLaunchKernelGGL(early_head_bf16_kernel<1>, dim3((unsigned)grid), dim3(kGemmThreads), kHeadLdsBytes, st,
                           hidden, vocab, B, cus, force, reinterpret_cast<const uint16_t *>(hidden_states),
                           reinterpret_cast<const uint16_t *>(head_weight), tb);
    } else {
      dim3 grid((unsigned)ws.row_cap, (unsigned)((vocab + 255) / 256));
      if (crit.kind == 0)
        hipLaunchKernelGGL(early_head_f32_kernel<0>, grid, dim3(256), 0, st, hidden, vocab, B,
                           reinterpret_cast<const float *>(hidden_states),
                           reinterpret_cast<const float *>(head_weight), tb);
      else
        hipLaunchKernelGGL(early_head_f32_kernel<1>, grid, dim3(256), 0, st, hidden, vocab, B,
                           reinterpret_cast<const float *>(hidden_states),
                           reinterpret_cast<const float *>(head_weight), tb);
    }
    if (crit.kind != 0)
      hipLaunchKernelGGL(row_lse_kernel, dim3((unsigned)ws.row_cap), dim3(kWave), 0, st, B, vocab, cus, force,
                         dt == PROPD_BF16 ? 1 : 0, tb, ws.logq);
  }
  if (!launch_ok()) return PROPD_ERR_DEVICE;
  hipLaunchKernelGGL(prune_compact_kernel, dim3(B), dim3(PROPD_MAX_TREE * kCompactSplit), 0, st, B, T_max,
                     vocab, cus, force, dt == PROPD_BF16 ? 1 : 0, crit, tree->n_nodes, tree->parent, tree->token,
                     tree->depth, tree->anc, scored ? ws.row_base : nullptr, ws.cnt_part, ws.logq,
                     keep_bits, new_index, orig_index, n_kept, tree_out->n_nodes, tree_out->parent,
                     tree_out->token, tree_out->depth, tree_out->anc, rank_out);
  if (n_payloads > 0) {
    pa.n = n_payloads;
    dim3 grid((unsigned)(total_blocks + 1));  // the extra block writes cu_nodes
    hipLaunchKernelGGL(gather_rows_kernel, grid, dim3(kGatherThreads), 0, st, pa, B, T_max,
                       orig_index, n_kept, cu_nodes);
  } else {
    hipLaunchKernelGGL(cu_nodes_kernel, dim3(1), dim3(kScanThreads), 0, st, B, n_kept, cu_nodes);
  }
  return launch_ok() ? PROPD_OK : PROPD_ERR_DEVICE;
}

extern "C" propd_status propd_early_prune(
    const propd_tree *tree, propd_dtype dt, int32_t hidden, int32_t vocab, int32_t top_k,
    const void *hidden_states, const void *head_weight, uint64_t *keep_bits, int32_t *new_index,
    int32_t *orig_index, int32_t *n_kept, int32_t *cu_nodes, const propd_tree_out *tree_out,
    int32_t *rank_out, int32_t n_payloads, const propd_payload *payloads, void *workspace,
    size_t workspace_bytes, void *hip_stream) {
  if (top_k < 1) return PROPD_ERR_INVALID_ARG;
  const propd::Criterion crit = {0, top_k, 0.f, 0, nullptr};
  return prune_impl(crit, tree, dt, hidden, vocab, hidden_states, head_weight, keep_bits, new_index,
                    orig_index, n_kept, cu_nodes, tree_out, rank_out, n_payloads, payloads,
                    workspace, workspace_bytes, hip_stream);
}

extern "C" propd_status propd_early_prune_prob(
    const propd_tree *tree, propd_dtype dt, int32_t hidden, int32_t vocab, propd_prob_mode mode,
    float threshold, int32_t keep_count, const void *hidden_states, const void *head_weight,
    uint64_t *keep_bits, int32_t *new_index, int32_t *orig_index, int32_t *n_kept,
    int32_t *cu_nodes, const propd_tree_out *tree_out, float *log_marginal, int32_t n_payloads,
    const propd_payload *payloads, void *workspace, size_t workspace_bytes, void *hip_stream) {
  propd::Criterion crit = {1, 1, 0.f, 0, log_marginal};
  if (mode == PROPD_PROB_THRESHOLD) {
    if (!(threshold >= 0.f) || threshold > 1.f) return PROPD_ERR_INVALID_ARG;
    crit.log_threshold = threshold > 0.f ? logf(threshold) : -INFINITY;
  } else if (mode == PROPD_PROB_RANK) {
    if (keep_count < 1) return PROPD_ERR_INVALID_ARG;
    crit.kind = 2;
    crit.keep_count = keep_count;
  } else {
    return PROPD_ERR_INVALID_ARG;
  }
  return prune_impl(crit, tree, dt, hidden, vocab, hidden_states, head_weight, keep_bits, new_index,
                    orig_index, n_kept, cu_nodes, tree_out, nullptr, n_payloads, payloads,
                    workspace, workspace_bytes, hip_stream);
}
