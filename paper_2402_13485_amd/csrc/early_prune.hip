// Early pruning of the token tree (Section 4.1: "Pruning Process" and
// "Implementation Optimization").
//
// Kernel chain, all on the caller's stream, no host round trip:
//   parent_rows_kernel    per sequence: which nodes have children (only those
//                         need early-head scores), compacted by wave ballot
//   row_table_kernel      prefix sum over sequences -> global row table
//   early_head_bf16_kernel  scores z = hidden[parent rows] . head_weight^T as a
//                         bf16 MFMA GEMM with fp32 accumulation (M = parent rows,
//                         N = vocabulary, K = hidden); fp32 scores go to scratch
//   early_head_f32_kernel plain fp32 variant
//   rank_count_kernel     per parent row: rank of every child's token by
//                         counting scores that beat it (the top-k membership test)
//   child_logprob_kernel  probability criterion: log-sum-exp of every parent row and the
//                         log-probability of every child's token
//   prob_decide_kernel    probability criterion: path marginals, threshold or rank test
//   prune_compact_kernel  per sequence: fail bits by ballot, branch elimination
//                         by testing the cached ancestor bitset against the fail
//                         bits, order-preserving compaction by prefix popcount,
//                         mask subsampling by bit extraction
//   cu_nodes_kernel       exclusive prefix sum of survivor counts (when there are payloads
//                         it rides along as one extra block of the gather launch)
//   gather_rows_kernel    survivor rows of the listed payload tensors
#include "common.h"

namespace propd {

// ------------------------------------------------------------------------------------
// scratch layout
// ------------------------------------------------------------------------------------
struct PruneScratch {
  int32_t *rank;        // [B*T_max]
  int32_t *n_par;       // [B]
  int32_t *local_list;  // [B*T_max]  per sequence: nodes with children, ascending
  int32_t *row_src;     // [B*T_max]  global row -> b*T_max + node
  int32_t *row_base;    // [B+1]      exclusive prefix of n_par; [B] = total rows
  float *logq;          // [B*T_max]  probability criterion: log q of every node's token
  float *scores;        // [row_cap * score_pitch]
  size_t row_cap, score_pitch, total_bytes;
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
  s.rank = reinterpret_cast<int32_t *>(take(nt * 4));
  s.n_par = reinterpret_cast<int32_t *>(take((size_t)B * 4));
  s.local_list = reinterpret_cast<int32_t *>(take(nt * 4));
  s.row_src = reinterpret_cast<int32_t *>(take(nt * 4));
  s.row_base = reinterpret_cast<int32_t *>(take((size_t)(B + 1) * 4));
  s.logq = reinterpret_cast<float *>(take(nt * 4));
  s.row_cap = (size_t)B * (T_max > 1 ? T_max - 1 : 1);  // a node with children is not a leaf
  s.score_pitch = align_up((size_t)vocab, 4);
  s.scores = reinterpret_cast<float *>(take(s.row_cap * s.score_pitch * 4));
  s.total_bytes = off;
  return s;
}

size_t early_prune_workspace_bytes(int B, int T_max, int vocab) {
  return carve_scratch(nullptr, B, T_max, vocab).total_bytes;
}

// ------------------------------------------------------------------------------------
// which nodes need scores
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(PROPD_MAX_TREE) void parent_rows_kernel(
    int T_max, const int32_t *__restrict__ n_nodes, const int32_t *__restrict__ parent,
    int32_t *__restrict__ n_par, int32_t *__restrict__ local_list, int32_t *__restrict__ rank) {
  const int b = blockIdx.x, i = threadIdx.x;
  int T = n_nodes[b];
  T = T < 1 ? 1 : (T > T_max ? T_max : T);
  __shared__ int s_has_child[PROPD_MAX_TREE];
  __shared__ int s_wave_count[2];
  s_has_child[i] = 0;
  __syncthreads();
  if (i > 0 && i < T) {
    const int p = parent[(size_t)b * T_max + i];
    if (p >= 0 && p < i) s_has_child[p] = 1;  // same value from every child: benign
  }
  __syncthreads();
  const bool is_par = i < T && s_has_child[i] != 0;
  const uint64_t bal = __ballot(is_par);
  if ((i & 63) == 0) s_wave_count[i >> 6] = __popcll(bal);
  __syncthreads();
  const int before = (i >= 64 ? s_wave_count[0] : 0) + __popcll(bal & ((1ull << (i & 63)) - 1ull));
  if (is_par) local_list[(size_t)b * T_max + before] = i;
  if (i == 0) n_par[b] = s_wave_count[0] + s_wave_count[1];
  // ranks default to 0 (root; everything when nothing is scored), padding to -1
  if (i < T_max) rank[(size_t)b * T_max + i] = i < T ? 0 : -1;
}

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

// Row table: row_base = exclusive prefix of n_par over the sequences (workgroup 0 writes it),
// row_src[row_base[b] + r] = node of the r-th parent of sequence b.  Every workgroup takes 256
// (sequence, r) slots and finds the base of its first sequence by a sum of its own, so the
// table is built by as many workgroups as there are slots instead of one.
__global__ __launch_bounds__(kScanThreads) void row_table_kernel(
    int B, int T_max, const int32_t *__restrict__ n_par, const int32_t *__restrict__ local_list,
    int32_t *__restrict__ row_base, int32_t *__restrict__ row_src) {
  const int tid = threadIdx.x;
  if (blockIdx.x == 0) {
    block_exclusive_scan(n_par, row_base, B);
    __syncthreads();
  }
  const int idx0 = blockIdx.x * kScanThreads;
  const int b_first = idx0 / T_max;
  int part = 0;
  for (int x = tid; x < b_first; x += kScanThreads) part += n_par[x];
  part = wave_reduce_sum(part);
  __shared__ int s_sum[kScanThreads / kWave];
  if ((tid & 63) == 0) s_sum[tid >> 6] = part;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int w = 0; w < kScanThreads / kWave; ++w) base += s_sum[w];
  const int idx = idx0 + tid;
  if (idx >= B * T_max) return;
  const int b = idx / T_max, r = idx - b * T_max;
  if (r >= n_par[b]) return;
  for (int x = b_first; x < b; ++x) base += n_par[x];
  row_src[base + r] = b * T_max + local_list[idx];
}

__global__ __launch_bounds__(kScanThreads) void cu_nodes_kernel(int B,
                                                                const int32_t *__restrict__ n_kept,
                                                                int32_t *__restrict__ cu_nodes) {
  block_exclusive_scan(n_kept, cu_nodes, B);
}

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
//   - K advances 32 per step through a ring of four 32 KB LDS stages filled by direct
//     global->LDS loads (no staging registers, no LDS stores), up to three steps ahead of
//     the math; one barrier per K step.  A row of a stage is 64 bytes (4 chunks of 16); the
//     lane that fills chunk c of LDS row r fetches chunk c ^ key(r) of the global row, with
//     key(r) = (r >> 2) & 3, so that the 16 rows one quarter-wave reads for a chunk column
//     fall into 16 different bank groups;
//   - operand fragments are double-buffered in registers: the LDS reads of one half step
//     are issued before the MFMAs of the half step before it, and the barrier sits between
//     two MFMA groups whose operands are already in registers, so the matrix core has work
//     queued while waves meet;
//   - the A rows are gathered through the row table by the loads themselves; rows past
//     the last one and vocabulary entries past the last re-read the last valid one and
//     are dropped when the scores are stored;
//   - the grid is one-dimensional and XCD-aware.  Workgroups are handed to the 8
//     XCDs round-robin, each XCD has its own L2: workgroup id -> (xcd, slot), and an
//     XCD walks its own vocabulary tiles with all row tiles of one vocabulary tile
//     adjacent in time, so a weight tile is fetched from HBM once and hits in that
//     XCD's L2 for the other row tiles.
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

// Waits until at most n of this wave's loads are outstanding (n = whole steps of 3 or 4 loads).
__device__ __forceinline__ void gemm_wait_outstanding(int n) {
  if (n >= 16) gemm_wait_vmem<16>();
  else if (n >= 12) gemm_wait_vmem<12>();
  else if (n >= 9) gemm_wait_vmem<9>();
  else if (n >= 8) gemm_wait_vmem<8>();
  else if (n >= 6) gemm_wait_vmem<6>();
  else if (n >= 4) gemm_wait_vmem<4>();
  else if (n >= 3) gemm_wait_vmem<3>();
  else gemm_wait_vmem<0>();
}

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

template <int FN>
__device__ __forceinline__ void early_head_tile(
    int hidden, int vocab, int m_total, int m0, int v0, const uint16_t *__restrict__ hidden_states,
    const uint16_t *__restrict__ head_weight, const int32_t *__restrict__ row_src,
    float *__restrict__ scores, size_t score_pitch, unsigned char *gemm_smem) {
  constexpr int BM = kGemmBM, BN = 64 * FN, WN = 32 * FN;
  constexpr int kStages = gemm_stages(FN), kStageBytes = gemm_stage_bytes(FN);
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void global_void;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void *)gemm_smem;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, g = lane >> 5;

  // ---- loader: a load instruction fills 16 rows (1 KB).  A stage has 16 such groups of A
  //      rows and 4*FN of W rows; wave w takes groups w and w+8 of each (the second W group
  //      only where it exists).
  const int ld_row = lane >> 2;
  const int ld_chunk = ((lane & 3) ^ ((lane >> 4) & 3)) << 4;  // byte offset in the global row
  const bool second_w = FN == 4 ? true : (FN == 2 ? false : wave < 4);
  const int per_step = second_w ? 4 : 3;  // loads of this wave per K step
  const unsigned char *a_src[2], *b_src[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    int m = m0 + 16 * (wave + 8 * j) + ld_row;
    m = m < m_total ? m : m_total - 1;
    a_src[j] = reinterpret_cast<const unsigned char *>(hidden_states + (size_t)row_src[m] * hidden) + ld_chunk;
    int v = v0 + 16 * (wave + 8 * j) + ld_row;
    v = v < vocab ? v : vocab - 1;
    b_src[j] = reinterpret_cast<const unsigned char *>(head_weight + (size_t)v * hidden) + ld_chunk;
  }
  auto issue = [&](int slot) {  // the next K step of every source pointer
    unsigned char *dst = gemm_smem + slot * kStageBytes + wave * 1024;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      __builtin_amdgcn_global_load_lds((global_void *)a_src[j], (lds_void *)(dst + j * 8192), 16, 0, 0);
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
  gemm_wait_outstanding((n_pro - 1) * per_step);
  __builtin_amdgcn_s_barrier();
  constexpr int kReads = 2 + FN;  // LDS reads of one half step
  Frag f0, f1;
  read(f0, 0, 0);
  uint32_t so = 0;  // byte offset of the stage being multiplied
  for (int step = 0; step + 1 < n_steps; ++step) {
    read(f1, so, 1);
    gemm_wait_frag<kReads>(f0);  // the reads just issued fly while the MFMAs below run
    mma(f0);
    __builtin_amdgcn_sched_barrier(0);
    gemm_wait_frag<0>(f1);  // this wave is done with the slot of this step
    // the next step has landed once at most the steps after it (kStages-2 of them were
    // issued) are outstanding
    {
      const int issued_after = n_steps - 2 - step < kStages - 2 ? n_steps - 2 - step : kStages - 2;
      gemm_wait_outstanding(issued_after * per_step);
    }
    __builtin_amdgcn_s_barrier();  // it is visible; every wave is done with this step's slot
    if (step + kStages < n_steps) {
      issue(slot_ld);  // into the slot of this step
      slot_ld = slot_ld + 1 == kStages ? 0 : slot_ld + 1;
    }
    so = so + kStageBytes == kStages * kStageBytes ? 0 : so + kStageBytes;
    read(f0, so, 0);
    mma(f1);
    __builtin_amdgcn_sched_barrier(0);
  }
  read(f1, so, 1);
  gemm_wait_frag<kReads>(f0);
  mma(f0);
  gemm_wait_frag<0>(f1);
  mma(f1);

  mfma_settle();
  // accumulator layout of the 32x32 MFMA: lane -> column l32, register r -> row
  // 8*(r/4) + 4*g + r%4
  const bool full = m0 + BM <= m_total && v0 + BN <= vocab;
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < FN; ++y) {
      const int col = v0 + wn * WN + y * 32 + l32;
      const int row0 = m0 + wm * 64 + x * 32 + 4 * g;
      float *out = scores + (size_t)row0 * score_pitch + col;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int dr = 8 * (r >> 2) + (r & 3);
        if (full || (row0 + dr < m_total && col < vocab)) out[(size_t)dr * score_pitch] = acc[x][y][r];
      }
    }
}

__global__ __launch_bounds__(kGemmThreads, 1) void early_head_bf16_kernel(
    int hidden, int vocab, int B, int cus, const uint16_t *__restrict__ hidden_states,
    const uint16_t *__restrict__ head_weight, const int32_t *__restrict__ row_src,
    const int32_t *__restrict__ row_base, float *__restrict__ scores, size_t score_pitch) {
  const int m_total = row_base[B];
  const int m_tiles = (m_total + kGemmBM - 1) / kGemmBM;
  if (m_tiles == 0) return;
  const int fn = gemm_pick_fn(m_tiles, vocab, cus);
  const int n_tiles = (vocab + 64 * fn - 1) / (64 * fn);
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int n_tile = (slot / m_tiles) * kXcds + xcd;
  if (n_tile >= n_tiles) return;
  const int m0 = (slot % m_tiles) * kGemmBM, v0 = n_tile * 64 * fn;
  extern __shared__ __attribute__((aligned(1024))) unsigned char gemm_smem[];
  if (fn == 2)
    early_head_tile<2>(hidden, vocab, m_total, m0, v0, hidden_states, head_weight, row_src, scores,
                       score_pitch, gemm_smem);
  else if (fn == 3)
    early_head_tile<3>(hidden, vocab, m_total, m0, v0, hidden_states, head_weight, row_src, scores,
                       score_pitch, gemm_smem);
  else
    early_head_tile<4>(hidden, vocab, m_total, m0, v0, hidden_states, head_weight, row_src, scores,
                       score_pitch, gemm_smem);
}

// fp32 variant: one score per thread, a plain sequential dot product.
__global__ __launch_bounds__(256) void early_head_f32_kernel(
    int hidden, int vocab, int B, const float *__restrict__ hidden_states,
    const float *__restrict__ head_weight, const int32_t *__restrict__ row_src,
    const int32_t *__restrict__ row_base, float *__restrict__ scores, size_t score_pitch) {
  const int m = blockIdx.x;
  if (m >= row_base[B]) return;
  const int v = blockIdx.y * 256 + threadIdx.x;
  if (v >= vocab) return;
  const float *h = hidden_states + (size_t)row_src[m] * hidden;
  const float *w = head_weight + (size_t)v * hidden;
  float acc = 0.f;
  for (int x = 0; x < hidden; ++x) acc = fmaf(h[x], w[x], acc);
  scores[(size_t)m * score_pitch + v] = acc;
}

// ------------------------------------------------------------------------------------
// top-k membership by counting
// ------------------------------------------------------------------------------------
constexpr int kRankThreads = 256;
constexpr int kRankChunk = 8;     // children compared per pass over the scores
constexpr int kRankSplit = 4;     // workgroups sharing one parent row (column slices)

// One pass over a slice of a score row for NC children at once: counts, per child, the scores
// that beat its token's (a higher score, or the same score at a lower id), adds the counts of
// the workgroup up in LDS and then onto the children's ranks.
template <int NC>
__device__ __forceinline__ void rank_pass(int b, int T_max, int vocab, int c0, int nchild, int part,
                                          int c_lo, int c_hi, int nvec, const float *__restrict__ z,
                                          const int32_t *__restrict__ token, const int *s_child,
                                          int *s_count, int32_t *__restrict__ rank) {
  const int tid = threadIdx.x;
  float thr[NC];
  int tok[NC], cnt[NC];
#pragma unroll
  for (int e = 0; e < NC; ++e) {
    thr[e] = INFINITY;  // unused slot: nothing beats +inf, nothing ties below id -1
    tok[e] = -1;
    cnt[e] = 0;
    if (c0 + e < nchild) {
      const int t = token[(size_t)b * T_max + s_child[c0 + e]];
      if (t >= 0 && t < vocab) {
        thr[e] = z[t];
        tok[e] = t;
      }
    }
  }
  if (tid < NC) s_count[tid] = 0;
  __syncthreads();
  // four loads of a lane in flight before the first is used (a position past the slice
  // re-reads the slice's first vector and is not counted)
  constexpr int kInFlight = 4;
  for (int c0 = c_lo + tid; c0 < c_hi; c0 += kInFlight * kRankThreads) {
    f32x4 u[kInFlight];
#pragma unroll
    for (int k = 0; k < kInFlight; ++k) {
      const int c = c0 + k * kRankThreads;
      u[k] = *reinterpret_cast<const f32x4 *>(z + 4 * (c < c_hi ? c : c_lo));
    }
#pragma unroll
    for (int k = 0; k < kInFlight; ++k) {
      const int c = c0 + k * kRankThreads;
      if (c >= c_hi) break;
      const int v = 4 * c;
#pragma unroll
      for (int e = 0; e < NC; ++e) {
        cnt[e] += (u[k].x > thr[e]) || (u[k].x == thr[e] && v < tok[e]);
        cnt[e] += (u[k].y > thr[e]) || (u[k].y == thr[e] && v + 1 < tok[e]);
        cnt[e] += (u[k].z > thr[e]) || (u[k].z == thr[e] && v + 2 < tok[e]);
        cnt[e] += (u[k].w > thr[e]) || (u[k].w == thr[e] && v + 3 < tok[e]);
      }
    }
  }
  if (part == kRankSplit - 1)
    for (int v = 4 * nvec + tid; v < vocab; v += kRankThreads) {
      const float x = z[v];
#pragma unroll
      for (int e = 0; e < NC; ++e) cnt[e] += (x > thr[e]) || (x == thr[e] && v < tok[e]);
    }
#pragma unroll
  for (int e = 0; e < NC; ++e) {
    const int sum = wave_reduce_sum(cnt[e]);
    if ((tid & 63) == 0 && sum) atomicAdd(&s_count[e], sum);
  }
  __syncthreads();
  if (tid < NC && c0 + tid < nchild) {
    int mine = 0;
    bool valid_tok = false;
#pragma unroll
    for (int e = 0; e < NC; ++e)
      if (e == tid) {
        mine = s_count[e];
        valid_tok = tok[e] >= 0;
      }
    int32_t *dst = &rank[(size_t)b * T_max + s_child[c0 + tid]];
    // a token id outside the vocabulary can be in no top-k list
    if (!valid_tok) {
      if (part == 0) atomicAdd(dst, vocab);
    } else if (mine) {
      atomicAdd(dst, mine);
    }
  }
  __syncthreads();
}

// One parent row is shared by kRankSplit workgroups, each counting over its own slice of
// the vocabulary and adding its counts to the children's ranks with integer atomics (the
// sum does not depend on the order).  ranks of children were zeroed by parent_rows_kernel.
// Children are taken up to kRankChunk at a time, in a pass specialised for 1, 2, 4 or 8 of
// them: most nodes have one or two children and the compare work goes with that number.
__global__ __launch_bounds__(kRankThreads) void rank_count_kernel(
    int B, int T_max, int vocab, const int32_t *__restrict__ n_nodes,
    const int32_t *__restrict__ parent, const int32_t *__restrict__ token,
    const int32_t *__restrict__ row_src, const int32_t *__restrict__ row_base,
    const float *__restrict__ scores, size_t score_pitch, int32_t *__restrict__ rank) {
  const int m = blockIdx.x / kRankSplit, part = blockIdx.x - m * kRankSplit;
  if (m >= row_base[B]) return;
  const int node = row_src[m];
  const int b = node / T_max, p = node - b * T_max;
  int T = n_nodes[b];
  T = T < 1 ? 1 : (T > T_max ? T_max : T);
  const int tid = threadIdx.x;
  __shared__ int s_child[PROPD_MAX_TREE];
  __shared__ int s_nchild;
  __shared__ int s_count[kRankChunk];
  if (tid == 0) s_nchild = 0;
  __syncthreads();
  if (tid > p && tid < T && parent[(size_t)b * T_max + tid] == p)
    s_child[atomicAdd(&s_nchild, 1)] = tid;
  __syncthreads();
  const int nchild = s_nchild;
  const float *z = scores + (size_t)m * score_pitch;
  // this workgroup's slice, in units of 4 scores; the last slice also takes the tail
  const int nvec = vocab >> 2;
  const int per = (nvec + kRankSplit - 1) / kRankSplit;
  const int c_lo = part * per, c_hi = (c_lo + per < nvec) ? c_lo + per : nvec;

  for (int c0 = 0; c0 < nchild; c0 += kRankChunk) {
    const int here = nchild - c0;
    if (here <= 1)
      rank_pass<1>(b, T_max, vocab, c0, nchild, part, c_lo, c_hi, nvec, z, token, s_child, s_count, rank);
    else if (here <= 2)
      rank_pass<2>(b, T_max, vocab, c0, nchild, part, c_lo, c_hi, nvec, z, token, s_child, s_count, rank);
    else if (here <= 4)
      rank_pass<4>(b, T_max, vocab, c0, nchild, part, c_lo, c_hi, nvec, z, token, s_child, s_count, rank);
    else
      rank_pass<kRankChunk>(b, T_max, vocab, c0, nchild, part, c_lo, c_hi, nvec, z, token, s_child, s_count, rank);
  }
}

// ------------------------------------------------------------------------------------
// probability-based selection (Section 4.1, "Pruning Criterion", second criterion)
// ------------------------------------------------------------------------------------
constexpr int kLseThreads = 256;

// (max, sum of exp(x - max)) of two parts of a row, merged
__device__ __forceinline__ void lse_merge(float &m, float &s, float m2, float s2) {
  const float mm = m > m2 ? m : m2;
  s = (m == -INFINITY ? 0.f : s * expf(m - mm)) + (m2 == -INFINITY ? 0.f : s2 * expf(m2 - mm));
  m = mm;
}

// One workgroup per parent row: one pass over the row's scores for log sum_v exp(z[v]), then
// logq = z[token] - that for every child of the row's node.  A token id outside the
// vocabulary has probability 0 (logq = -inf).
__global__ __launch_bounds__(kLseThreads) void child_logprob_kernel(
    int B, int T_max, int vocab, const int32_t *__restrict__ n_nodes,
    const int32_t *__restrict__ parent, const int32_t *__restrict__ token,
    const int32_t *__restrict__ row_src, const int32_t *__restrict__ row_base,
    const float *__restrict__ scores, size_t score_pitch, float *__restrict__ logq) {
  const int m = blockIdx.x;
  if (m >= row_base[B]) return;
  const int node = row_src[m];
  const int b = node / T_max, p = node - b * T_max;
  int T = n_nodes[b];
  T = T < 1 ? 1 : (T > T_max ? T_max : T);
  const int tid = threadIdx.x;
  const float *z = scores + (size_t)m * score_pitch;
  float mx = -INFINITY, sum = 0.f;
  const int nvec = vocab >> 2;
  for (int c = tid; c < nvec; c += kLseThreads) {
    const f32x4 u = *reinterpret_cast<const f32x4 *>(z + 4 * c);
    const float m4 = fmaxf(fmaxf(u.x, u.y), fmaxf(u.z, u.w));
    const float s4 = expf(u.x - m4) + expf(u.y - m4) + expf(u.z - m4) + expf(u.w - m4);
    lse_merge(mx, sum, m4, s4);
  }
  for (int v = 4 * nvec + tid; v < vocab; v += kLseThreads) lse_merge(mx, sum, z[v], 1.f);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float m2 = __shfl_xor(mx, o, kWave), s2 = __shfl_xor(sum, o, kWave);
    lse_merge(mx, sum, m2, s2);
  }
  __shared__ float s_m[kLseThreads / kWave], s_s[kLseThreads / kWave];
  if ((tid & 63) == 0) {
    s_m[tid >> 6] = mx;
    s_s[tid >> 6] = sum;
  }
  __syncthreads();
  mx = s_m[0];
  sum = s_s[0];
#pragma unroll
  for (int w = 1; w < kLseThreads / kWave; ++w) lse_merge(mx, sum, s_m[w], s_s[w]);
  const float lse = mx + logf(sum);
  if (tid > p && tid < T && parent[(size_t)b * T_max + tid] == p) {
    const int t = token[(size_t)b * T_max + tid];
    logq[(size_t)b * T_max + tid] = (t >= 0 && t < vocab) ? z[t] - lse : -INFINITY;
  }
}

// One workgroup per sequence, one lane per node: the log marginal of a node's sequence is the
// sum of logq over its root path (the cached ancestor set, root excluded, in root-to-node
// order); then the test.  mode 0: pruned when the marginal is below the threshold; mode 1:
// pruned when `keep_count` or more sequences of the tree are more probable (equal marginals:
// the lower node index counts as more probable).  A marginal of zero probability is always
// pruned.  The result is written as a 0/1 "rank" for prune_compact_kernel with k = 1.
__global__ __launch_bounds__(PROPD_MAX_TREE) void prob_decide_kernel(
    int T_max, int mode, float log_threshold, int keep_count, const int32_t *__restrict__ n_nodes,
    const uint64_t *__restrict__ anc, const float *__restrict__ logq, int32_t *__restrict__ rank,
    float *__restrict__ log_marginal) {
  const int b = blockIdx.x, i = threadIdx.x;
  int T = n_nodes[b];
  T = T < 1 ? 1 : (T > T_max ? T_max : T);
  const size_t base = (size_t)b * T_max;
  const bool valid = i < T;
  __shared__ float s_q[PROPD_MAX_TREE], s_lm[PROPD_MAX_TREE];
  s_q[i] = (valid && i > 0) ? logq[base + i] : 0.f;
  __syncthreads();
  float lm = 0.f;
  if (valid && i > 0) {
    uint64_t lo = anc[(base + i) * 2] & ~1ull, hi = anc[(base + i) * 2 + 1];
    while (lo) {
      lm += s_q[__ffsll((long long)lo) - 1];
      lo &= lo - 1;
    }
    while (hi) {
      lm += s_q[64 + __ffsll((long long)hi) - 1];
      hi &= hi - 1;
    }
  }
  s_lm[i] = valid ? lm : -INFINITY;
  __syncthreads();
  bool fail = false;
  if (valid && i > 0) {
    if (mode == 0) {
      fail = !(lm >= log_threshold);
    } else {
      int ahead = 0;
      for (int j = 0; j < T; ++j) ahead += (s_lm[j] > lm) || (s_lm[j] == lm && j < i);
      fail = ahead >= keep_count;
    }
    fail = fail || !(lm > -INFINITY);
  }
  if (i < T_max) {
    rank[base + i] = valid ? (fail ? 1 : 0) : -1;
    if (log_marginal) log_marginal[base + i] = valid ? lm : 0.f;
  }
}

// ------------------------------------------------------------------------------------
// branch elimination, compaction, mask subsampling
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(PROPD_MAX_TREE) void prune_compact_kernel(
    int T_max, int top_k, const int32_t *__restrict__ n_nodes, const int32_t *__restrict__ parent,
    const int32_t *__restrict__ token, const int32_t *__restrict__ depth,
    const uint64_t *__restrict__ anc, const int32_t *__restrict__ rank,
    uint64_t *__restrict__ keep_bits, int32_t *__restrict__ new_index,
    int32_t *__restrict__ orig_index, int32_t *__restrict__ n_kept,
    int32_t *__restrict__ out_n_nodes, int32_t *__restrict__ out_parent,
    int32_t *__restrict__ out_token, int32_t *__restrict__ out_depth,
    uint64_t *__restrict__ out_anc, int32_t *__restrict__ rank_out) {
  const int b = blockIdx.x, i = threadIdx.x;
  int T = n_nodes[b];
  T = T < 1 ? 1 : (T > T_max ? T_max : T);
  const size_t base = (size_t)b * T_max;
  const bool valid = i < T;
  __shared__ uint64_t s_fail[2], s_keep[2];

  int my_rank = -1;
  uint64_t a_lo = 0, a_hi = 0;
  if (valid) {
    my_rank = rank[base + i];
    a_lo = anc[(base + i) * 2];
    a_hi = anc[(base + i) * 2 + 1];
  }
  if (rank_out && i < T_max) rank_out[base + i] = my_rank;
  const bool fail = valid && i > 0 && my_rank >= top_k;
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
    out_token[base + ni] = token[base + i];
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

__global__ void fill_rank_kernel(int n, int T_max, const int32_t *__restrict__ n_nodes,
                                 int32_t *__restrict__ rank) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n) return;
  const int b = idx / T_max, i = idx - b * T_max;
  rank[idx] = i < n_nodes[b] ? 0 : -1;
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

namespace {
// which criterion decides (Section 4.1, "Pruning Criterion")
struct Criterion {
  int kind;             // 0 top-k, 1 probability threshold, 2 probability rank
  int top_k;            // kind 0
  float log_threshold;  // kind 1
  int keep_count;       // kind 2
  float *log_marginal;  // kinds 1, 2: optional output
};
}  // namespace

static propd_status prune_impl(
    const Criterion &crit, const propd_tree *tree, propd_dtype dt, int32_t hidden, int32_t vocab,
    const void *hidden_states, const void *head_weight, uint64_t *keep_bits, int32_t *new_index,
    int32_t *orig_index, int32_t *n_kept, int32_t *cu_nodes, const propd_tree_out *tree_out,
    int32_t *rank_out, int32_t n_payloads, const propd_payload *payloads, void *workspace,
    size_t workspace_bytes, void *hip_stream) {
  using namespace propd;
  const int top_k = crit.kind == 0 ? crit.top_k : 1;  // the 0/1 flags of the other kinds pass below 1
  if (!tree || tree->B < 1 || tree->T_max < 1 || tree->T_max > PROPD_MAX_TREE || hidden < 1 ||
      vocab < 1 || top_k < 1)
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
  const int B = tree->B, T_max = tree->T_max;
  if ((long long)B * T_max > (1ll << 27)) return PROPD_ERR_UNSUPPORTED;
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

  if (crit.kind == 0 && top_k >= vocab) {
    // every id is inside the list: nothing can fail, no scores are needed
    const int n = B * T_max;
    hipLaunchKernelGGL(fill_rank_kernel, dim3((n + 255) / 256), dim3(256), 0, st, n, T_max,
                       tree->n_nodes, ws.rank);
  } else {
    hipLaunchKernelGGL(parent_rows_kernel, dim3(B), dim3(PROPD_MAX_TREE), 0, st, T_max,
                       tree->n_nodes, tree->parent, ws.n_par, ws.local_list, ws.rank);
    hipLaunchKernelGGL(row_table_kernel, dim3((unsigned)((B * T_max + kScanThreads - 1) / kScanThreads)),
                       dim3(kScanThreads), 0, st, B, T_max, ws.n_par,
                       ws.local_list, ws.row_base, ws.row_src);
    if (dt == PROPD_BF16) {
      constexpr int BM = kGemmBM, BN = 64 * kGemmMinFN;  // the grid covers the narrowest tiles
      static bool attr_set = false;
      if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&early_head_bf16_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kGemmLdsBytes) != hipSuccess)
          return PROPD_ERR_DEVICE;
        attr_set = true;
      }
      const long long m_tiles_cap = (ws.row_cap + BM - 1) / BM;
      const long long n_groups = ((vocab + BN - 1) / BN + kXcds - 1) / kXcds;
      const long long grid = kXcds * n_groups * m_tiles_cap;
      if (grid > (1ll << 31) - 1) return PROPD_ERR_UNSUPPORTED;
      hipLaunchKernelGGL(early_head_bf16_kernel, dim3((unsigned)grid), dim3(kGemmThreads),
                         kGemmLdsBytes, st, hidden, vocab, B, prune_compute_units(),
                         reinterpret_cast<const uint16_t *>(hidden_states),
                         reinterpret_cast<const uint16_t *>(head_weight), ws.row_src, ws.row_base,
                         ws.scores, ws.score_pitch);
    } else {
      dim3 grid((unsigned)ws.row_cap, (unsigned)((vocab + 255) / 256));
      hipLaunchKernelGGL(early_head_f32_kernel, grid, dim3(256), 0, st, hidden, vocab, B,
                         reinterpret_cast<const float *>(hidden_states),
                         reinterpret_cast<const float *>(head_weight), ws.row_src, ws.row_base,
                         ws.scores, ws.score_pitch);
    }
    if (crit.kind == 0) {
      hipLaunchKernelGGL(rank_count_kernel, dim3((unsigned)(ws.row_cap * kRankSplit)), dim3(kRankThreads), 0, st, B,
                         T_max, vocab, tree->n_nodes, tree->parent, tree->token, ws.row_src,
                         ws.row_base, ws.scores, ws.score_pitch, ws.rank);
    } else {
      hipLaunchKernelGGL(child_logprob_kernel, dim3((unsigned)ws.row_cap), dim3(kLseThreads), 0, st, B,
                         T_max, vocab, tree->n_nodes, tree->parent, tree->token, ws.row_src,
                         ws.row_base, ws.scores, ws.score_pitch, ws.logq);
      hipLaunchKernelGGL(prob_decide_kernel, dim3(B), dim3(PROPD_MAX_TREE), 0, st, T_max,
                         crit.kind == 1 ? 0 : 1, crit.log_threshold, crit.keep_count, tree->n_nodes,
                         tree->anc, ws.logq, ws.rank, crit.log_marginal);
    }
  }
  if (!launch_ok()) return PROPD_ERR_DEVICE;
  hipLaunchKernelGGL(prune_compact_kernel, dim3(B), dim3(PROPD_MAX_TREE), 0, st, T_max, top_k,
                     tree->n_nodes, tree->parent, tree->token, tree->depth, tree->anc, ws.rank,
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
  const Criterion crit = {0, top_k, 0.f, 0, nullptr};
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
  Criterion crit = {1, 1, 0.f, 0, log_marginal};
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
