// Tree-masked attention over the cached prefix plus each node's own root path
// (Section 2, "Verification"; Figure 2(b,c)).
//
// bf16 path (d = 128).  The work is a stream of K/V rows from HBM that all T
// tree queries of a (sequence, head) pair share, so the kernel is organised
// around reading every K and V row exactly once, as fast as HBM delivers them:
//   - the work of a call is the list of 32-row K/V stages of all (sequence, head)
//     units in order (cached rows, then tree rows); a persistent grid of two
//     workgroups per compute unit cuts that list into equal contiguous ranges, so
//     ragged sequence lengths balance by construction;
//   - a workgroup streams its range through a ring of LDS stages with direct
//     global->LDS loads (no registers, no LDS store instructions), issued NS-1
//     stages ahead of the math and running straight across unit boundaries; rows
//     are unpadded in LDS and their 16-byte chunks are XOR-swizzled by the load
//     addresses so that both MFMA operand read patterns are bank-conflict free;
//   - scores are computed transposed, S^T = K . Q^T, with the 32x32x16 bf16 MFMA,
//     so that a lane owns one query column: the running max / sum of the online
//     softmax are per-lane scalars, and the fp32 score registers, once
//     exponentiated and rounded to bf16, ARE the B operand of the second MFMA
//     O^T += V^T . P^T, with no shuffle or LDS round trip; V^T is read from
//     row-major V in LDS with the transposing LDS read;
//   - the cached prefix needs no mask; tree stages keep a score only where the
//     node's 128-bit ancestor set has the bit;
//   - the four waves of a workgroup split the query columns (32 each); a wave whose
//     columns lie beyond the tree only helps with the loads;
//   - a unit cut by a range boundary leaves fp32 partials (O, max, sum), at most
//     two per workgroup, and the workgroup holding its first piece leaves a record of the
//     cut; a second kernel merges the pieces of every recorded cut, in their order.
// fp32 path: a plain one-wave-per-query kernel, fp32 throughout.
#include <type_traits>

#include "common.h"

namespace propd {

constexpr int kD = 128;
constexpr int kAttnThreads = 256;
constexpr int kMaxGrid = 1024;                 // workgroups of the persistent kernel, at most
constexpr int kStageRows = 32;                 // K/V rows per ring stage
constexpr int kRowBytes = kD * 2;              // one bf16 row
constexpr int kHalfStage = kStageRows * kRowBytes;  // K part of a stage; the V part follows
constexpr int kStageBytes = 2 * kHalfStage;
constexpr int kRingStages = 5;  // 16 KB each; two workgroups per CU share 160 KB

struct AttnParams {
  const uint16_t *q, *k_cache, *v_cache, *k_tree, *v_tree;
  uint16_t *out;
  const int32_t *seq_lens, *n_nodes;
  const uint64_t *anc;
  int B, H, T_max, L_max;
  float scale_log2e;
  float *part_o;   // [2 * grid][4 waves][16 blocks][64 lanes][4]
  float *part_ml;  // [2 * grid][4 waves][m | l][64 lanes]
  int32_t *cuts;   // [grid][4] per workgroup: the unit whose first piece it holds (CutRecord)
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two floats -> packed bf16 pair (round to nearest even), one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  const f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// Transposing LDS read (ds_read_b64_tr_b16), issued as assembly so that the compiler does
// not fence it against the ring's direct loads in flight (the builtin counts as a possible
// LDS write, which would drain them).  The result is valid only after wait_lds<>().
template <int OFFSET>
__device__ __forceinline__ u32x2 lds_read_tr16(uint32_t addr) {
  u32x2 r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET));
  return r;
}

// wait until at most N LDS operations of this wave are outstanding; the registers named
// are the results being waited for, so that their uses cannot be scheduled above the wait
template <int N>
__device__ __forceinline__ void wait_lds(u32x2 (&a)[8]) {
  asm volatile("s_waitcnt lgkmcnt(%8)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]),
                 "+v"(a[7])
               : "n"(N));
}

// wait until at most N of this wave's vector memory operations are outstanding
template <int N>
__device__ __forceinline__ void wait_vmem() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Global loads and stores issued as assembly.  The main kernel waits for its vector memory
// operations itself, with explicit counts; the compiler's own bookkeeping would fence the
// ring's loads in flight at every use of a loaded register.  The compiler's hazard
// recognizer does not look inside assembly either: the stores carry their own wait states
// for data registers written just before by vector or cross-lane instructions, and after
// themselves, because a store wider than 8 bytes still reads its data registers when the
// next instruction issues.
__device__ __forceinline__ u32x4 global_load16_untracked(const void *ptr) {
  u32x4 r;
  asm volatile("s_nop 3\n\tglobal_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(ptr) : "memory");
  return r;
}
__device__ __forceinline__ void global_store16_untracked(void *ptr, u32x4 v) {
  asm volatile("s_nop 7\n\tglobal_store_dwordx4 %0, %1, off sc1\n\ts_nop 3" ::"v"(ptr), "v"(v) : "memory");
}
__device__ __forceinline__ void global_store4_untracked(void *ptr, float v) {
  asm volatile("s_nop 7\n\tglobal_store_dword %0, %1, off sc1\n\ts_nop 3" ::"v"(ptr), "v"(v) : "memory");
}

// Exchange between the two 32-lane halves of a wave (v_permlane32_swap): afterwards lane
// l < 32 holds (a[l], a[l+32]) and lane l >= 32 holds (b[l-32], b[l]) in (a, b).
__device__ __forceinline__ void swap_halves(uint32_t &a, uint32_t &b) {
  const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  a = r[0];
  b = r[1];
}

// A lane of the main kernel holds, for its query t = 32*wave + lane%32, the 64 values
// d = 32*mb + 8*q4 + 4*(lane/32) + j of O^T in o_acc[mb][4*q4 + j].
// Output rows: neighbouring q4 of the two lane halves are exchanged so that every lane
// writes 8 consecutive bf16 values (16 bytes) per store.
template <bool kUntracked>
__device__ __forceinline__ void store_out_block(uint16_t *orow, const f32x16 &o, float inv, int g, int mb) {
#pragma unroll
  for (int jp = 0; jp < 2; ++jp) {
    const int e = 8 * jp, od = 8 * jp + 4;  // first register of the even / odd q4 of the pair
    uint32_t a0 = cvt_pk_bf16(o[e] * inv, o[e + 1] * inv);
    uint32_t a1 = cvt_pk_bf16(o[e + 2] * inv, o[e + 3] * inv);
    uint32_t b0 = cvt_pk_bf16(o[od] * inv, o[od + 1] * inv);
    uint32_t b1 = cvt_pk_bf16(o[od + 2] * inv, o[od + 3] * inv);
    swap_halves(a0, b0);
    swap_halves(a1, b1);
    // lower half: d = 32*mb + 16*jp + 0..7, upper half: the 8 values after those
    const u32x4 w4 = {a0, a1, b0, b1};
    if (kUntracked) global_store16_untracked(orow + mb * 32 + 16 * jp + 8 * g, w4);
    else *reinterpret_cast<u32x4 *>(orow + mb * 32 + 16 * jp + 8 * g) = w4;
  }
}

template <bool kUntracked>
__device__ __forceinline__ void store_out_row(uint16_t *orow, const f32x16 (&o)[4], float inv, int g) {
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) store_out_block<kUntracked>(orow, o[mb], inv, g, mb);
}

// Partial results keep the register layout, so that a wave writes and reads them as
// contiguous 1 KB blocks: part_o[slot][wave][4*mb + q4][lane][j], part_ml[slot][wave][m|l][lane].
constexpr size_t kPartOFloats = 4 * 16 * 64 * 4;  // floats of part_o per slot
constexpr size_t kPartMlFloats = 4 * 2 * 64;     // floats of part_ml per slot
__device__ __forceinline__ size_t part_o_index(size_t slot, int wave, int blk, int lane) {
  return (((slot * 4 + wave) * 16 + blk) * 64 + lane) * 4;
}
__device__ __forceinline__ size_t part_ml_index(size_t slot, int wave, int which, int lane) {
  return ((slot * 4 + wave) * 2 + which) * 64 + lane;
}

// Work decomposition shared by the main kernel and the merge kernel.  The work of one
// call is made of K/V stages; a (sequence, head) unit is its cached stages followed by its
// tree stages.  Workgroup w of G does, in this order,
//   - k whole units w, w+G, ..., when all sequences have the same lengths (k = units / G):
//     no partial results, and all workgroups write their outputs at the same moments, which
//     the memory system takes far better than a trickle of stores into the read stream;
//   - the contiguous range [w*N/G, (w+1)*N/G) of the list of the N stages of the remaining
//     units (all units when lengths differ, so that every workgroup streams the same number
//     of rows whatever the mix); a unit cut by a range boundary is finished by the merge
//     kernel from per-workgroup partial results.
// A wave-uniform 32-bit load on the scalar path.  Issued as assembly: the compiler would
// use a vector load here and wait for it with vmcnt(0), which drains the ring.  The
// scalar cache is invalidated when a kernel starts, like the vector caches, so values
// that an earlier kernel or the caller rewrote in place are seen.
__device__ __forceinline__ int32_t uniform_load_i32(const int32_t *ptr) {
  const uint64_t a = (uint64_t)(uintptr_t)ptr;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  const uint64_t sa = ((uint64_t)hi << 32) | lo;  // in scalar registers
  int32_t v;
  asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(sa) : "memory");
  return v;
}

struct StageMap {
  int B, H;
  const int32_t *seq_lens, *n_nodes;
  int L_max, T_max;
  __device__ __forceinline__ int len(int b) const {
    const int L = uniform_load_i32(seq_lens + b);
    return L < 0 ? 0 : (L > L_max ? L_max : L);
  }
  __device__ __forceinline__ int nodes(int b) const {
    const int T = uniform_load_i32(n_nodes + b);
    return T < 1 ? 1 : (T > T_max ? T_max : T);
  }
  __device__ __forceinline__ int cache_stages(int b) const {
    return (len(b) + kStageRows - 1) / kStageRows;
  }
  __device__ __forceinline__ int tree_stages(int b) const {
    return (nodes(b) + kStageRows - 1) / kStageRows;
  }
  __device__ __forceinline__ int unit_stages(int b) const { return cache_stages(b) + tree_stages(b); }
  // the same for a sequence index that differs between lanes (plain loads); 0 past the batch
  __device__ __forceinline__ int unit_stages_lane(int b) const {
    if (b >= B) return 0;
    int L = seq_lens[b], T = n_nodes[b];
    L = L < 0 ? 0 : (L > L_max ? L_max : L);
    T = T < 1 ? 1 : (T > T_max ? T_max : T);
    return (L + kStageRows - 1) / kStageRows + (T + kStageRows - 1) / kStageRows;
  }
  // Sequence that holds stage x of the list of all units, and the stages before that
  // sequence; the last sequence if x lies past the end.  Every lane of the wave takes part:
  // 64 sequences are sized per pass, with a wave prefix sum.
  __device__ void locate(long long x, int &b_out, long long &b_start_out) const {
    const int lane = threadIdx.x & 63;
    long long base = 0;
    int b_found = B - 1;
    long long start_found = 0;
    bool found = false;
    for (int b0 = 0; b0 < B && !found; b0 += 64) {
      const long long mine = (long long)H * unit_stages_lane(b0 + lane);
      long long incl = mine;  // inclusive prefix over the lanes
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const long long up = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += up;
      }
      const long long excl = base + incl - mine;
      // the holder is the last sequence that starts at or before x
      const uint64_t le = __ballot(b0 + lane < B && excl <= x);
      const int n_le = __popcll(le);
      const long long total = __shfl(incl, 63, kWave);
      if (x < base + total || b0 + 64 >= B) {
        const int src = n_le > 0 ? n_le - 1 : 0;
        b_found = b0 + src;
        start_found = __shfl(excl, src, kWave);
        found = true;
      }
      base += total;
    }
    b_out = __builtin_amdgcn_readfirstlane(b_found);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)start_found);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)start_found >> 32));
    b_start_out = (long long)(((uint64_t)hi << 32) | lo);
  }
  // stages of all units before unit (b, h) in the list of all units
  __device__ long long stages_before(int b, int h) const {
    const int lane = threadIdx.x & 63;
    long long n = 0;
    for (int b0 = 0; b0 < b; b0 += 64)
      n += wave_reduce_sum(b0 + lane < b ? (long long)H * unit_stages_lane(b0 + lane) : 0ll);
    n += (long long)h * unit_stages(b);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)n);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)n >> 32));
    return (long long)(((uint64_t)hi << 32) | lo);
  }
};


struct Schedule {
  int k;                  // whole units per workgroup, done first
  long long first_split;  // first unit of the split list (= k * G)
  long long split_base;   // stages of the units before it
  long long n_split;      // stages of the split list
  // The split list is cut into G contiguous ranges: the first `rem` workgroups take
  // `quot` + 1 stages, the others `quot` (one division per kernel, none per range).
  long long quot, rem;
  __device__ __forceinline__ long long range_start(long long w) const {
    return w * quot + (w < rem ? w : rem);
  }
  // workgroup whose range holds stage x of the split list
  __device__ __forceinline__ long long range_owner(long long x) const {
    const long long big = rem * (quot + 1);  // stages held by the larger ranges
    if (n_split < (1ll << 31)) {             // the usual case: 32-bit divisions
      const uint32_t xx = (uint32_t)x, bb = (uint32_t)big, qq = (uint32_t)quot;
      return xx < bb ? xx / (qq + 1u) : (uint32_t)rem + (xx - bb) / qq;
    }
    return x < big ? x / (quot + 1) : rem + (x - big) / quot;
  }
};

// What the workgroup that holds the FIRST piece of a cut unit leaves for the merge kernel
// (every workgroup of the grid writes its record in every call; unit < 0: none).  The pieces
// of the unit lie in workgroups w .. w_last: the first in the second partial slot of w, the
// others in the first slot of theirs.
struct CutRecord {
  int32_t unit;
  int32_t w_last_and_nodes;  // w_last | (tree nodes of the unit's sequence << 16)
  int32_t pad[2];
};

__device__ __forceinline__ Schedule make_schedule(const StageMap &m, long long G) {
  Schedule sc;
  const int lane = threadIdx.x & 63;
  int us_min = 1 << 30, us_max = 0;
  long long n_all = 0;
  for (int b0 = 0; b0 < m.B; b0 += 64) {  // 64 sequences per pass, one per lane
    const bool in = b0 + lane < m.B;
    const int us = m.unit_stages_lane(b0 + lane);
    us_min = min(us_min, -wave_reduce_max(in ? -us : -(1 << 30)));
    us_max = max(us_max, wave_reduce_max(in ? us : 0));
    n_all += wave_reduce_sum((long long)m.H * us);
  }
  us_min = __builtin_amdgcn_readfirstlane(us_min);
  us_max = __builtin_amdgcn_readfirstlane(us_max);
  {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)n_all);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)n_all >> 32));
    n_all = (long long)(((uint64_t)hi << 32) | lo);
  }
  // whole units first only where they are (nearly) equally long: a workgroup's k of them
  // then differ by at most a few percent between workgroups
  const long long U = (long long)m.B * m.H;
  sc.k = (us_max - us_min) * 32 <= us_max ? (int)(U / G) : 0;
  sc.first_split = (long long)sc.k * G;
  sc.split_base = sc.k > 0 ? m.stages_before((int)(sc.first_split / m.H), (int)(sc.first_split % m.H)) : 0;
  sc.n_split = n_all - sc.split_base;
  sc.quot = sc.n_split / G;
  sc.rem = sc.n_split - sc.quot * G;
  return sc;
}

// Position of a workgroup in its own sequence of stages: stage s of unit (b, h).
struct Walk {
  long long unit;  // b * H + h
  int b, s;
  int L, T, cs, ts;         // cached rows, tree nodes, cached stages, tree stages of sequence b
  int whole_left;           // whole units still to do, this one included; 0 = in the split range
  long long split_unit;     // where this workgroup's split range starts
  int split_s;
  long long x_end;          // end of this workgroup's range in the split list
  __device__ __forceinline__ void load_sizes(const StageMap &m) {
    L = m.len(b);
    T = m.nodes(b);
    cs = (L + kStageRows - 1) / kStageRows;
    ts = (T + kStageRows - 1) / kStageRows;
  }
  __device__ __forceinline__ void set_unit(const StageMap &m, long long u) {
    unit = u;
    const int nb = (int)(u / m.H);
    if (nb != b) {
      b = nb;
      load_sizes(m);
    }
  }
  // the workgroup's first stage; returns the number of stages it will do
  __device__ int start(const StageMap &m, const Schedule &sc, long long w, long long G) {
    const long long U = (long long)m.B * m.H;
    const long long x0 = sc.range_start(w);
    int n_my = (int)(sc.range_start(w + 1) - x0);
    x_end = x0 + n_my;
    // locate stage split_base + x0 of the list of all units
    const long long x = sc.split_base + x0;
    long long b_start;
    m.locate(x, b, b_start);
    load_sizes(m);
    {
      const int us = cs + ts;
      const long long hh = (x - b_start) / us;
      split_unit = (long long)b * m.H + hh;
      split_s = (int)((x - b_start) - hh * us);
    }
    if (split_unit >= U) {  // an empty range at the very end: stay on valid memory
      split_unit = U - 1;
      split_s = 0;
    }
    whole_left = sc.k;
    if (sc.k > 0) {
      for (int j = 0; j < sc.k; ++j) n_my += m.unit_stages((int)((w + j * G) / m.H));
      b = -1;
      set_unit(m, w);
      s = 0;
    } else {
      b = -1;
      set_unit(m, split_unit);
      s = split_s;
    }
    return n_my;
  }
  __device__ __forceinline__ void advance(const StageMap &m, long long G, int n) {
    s += n;  // n <= stages left in the unit
    if (s < cs + ts) return;
    s = 0;
    if (whole_left > 0) {
      if (--whole_left > 0) {
        set_unit(m, unit + G);
      } else {
        set_unit(m, split_unit);
        s = split_s;
      }
    } else if (unit + 1 < (long long)m.B * m.H) {
      set_unit(m, unit + 1);
    }
  }
};

template <int NS>
__global__ __launch_bounds__(kAttnThreads, 2) void tree_attn_bf16_kernel(AttnParams p) {
  static_assert(NS >= 4, "three stages are in use by the math, the rest is in flight");
  constexpr int kAhead = NS - 3;  // stages in flight beyond the newest one the math uses
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void *)smem;  // LDS byte address of the ring

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  const int t = wave * 32 + l32;  // this lane's query column

  const StageMap map = {p.B, p.H, p.seq_lens, p.n_nodes, p.L_max, p.T_max};
  const long long G = gridDim.x, w = blockIdx.x;
  const Schedule sch = make_schedule(map, G);
  Walk cp;
  const int n_my = cp.start(map, sch, w, G);
  CutRecord cut = {-1, 0, {0, 0}};
  auto leave_record = [&]() {
    if (tid == 0) *reinterpret_cast<CutRecord *>(p.cuts + 4 * w) = cut;
  };
  if (n_my <= 0) {
    leave_record();
    return;
  }

  // ---- loader.  It walks the same stage list ahead of the math, one segment (the cached
  //      rows or the tree rows of a unit) at a time.  One direct load moves 64 lanes x 16
  //      bytes = 4 rows into 1 KB of LDS that is contiguous in lane order, so the swizzle is
  //      applied on the global side: the lane that fills chunk c of LDS row r fetches chunk
  //      c ^ key(r) of the global row.  Keys: K rows r & 15 (a 16-byte read of one chunk
  //      column over 16 rows touches 16 distinct chunks); V rows ((r & 3) << 2) | ((r >> 2) & 3)
  //      (the 4 rows x 64 bytes of one transposing read land in 4 distinct 64-byte bank
  //      groups).  A wave fills rows 4*wave + lane/16 of each 16-row half, so its keys do not
  //      depend on the half.  Rows past the last valid one of a segment re-read that last
  //      row: finite data that the mask discards (K) or that meets a zero weight (V);
  //      padding is never touched.
  const int ld_row = 4 * wave + (lane >> 4);
  const int k_lane_chunk = ((lane & 15) ^ ld_row) << 4;
  const int v_lane_chunk = ((lane & 15) ^ (((lane >> 4) << 2) | wave)) << 4;
  Walk lw = cp;  // the next stage to issue
  int ld_rows;                       // rows left in the segment, from the next stage to issue
  const unsigned char *ld_k, *ld_v;  // first row of the next stage to issue
  auto ld_segment = [&]() {          // the segment (cached or tree rows) that stage lw.s starts
    const bool tree = lw.s >= lw.cs;
    const int first_row = (tree ? lw.s - lw.cs : lw.s) * kStageRows;
    ld_rows = (tree ? lw.T : lw.L) - first_row;
    const size_t row0 = (size_t)lw.unit * (tree ? p.T_max : p.L_max) + first_row;
    ld_k = reinterpret_cast<const unsigned char *>(tree ? p.k_tree : p.k_cache) + row0 * kRowBytes;
    ld_v = reinterpret_cast<const unsigned char *>(tree ? p.v_tree : p.v_cache) + row0 * kRowBytes;
  };
  ld_segment();
  auto dma16 = [&](const unsigned char *src, unsigned char *dst) {
    __builtin_amdgcn_global_load_lds((global_void *)src, (lds_void *)dst, 16, 0, 2 /* nt */);
  };
  auto issue = [&](int slot) {
    unsigned char *dst = smem + slot * kStageBytes + (4 * wave) * kRowBytes;
    if (ld_rows >= kStageRows) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int ro = (16 * i + ld_row) * kRowBytes;
        dma16(ld_k + (ro + k_lane_chunk), dst + i * 16 * kRowBytes);
        dma16(ld_v + (ro + v_lane_chunk), dst + kHalfStage + i * 16 * kRowBytes);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        int row = 16 * i + ld_row;
        row = row < ld_rows ? row : ld_rows - 1;
        dma16(ld_k + (row * kRowBytes + k_lane_chunk), dst + i * 16 * kRowBytes);
        dma16(ld_v + (row * kRowBytes + v_lane_chunk), dst + kHalfStage + i * 16 * kRowBytes);
      }
    }
    lw.advance(map, G, 1);
    if (ld_rows > kStageRows) {
      ld_rows -= kStageRows;
      ld_k += kHalfStage;
      ld_v += kHalfStage;
    } else {
      ld_segment();  // the tree rows of the unit, or another unit
    }
  };

  // ---- per-lane LDS read offsets within a stage
  // K as the A operand of S^T: lane = row l32, 8 consecutive d from 16*ks + 8*g (chunk 2*ks + g)
  uint32_t k_rd[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks)
    k_rd[ks] = smem_base + l32 * kRowBytes + (((2 * ks + g) ^ (l32 & 15)) << 4);
  // V^T as the A operand of O^T: transposing read; in each group of 16 lanes, lane i points at
  // row i/4, 4 columns from 4*(i%4), and receives column i of those 4 rows.  Per MFMA k-step
  // (16 rows): slots 0..3 = rows 4g + 0..3, slots 4..7 = those rows + 8.
  uint32_t v_rd[4][2];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
      const int r = 4 * g + ((lane & 15) >> 2) + 8 * hi;
      const int key = ((r & 3) << 2) | ((r >> 2) & 3);
      const int chunk = mb * 4 + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
      v_rd[mb][hi] = smem_base + kHalfStage + r * kRowBytes + ((chunk ^ key) << 4) + 8 * (lane & 1);
    }

  // ---- ring bookkeeping.  acquire() is called once per stage of the range, in order, by
  //      every wave: it waits for the stage's loads, meets the other waves, and refills the
  //      slot whose stage every wave finished two acquires ago.  Vector memory loads of a
  //      wave complete in issue order, so "stage x has landed" is "at most 4 operations
  //      outstanding": the loads of stage x+1.  Query loads and output stores that the wave
  //      issued since then are waited for as well (loads and stores are not ordered against
  //      each other, so the stores cannot be counted off).
  static_assert(kAhead == 2, "the wait below allows exactly one younger stage in flight");
  int n_acq = 0;              // stages acquired so far
  int slot_acq = 0;           // slot of the next stage to acquire
  int slot_ld = 0;            // slot of the next stage to issue
  auto next_slot = [](int sl) { return sl + 1 == NS ? 0 : sl + 1; };
#pragma unroll
  for (int i = 0; i < kAhead; ++i)
    if (i < n_my) {
      issue(slot_ld);
      slot_ld = next_slot(slot_ld);
    }
  auto acquire = [&]() -> int {
    if (n_acq + 1 < n_my) wait_vmem<4>(); else wait_vmem<0>();
    __builtin_amdgcn_s_barrier();
    if (n_acq + kAhead < n_my) {
      issue(slot_ld);
      slot_ld = next_slot(slot_ld);
    }
    const int sl = slot_acq;
    slot_acq = next_slot(slot_acq);
    ++n_acq;
    return sl;
  };

  // ---- a piece: the part of one unit that lies in this range
  struct Piece {
    int L, T, n_cache, s0, n_st, unit, b, n_cmp;
    bool whole;
  };
  auto piece_at = [&](const Walk &c, int n_done) {
    Piece pc;
    pc.L = c.L;
    pc.T = c.T;
    pc.n_cache = c.cs;
    pc.s0 = c.s;
    const int us = c.cs + c.ts;
    pc.n_st = us - c.s < n_my - n_done ? us - c.s : n_my - n_done;
    pc.whole = c.s == 0 && pc.n_st == us;
    pc.unit = (int)c.unit;
    pc.b = c.b;
    // Stages this wave has math for: none if its 32 query columns lie beyond the tree; tree
    // rows after its last query are descendants or strangers of all its queries, and those
    // stages are the last of the unit.
    pc.n_cmp = 0;
    if (wave * 32 < c.T) {
      pc.n_cmp = c.cs + wave + 1 - c.s;
      pc.n_cmp = pc.n_cmp > pc.n_st ? pc.n_st : (pc.n_cmp < 0 ? 0 : pc.n_cmp);
    }
    return pc;
  };

  // Q^T fragments (B operand: lane = query column, 8 consecutive d per K step) and the
  // ancestor set of this lane's node.  Lanes past the tree take node 0: valid memory, and
  // their columns are never stored.
  u32x4 qf[8], ancv;
  auto load_queries = [&](const Piece &pc) {
    const int tq = t < pc.T ? t : 0;
    const uint16_t *qrow = p.q + ((size_t)pc.unit * p.T_max + tq) * kD + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = global_load16_untracked(qrow + ks * 16);
    ancv = global_load16_untracked(p.anc + ((size_t)pc.b * p.T_max + tq) * 2);
  };
  auto wait_queries = [&]() {
    // the registers are named so that their uses cannot be scheduled above the wait
    auto tie = [&]() {
      asm volatile("" : "+v"(qf[0]), "+v"(qf[1]), "+v"(qf[2]), "+v"(qf[3]), "+v"(qf[4]), "+v"(qf[5]),
                        "+v"(qf[6]), "+v"(qf[7]), "+v"(ancv));
    };
    tie();
    wait_vmem<0>();
    tie();
  };

  float m_run, l_run;
  f32x16 o_acc[4];
  u32x2 vt[2][8];
  // S^T = K . Q^T of one stage
  auto scores = [&](int sl) -> f32x16 {
    const uint32_t so = (uint32_t)sl * kStageBytes;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 a = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8 *>(
          (uintptr_t)(k_rd[ks] + so));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, qf[ks]), acc, 0, 0, 0);
    }
    return acc;
  };
  // start the transposing reads of a whole V stage: vt[ks2][2*mb + hi]
  auto read_v = [&](int sl) {
    const uint32_t so = (uint32_t)sl * kStageBytes;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      vt[0][2 * mb] = lds_read_tr16<0>(v_rd[mb][0] + so);
      vt[0][2 * mb + 1] = lds_read_tr16<0>(v_rd[mb][1] + so);
    }
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      vt[1][2 * mb] = lds_read_tr16<16 * kRowBytes>(v_rd[mb][0] + so);
      vt[1][2 * mb + 1] = lds_read_tr16<16 * kRowBytes>(v_rd[mb][1] + so);
    }
  };
  // O^T += V^T . P^T with the V registers read last and the given weights
  auto weighted_sum = [&](const uint32_t (&pw)[8]) {
    wait_lds<0>(vt[0]);
    wait_lds<0>(vt[1]);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      const u32x4 pv = {pw[4 * ks2], pw[4 * ks2 + 1], pw[4 * ks2 + 2], pw[4 * ks2 + 3]};
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pv);
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        const u32x4 aw = {vt[ks2][2 * mb].x, vt[ks2][2 * mb].y, vt[ks2][2 * mb + 1].x,
                          vt[ks2][2 * mb + 1].y};
        o_acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw), pf,
                                                            o_acc[mb], 0, 0, 0);
      }
    }
  };

  const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
  // a new running maximum is adopted only when it exceeds the reference by 2^8 in the
  // exponent; below that the weights simply exceed 1, by a factor fp32 sums and bf16 hold
  const float tau = 8.f / p.scale_log2e;

  Piece pc = piece_at(cp, 0);
  if (pc.n_cmp > 0) load_queries(pc);
  while (n_acq < n_my) {
    const int L = pc.L, T = pc.T, n_cache = pc.n_cache, s0 = pc.s0;
    m_run = -INFINITY;
    l_run = 0.f;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[mb][r] = 0.f;

    if (pc.n_cmp > 0) {
      // The loop is software-pipelined over stages so that matrix and vector work of
      // different stages sit in one basic block: iteration i computes the scores of stage
      // i+1 (MFMA), the softmax weights of stage i (VALU), and adds stage i-1 to O (MFMA).
      int sl_cur = acquire();
      wait_queries();
      const uint64_t anc_lo = ((uint64_t)ancv.y << 32) | ancv.x, anc_hi = ((uint64_t)ancv.w << 32) | ancv.z;
      f32x16 sc = scores(sl_cur);
      uint32_t pw_prev[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) pw_prev[r] = 0u;

      auto stage = [&](int i, auto has_next, auto has_prev) {
        constexpr bool kNext = decltype(has_next)::value, kPrev = decltype(has_prev)::value;
        int sl_next = 0;
        if (kNext) sl_next = acquire();
        mfma_settle();  // sc was written by MFMAs of the previous iteration or the prologue

        const int s = s0 + i;
        const bool is_tree = s >= n_cache;
        const int j0 = (is_tree ? s - n_cache : s) * kStageRows;
        int n_valid = (is_tree ? T : L) - j0;
        n_valid = n_valid > kStageRows ? kStageRows : n_valid;
        // ---- mask (the softmax scale is positive, so it commutes with max and is applied
        //      inside the exponent).  Register r of a 32x32 accumulator holds row
        //      8*(r/4) + 4*g + r%4 of the block, i.e. K/V row j0 + that.
        if (is_tree || n_valid < kStageRows) {  // uniform over the workgroup
          // visibility of the stage's rows to this lane's query: cached rows below L for
          // every query, tree rows only where the node's ancestor set has the bit
          uint32_t vis = n_valid >= 32 ? ~0u : ((1u << n_valid) - 1u);
          const uint64_t word = j0 >= 64 ? anc_hi : anc_lo;  // tree stages start at 0, 32, 64, 96
          vis &= is_tree ? (uint32_t)(word >> (j0 & 32)) : ~0u;
          vis >>= 4 * g;
#pragma unroll
          for (int r = 0; r < 16; ++r)
            sc[r] = ((vis >> (8 * (r >> 2) + (r & 3))) & 1u) ? sc[r] : -INFINITY;
        }
        // ---- running maximum
        float m_blk = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) m_blk = fmaxf(m_blk, sc[r]);
        {  // the other half of the stage's rows is in the lane 32 away
          uint32_t lo = __float_as_uint(m_blk), hi = lo;
          swap_halves(lo, hi);
          m_blk = fmaxf(__uint_as_float(lo), __uint_as_float(hi));
        }
        if (__builtin_amdgcn_ballot_w64(m_blk > m_run + tau) != 0) {
          // rare: move the reference.  O must first receive the stage still pending, whose
          // weights are relative to the old reference.
          if (kPrev) {
            weighted_sum(pw_prev);
#pragma unroll
            for (int r = 0; r < 8; ++r) pw_prev[r] = 0u;
            mfma_settle();
          }
          const float m_new = fmaxf(m_run, m_blk);
          const float m_safe = m_new == -INFINITY ? 0.f : m_new;
          const float alpha = fast_exp2((m_run - m_safe) * p.scale_log2e);
          l_run *= alpha;
#pragma unroll
          for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[mb][r] *= alpha;
          m_run = m_new;
        }
        const float neg_m = -(m_run == -INFINITY ? 0.f : m_run) * p.scale_log2e;

        // ---- one block: scores of the next stage, weights of this one, O update of the last
        f32x16 sc_next;
        if (kNext) sc_next = scores(sl_next);
        uint32_t pw[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0 = fast_exp2(fmaf(sc[r], p.scale_log2e, neg_m));
          const float p1 = fast_exp2(fmaf(sc[r + 1], p.scale_log2e, neg_m));
          pw[r >> 1] = cvt_pk_bf16(p0, p1);
          // the row sums are taken over the rounded bf16 weights, the values the MFMA multiplies
          l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[r >> 1]), ones,
                                                  l_run, false);
        }
        if (kPrev) weighted_sum(pw_prev);
        read_v(sl_cur);  // V of this stage, used by the next iteration or the drain
#pragma unroll
        for (int r = 0; r < 8; ++r) pw_prev[r] = pw[r];
        if (kNext) {
          sc = sc_next;
          sl_cur = sl_next;
        }
      };
      using yes = std::true_type;
      using no = std::false_type;
      if (pc.n_cmp == 1) {
        stage(0, no{}, no{});
      } else {
        stage(0, yes{}, no{});
        for (int i = 1; i < pc.n_cmp - 1; ++i) stage(i, yes{}, yes{});
        stage(pc.n_cmp - 1, no{}, yes{});
      }
      weighted_sum(pw_prev);  // drain
      mfma_settle();
    }
    // stages of the piece without math for this wave: keep the ring and the barriers going
    for (int i = pc.n_cmp; i < pc.n_st; ++i) acquire();

    // ---- the next piece's queries are requested before this piece's results are stored:
    //      waiting for them later then does not wait for the stores
    const Piece done = pc;
    cp.advance(map, G, done.n_st);
    if (n_acq < n_my) {
      pc = piece_at(cp, n_acq);
      if (pc.n_cmp > 0) load_queries(pc);
    }

    // ---- write: lane holds d = mb*32 + 8*(r/4) + 4*g + r%4 for its query t
    l_run += __shfl_xor(l_run, 32, kWave);
    m_run *= p.scale_log2e;  // from here on the maximum is in the exponent's (log2) domain
    if (wave * 32 < T) {
      if (done.whole) {
        if (t < T)
          store_out_row<true>(p.out + ((size_t)done.unit * p.T_max + t) * kD, o_acc, 1.f / l_run, g);
      } else {
        // a range starts inside at most one unit and ends inside at most one
        const size_t ps = 2 * (size_t)w + (s0 > 0 ? 0 : 1);
        if (s0 == 0) {
          // the unit starts here and runs past the end of this range, which is the end of
          // this workgroup's work: its last stage lies us - n_st stages further
          const int us = n_cache + (T + kStageRows - 1) / kStageRows;
          cut.unit = done.unit;
          cut.w_last_and_nodes = (int32_t)sch.range_owner(cp.x_end - 1 + (us - done.n_st)) | (T << 16);
        }
        if (t < T) {
#pragma unroll
          for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const f32x4 w4 = {o_acc[mb][4 * q4], o_acc[mb][4 * q4 + 1], o_acc[mb][4 * q4 + 2],
                                o_acc[mb][4 * q4 + 3]};
              global_store16_untracked(p.part_o + part_o_index(ps, wave, 4 * mb + q4, lane),
                                       __builtin_bit_cast(u32x4, w4));
            }
          global_store4_untracked(p.part_ml + part_ml_index(ps, wave, 0, lane), m_run);
          global_store4_untracked(p.part_ml + part_ml_index(ps, wave, 1, lane), l_run);
        }
      }
    }
  }
  leave_record();
}

// Finish the units that a range boundary cut: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s
// over the pieces s of the unit, always in the order of the pieces.  One wave per (workgroup of
// the main kernel, group of 32 queries, quarter of the head dimension): it reads that
// workgroup's record, returns at once when it names no unit, and otherwise merges the partials
// of workgroups w .. w_last, four pieces at a time with all their loads in flight together.
// Lanes map to (query, d) exactly as in the main kernel; a wave owns one 32-wide block mb of d.
constexpr int kCombinePieces = 4;

__global__ __launch_bounds__(kWave) void tree_attn_combine_kernel(AttnParams p) {
  const int w = blockIdx.x >> 4, dw = (blockIdx.x >> 2) & 3, mb = blockIdx.x & 3;
  const CutRecord cut = *reinterpret_cast<const CutRecord *>(p.cuts + 4 * w);
  if (cut.unit < 0) return;
  const int T = cut.w_last_and_nodes >> 16, w_last = cut.w_last_and_nodes & 0xffff;
  if (dw * 32 >= T) return;
  const int lane = threadIdx.x;
  const int t = dw * 32 + (lane & 31), g = lane >> 5;
  // lanes beyond the tree read lane 0's data (valid memory) and store nothing
  const int ln = t < T ? lane : 0;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  float M = -INFINITY, lsum = 0.f;
  for (int w0 = w; w0 <= w_last; w0 += kCombinePieces) {
    f32x4 o[kCombinePieces][4];
    float m[kCombinePieces], l[kCombinePieces];
#pragma unroll
    for (int k = 0; k < kCombinePieces; ++k) {
      const int wg = w0 + k <= w_last ? w0 + k : w_last;  // past the last piece: re-read it, weight 0
      const size_t ps = 2 * (size_t)wg + (wg == w ? 1 : 0);
      m[k] = p.part_ml[part_ml_index(ps, dw, 0, ln)];
      l[k] = p.part_ml[part_ml_index(ps, dw, 1, ln)];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        o[k][q4] = *reinterpret_cast<const f32x4 *>(p.part_o + part_o_index(ps, dw, 4 * mb + q4, ln));
    }
#pragma unroll
    for (int k = 0; k < kCombinePieces; ++k) {
      if (w0 + k > w_last) break;  // uniform
      const float M_new = fmaxf(M, m[k]);
      const float M_safe = M_new == -INFINITY ? 0.f : M_new;
      const float a_old = fast_exp2(M - M_safe), a_new = fast_exp2(m[k] - M_safe);
      lsum = lsum * a_old + l[k] * a_new;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[4 * q4 + j] = acc[4 * q4 + j] * a_old + o[k][q4][j] * a_new;
      M = M_new;
    }
  }
  // the two lanes of an exchange pair hold the same query, so they are active together
  if (t < T) store_out_block<false>(p.out + ((size_t)cut.unit * p.T_max + t) * kD, acc, 1.f / lsum, g, mb);
}

// ------------------------------------------------------------------------------------
// Plain path: one wave per (sequence, head, node); products, softmax and output sums in fp32.
// Serves fp32 operands (d = 64 or 128) and bf16 operands with d = 64, the head size the
// tiled kernel above is not written for; the result is stored in the operands' type.
// ------------------------------------------------------------------------------------
template <typename E>
struct AttnParamsPlain {
  const E *q, *k_cache, *v_cache, *k_tree, *v_tree;
  E *out;
  const int32_t *seq_lens, *n_nodes;
  const uint64_t *anc;
  int H, T_max, L_max, d;
  float scale;
};

__device__ __forceinline__ float plain_load(const float *p) { return *p; }
__device__ __forceinline__ float plain_load(const uint16_t *p) { return bf16_bits_to_f32(*p); }
__device__ __forceinline__ void plain_store(float *p, float x) { *p = x; }
__device__ __forceinline__ void plain_store(uint16_t *p, float x) { *p = (uint16_t)f32_to_bf16_bits(x); }

template <typename E>
__global__ __launch_bounds__(kWave) void tree_attn_plain_kernel(AttnParamsPlain<E> p) {
  const int unit = blockIdx.x / p.T_max, i = blockIdx.x - unit * p.T_max;
  const int b = unit / p.H;
  int L = p.seq_lens[b];
  L = L < 0 ? 0 : (L > p.L_max ? p.L_max : L);
  int T = p.n_nodes[b];
  T = T < 1 ? 1 : (T > p.T_max ? p.T_max : T);
  if (i >= T) return;
  const int lane = threadIdx.x, d = p.d;
  const uint64_t a_lo = p.anc[((size_t)b * p.T_max + i) * 2];
  const uint64_t a_hi = p.anc[((size_t)b * p.T_max + i) * 2 + 1];
  const E *q = p.q + ((size_t)unit * p.T_max + i) * d;
  const E *kc = p.k_cache + (size_t)unit * p.L_max * d;
  const E *vc = p.v_cache + (size_t)unit * p.L_max * d;
  const E *kt = p.k_tree + (size_t)unit * p.T_max * d;
  const E *vt = p.v_tree + (size_t)unit * p.T_max * d;

  float m_run = -INFINITY, l_run = 0.f, o0 = 0.f, o1 = 0.f;  // lane owns columns lane, lane+64
  const int total = L + T;
  for (int j0 = 0; j0 < total; j0 += kWave) {
    const int j = j0 + lane;
    const bool in_cache = j < L;
    const int jt = j - L;
    const bool ok = in_cache || (j < total && test_bit128(a_lo, a_hi, jt));
    float s = -INFINITY;
    if (ok) {
      const E *kr = in_cache ? kc + (size_t)j * d : kt + (size_t)jt * d;
      float acc = 0.f;
      for (int x = 0; x < d; ++x) acc = fmaf(plain_load(q + x), plain_load(kr + x), acc);
      s = acc * p.scale;
    }
    const float m_new = fmaxf(m_run, wave_reduce_max(s));
    if (m_new == -INFINITY) continue;  // nothing visible in this chunk (uniform across the wave)
    const float alpha = expf(m_run - m_new);
    const float w = ok ? expf(s - m_new) : 0.f;
    l_run = l_run * alpha + wave_reduce_sum(w);
    o0 *= alpha;
    o1 *= alpha;
    m_run = m_new;
    const uint64_t live = __ballot(w != 0.f);
    for (uint64_t rest = live; rest; rest &= rest - 1) {
      const int src = __ffsll((long long)rest) - 1;
      const float wj = __shfl(w, src, kWave);
      const int jj = j0 + src;
      const E *vr = jj < L ? vc + (size_t)jj * d : vt + (size_t)(jj - L) * d;
      if (lane < d) o0 = fmaf(wj, plain_load(vr + lane), o0);
      if (lane + 64 < d) o1 = fmaf(wj, plain_load(vr + lane + 64), o1);
    }
  }
  E *o = p.out + ((size_t)unit * p.T_max + i) * d;
  if (lane < d) plain_store(o + lane, o0 / l_run);
  if (lane + 64 < d) plain_store(o + lane + 64, o1 / l_run);
}

template <typename E>
static bool launch_plain(const propd_tree *tree, int H, int d, float scale, const void *q, const void *k_cache,
                         const void *v_cache, const void *k_tree, const void *v_tree, const int32_t *seq_lens,
                         int L_max, void *out, hipStream_t st) {
  AttnParamsPlain<E> p;
  p.q = reinterpret_cast<const E *>(q);
  p.k_cache = reinterpret_cast<const E *>(k_cache);
  p.v_cache = reinterpret_cast<const E *>(v_cache);
  p.k_tree = reinterpret_cast<const E *>(k_tree);
  p.v_tree = reinterpret_cast<const E *>(v_tree);
  p.out = reinterpret_cast<E *>(out);
  p.seq_lens = seq_lens;
  p.n_nodes = tree->n_nodes;
  p.anc = tree->anc;
  p.H = H;
  p.T_max = tree->T_max;
  p.L_max = L_max;
  p.d = d;
  p.scale = scale;
  const long long units = (long long)tree->B * H;
  hipLaunchKernelGGL(tree_attn_plain_kernel<E>, dim3((unsigned)(units * tree->T_max)), dim3(kWave), 0, st, p);
  return launch_ok();
}

// ------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------
static int compute_units() {
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

// Workgroups of the persistent kernel: at most one per two stages of the call, a bound the
// host can compute without a device (the workspace is sized by it) ...
static int grid_bound(int B, int H, int L_max, int T_max) {
  const long long per_unit = (L_max + kStageRows - 1) / kStageRows + (T_max + kStageRows - 1) / kStageRows;
  const long long stages = (long long)B * H * per_unit;
  long long grid = kMaxGrid;
  if (grid > (stages + 1) / 2) grid = (stages + 1) / 2;
  return (int)(grid < 1 ? 1 : grid);
}

// ... and two per compute unit (what LDS allows to be resident).
static int pick_grid(int B, int H, int L_max, int T_max) {
  const int bound = grid_bound(B, H, L_max, T_max), resident = 2 * compute_units();
  return bound < resident ? bound : resident;
}

// Partial slots (two per workgroup) and cut records (one per workgroup) of the largest grid
// a call with these dimensions can use.
size_t tree_attention_workspace_bytes(int B, int H, int L_max, int T_max) {
  const size_t grid = (size_t)grid_bound(B, H, L_max, T_max), slots = 2 * grid;
  return align_up(slots * kPartOFloats * 4, 256) + align_up(slots * kPartMlFloats * 4, 256) +
         align_up(grid * sizeof(CutRecord), 256);
}

static bool launch_bf16(const AttnParams &p, int grid, hipStream_t st) {
  constexpr int lds_bytes = kRingStages * kStageBytes;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_attn_bf16_kernel<kRingStages>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
      return false;
    attr_set = true;
  }
  hipLaunchKernelGGL(tree_attn_bf16_kernel<kRingStages>, dim3((unsigned)grid), dim3(kAttnThreads),
                     lds_bytes, st, p);
  if (!launch_ok()) return false;
  hipLaunchKernelGGL(tree_attn_combine_kernel, dim3((unsigned)grid * 16), dim3(kWave), 0, st, p);
  return launch_ok();
}

}  // namespace propd

extern "C" propd_status propd_tree_attention(const propd_tree *tree, propd_dtype dt, int32_t H,
                                             int32_t d, float scale, const void *q,
                                             const void *k_cache, const void *v_cache,
                                             const void *k_tree, const void *v_tree,
                                             const int32_t *seq_lens, int32_t L_max, void *out,
                                             void *workspace, size_t workspace_bytes,
                                             void *hip_stream) {
  using namespace propd;
  if (!tree || tree->B < 1 || tree->T_max < 1 || tree->T_max > PROPD_MAX_TREE || H < 1 ||
      L_max < 0 || !tree->n_nodes || !tree->anc || !q || !k_tree || !v_tree || !seq_lens || !out ||
      (L_max > 0 && (!k_cache || !v_cache)))
    return PROPD_ERR_INVALID_ARG;
  if (dt != PROPD_BF16 && dt != PROPD_F32) return PROPD_ERR_INVALID_ARG;
  if (!(scale > 0.f)) return PROPD_ERR_INVALID_ARG;  // the kernels take max before scaling
  const long long units = (long long)tree->B * H;
  if (units * tree->T_max > (1ll << 30) || units > (1ll << 28)) return PROPD_ERR_UNSUPPORTED;
  hipStream_t st = as_stream(hip_stream);

  if (dt == PROPD_F32) {
    if (d != 64 && d != 128) return PROPD_ERR_UNSUPPORTED;
    return launch_plain<float>(tree, H, d, scale, q, k_cache, v_cache, k_tree, v_tree, seq_lens, L_max, out, st)
               ? PROPD_OK
               : PROPD_ERR_DEVICE;
  }
  if (d == 64)  // bf16, the smaller head: no workspace is used
    return launch_plain<uint16_t>(tree, H, d, scale, q, k_cache, v_cache, k_tree, v_tree, seq_lens, L_max, out, st)
               ? PROPD_OK
               : PROPD_ERR_DEVICE;

  if (d != kD) return PROPD_ERR_UNSUPPORTED;
  // rows are moved 16 bytes per lane, by direct loads to LDS and four-dword loads and stores
  for (const void *ptr : {q, k_cache, v_cache, k_tree, v_tree, (const void *)out, (const void *)tree->anc,
                          (const void *)workspace})
    if (reinterpret_cast<uintptr_t>(ptr) % 16 != 0) return PROPD_ERR_INVALID_ARG;
  const size_t need = tree_attention_workspace_bytes(tree->B, H, L_max, tree->T_max);
  if (!workspace || workspace_bytes < need) return PROPD_ERR_WORKSPACE;
  AttnParams p;
  p.q = reinterpret_cast<const uint16_t *>(q);
  p.k_cache = reinterpret_cast<const uint16_t *>(k_cache);
  p.v_cache = reinterpret_cast<const uint16_t *>(v_cache);
  p.k_tree = reinterpret_cast<const uint16_t *>(k_tree);
  p.v_tree = reinterpret_cast<const uint16_t *>(v_tree);
  p.out = reinterpret_cast<uint16_t *>(out);
  p.seq_lens = seq_lens;
  p.n_nodes = tree->n_nodes;
  p.anc = tree->anc;
  p.H = H;
  p.T_max = tree->T_max;
  p.L_max = L_max;
  p.B = tree->B;
  p.scale_log2e = scale * 1.4426950408889634f;
  const int grid = pick_grid(tree->B, H, L_max, tree->T_max);
  const size_t slots = 2 * (size_t)grid_bound(tree->B, H, L_max, tree->T_max);
  char *ws = reinterpret_cast<char *>(workspace);
  p.part_o = reinterpret_cast<float *>(ws);
  ws += align_up(slots * kPartOFloats * 4, 256);
  p.part_ml = reinterpret_cast<float *>(ws);
  ws += align_up(slots * kPartMlFloats * 4, 256);
  p.cuts = reinterpret_cast<int32_t *>(ws);
  if (!launch_bf16(p, grid, st)) return PROPD_ERR_DEVICE;
  return PROPD_OK;
}

extern "C" size_t propd_workspace_bytes(propd_ws_kind which, int32_t B, int32_t T_max, int32_t H,
                                        int32_t d, int32_t L_max, int32_t hidden, int32_t vocab) {
  (void)d;
  (void)hidden;
  if (B < 1 || T_max < 1 || T_max > PROPD_MAX_TREE) return 0;
  switch (which) {
    case PROPD_WS_TREE_ATTENTION:
      if (H < 1 || L_max < 0) return 0;
      return propd::tree_attention_workspace_bytes(B, H, L_max, T_max);
    case PROPD_WS_EARLY_PRUNE:
      if (vocab < 1) return 0;
      return propd::early_prune_workspace_bytes(B, T_max, vocab);
    case PROPD_WS_ACCEPT_PATH:
      return propd::accept_path_workspace_bytes(B, T_max);
  }
  return 0;
}
