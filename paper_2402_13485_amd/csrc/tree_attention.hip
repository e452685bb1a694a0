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
//     two per workgroup; a second kernel merges them.
// fp32 path: a plain one-wave-per-query kernel, fp32 throughout.
#include "common.h"

namespace propd {

constexpr int kD = 128;
constexpr int kAttnThreads = 256;
constexpr int kMaxGrid = 1024;                 // workgroups of the persistent kernel, at most
constexpr int kStageRows = 32;                 // K/V rows per ring stage
constexpr int kRowBytes = kD * 2;              // one bf16 row
constexpr int kHalfStage = kStageRows * kRowBytes;  // K part of a stage; the V part follows
constexpr int kStageBytes = 2 * kHalfStage;
#ifndef PROPD_RING_STAGES
#define PROPD_RING_STAGES 5
#endif
constexpr int kRingStages = PROPD_RING_STAGES;  // 16 KB each; two workgroups per CU share 160 KB

struct AttnParams {
  const uint16_t *q, *k_cache, *v_cache, *k_tree, *v_tree;
  uint16_t *out;
  const int32_t *seq_lens, *n_nodes;
  const uint64_t *anc;
  int B, H, T_max, L_max;
  float scale_log2e;
  float *part_o;   // [2 * grid][128][128]
  float *part_ml;  // [2 * grid][128][2]
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

// Work decomposition shared by the main kernel and the merge kernel.  The work of one
// call is the list of K/V stages of all (sequence, head) units in order, each unit's
// cached stages followed by its tree stages.  Workgroup w of G owns the contiguous range
// [w*N/G, (w+1)*N/G) of that list, so every workgroup streams the same number of rows
// whatever the mix of sequence lengths; a unit cut by a range boundary is finished by
// the merge kernel from per-workgroup partial results.
struct StageMap {
  int B, H;
  const int32_t *seq_lens, *n_nodes;
  int L_max, T_max;
  __device__ __forceinline__ int len(int b) const {
    const int L = seq_lens[b];
    return L < 0 ? 0 : (L > L_max ? L_max : L);
  }
  __device__ __forceinline__ int nodes(int b) const {
    const int T = n_nodes[b];
    return T < 1 ? 1 : (T > T_max ? T_max : T);
  }
  __device__ __forceinline__ int cache_stages(int b) const {
    return (len(b) + kStageRows - 1) / kStageRows;
  }
  __device__ __forceinline__ int tree_stages(int b) const {
    return (nodes(b) + kStageRows - 1) / kStageRows;
  }
  __device__ __forceinline__ int unit_stages(int b) const { return cache_stages(b) + tree_stages(b); }
  __device__ long long total() const {
    long long n = 0;
    for (int b = 0; b < B; ++b) n += (long long)H * unit_stages(b);
    return n;
  }
};

__device__ __forceinline__ long long range_start(long long w, long long n, long long g) {
  return w * n / g;
}

// Position in the stage list: stage s of unit (b, h), with the sizes of sequence b.
struct Cursor {
  int b, h, s;
  int L, T, cs, ts;  // cached rows, tree nodes, cached stages, tree stages of sequence b
  __device__ __forceinline__ void load_sizes(const StageMap &m) {
    L = m.len(b);
    T = m.nodes(b);
    cs = (L + kStageRows - 1) / kStageRows;
    ts = (T + kStageRows - 1) / kStageRows;
  }
  __device__ __forceinline__ void advance(const StageMap &m, int n) {  // n <= stages left in the unit
    s += n;
    if (s == cs + ts) {
      s = 0;
      if (++h == m.H) {
        h = 0;
        if (b + 1 < m.B) {
          ++b;
          load_sizes(m);
        }
      }
    }
  }
};

template <int NS>
__global__ __launch_bounds__(kAttnThreads, 2) void tree_attn_bf16_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void *)smem;  // LDS byte address of the ring

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  const int t = wave * 32 + l32;  // this lane's query column

  const StageMap map = {p.B, p.H, p.seq_lens, p.n_nodes, p.L_max, p.T_max};
  const long long n_total = map.total();
  const long long G = gridDim.x, w = blockIdx.x;
  const long long x0 = range_start(w, n_total, G);
  const int n_my = (int)(range_start(w + 1, n_total, G) - x0);
  if (n_my <= 0) return;

  // ---- the first stage of this range
  Cursor cp;
  {
    cp.b = 0;
    long long b_start = 0;
    while (cp.b < p.B - 1 && x0 >= b_start + (long long)p.H * map.unit_stages(cp.b)) {
      b_start += (long long)p.H * map.unit_stages(cp.b);
      ++cp.b;
    }
    cp.load_sizes(map);
    const int us = cp.cs + cp.ts;
    cp.h = (int)((x0 - b_start) / us);
    cp.s = (int)((x0 - b_start) - (long long)cp.h * us);
  }
  Cursor ld = cp;  // the loader runs ahead of the math over the same list

  // ---- loader.  One direct load moves 64 lanes x 16 bytes = 4 rows into 1 KB of LDS that
  //      is contiguous in lane order, so the swizzle is applied on the global side: the lane
  //      that fills chunk c of LDS row r fetches chunk c ^ key(r) of the global row.  Keys:
  //      K rows r & 15 (a 16-byte read of one chunk column over 16 rows touches 16 distinct
  //      chunks); V rows ((r & 3) << 2) | ((r >> 2) & 3) (the 4 rows x 64 bytes of one
  //      transposing read land in 4 distinct 64-byte bank groups).  A wave fills rows
  //      4*wave + lane/16 of each 16-row half, so its keys do not depend on the half.
  //      Rows past the last valid one re-read that last row: finite data that the mask
  //      discards (K) or that meets a zero weight (V); padding is never touched.
  const int ld_row = 4 * wave + (lane >> 4);
  const int k_src_chunk = ((lane & 15) ^ ld_row) << 4;
  const int v_src_chunk = ((lane & 15) ^ (((lane >> 4) << 2) | wave)) << 4;
  auto issue = [&](int slot) {
    const bool is_tree = ld.s >= ld.cs;
    const int j0 = (is_tree ? ld.s - ld.cs : ld.s) * kStageRows;
    const int last = (is_tree ? ld.T : ld.L) - 1;
    const size_t unit = (size_t)ld.b * p.H + ld.h;
    const unsigned char *kb = reinterpret_cast<const unsigned char *>(
        is_tree ? p.k_tree + unit * p.T_max * kD : p.k_cache + unit * p.L_max * kD);
    const unsigned char *vb = reinterpret_cast<const unsigned char *>(
        is_tree ? p.v_tree + unit * p.T_max * kD : p.v_cache + unit * p.L_max * kD);
    unsigned char *dst = smem + slot * kStageBytes + (4 * wave) * kRowBytes;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      int row = j0 + 16 * i + ld_row;
      row = row > last ? last : row;
      const size_t ro = (size_t)row * kRowBytes;
      __builtin_amdgcn_global_load_lds((global_void *)(kb + ro + k_src_chunk),
                                       (lds_void *)(dst + i * 16 * kRowBytes), 16, 0, 2);
      __builtin_amdgcn_global_load_lds((global_void *)(vb + ro + v_src_chunk),
                                       (lds_void *)(dst + kHalfStage + i * 16 * kRowBytes), 16, 0, 2);
    }
    ld.advance(map, 1);
  };

  // ---- per-lane LDS read offsets within a stage
  // K as the A operand of S^T: lane = row l32, 8 consecutive d from 16*ks + 8*g (chunk 2*ks + g)
  int k_rd[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k_rd[ks] = l32 * kRowBytes + (((2 * ks + g) ^ (l32 & 15)) << 4);
  // V^T as the A operand of O^T: transposing read; in each group of 16 lanes, lane i points at
  // row i/4, 4 columns from 4*(i%4), and receives column i of those 4 rows.  Per MFMA k-step
  // (16 rows): slots 0..3 = rows 4g + 0..3, slots 4..7 = those rows + 8.
  int v_rd[4][2];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
      const int r = 4 * g + ((lane & 15) >> 2) + 8 * hi;
      const int key = ((r & 3) << 2) | ((r >> 2) & 3);
      const int chunk = mb * 4 + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
      v_rd[mb][hi] = kHalfStage + r * kRowBytes + ((chunk ^ key) << 4) + 8 * (lane & 1);
    }

  // ---- fill the ring
  int slot_ld = 0;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < n_my) {
      issue(slot_ld);
      slot_ld = slot_ld + 1 == NS ? 0 : slot_ld + 1;
    }

  int it = 0, slot = 0;
  while (it < n_my) {
    // ---- the piece of one unit that lies in this range
    const int L = cp.L, T = cp.T, n_cache = cp.cs;
    const int us = cp.cs + cp.ts, s0 = cp.s;
    const int n_st = us - s0 < n_my - it ? us - s0 : n_my - it;
    const bool whole = s0 == 0 && n_st == us;
    const int unit = cp.b * p.H + cp.h;
#ifdef PROPD_TIMING_NO_MATH  // timing experiment: stream only
    const bool active = false;
#else
    const bool active = wave * 32 < T;  // wave-uniform: some query of this wave exists
#endif

    // Q^T fragments: B operand, lane = query column, 8 consecutive d per K step
    bf16x8 qf[8];
    uint64_t anc_lo = 0, anc_hi = 0;
    {
      const u32x4 zero4 = {0u, 0u, 0u, 0u};
      const uint16_t *qrow = p.q + ((size_t)unit * p.T_max + (t < T ? t : 0)) * kD + g * 8;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        u32x4 v = t < T ? *reinterpret_cast<const u32x4 *>(qrow + ks * 16) : zero4;
        qf[ks] = __builtin_bit_cast(bf16x8, v);
      }
      if (t < T) {
        anc_lo = p.anc[((size_t)cp.b * p.T_max + t) * 2];
        anc_hi = p.anc[((size_t)cp.b * p.T_max + t) * 2 + 1];
      }
      // Touch the loaded registers here, so that the wait for them is placed before the
      // stage loop and not inside it, where it would also drain the ring's loads in flight.
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(qf[ks]));
      asm volatile("" ::"v"(anc_lo), "v"(anc_hi));
    }

    float m_run = -INFINITY, l_run = 0.f;
    f32x16 o_acc[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[mb][r] = 0.f;

    for (int i = 0; i < n_st; ++i, ++it) {
      // stage `it` has landed once at most the loads of the NS-2 stages issued after it
      // (4 per wave and stage) are outstanding; near the end of the range fewer follow it
      if (it + NS - 2 <= n_my - 1) wait_vmem<4 * (NS - 2)>(); else wait_vmem<0>();
      __builtin_amdgcn_s_barrier();  // stage `it` is visible; every wave is done with stage it-1
#ifdef PROPD_TIMING_NO_LOADS  // timing experiment: math on whatever the ring holds
      if (false) {
#else
      if (it + NS - 1 < n_my) {
#endif
        issue(slot_ld);  // refill the slot of stage it-1
        slot_ld = slot_ld + 1 == NS ? 0 : slot_ld + 1;
      }
      const unsigned char *st = smem + slot * kStageBytes;
      slot = slot + 1 == NS ? 0 : slot + 1;

      const int s = s0 + i;
      const bool is_tree = s >= n_cache;
      const int j0 = (is_tree ? s - n_cache : s) * kStageRows;
      // tree rows after this wave's last query are descendants or strangers of all its queries
      if (!active || (is_tree && j0 > wave * 32 + 31)) continue;
      int n_valid = (is_tree ? T : L) - j0;
      n_valid = n_valid > kStageRows ? kStageRows : n_valid;
      const bool partial = is_tree || n_valid < kStageRows;  // uniform over the workgroup

      // ---- S^T = K . Q^T
      f32x16 sc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(st + k_rd[ks]);
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sc, 0, 0, 0);
      }
      mfma_settle();

      // ---- start the transposing reads of the whole V stage now; they complete while the
      //      softmax below runs.  vt[ks2][2*mb + hi]: k-step ks2 (16 rows), d block mb.
      u32x2 vt[2][8];
      {
        const uint32_t vs = smem_base + (uint32_t)(st - smem);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
          vt[0][2 * mb] = lds_read_tr16<0>(vs + v_rd[mb][0]);
          vt[0][2 * mb + 1] = lds_read_tr16<0>(vs + v_rd[mb][1]);
        }
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
          vt[1][2 * mb] = lds_read_tr16<16 * kRowBytes>(vs + v_rd[mb][0]);
          vt[1][2 * mb + 1] = lds_read_tr16<16 * kRowBytes>(vs + v_rd[mb][1]);
        }
      }

      // ---- mask and running max on the raw scores (the softmax scale is positive, so it
      //      commutes with max and is applied inside the exponent).  Register r of a 32x32
      //      accumulator holds row 8*(r/4) + 4*g + r%4 of the block, i.e. K/V row j0 + that.
      if (partial) {
        // visibility of the stage's rows to this lane's query: cached rows below L for every
        // query, tree rows only where the node's ancestor set has the bit
        uint32_t vis = n_valid >= 32 ? ~0u : ((1u << n_valid) - 1u);
        const uint64_t word = j0 >= 64 ? anc_hi : anc_lo;  // tree stages start at 0, 32, 64, 96
        vis &= is_tree ? (uint32_t)(word >> (j0 & 32)) : ~0u;
        vis >>= 4 * g;
#pragma unroll
        for (int r = 0; r < 16; ++r)
          sc[r] = ((vis >> (8 * (r >> 2) + (r & 3))) & 1u) ? sc[r] : -INFINITY;
      }
      float m_blk = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) m_blk = fmaxf(m_blk, sc[r]);
      m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32, kWave));
      const float m_new = fmaxf(m_run, m_blk);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      // rescale only when some query of this wave saw a new maximum
      if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
        const float alpha = fast_exp2((m_run - m_safe) * p.scale_log2e);
        l_run *= alpha;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) o_acc[mb][r] *= alpha;
        m_run = m_new;
      }
      const float neg_m = -m_safe * p.scale_log2e;

      // ---- P^T (bf16) straight from the score registers, then O^T += V^T . P^T.  The row
      //      sums are taken over the rounded bf16 weights, the same values the MFMA multiplies.
      const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
      uint32_t pw[8];
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const float p0 = fast_exp2(fmaf(sc[r], p.scale_log2e, neg_m));
        const float p1 = fast_exp2(fmaf(sc[r + 1], p.scale_log2e, neg_m));
        pw[r >> 1] = cvt_pk_bf16(p0, p1);
        l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[r >> 1]), ones, l_run,
                                                false);
      }
      wait_lds<8>(vt[0]);  // LDS reads return in order: the first eight are in
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2) {
        if (ks2 == 1) wait_lds<0>(vt[1]);
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
    }

    // ---- write: lane holds d = mb*32 + 8*(r/4) + 4*g + r%4 for its query t
    mfma_settle();
    l_run += __shfl_xor(l_run, 32, kWave);
    m_run *= p.scale_log2e;  // from here on the maximum is in the exponent's (log2) domain
    if (t < T) {
      if (whole) {
        const float inv = 1.f / l_run;
        uint16_t *orow = p.out + ((size_t)unit * p.T_max + t) * kD;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            u32x2 w2;
            w2.x = cvt_pk_bf16(o_acc[mb][4 * q4] * inv, o_acc[mb][4 * q4 + 1] * inv);
            w2.y = cvt_pk_bf16(o_acc[mb][4 * q4 + 2] * inv, o_acc[mb][4 * q4 + 3] * inv);
            *reinterpret_cast<u32x2 *>(orow + mb * 32 + 8 * q4 + 4 * g) = w2;
          }
      } else {
        // a range starts inside at most one unit and ends inside at most one
        const size_t ps = 2 * (size_t)w + (s0 > 0 ? 0 : 1);
        float *po = p.part_o + (ps * 128 + t) * kD;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const f32x4 w4 = {o_acc[mb][4 * q4], o_acc[mb][4 * q4 + 1], o_acc[mb][4 * q4 + 2],
                              o_acc[mb][4 * q4 + 3]};
            *reinterpret_cast<f32x4 *>(po + mb * 32 + 8 * q4 + 4 * g) = w4;
          }
        if (g == 0) {
          p.part_ml[(ps * 128 + t) * 2] = m_run;
          p.part_ml[(ps * 128 + t) * 2 + 1] = l_run;
        }
      }
    }
    cp.advance(map, n_st);
  }
}

// Finish the units that a range boundary cut: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s
// over the workgroups s that hold a piece.  One workgroup per unit; whole units return at once.
__global__ __launch_bounds__(kAttnThreads) void tree_attn_combine_kernel(AttnParams p, int G) {
  const int unit = blockIdx.x;
  const int b = unit / p.H, h = unit - b * p.H;
  const StageMap map = {p.B, p.H, p.seq_lens, p.n_nodes, p.L_max, p.T_max};
  long long n_total = 0, b_start = 0;
  for (int bb = 0; bb < p.B; ++bb) {
    if (bb == b) b_start = n_total;
    n_total += (long long)p.H * map.unit_stages(bb);
  }
  const int ut = map.unit_stages(b), T = map.nodes(b);
  const long long S = b_start + (long long)h * ut, E = S + ut;
  // workgroup that owns tile x: the largest w with range_start(w) <= x
  auto owner = [&](long long x) {
    long long w = x * G / n_total;
    while (w + 1 < G && range_start(w + 1, n_total, G) <= x) ++w;
    while (w > 0 && range_start(w, n_total, G) > x) --w;
    return w;
  };
  const long long w_first = owner(S), w_last = owner(E - 1);
  if (w_first == w_last) return;  // the unit was finished by one workgroup
  // partial slots of the pieces, worked out once per workgroup
  __shared__ int s_slot[kMaxGrid];
  const int pieces = (int)(w_last - w_first + 1);
  for (int i = threadIdx.x; i < pieces; i += kAttnThreads) {
    const long long w = w_first + i;
    s_slot[i] = (int)(2 * w + (range_start(w, n_total, G) > S ? 0 : 1));
  }
  __syncthreads();
  for (int item = threadIdx.x; item < T * (kD / 4); item += kAttnThreads) {
    const int t = item / (kD / 4), d4 = (item - t * (kD / 4)) * 4;
    float M = -INFINITY;
    for (int i = 0; i < pieces; ++i)
      M = fmaxf(M, p.part_ml[((size_t)s_slot[i] * 128 + t) * 2]);
    if (M == -INFINITY) M = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float lsum = 0.f;
    for (int i = 0; i < pieces; ++i) {
      const size_t slot = (size_t)s_slot[i];
      const float wgt = fast_exp2(p.part_ml[(slot * 128 + t) * 2] - M);
      lsum += wgt * p.part_ml[(slot * 128 + t) * 2 + 1];
      if (wgt != 0.f) {
        const f32x4 o = *reinterpret_cast<const f32x4 *>(p.part_o + (slot * 128 + t) * kD + d4);
        acc += o * wgt;
      }
    }
    const float inv = 1.f / lsum;
    u32x2 w2;
    w2.x = cvt_pk_bf16(acc.x * inv, acc.y * inv);
    w2.y = cvt_pk_bf16(acc.z * inv, acc.w * inv);
    *reinterpret_cast<u32x2 *>(p.out + ((size_t)unit * p.T_max + t) * kD + d4) = w2;
  }
}

// ------------------------------------------------------------------------------------
// fp32 path: one wave per (sequence, head, node); fp32 loads, products, softmax, output.
// ------------------------------------------------------------------------------------
struct AttnParamsF32 {
  const float *q, *k_cache, *v_cache, *k_tree, *v_tree;
  float *out;
  const int32_t *seq_lens, *n_nodes;
  const uint64_t *anc;
  int H, T_max, L_max, d;
  float scale;
};

__global__ __launch_bounds__(kWave) void tree_attn_f32_kernel(AttnParamsF32 p) {
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
  const float *q = p.q + ((size_t)unit * p.T_max + i) * d;
  const float *kc = p.k_cache + (size_t)unit * p.L_max * d;
  const float *vc = p.v_cache + (size_t)unit * p.L_max * d;
  const float *kt = p.k_tree + (size_t)unit * p.T_max * d;
  const float *vt = p.v_tree + (size_t)unit * p.T_max * d;

  float m_run = -INFINITY, l_run = 0.f, o0 = 0.f, o1 = 0.f;  // lane owns columns lane, lane+64
  const int total = L + T;
  for (int j0 = 0; j0 < total; j0 += kWave) {
    const int j = j0 + lane;
    const bool in_cache = j < L;
    const int jt = j - L;
    const bool ok = in_cache || (j < total && test_bit128(a_lo, a_hi, jt));
    float s = -INFINITY;
    if (ok) {
      const float *kr = in_cache ? kc + (size_t)j * d : kt + (size_t)jt * d;
      float acc = 0.f;
      for (int x = 0; x < d; ++x) acc = fmaf(q[x], kr[x], acc);
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
      const float *vr = jj < L ? vc + (size_t)jj * d : vt + (size_t)(jj - L) * d;
      if (lane < d) o0 = fmaf(wj, vr[lane], o0);
      if (lane + 64 < d) o1 = fmaf(wj, vr[lane + 64], o1);
    }
  }
  float *o = p.out + ((size_t)unit * p.T_max + i) * d;
  if (lane < d) o[lane] = o0 / l_run;
  if (lane + 64 < d) o[lane + 64] = o1 / l_run;
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

// Workgroups of the persistent kernel: two per compute unit (what LDS allows to be
// resident), fewer when the whole call has fewer than two stages per workgroup.
static int pick_grid(int B, int H, int L_max, int T_max) {
  const long long per_unit = (L_max + kStageRows - 1) / kStageRows + (T_max + kStageRows - 1) / kStageRows;
  const long long stages = (long long)B * H * per_unit;
  long long grid = 2ll * compute_units();
  if (grid > kMaxGrid) grid = kMaxGrid;
  if (grid > (stages + 1) / 2) grid = (stages + 1) / 2;
  return (int)(grid < 1 ? 1 : grid);
}

// Partial slots: two per workgroup of the grid this call will use.
size_t tree_attention_workspace_bytes(int B, int H, int L_max, int T_max) {
  const size_t slots = 2 * (size_t)pick_grid(B, H, L_max, T_max);
  return align_up(slots * 128 * kD * 4, 256) + align_up(slots * 128 * 2 * 4, 256);
}

static bool launch_bf16(const AttnParams &p, int grid, int units, hipStream_t st) {
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
  hipLaunchKernelGGL(tree_attn_combine_kernel, dim3((unsigned)units), dim3(kAttnThreads), 0, st, p,
                     grid);
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
  if (units * tree->T_max > (1ll << 30)) return PROPD_ERR_UNSUPPORTED;
  hipStream_t st = as_stream(hip_stream);

  if (dt == PROPD_F32) {
    if (d != 64 && d != 128) return PROPD_ERR_UNSUPPORTED;
    AttnParamsF32 p;
    p.q = reinterpret_cast<const float *>(q);
    p.k_cache = reinterpret_cast<const float *>(k_cache);
    p.v_cache = reinterpret_cast<const float *>(v_cache);
    p.k_tree = reinterpret_cast<const float *>(k_tree);
    p.v_tree = reinterpret_cast<const float *>(v_tree);
    p.out = reinterpret_cast<float *>(out);
    p.seq_lens = seq_lens;
    p.n_nodes = tree->n_nodes;
    p.anc = tree->anc;
    p.H = H;
    p.T_max = tree->T_max;
    p.L_max = L_max;
    p.d = d;
    p.scale = scale;
    hipLaunchKernelGGL(tree_attn_f32_kernel, dim3((unsigned)(units * tree->T_max)), dim3(kWave), 0,
                       st, p);
    return launch_ok() ? PROPD_OK : PROPD_ERR_DEVICE;
  }

  if (d != kD) return PROPD_ERR_UNSUPPORTED;
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
  const size_t slots = 2 * (size_t)grid;
  p.part_o = reinterpret_cast<float *>(workspace);
  p.part_ml = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) +
                                        align_up(slots * 128 * kD * 4, 256));
  if (!launch_bf16(p, grid, (int)units, st)) return PROPD_ERR_DEVICE;
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
      return propd::align_up((size_t)B * T_max * 4, 256);
  }
  return 0;
}
