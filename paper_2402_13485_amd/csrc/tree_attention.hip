// Tree-masked attention over the cached prefix plus each node's own root path
// (Section 2, "Verification"; Figure 2(b,c)).
//
// bf16 path (d = 128).  The work is a stream of K/V rows from HBM that all T
// tree queries of a (sequence, head) pair share, so the kernel is organised
// around reading every K and V row exactly once:
//   - a persistent grid (two workgroups of 4 waves per compute unit); the list of
//     all K/V tiles of the call is cut into equal contiguous ranges, one per
//     workgroup, so ragged sequence lengths balance by construction;
//   - K/V tiles go global -> registers -> LDS, 16 bytes per lane, fully coalesced,
//     double buffered: one barrier per tile, the tile after next in flight;
//   - scores are computed transposed, S^T = K . Q^T, with the 32x32x16 bf16 MFMA,
//     so that a lane owns one query column: the running max / sum of the online
//     softmax are per-lane scalars, and the fp32 score registers, once
//     exponentiated and rounded to bf16, ARE the B operand of the second MFMA
//     O^T += V^T . P^T, with no shuffle or LDS round trip; V^T is read from
//     row-major V in LDS with the transposing LDS read;
//   - the cached prefix needs no mask; the tree part is one extra tile whose
//     scores are kept only where the node's 128-bit ancestor set has the bit;
//   - waves split the query columns (32 per wave) and, when the tree is small,
//     also the rows of a tile; row groups are merged through LDS at the end;
//   - a unit cut by a range boundary leaves fp32 partials (O, max, sum), at most
//     two per workgroup; a second kernel merges them.
// fp32 path: a plain one-wave-per-query kernel, fp32 throughout.
#include "common.h"

namespace propd {

#ifndef PROPD_EXP
#define PROPD_EXP 0  // timing experiments: 1 no S MFMAs, 2 no exp, 4 no PV, 8 no settle
#endif
constexpr int kD = 128;
constexpr int kAttnThreads = 256;
constexpr int kMaxGrid = 1024;  // workgroups of the persistent kernel, at most
constexpr int kKPitch = kD + 8;   // bf16 elements per K row in LDS: 272 B, conflict-free b128 reads
constexpr int kVPitch = kD + 32;  // bf16 elements per V row in LDS: 320 B, conflict-free transpose reads

template <int TG>
struct AttnCfg {
  static constexpr int KG = 4 / TG;              // waves sharing one query group, splitting rows
  static constexpr int NBW = (TG == 4) ? 2 : 1;  // 32-row blocks per wave per tile
  static constexpr int TILE_J = 32 * KG * NBW;   // K/V rows per tile: 64, 64, 128
  static constexpr int CH = TILE_J * 16 / kAttnThreads;  // 16-byte chunks per thread per tensor
  static constexpr int k_elems = TILE_J * kKPitch;
  static constexpr int v_elems = TILE_J * kVPitch;
  static constexpr size_t buf_bytes = (size_t)(k_elems + v_elems) * 2;
  static constexpr size_t tile_bytes = 2 * buf_bytes;  // double buffered
  static constexpr size_t merge_bytes = (size_t)(4 - TG) * 64 * 66 * 4;  // o[64] + m + l per lane
  static constexpr size_t lds_bytes = tile_bytes > merge_bytes ? tile_bytes : merge_bytes;
};

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

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two floats -> packed bf16 pair (round to nearest even), one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  const f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// Work decomposition shared by the main kernel and the merge kernel.  The work of one
// call is the list of K/V tiles of all (sequence, head) units in order, each unit's
// cached tiles followed by its tree tiles.  Workgroup w of G owns the contiguous range
// [w*N/G, (w+1)*N/G) of that list, so every workgroup streams the same number of rows
// whatever the mix of sequence lengths; a unit cut by a range boundary is finished by
// the merge kernel from per-workgroup partial results.
template <int TILE_J>
struct TileMap {
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
  __device__ __forceinline__ int cache_tiles(int b) const { return (len(b) + TILE_J - 1) / TILE_J; }
  __device__ __forceinline__ int tree_tiles(int b) const { return (nodes(b) + TILE_J - 1) / TILE_J; }
  __device__ __forceinline__ int unit_tiles(int b) const { return cache_tiles(b) + tree_tiles(b); }
  __device__ long long total() const {
    long long n = 0;
    for (int b = 0; b < B; ++b) n += (long long)H * unit_tiles(b);
    return n;
  }
};

__device__ __forceinline__ long long range_start(long long w, long long n, long long g) {
  return w * n / g;
}

template <int TG>
__global__ __launch_bounds__(kAttnThreads, TG == 1 ? 1 : 2) void tree_attn_bf16_kernel(AttnParams p) {
  using C = AttnCfg<TG>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t *lds = reinterpret_cast<uint16_t *>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int tg = wave % TG, kg = wave / TG;
  const int t = tg * 32 + l32;  // this lane's query column

  const TileMap<C::TILE_J> map = {p.B, p.H, p.seq_lens, p.n_nodes, p.L_max, p.T_max};
  const long long n_total = map.total();
  const long long G = gridDim.x, w = blockIdx.x;
  long long x = range_start(w, n_total, G);
  const long long x_end = range_start(w + 1, n_total, G);

  int b = 0;
  long long b_start = 0;  // first tile of sequence b in the global list
  while (x < x_end) {
    // ---- locate the unit that owns tile x (x only grows, so b only grows)
    while (b < p.B - 1 && x >= b_start + (long long)p.H * map.unit_tiles(b)) {
      b_start += (long long)p.H * map.unit_tiles(b);
      ++b;
    }
    const int L = map.len(b), T = map.nodes(b);
    const int ut = map.unit_tiles(b), n_cache_tiles = map.cache_tiles(b);
    const int h = (int)((x - b_start) / ut);
    const int tile0 = (int)((x - b_start) - (long long)h * ut);
    const long long unit_end = b_start + (long long)(h + 1) * ut;
    const int n_tiles = (int)((unit_end < x_end ? unit_end : x_end) - x);
    const bool whole = tile0 == 0 && n_tiles == ut;
    const int unit = b * p.H + h;

    const uint16_t *kc = p.k_cache + (size_t)unit * p.L_max * kD;
    const uint16_t *vc = p.v_cache + (size_t)unit * p.L_max * kD;
    const uint16_t *kt = p.k_tree + (size_t)unit * p.T_max * kD;
    const uint16_t *vt = p.v_tree + (size_t)unit * p.T_max * kD;

    // Q^T fragments: B operand, lane = query column, 8 consecutive d per K step
    bf16x8 qf[8];
    {
      const u32x4 zero4 = {0u, 0u, 0u, 0u};
      const uint16_t *qrow = p.q + ((size_t)unit * p.T_max + (t < T ? t : 0)) * kD + g * 8;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        u32x4 v = t < T ? *reinterpret_cast<const u32x4 *>(qrow + ks * 16) : zero4;
        qf[ks] = __builtin_bit_cast(bf16x8, v);
      }
    }
    uint64_t anc_lo = 0, anc_hi = 0;
    if (t < T) {
      anc_lo = p.anc[((size_t)b * p.T_max + t) * 2];
      anc_hi = p.anc[((size_t)b * p.T_max + t) * 2 + 1];
    }

    float m_run = -INFINITY, l_run = 0.f;
    f32x16 o_acc[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[mb][r] = 0.f;

    // ---- tile fetch: 16-byte chunks, chunk c -> row c/16, columns (c%16)*8 .. +8
    u32x4 k_reg[C::CH], v_reg[C::CH];
    auto fetch = [&](int it) {
      const int tile = tile0 + it;
      const bool is_tree = tile >= n_cache_tiles;
      const int j0 = (is_tree ? tile - n_cache_tiles : tile) * C::TILE_J;
      const int rows_valid = (is_tree ? T : L) - j0;
      const uint16_t *ksrc = (is_tree ? kt : kc) + (size_t)j0 * kD;
      const uint16_t *vsrc = (is_tree ? vt : vc) + (size_t)j0 * kD;
      const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int i = 0; i < C::CH; ++i) {
        const int c = i * kAttnThreads + tid;
        const bool ok = (c >> 4) < rows_valid;  // rows beyond the valid ones read as zero
        k_reg[i] = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(ksrc) + c) : zero4;
        v_reg[i] = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vsrc) + c) : zero4;
      }
    };
    auto stash = [&](int buf) {
      uint16_t *Ks = lds + buf * (C::k_elems + C::v_elems);
      uint16_t *Vs = Ks + C::k_elems;
#pragma unroll
      for (int i = 0; i < C::CH; ++i) {
        const int c = i * kAttnThreads + tid;
        const int row = c >> 4, col = (c & 15) * 8;
        *reinterpret_cast<u32x4 *>(&Ks[row * kKPitch + col]) = k_reg[i];
        *reinterpret_cast<u32x4 *>(&Vs[row * kVPitch + col]) = v_reg[i];
      }
    };

    fetch(0);
    stash(0);
    if (n_tiles > 1) fetch(1);
    __syncthreads();

    for (int it = 0; it < n_tiles; ++it) {
      const int cur = it & 1;
      // tile it+1 is in registers: park it in the other buffer (free since the last
      // barrier), then start loading tile it+2; both overlap with the math below
      if (it + 1 < n_tiles) stash(cur ^ 1);
      if (it + 2 < n_tiles) fetch(it + 2);

      const uint16_t *Ks = lds + cur * (C::k_elems + C::v_elems);
      const uint16_t *Vs = Ks + C::k_elems;
      const int tile = tile0 + it;
      const bool is_tree = tile >= n_cache_tiles;
      const int j0 = (is_tree ? tile - n_cache_tiles : tile) * C::TILE_J;
      int n_valid = (is_tree ? T : L) - j0;
      n_valid = n_valid > C::TILE_J ? C::TILE_J : n_valid;
      const bool partial = is_tree || n_valid < C::TILE_J;  // uniform over the workgroup

      // ---- S^T = K . Q^T for this wave's row blocks
      f32x16 s[C::NBW];
#pragma unroll
      for (int nb = 0; nb < C::NBW; ++nb) {
        const int jb = kg * C::NBW + nb;
#pragma unroll
        for (int r = 0; r < 16; ++r)
          s[nb][r] = (PROPD_EXP & 1) ? (float)__builtin_bit_cast(u32x4, qf[r & 7]).x * 1e-12f : 0.f;
#pragma unroll
        for (int ks = 0; ks < ((PROPD_EXP & 1) ? 0 : 8); ++ks) {
          const bf16x8 a =
              *reinterpret_cast<const bf16x8 *>(&Ks[(jb * 32 + l32) * kKPitch + ks * 16 + g * 8]);
          s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[nb], 0, 0, 0);
        }
      }
      if (!(PROPD_EXP & 8)) mfma_settle();

      // ---- mask and running max on the raw scores (the softmax scale is positive, so it
      //      commutes with max and is applied inside the exponent).  Register r of a 32x32
      //      accumulator holds row 8*(r/4) + 4*g + r%4 of the block, i.e. K/V row j of the tile.
      if (partial) {
        // tile-local visibility of this lane's query: cached rows below L for every
        // query, tree rows only where the node's ancestor set has the bit
        uint64_t vis_lo, vis_hi;
        mask_below(n_valid, vis_lo, vis_hi);
        const uint64_t t_lo = j0 >= 64 ? anc_hi : anc_lo;  // tree tiles start at row 0 or 64
        const uint64_t t_hi = j0 >= 64 ? 0ull : anc_hi;
        vis_lo &= is_tree ? t_lo : ~0ull;
        vis_hi &= is_tree ? t_hi : ~0ull;
#pragma unroll
        for (int nb = 0; nb < C::NBW; ++nb) {
          const int jb = kg * C::NBW + nb;
          const uint64_t word = (jb & 2) ? vis_hi : vis_lo;
          const uint32_t vis = (uint32_t)(word >> ((jb & 1) * 32)) >> (4 * g);
#pragma unroll
          for (int r = 0; r < 16; ++r)
            s[nb][r] = ((vis >> (8 * (r >> 2) + (r & 3))) & 1u) ? s[nb][r] : -INFINITY;
        }
      }
      float m_blk = -INFINITY;
#pragma unroll
      for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) m_blk = fmaxf(m_blk, s[nb][r]);
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

      // ---- P^T (bf16) straight from the score registers, then O^T += V^T . P^T.
      //      The A operand V^T comes from row-major V in LDS through the transposing
      //      read: in each group of 16 lanes, lane i points at row i/4, 4 columns from
      //      4*(i%4), and receives column i of those 4 rows.  The row sums are taken over
      //      the rounded bf16 weights, the same values the MFMA multiplies.
      const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
#pragma unroll
      for (int nb = 0; nb < C::NBW; ++nb) {
        const int jb = kg * C::NBW + nb;
        uint32_t pw[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          float p0 = fmaf(s[nb][r], p.scale_log2e, neg_m), p1 = fmaf(s[nb][r + 1], p.scale_log2e, neg_m);
          if (!(PROPD_EXP & 2)) {
            p0 = fast_exp2(p0);
            p1 = fast_exp2(p1);
          }
          pw[r >> 1] = cvt_pk_bf16(p0, p1);
          l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[r >> 1]), ones,
                                                  l_run, false);
        }
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
          const u32x4 pv = {pw[4 * ks2], pw[4 * ks2 + 1], pw[4 * ks2 + 2], pw[4 * ks2 + 3]};
          const bf16x8 pf = __builtin_bit_cast(bf16x8, pv);
          // slots 0..3: rows 16*ks2 + 4g + 0..3; slots 4..7: those rows + 8
          const int row = jb * 32 + 16 * ks2 + 4 * g + ((lane & 15) >> 2);
          const int col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
          for (int mb = 0; mb < ((PROPD_EXP & 4) ? 0 : 4); ++mb) {
            const uint16_t *src = &Vs[row * kVPitch + mb * 32 + col];
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4 *)(src));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4 *)(src + 8 * kVPitch));
            const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
            const u32x4 aw = {lo2.x, lo2.y, hi2.x, hi2.y};
            o_acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw), pf,
                                                                o_acc[mb], 0, 0, 0);
          }
        }
      }
      __syncthreads();  // tile it is consumed, tile it+1 is visible
    }

    // ---- merge the row groups of one query group through LDS (lane-wise)
    mfma_settle();
    l_run += __shfl_xor(l_run, 32, kWave);
    m_run *= p.scale_log2e;  // from here on the maximum is in the exponent's (log2) domain
    if (C::KG > 1) {
      float *mg = reinterpret_cast<float *>(smem);
      if (kg > 0) {
        float *slot = mg + (size_t)((kg - 1) * TG + tg) * 66 * 64;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) slot[(mb * 16 + r) * 64 + lane] = o_acc[mb][r];
        slot[64 * 64 + lane] = m_run;
        slot[65 * 64 + lane] = l_run;
      }
      __syncthreads();
      if (kg == 0) {
#pragma unroll
        for (int k2 = 1; k2 < C::KG; ++k2) {
          const float *slot = mg + (size_t)((k2 - 1) * TG + tg) * 66 * 64;
          const float m2 = slot[64 * 64 + lane], l2 = slot[65 * 64 + lane];
          const float m_new = fmaxf(m_run, m2);
          const float m_safe = m_new == -INFINITY ? 0.f : m_new;
          const float a1 = fast_exp2(m_run - m_safe), a2 = fast_exp2(m2 - m_safe);
          l_run = l_run * a1 + l2 * a2;
          m_run = m_new;
#pragma unroll
          for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              o_acc[mb][r] = o_acc[mb][r] * a1 + slot[(mb * 16 + r) * 64 + lane] * a2;
        }
      }
      __syncthreads();  // the buffers are reused by the next segment
    }

    // ---- write: lane holds d = mb*32 + 8*(r/4) + 4*g + r%4 for its query t
    if (kg == 0 && t < T) {
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
        const size_t slot = 2 * (size_t)w + (tile0 > 0 ? 0 : 1);
        float *po = p.part_o + (slot * 128 + t) * kD;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const f32x4 w4 = {o_acc[mb][4 * q4], o_acc[mb][4 * q4 + 1], o_acc[mb][4 * q4 + 2],
                              o_acc[mb][4 * q4 + 3]};
            *reinterpret_cast<f32x4 *>(po + mb * 32 + 8 * q4 + 4 * g) = w4;
          }
        if (g == 0) {
          p.part_ml[(slot * 128 + t) * 2] = m_run;
          p.part_ml[(slot * 128 + t) * 2 + 1] = l_run;
        }
      }
    }
    x += n_tiles;
  }
}

// Finish the units that a range boundary cut: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s
// over the workgroups s that hold a piece.  One workgroup per unit; whole units return at once.
template <int TILE_J>
__global__ __launch_bounds__(kAttnThreads) void tree_attn_combine_kernel(AttnParams p, int G) {
  const int unit = blockIdx.x;
  const int b = unit / p.H, h = unit - b * p.H;
  const TileMap<TILE_J> map = {p.B, p.H, p.seq_lens, p.n_nodes, p.L_max, p.T_max};
  long long n_total = 0, b_start = 0;
  for (int bb = 0; bb < p.B; ++bb) {
    if (bb == b) b_start = n_total;
    n_total += (long long)p.H * map.unit_tiles(bb);
  }
  const int ut = map.unit_tiles(b), T = map.nodes(b);
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
static int pick_tg(int T_max) { return T_max <= 32 ? 1 : (T_max <= 64 ? 2 : 4); }

static int tile_rows(int tg) { return tg == 1 ? AttnCfg<1>::TILE_J : AttnCfg<4>::TILE_J; }

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

// Workgroups of the persistent kernel: two per compute unit (what LDS and registers
// allow to be resident), fewer when the whole call has fewer than two tiles per workgroup.
static int pick_grid(int B, int H, int L_max, int T_max) {
  const int tile = tile_rows(pick_tg(T_max));
  const long long per_unit = (L_max + tile - 1) / tile + (T_max + tile - 1) / tile;
  const long long tiles = (long long)B * H * per_unit;
  long long grid = 2ll * compute_units();
  if (grid > kMaxGrid) grid = kMaxGrid;
  if (grid > (tiles + 1) / 2) grid = (tiles + 1) / 2;
  return (int)(grid < 1 ? 1 : grid);
}

// Partial slots: two per workgroup of the grid this call will use.
size_t tree_attention_workspace_bytes(int B, int H, int L_max, int T_max) {
  const size_t slots = 2 * (size_t)pick_grid(B, H, L_max, T_max);
  return align_up(slots * 128 * kD * 4, 256) + align_up(slots * 128 * 2 * 4, 256);
}

template <int TG>
static bool launch_bf16(const AttnParams &p, int grid, int units, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_attn_bf16_kernel<TG>),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)AttnCfg<TG>::lds_bytes) != hipSuccess)
      return false;
    attr_set = true;
  }
  hipLaunchKernelGGL(tree_attn_bf16_kernel<TG>, dim3((unsigned)grid), dim3(kAttnThreads),
                     AttnCfg<TG>::lds_bytes, st, p);
  if (!launch_ok()) return false;
  hipLaunchKernelGGL(tree_attn_combine_kernel<AttnCfg<TG>::TILE_J>, dim3((unsigned)units),
                     dim3(kAttnThreads), 0, st, p, grid);
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
  bool ok;
  switch (pick_tg(tree->T_max)) {
    case 1: ok = launch_bf16<1>(p, grid, (int)units, st); break;
    case 2: ok = launch_bf16<2>(p, grid, (int)units, st); break;
    default: ok = launch_bf16<4>(p, grid, (int)units, st); break;
  }
  if (!ok) return PROPD_ERR_DEVICE;
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
