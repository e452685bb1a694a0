// Early-head scoring, second tile shape: 352 rows x 256 vocabulary entries per workgroup.
// Included by early_prune.hip inside namespace propd, after the helpers it uses.
//
// Why a second shape.  The scoring GEMM has few rows (the nodes that have children: 704 at
// B = 16, T = 128) against a wide vocabulary, and it is bound by operand delivery, not by the
// matrix cores.  With 256-row tiles those 704 rows need three row tiles (8 % padding) and
// 501 workgroups, two rounds of the chip.  Two 352-row tiles have no padding, 250 workgroups
// of 352 x 256 fill the 256 compute units in ONE round, every weight tile is fetched by two
// workgroups instead of three, and a workgroup moves (352 + 256) / (352 * 256) operand
// bytes per output instead of (256 + 192) / (256 * 192): 26 % fewer bytes into LDS and 18 %
// fewer out of it per FLOP.  The accumulators (352 x 256 fp32 = 360 KB) take 176 registers
// in each of the 8 waves, which leaves room for operands only if they are streamed.
//   - 8 waves as 2 (rows) x 4 (columns), a wave owns 176 x 64 as 11 x 4 tiles of the
//     16x16x32 bf16 MFMA (176 = 11 x 16 is no multiple of 32);
//   - K advances 32 per step through a ring of four 38 KB LDS stages (352 + 256 rows of 64
//     bytes), filled by direct global->LDS loads three steps ahead.  The 16-byte chunks of a
//     row are XOR-swizzled with key(row) = (row >> 1) & 3: a fragment read of this MFMA has
//     lane -> (row lane % 16, chunk lane / 16), and with the other shape's key (row >> 2) & 3
//     every such read took twice its time in bank conflicts (measured: 64 against 38 ticks);
//   - per step a wave reads its four B fragments and then streams the eleven A fragments
//     through a four-deep register ring: the read of fragment i + 3 is issued behind the four
//     MFMAs of fragment i, waits are placed by hand (LDS reads return in order);
//   - the epilogues are the same two as for the other shape, on this accumulator layout: a
//     row of the tile lives in the 16 lanes of a quarter wave (column = lane % 16 + 16 j), a
//     lane holds rows 16 i + 4 (lane / 16) + r.
#pragma once

constexpr int kTallBM = 352, kTallBN = 256, kTallStages = 4;
constexpr int kTallWaveRows = kTallBM / 2, kTallWaveCols = kTallBN / 4;  // 176 x 64
constexpr int kTallMI = kTallWaveRows / 16, kTallNJ = kTallWaveCols / 16;  // 11 x 4 MFMA tiles
constexpr int kTallRows = kTallBM + kTallBN;                 // LDS rows of a stage
constexpr int kTallStageBytes = kTallRows * kGemmRowBytes;   // 38912
constexpr int kTallLdsBytes = kTallStages * kTallStageBytes; // 155648
constexpr int kTallGroups = kTallRows / 16;                  // 16-row groups, one load instruction each
constexpr int kTallAGroups = kTallBM / 16;
constexpr int kTallEpiChildren = 12;                         // children of a row per epilogue pass
static_assert(kTallLdsBytes <= 160 * 1024, "ring");

template <int N>
__device__ __forceinline__ void tall_wait_lds(u32x4 &a) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N));
}
template <int N>
__device__ __forceinline__ void tall_wait_lds5(u32x4 &a, u32x4 &b0, u32x4 &b1, u32x4 &b2, u32x4 &b3) {
  asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(a), "+v"(b0), "+v"(b1), "+v"(b2), "+v"(b3) : "n"(N));
}

// Waits until at most n of this wave's loads are outstanding (n = whole steps of 4 or 5 loads).
__device__ __forceinline__ void tall_wait_outstanding(int n) {
  if (n >= 10) gemm_wait_vmem<10>();
  else if (n >= 8) gemm_wait_vmem<8>();
  else if (n >= 5) gemm_wait_vmem<5>();
  else if (n >= 4) gemm_wait_vmem<4>();
  else gemm_wait_vmem<0>();
}

typedef f32x4 TallAcc[kTallMI][kTallNJ];

// LDS accesses with the row's offset as an immediate of the instruction: one address register
// serves all rows of a lane.  (Left to itself the compiler materialises an address per row,
// keeps all of them across the passes and spills the accumulators for it.)
template <int OFFSET>
__device__ __forceinline__ uint32_t tall_lds_read4(uint32_t addr) {
  uint32_t r;
  asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET));
  return r;
}
template <int OFFSET>
__device__ __forceinline__ void tall_lds_write4(uint32_t addr, uint32_t v) {
  asm volatile("ds_write_b32 %0, %1 offset:%2" ::"v"(addr), "v"(v), "n"(OFFSET) : "memory");
}
__device__ __forceinline__ void tall_wait_row(uint32_t &meta, u32x4 &thr) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(meta), "+v"(thr));
}
__device__ __forceinline__ int opaque(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

// Sum over the 16 lanes of each quarter wave, left in lanes 15, 31, 47 and 63.
__device__ __forceinline__ int quarter_wave_sum_to_last(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);  // row_shr:8
  return v;
}

// Counting epilogue on the 16x16 accumulator layout; the method is that of epilogue_count.
__device__ __forceinline__ void tall_epilogue_count(TallAcc &acc, int m0, int v0, int n_tile, int vocab,
                                                    int tid_in, int my_pos, int my_cc,
                                                    const HeadTables &tb, unsigned char *smem) {
  constexpr int BM = kTallBM, WN = kTallWaveCols, E = kTallEpiChildren, NW = 4;
  static_assert(E % 4 == 0 && WN < 256, "four byte-sized counts per word");
  int tid = tid_in;  // see epilogue_count: keeps the addresses below out of the K loop
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, c16 = lane & 15, q = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave >> 2, wn = wave & 3;
  int *s_max = reinterpret_cast<int *>(smem);
  int *s_cc = s_max + 64;                                // [BM] children in this pass | flags << 8
  int *s_pos = s_cc + BM;                                // [BM]
  float *s_thr = reinterpret_cast<float *>(s_pos + BM);  // [NW][BM][E]
  float *s_own = s_thr + NW * BM * E;                    // [BM][E]
  int *s_tok = reinterpret_cast<int *>(s_own + BM * E);  // [BM][E]
  int *s_node = s_tok + BM * E;                          // [BM][E]
  int *s_count = s_node + BM * E;                        // [NW][BM][E/4]
  static_assert((64 + 2 * BM + (NW + 3) * BM * E + NW * BM * (E / 4)) * 4 <= kTallLdsBytes, "epilogue tables");
  if (v0 + kTallBN > vocab) {  // columns past the vocabulary can beat nothing
#pragma unroll
    for (int j = 0; j < kTallNJ; ++j) {
      const bool out = v0 + wn * WN + 16 * j + c16 >= vocab;
#pragma unroll
      for (int i = 0; i < kTallMI; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][j][r] = out ? -INFINITY : acc[i][j][r];
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
  const int row0 = wm * kTallWaveRows + 4 * q;  // this lane's rows: row0 + 16 i + r
  for (int e0 = 0; e0 < max_cc; e0 += E) {
    if (tid < BM) {
      int n = my_cc - e0;
      s_cc[tid] = n < 0 ? 0 : (n > E ? E : n);
      s_pos[tid] = my_pos + e0;
    }
    __syncthreads();
    {
      constexpr int kSlots = (BM * E + kGemmThreads - 1) / kGemmThreads, kChunk = 3;
      static_assert(kSlots % kChunk == 0, "slots per thread");
#pragma unroll 1  // three slots at a time: more would not fit beside the accumulators
      for (int j0 = 0; j0 < kSlots; j0 += kChunk) {
        int c[kChunk], t[kChunk];
        float o[kChunk];
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
          const int slot = tid + kGemmThreads * (j0 + j), row = slot / E, e = slot - row * E;
          c[j] = (slot < BM * E && e < (s_cc[row] & 255)) ? tb.child_list[s_pos[row] + e] : -1;
        }
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
          t[j] = c[j] >= 0 ? tb.token[c[j]] : -1;
          o[j] = c[j] >= 0 ? tb.own[c[j]] : INFINITY;
        }
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
          const int slot = tid + kGemmThreads * (j0 + j), row = slot / E;
          if (slot < BM * E) {
            const bool ok = t[j] >= 0 && t[j] < vocab;
            s_own[slot] = ok ? o[j] : INFINITY;
            s_tok[slot] = ok ? t[j] : -1;
            s_node[slot] = c[j];
#pragma unroll
            for (int w4 = 0; w4 < NW; ++w4) {
              const int c0 = v0 + w4 * WN;
              float thr = INFINITY;
              if (ok) {
                const bool inside = t[j] >= c0 && t[j] < c0 + WN;
                thr = t[j] < c0 ? o[j] : (inside ? __uint_as_float(0x7fc00000u) : float_pred(o[j]));
                if (inside) atomicOr(&s_cc[row], 256 << w4);
              }
              s_thr[w4 * BM * E + slot] = thr;
            }
          }
        }
      }
    }
    __syncthreads();
    // this lane's 44 rows in the order (i, r)
    typedef __attribute__((address_space(3))) void lds_void;
    const uint32_t cc_addr = (uint32_t)(uintptr_t)(lds_void *)(s_cc + row0);
    const uint32_t thr_addr = (uint32_t)(uintptr_t)(lds_void *)(s_thr + wn * BM * E + row0 * E);
    const uint32_t count_addr = (uint32_t)(uintptr_t)(lds_void *)(s_count + wn * BM * (E / 4) + row0 * (E / 4));
    static_for<kTallMI * 4>([&](auto idx_c) {
      constexpr int idx = decltype(idx_c)::value;
      constexpr int i = idx >> 2, r = idx & 3, off = 16 * i + r;
      uint32_t meta = tall_lds_read4<off * 4>(cc_addr);
      u32x4 thr_u = gemm_lds_read16<off * E * 4>(thr_addr);
      tall_wait_row(meta, thr_u);
      f32x4 thr4 = __builtin_bit_cast(f32x4, thr_u);
      const int m0q = __builtin_amdgcn_readlane((int)meta, 0), m1q = __builtin_amdgcn_readlane((int)meta, 16);
      const int m2q = __builtin_amdgcn_readlane((int)meta, 32), m3q = __builtin_amdgcn_readlane((int)meta, 48);
      int n_all = m0q & 255;
      n_all = (m1q & 255) > n_all ? (m1q & 255) : n_all;
      n_all = (m2q & 255) > n_all ? (m2q & 255) : n_all;
      n_all = (m3q & 255) > n_all ? (m3q & 255) : n_all;
      const bool side_path = (((m0q | m1q | m2q | m3q) >> (8 + wn)) & 1) != 0;
      for (int e4 = 0; e4 < n_all; e4 += 4) {
        if (e4 > 0) thr4 = *reinterpret_cast<const f32x4 *>(s_thr + wn * BM * E + (row0 + opaque(off)) * E + e4);
        int packed = 0;
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) {
          const float thr = thr4[j4];
          int cnt = 0;
#pragma unroll
          for (int j = 0; j < kTallNJ; ++j) cnt += acc[i][j][r] > thr ? 1 : 0;
          if (side_path && thr != thr) {
            const int ent = (row0 + opaque(off)) * E + e4 + j4;
            const float own = s_own[ent];
            const int tok = s_tok[ent];
#pragma unroll
            for (int j = 0; j < kTallNJ; ++j) {
              const int col = v0 + wn * WN + 16 * j + c16;
              const float z = acc[i][j][r];
              cnt += (col != tok && (z > own || (z == own && col < tok))) ? 1 : 0;
            }
          }
          packed += cnt << (8 * j4);
        }
        packed = quarter_wave_sum_to_last(packed);
        if (c16 == 15) {
          if (e4 == 0) tall_lds_write4<off * (E / 4) * 4>(count_addr, (uint32_t)packed);
          else s_count[wn * BM * (E / 4) + (row0 + opaque(off)) * (E / 4) + (e4 >> 2)] = packed;
        }
      }
    });
    __syncthreads();
    for (int slot = tid; slot < BM * E; slot += kGemmThreads) {
      const int c = s_node[slot];
      if (c >= 0) {
        const int word = slot >> 2, sh = 8 * (slot & 3);
        int cnt = 0;
#pragma unroll
        for (int w4 = 0; w4 < NW; ++w4) cnt += (s_count[w4 * BM * (E / 4) + word] >> sh) & 255;
        tb.cnt_part[(size_t)n_tile * tb.cnt_stride + c] = cnt;
      }
    }
    __syncthreads();  // the next pass, or the next tile's loads, reuse this memory
  }
}

// (max, sum of exponentials) per row and wave column, four column parts per tile
__device__ __forceinline__ void tall_epilogue_lse(const TallAcc &acc, int m0, int v0, int m_total, int vocab,
                                                  int n_tile, int wm, int wn, int lane, const HeadTables &tb) {
  const int c16 = lane & 15, q = lane >> 4;
#pragma unroll
  for (int i = 0; i < kTallMI; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < kTallNJ; ++j)
        if (v0 + wn * kTallWaveCols + 16 * j + c16 < vocab) mx = fmaxf(mx, acc[i][j][r]);
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, kWave));
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < kTallNJ; ++j)
        if (v0 + wn * kTallWaveCols + 16 * j + c16 < vocab) sum += expf(acc[i][j][r] - mx);
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o, kWave);
      const int m = m0 + wm * kTallWaveRows + 16 * i + 4 * q + r;
      if (c16 == 0 && m < m_total) {
        float *dst = tb.lse_part + ((size_t)m * tb.parts + 4 * n_tile + wn) * 2;
        dst[0] = mx;
        dst[1] = sum;
      }
    }
}

template <int KIND>
__device__ __forceinline__ void early_head_tall_tile(
    int hidden, int vocab, int m_total, int m0, int v0, int n_tile,
    const uint16_t *__restrict__ hidden_states, const uint16_t *__restrict__ head_weight,
    const HeadTables &tb, unsigned char *smem) {
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void global_void;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void *)smem;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  int my_pos = 0, my_cc = 0;
  if (KIND == 0 && tid < kTallBM && m0 + tid < m_total) {
    my_pos = tb.row_info[2 * (m0 + tid)];
    my_cc = tb.row_info[2 * (m0 + tid) + 1];
  }

  // ---- loader: group gi = wave + 8 j (16 rows, 1 KB) for j = 0 .. n_groups - 1
  const int ld_row = lane >> 2;
  const int ld_chunk = ((lane & 3) ^ ((lane >> 3) & 3)) << 4;  // byte offset in the global row: chunk ^ key(row)
  const int n_groups = wave + 32 < kTallGroups ? 5 : 4;         // loads of this wave per K step
  const unsigned char *src[5];
#pragma unroll
  for (int j = 0; j < 5; ++j) {
    const int gi = wave + 8 * j;
    if (gi < kTallAGroups) {
      int m = m0 + 16 * gi + ld_row;
      m = m < m_total ? m : m_total - 1;
      src[j] = reinterpret_cast<const unsigned char *>(hidden_states + (size_t)tb.row_src[m] * hidden) + ld_chunk;
    } else {
      int v = v0 + 16 * (gi - kTallAGroups) + ld_row;
      v = v < vocab ? v : vocab - 1;
      src[j] = reinterpret_cast<const unsigned char *>(head_weight + (size_t)v * hidden) + ld_chunk;
    }
  }
  int k_off = 0;  // bytes into the rows of the next step to issue
  auto issue = [&](int slot) {
    unsigned char *dst = smem + slot * kTallStageBytes + wave * 1024;
#pragma unroll
    for (int j = 0; j < 5; ++j)
      if (j < n_groups)
        __builtin_amdgcn_global_load_lds((global_void *)(src[j] + k_off), (lds_void *)(dst + j * 8192), 16, 0, 0);
    k_off += kGemmRowBytes;
  };

  // ---- per-lane LDS read addresses: row lane % 16 of a 16-row block, chunk lane / 16 (swizzled)
  const int c16 = lane & 15, kq = lane >> 4;
  const uint32_t frag_off = c16 * kGemmRowBytes + ((kq ^ ((c16 >> 1) & 3)) << 4);
  const uint32_t a_rd = smem_base + wm * kTallWaveRows * kGemmRowBytes + frag_off;
  const uint32_t b_rd = smem_base + (kTallBM + wn * kTallWaveCols) * kGemmRowBytes + frag_off;

  TallAcc acc;
#pragma unroll
  for (int i = 0; i < kTallMI; ++i)
#pragma unroll
    for (int j = 0; j < kTallNJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // The ring: the step being multiplied, the next one (landed or landing) and one or two more
  // in flight.  The loads of step s + 3 are issued in the MIDDLE of step s, into the slot that
  // step s - 1 left at the last barrier: the address arithmetic and the issue then run in the
  // shadow of this wave's queued MFMAs instead of right after the barrier, where every wave
  // of the workgroup would do them at the same time with the matrix cores idle.
  const int n_steps = hidden / kBK;
  const int n_pro = n_steps < kTallStages - 1 ? n_steps : kTallStages - 1;
  int slot_ld = 0;
  for (int i = 0; i < n_pro; ++i) {
    issue(slot_ld);
    slot_ld = slot_ld + 1 == kTallStages ? 0 : slot_ld + 1;
  }
  tall_wait_outstanding((n_pro - 1) * n_groups);
  __builtin_amdgcn_s_barrier();
  uint32_t so = 0;  // byte offset of the stage being multiplied
  for (int step = 0; step < n_steps; ++step) {
    const uint32_t pa = a_rd + so, pb = b_rd + so;
    u32x4 bf[kTallNJ], af[4];
    // the first product needs only A0 and B0: they are read first
    af[0] = gemm_lds_read16<0>(pa);
    bf[0] = gemm_lds_read16<0>(pb);
    bf[1] = gemm_lds_read16<1024>(pb);
    bf[2] = gemm_lds_read16<2048>(pb);
    bf[3] = gemm_lds_read16<3072>(pb);
    af[1] = gemm_lds_read16<1024>(pa);
    af[2] = gemm_lds_read16<2048>(pa);
    tall_wait_lds5<5>(af[0], bf[0], bf[1], bf[2], bf[3]);  // A0, B0 (the B registers are only named)
    acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[0]),
                                                        __builtin_bit_cast(bf16x8, bf[0]), acc[0][0], 0, 0, 0);
    static_for<kTallMI>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      constexpr int allowed = kTallMI - 1 - i < 2 ? kTallMI - 1 - i : 2;  // younger A reads in flight
      if (i == 0) tall_wait_lds5<allowed>(af[0], bf[0], bf[1], bf[2], bf[3]);
      else tall_wait_lds<allowed>(af[i & 3]);
#pragma unroll
      for (int j = (i == 0 ? 1 : 0); j < kTallNJ; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[i & 3]),
                                                            __builtin_bit_cast(bf16x8, bf[j]), acc[i][j], 0, 0, 0);
      if (i + 3 < kTallMI) af[(i + 3) & 3] = gemm_lds_read16<(i + 3) * 1024>(pa);
      if (i == 4 && step + kTallStages - 1 < n_steps) {
        issue(slot_ld);  // step + 3, into the slot of step - 1
        slot_ld = slot_ld + 1 == kTallStages ? 0 : slot_ld + 1;
      }
    });
    if (step + 1 < n_steps) {
      // this wave has read everything of this step's slot; the next step has landed once at
      // most the steps after it that were issued (up to two) are outstanding
      const int issued_after = n_steps - 2 - step < kTallStages - 2 ? n_steps - 2 - step : kTallStages - 2;
      tall_wait_outstanding(issued_after * n_groups);
      __builtin_amdgcn_s_barrier();  // it is visible; every wave is done with this step's slot
      so = so + kTallStageBytes == kTallStages * kTallStageBytes ? 0 : so + kTallStageBytes;
    }
  }
  mfma_settle();
  if (KIND == 0) tall_epilogue_count(acc, m0, v0, n_tile, vocab, tid, my_pos, my_cc, tb, smem);
  else tall_epilogue_lse(acc, m0, v0, m_total, vocab, n_tile, wm, wn, lane, tb);
}
