// Shared device helpers for the gfx950 kernels (wave64, CDNA4).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/propd.h"

namespace propd {

constexpr int kWave = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) {
  return __uint_as_float(b << 16);
}

// Round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

template <typename T>
__device__ __forceinline__ T wave_reduce_max(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    T other = __shfl_xor(v, o, kWave);
    v = other > v ? other : v;
  }
  return v;
}

template <typename T>
__device__ __forceinline__ T wave_reduce_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Bits of a 128-bit set strictly below position i (0 <= i <= 128).
__device__ __forceinline__ void mask_below(int i, uint64_t &lo, uint64_t &hi) {
  lo = i >= 64 ? ~0ull : ((1ull << i) - 1ull);
  hi = i <= 64 ? 0ull : (i >= 128 ? ~0ull : ((1ull << (i - 64)) - 1ull));
}

__device__ __forceinline__ int popc128_below(uint64_t lo, uint64_t hi, int i) {
  uint64_t ml, mh;
  mask_below(i, ml, mh);
  return __popcll(lo & ml) + __popcll(hi & mh);
}

__device__ __forceinline__ bool test_bit128(uint64_t lo, uint64_t hi, int j) {
  return ((j < 64 ? (lo >> j) : (hi >> (j - 64))) & 1ull) != 0;
}

// Results of an MFMA chain are read by vector ALU code right after it.  Observed on
// gfx950 with this toolchain: when a branch sits between the last MFMA and the first
// read, the reads can be issued before the matrix core has written the registers
// back (stale accumulator values, no error).  An explicit wait covering the longest
// MFMA used here (8 passes of 4 cycles) closes the window; the scheduling barriers
// keep the compiler from moving either side across it.
__device__ __forceinline__ void mfma_settle() {
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline bool launch_ok() { return hipGetLastError() == hipSuccess; }

// scratch sizes (host arithmetic), defined next to the kernels that use the scratch
size_t early_prune_workspace_bytes(int B, int T_max, int vocab);
size_t tree_attention_workspace_bytes(int B, int H, int L_max, int T_max);
size_t accept_path_workspace_bytes(int B, int T_max);

}  // namespace propd
