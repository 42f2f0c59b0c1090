// Device-side building blocks shared by the gfx950 kernels of the sparse-sketch
// codec: the row hashes (Section 3.1: bucket hash h, sign hash s) and wave64
// helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s2r {

constexpr int kWave = 64;
constexpr int kMaxRows = 16;

// Hash parameters of all rows, passed to kernels by value (kernarg, read with
// scalar loads).  Row j: bucket h_j(i) = (a[j]*i + b[j]) >> (64 - log2 w),
// sign s_j(i) = bit 63 of (c[j]*i + e[j]).
struct HashRows {
  uint64_t a[kMaxRows];
  uint64_t b[kMaxRows];
  uint64_t c[kMaxRows];
  uint64_t e[kMaxRows];
};

// Bucket of index i in a row with parameters (a, b); log2w in [0, 31].
__device__ __forceinline__ uint32_t bucket_of(uint32_t i, uint64_t a, uint64_t b, uint32_t log2w) {
  const uint64_t u = a * (uint64_t)i + b;
  return (uint32_t)((u >> 32) >> (32u - log2w));   // shift count 1..32 on a 64-bit operand
}

// 0x80000000 if s(i) = -1, else 0: XOR it into the float's bit pattern.
__device__ __forceinline__ uint32_t signbit_of(uint32_t i, uint64_t c, uint64_t e) {
  const uint64_t v = c * (uint64_t)i + e;
  return (uint32_t)(v >> 32) & 0x80000000u;
}

__device__ __forceinline__ uint32_t lane_id() {
  return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Number of set bits of m at positions below the calling lane.
__device__ __forceinline__ uint32_t bits_below_lane(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t x, uint32_t lane) {
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint32_t t = __shfl_up(x, off, kWave);
    if (lane >= (uint32_t)off) x += t;
  }
  return x;
}

// Position (0..63) of the r-th (0-based) set bit of m; r < popcount(m).
__device__ __forceinline__ uint32_t select_bit(uint64_t m, uint32_t r) {
  uint32_t x = (uint32_t)m, pos = 0;
  const uint32_t pl = __popc(x);
  if (r >= pl) { x = (uint32_t)(m >> 32); r -= pl; pos = 32; }
#pragma unroll
  for (int sh = 16; sh >= 1; sh >>= 1) {
    const uint32_t c = __popc(x & ((1u << sh) - 1u));
    if (r >= c) { x >>= sh; r -= c; pos += sh; }
  }
  return pos;
}

}  // namespace s2r
