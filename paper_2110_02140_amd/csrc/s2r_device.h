// Device-side building blocks shared by the gfx950 kernels of the sparse-sketch
// codec: the row hashes (Section 3.1: bucket hash h, sign hash s), wave64
// helpers, and the single-pass chained prefix ("decoupled look-back") that gives
// every tile the number of selected items before it, so that index lists come
// out ascending without a second pass over the input.
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

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += (uint64_t)__shfl_xor((unsigned long long)x, off, kWave);
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

// ---------------------------------------------------------------------------
// Chained prefix over tiles.
//
// status[t] packs a 2-bit flag (bits 63..62) and a 62-bit value in one word, so
// one relaxed 64-bit atomic carries both and no ordering between two locations
// is needed.  A tile first publishes AGGREGATE(its own count), then walks back
// over its predecessors, a wave-wide window of 64 tiles at a time, summing
// aggregates until it meets a PREFIX (inclusive count up to and including that
// tile), and finally publishes its own PREFIX.  Tile ids are handed out by an
// atomic counter in launch order, so every predecessor of a running tile has
// itself started and publishes its aggregate without waiting for anybody: the
// waits below end.  As a second line of defence each wait is bounded; if the
// bound is ever hit the caller poisons its count output instead of hanging.
// ---------------------------------------------------------------------------
constexpr uint64_t kFlagEmpty = 0, kFlagAggregate = 1, kFlagPrefix = 2;
constexpr uint64_t kValueMask = (1ull << 62) - 1;
constexpr uint32_t kSpinLimit = 1u << 22;

__device__ __forceinline__ void status_store(uint64_t* p, uint64_t flag, uint64_t value) {
  __hip_atomic_store(p, (flag << 62) | value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t status_load(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by all 64 lanes of one wave.  Publishes the tile's aggregate, returns
// the exclusive prefix (same value in every lane), publishes the inclusive
// prefix.  *timed_out is set (by any lane) if a bounded wait gave up.
__device__ __forceinline__ uint64_t chained_exclusive_prefix(uint64_t* status, uint32_t tile,
                                                             uint64_t aggregate, bool* timed_out) {
  const uint32_t lane = lane_id();
  if (tile == 0) {
    if (lane == 0) status_store(&status[0], kFlagPrefix, aggregate);
    return 0;
  }
  if (lane == 0) status_store(&status[tile], kFlagAggregate, aggregate);
  uint64_t excl = 0;
  int64_t window_end = (int64_t)tile - 1;          // newest tile of the current window
  bool bad = false;
  while (true) {
    const int64_t t = window_end - (int64_t)lane;  // lane 0 looks at the nearest predecessor
    uint64_t s = (kFlagPrefix << 62);              // tiles before 0: prefix 0
    if (t >= 0) {
      uint32_t spins = 0;
      s = status_load(&status[t]);
      while ((s >> 62) == kFlagEmpty) {
        if (++spins > kSpinLimit) { bad = true; s = (kFlagPrefix << 62); break; }
        __builtin_amdgcn_s_sleep(1);
        s = status_load(&status[t]);
      }
    }
    const uint64_t has_prefix = __ballot((s >> 62) == kFlagPrefix);
    // lanes up to and including the nearest PREFIX contribute
    const uint32_t first = has_prefix ? (uint32_t)__ffsll((unsigned long long)has_prefix) - 1u : 63u;
    excl += wave_sum_u64(lane <= first ? (s & kValueMask) : 0ull);
    if (has_prefix) break;
    window_end -= kWave;
  }
  if (__ballot(bad)) *timed_out = true;
  if (lane == 0) status_store(&status[tile], kFlagPrefix, excl + aggregate);
  return excl;
}

}  // namespace s2r
