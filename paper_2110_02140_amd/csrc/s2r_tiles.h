// From a bitmap to ascending lists without any workgroup waiting for another:
// per-piece popcounts, the prefix over the tiles, a bitmap tile in LDS, and the
// expansion Sparse(g) (indices, and values gathered at the set bits).
// Included by s2r_kernels.hip only (one translation unit).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/s2r.h"
#include "s2r_layout.h"

namespace s2r {

// ------------------------------------------------------------------ per-piece popcounts (decode)
// One wave per tile: lane l reads words l, l + 64, ... of the tile (coalesced), so
// word q of a lane belongs to piece 2q (lanes 0..31) or 2q + 1 (lanes 32..63).
// The eight popcounts travel as four pairs of 16-bit fields through a butterfly
// over each half of the wave (a field holds at most 32 * 64); lane 0 then owns
// the even pieces, fetches the odd ones from lane 32 and stores the tile's 16
// counts as 32 contiguous bytes.
__device__ __forceinline__ void count_tile_pieces(const uint64_t* __restrict__ bitmap, uint64_t nwords, uint32_t ntiles,
                                                  uint16_t* __restrict__ piece_count) {
  constexpr int kPer = kTileWords / kWave;                   // 8
  static_assert(kScanWords == kWave / 2 && kScansPerTile == 2 * kPer, "a piece is the words of half a wave");
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t tile = blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  if (tile >= ntiles) return;                                // uniform over the wave
  const uint64_t w0 = (uint64_t)tile * kTileWords;
  uint32_t pk[kPer / 2];
#pragma unroll
  for (int r = 0; r < kPer / 2; ++r) {
    const uint64_t wa = w0 + (2 * r) * kWave + lane, wb = wa + kWave;
    const uint32_t ca = wa < nwords ? (uint32_t)__popcll(bitmap[wa]) : 0u;
    const uint32_t cb = wb < nwords ? (uint32_t)__popcll(bitmap[wb]) : 0u;
    pk[r] = ca | (cb << 16);
  }
#pragma unroll
  for (int step = 1; step < kWave / 2; step <<= 1) {
#pragma unroll
    for (int r = 0; r < kPer / 2; ++r) pk[r] += (uint32_t)__shfl_xor((int)pk[r], step);
  }
  uint32_t odd[kPer / 2];
#pragma unroll
  for (int r = 0; r < kPer / 2; ++r) odd[r] = (uint32_t)__shfl_xor((int)pk[r], kWave / 2);
  if (lane == 0) {
    uint32_t o[kPer];                                        // o[q] = piece 2q | piece 2q + 1 << 16
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      const uint32_t sh = 16u * (q & 1);
      o[q] = ((pk[q / 2] >> sh) & 0xFFFFu) | (((odd[q / 2] >> sh) & 0xFFFFu) << 16);
    }
    uint4* dst = reinterpret_cast<uint4*>(piece_count + (uint64_t)tile * kScansPerTile);    // 32-byte aligned
    dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
    dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
  }
}

__global__ __launch_bounds__(kBlock) void bitmap_count_kernel(const uint64_t* __restrict__ bitmap, uint64_t nwords,
                                                              uint32_t ntiles, uint16_t* __restrict__ piece_count) {
  count_tile_pieces(bitmap, nwords, ntiles, piece_count);
}

// The same for the (block) bitmaps of the workers of an encode batch.
__global__ __launch_bounds__(kBlock) void bitmap_count_batch_kernel(const EncodeBatch B) {
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;
  count_tile_pieces(B.w[k].bitmap, B.nwords, B.ntiles, ws_piece_count(B, k));
}

// ------------------------------------------------------------------ prefix of the tile counts
// Single workgroup.  A tile's count is the sum of its kScansPerTile 16-bit piece
// counts (32 bytes, two 16-byte loads).  prefix[t] = sum of the counts of tiles
// 0..t-1, prefix[ntiles] = total, also written to *total_out.  A round covers
// kPrefixPer rows of 1024 consecutive tiles; thread t owns column t of every row,
// and its 2 * kPrefixPer loads are in flight together.  Each row is scanned inside
// its waves, the kPrefixPer x 16 wave totals are scanned by wave 0, and every
// element adds the offset of its (row, wave).  n <= 2^32 gives at most 2^17 tiles:
// sixteen rounds.
// Tiles with more than kGroupSlots set bits are also entered in the problem's
// dense-tile list: one entry (tile | group << 20) for every further group of
// kGroupSlots list positions, in arbitrary order, preceded by the entry count
// (at dense_off: the count, 256 bytes later the entries).  The expansion kernels
// give each entry a workgroup of its own.
// blockIdx.y selects one of several independent problems (the workers of an
// encode batch): its piece counts are at ws + y*ws_stride, its prefix at
// prefix_off bytes after them, its total at total_out[y].
__device__ __forceinline__ uint32_t sum_u16x8(const uint4 x) {
  const uint32_t lo = (x.x & 0xFFFFu) + (x.y & 0xFFFFu) + (x.z & 0xFFFFu) + (x.w & 0xFFFFu);
  const uint32_t hi = (x.x >> 16) + (x.y >> 16) + (x.z >> 16) + (x.w >> 16);
  return lo + hi;
}

__global__ __launch_bounds__(kPrefixBlock) void tile_prefix_kernel(char* __restrict__ ws, uint64_t ws_stride,
                                                                   uint64_t prefix_off, uint64_t dense_off,
                                                                   uint32_t ntiles, uint64_t* __restrict__ total_out) {
  const uint4* __restrict__ pieces = reinterpret_cast<const uint4*>(ws + blockIdx.y * ws_stride);
  uint64_t* __restrict__ prefix = reinterpret_cast<uint64_t*>(ws + blockIdx.y * ws_stride + prefix_off);
  uint32_t* __restrict__ dense_count = reinterpret_cast<uint32_t*>(ws + blockIdx.y * ws_stride + dense_off);
  uint32_t* __restrict__ dense_list = dense_count + 64;
  __shared__ uint32_t s_dense;
  if (threadIdx.x == 0) s_dense = 0u;
  __syncthreads();
  constexpr int kWaves = kPrefixBlock / kWave;               // 16
  constexpr int kCells = kPrefixPer * kWaves;                // (row, wave) totals per round
  constexpr int kPerLane = kCells / kWave;
  static_assert(kCells % kWave == 0, "wave 0 scans the totals, kPerLane per lane");
  __shared__ uint32_t s_tot[kCells + 1];
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  uint64_t carry = 0;
  for (uint32_t base = 0; base < ntiles; base += kPrefixBlock * kPrefixPer) {
    uint4 lo16[kPrefixPer], hi16[kPrefixPer];
    uint32_t c[kPrefixPer], incl[kPrefixPer];
#pragma unroll
    for (int q = 0; q < kPrefixPer; ++q) {
      const uint32_t i = base + q * kPrefixBlock + threadIdx.x;
      lo16[q] = i < ntiles ? pieces[2 * (uint64_t)i] : make_uint4(0u, 0u, 0u, 0u);
      hi16[q] = i < ntiles ? pieces[2 * (uint64_t)i + 1] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int q = 0; q < kPrefixPer; ++q) {
      c[q] = sum_u16x8(lo16[q]) + sum_u16x8(hi16[q]);
      if (c[q] > (uint32_t)kTileElems) c[q] = (uint32_t)kTileElems;   // (never, with counts this library wrote)
      if (c[q] > (uint32_t)kGroupSlots) {          // at most kGroupsPerTile - 1 further groups
        const uint32_t more = (c[q] - 1u) / kGroupSlots;
        const uint32_t at = __hip_atomic_fetch_add(&s_dense, more, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const uint32_t tile = base + q * kPrefixBlock + threadIdx.x;
        for (uint32_t g = 1; g <= more; ++g) dense_list[at + g - 1] = tile | (g << 20);
      }
      incl[q] = wave_inclusive_scan_u32(c[q], lane);
      if (lane == kWave - 1) s_tot[q * kWaves + wv] = incl[q];
    }
    __syncthreads();
    if (wv == 0) {             // exclusive scan of the totals; a round holds < 2^31 non-zeros
      uint32_t t[kPerLane], sum = 0;
#pragma unroll
      for (int r = 0; r < kPerLane; ++r) { t[r] = s_tot[lane * kPerLane + r]; sum += t[r]; }
      const uint32_t lane_incl = wave_inclusive_scan_u32(sum, lane);
      uint32_t run = lane_incl - sum;
#pragma unroll
      for (int r = 0; r < kPerLane; ++r) { s_tot[lane * kPerLane + r] = run; run += t[r]; }
      if (lane == kWave - 1) s_tot[kCells] = lane_incl;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kPrefixPer; ++q) {
      const uint32_t i = base + q * kPrefixBlock + threadIdx.x;
      if (i < ntiles) prefix[i] = carry + s_tot[q * kWaves + wv] + (incl[q] - c[q]);
    }
    carry += s_tot[kCells];
    __syncthreads();               // s_tot is rewritten in the next round
  }
  if (threadIdx.x == 0) {                          // (after the last round's closing barrier)
    prefix[ntiles] = carry;
    total_out[blockIdx.y] = carry;
    *dense_count = s_dense;
  }
}

// ------------------------------------------------------------------ bitmap tile in LDS
// A workgroup of THREADS threads (a multiple of 64 that divides kTileWords) takes
// one tile.  read_tile_words issues the loads of the tile's words (thread t owns
// the kTileWords / THREADS consecutive words starting at that multiple of t);
// scan_tile_words leaves them in T.words and the exclusive prefix of their
// popcounts in T.prefix (T.prefix[kTileWords] = tile total).  All threads of the
// workgroup call both; the second ends with a barrier.  They are separate so
// that a kernel can have its other loads in flight together with the words'.
struct TileBits {
  uint64_t words[kTileWords];
  uint16_t prefix[kTileWords + 2];     // a tile has at most 32768 = 0x8000 set bits
  uint32_t wave_count[kBlock / kWave];
};

template <int THREADS>
__device__ __forceinline__ void read_tile_words(uint64_t (&wd)[kTileWords / THREADS], const uint64_t* __restrict__ bitmap,
                                                uint64_t nwords, uint64_t word0) {
  constexpr int kPer = kTileWords / THREADS;
  const uint64_t w0 = word0 + (uint64_t)threadIdx.x * kPer;
  if (w0 + kPer <= nwords) {
#pragma unroll
    for (int q = 0; q < kPer; ++q) wd[q] = bitmap[w0 + q];
  } else {
#pragma unroll
    for (int q = 0; q < kPer; ++q) wd[q] = w0 + q < nwords ? bitmap[w0 + q] : 0ull;
  }
}

template <int THREADS>
__device__ __forceinline__ void scan_tile_words(TileBits& T, const uint64_t (&wd)[kTileWords / THREADS]) {
  constexpr int kPer = kTileWords / THREADS;
  constexpr int kWaves = THREADS / kWave;
  static_assert(THREADS % kWave == 0 && kTileWords % THREADS == 0 && THREADS <= kBlock, "unsupported workgroup size");
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  uint32_t pc[kPer];
  uint32_t cnt = 0;
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    pc[q] = (uint32_t)__popcll(wd[q]);
    cnt += pc[q];
  }
  const uint32_t incl = wave_inclusive_scan_u32(cnt, lane);
  uint32_t run = incl - cnt;
  if (kWaves > 1) {
    if (lane == kWave - 1) T.wave_count[wv] = incl;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kWaves; ++q) run += (uint32_t)q < wv ? T.wave_count[q] : 0u;
  }
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    T.words[threadIdx.x * kPer + q] = wd[q];
    T.prefix[threadIdx.x * kPer + q] = (uint16_t)run;
    run += pc[q];
  }
  if (threadIdx.x == THREADS - 1) T.prefix[kTileWords] = (uint16_t)run;
  __syncthreads();
}

// Element index (relative to the tile) of the t-th set bit of the tile, t < total.
__device__ __forceinline__ uint32_t locate_set_bit(const TileBits& T, uint32_t t) {
  static_assert(kTileWords == 512, "the search below takes log2(kTileWords) = 9 steps");
  uint32_t lo = 0, hi = kTileWords;               // invariant: prefix[lo] <= t < prefix[hi]
#pragma unroll
  for (int step = 0; step < 9; ++step) {
    const uint32_t mid = (lo + hi) >> 1;
    if (T.prefix[mid] <= t) lo = mid; else hi = mid;
  }
  return lo * 64 + select_bit(T.words[lo], t - T.prefix[lo]);
}

// ------------------------------------------------------------------ encode: Sparse(g)
// List positions [group * kGroupSlots, (group + 1) * kGroupSlots) of one tile, by
// one workgroup of kBlock threads.  All threads call it with the same arguments.
// VALUES: the values at the set bits are gathered too (expansions of aggregated or block bitmaps carry none).
template <bool VALUES>
__device__ __forceinline__ void compact_group(const EncodeBatch& B, const WorkerPtrs& P, const uint64_t* prefix,
                                              TileBits& T, uint32_t tile, uint32_t group) {
  const uint64_t word0 = (uint64_t)tile * kTileWords;
  uint64_t wd[kWordsPerThread];
  read_tile_words<kBlock>(wd, P.bitmap, B.nwords, word0);      // in flight together with the two prefix loads
  const uint64_t base = prefix[tile];
  const uint32_t total = (uint32_t)(prefix[tile + 1] - base);
  const uint32_t first = group * kGroupSlots;
  if (first >= total || base + first >= B.cap) return;          // uniform over the workgroup
  const uint32_t last = total - first > (uint32_t)kGroupSlots ? first + kGroupSlots : total;
  scan_tile_words<kBlock>(T, wd);
  // four output slots per thread and trip, so that the four value gathers are in flight together
  constexpr int kSlots = 4;
  for (uint32_t t0 = first + threadIdx.x; t0 < last; t0 += kBlock * kSlots) {
    uint32_t i[kSlots], v[kSlots];
    bool live[kSlots];
#pragma unroll
    for (int u = 0; u < kSlots; ++u) {
      const uint32_t t = t0 + u * kBlock;
      live[u] = t < last && base + t < B.cap;
      i[u] = live[u] ? (uint32_t)(word0 * 64 + locate_set_bit(T, t)) : 0u;
    }
#pragma unroll
    for (int u = 0; u < kSlots; ++u) v[u] = VALUES && live[u] ? P.grad[i[u]] : 0u;
#pragma unroll
    for (int u = 0; u < kSlots; ++u) {
      if (!live[u]) continue;
      const uint64_t pos = base + t0 + u * kBlock;
      P.nz_idx[pos] = i[u];
      if (VALUES) P.nz_val[pos] = v[u];
    }
  }
}

// The first `helpers` workgroups of a worker take the further groups of the tiles
// in the dense-tile list, one entry per trip (they start first: theirs is the
// longest work); workgroup helpers + t takes the first kGroupSlots list positions
// of tile t.
template <bool VALUES>
__global__ __launch_bounds__(kBlock) void encode_compact_kernel(const EncodeBatch B, uint32_t helpers) {
  __shared__ TileBits T;
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;                           // uniform over the workgroup
  if (blockIdx.x >= helpers) {
    compact_group<VALUES>(B, B.w[k], ws_prefix(B, k), T, blockIdx.x - helpers, 0u);
    return;
  }
  const uint32_t* dense = ws_dense_list(B, k);
  const uint32_t entries = dense[0];
  for (uint32_t e = blockIdx.x; e < entries; e += helpers) {
    const uint32_t entry = dense[64 + e];
    __syncthreads();                                     // T may still be read by the previous trip
    compact_group<VALUES>(B, B.w[k], ws_prefix(B, k), T, entry & 0xFFFFFu, entry >> 20);
  }
}

}  // namespace s2r
