// Decompress (Algorithm 1, recovery line and query loops): the gather route and
// the route that answers the queries from sketch slices held in LDS.
// Included by s2r_kernels.hip only (one translation unit).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/s2r.h"
#include "s2r_slices.h"

namespace s2r {

// ------------------------------------------------------------------ decode
struct DecodeArgs {
  const float* sketch;
  const uint64_t* bitmap;
  uint64_t n;
  uint64_t nwords;
  uint32_t d;
  uint32_t log2w;
  const uint64_t* prefix;    // [ntiles + 1]
  const uint32_t* dense;     // dense-tile list: count, 64 words later the entries
  uint32_t* idx_out;         // may be null
  float* val_out;            // may be null
  uint64_t cap;
  float* dense_out;          // may be null
  float* params;             // may be null; else params[i] += scale * estimate at every union index
  float scale;
};

// Median of D values by a fully unrolled exchange network: every output is one
// of the inputs (odd D); even D averages the two middle ones in float32.  The
// order is the total order a sort gives: NaN after everything else (a gradient
// that holds a NaN or opposite infinities poisons its d buckets, and the indices
// that read them, exactly as it does in a sort-based median), -0.0 and +0.0 equal.
template <int D>
__device__ __forceinline__ float median_fixed(float (&x)[D]) {
#pragma unroll
  for (int a = 0; a < D - 1; ++a) {
#pragma unroll
    for (int b = 0; b < D - 1 - a; ++b) {
      const float p = x[b], q = x[b + 1];
      const bool swap = !(p <= q) && (q == q);     // p > q, or p is NaN and q is not
      x[b] = swap ? q : p;
      x[b + 1] = swap ? p : q;
    }
  }
  if constexpr ((D & 1) != 0) return x[D / 2];
  else return 0.5f * (x[D / 2 - 1] + x[D / 2]);
}

template <int D>
__device__ __forceinline__ float query(const DecodeArgs& A, const HashRows& hp, uint32_t i) {
  float est[D];
#pragma unroll
  for (int j = 0; j < D; ++j) {
    const uint32_t h = bucket_of(i, hp.a[j], hp.b[j], A.log2w);
    const uint32_t raw = __float_as_uint(A.sketch[((uint64_t)j << A.log2w) + h]);
    est[j] = __uint_as_float(raw ^ signbit_of(i, hp.c[j], hp.e[j]));
  }
  return median_fixed<D>(est);
}

// List positions [group * kGroupSlots, (group + 1) * kGroupSlots) of one tile, by
// one workgroup of kBlock threads; group 0 also clears the tile's part of the
// dense output first (the kernel that handles the further groups runs afterwards).
template <int D>
__device__ __forceinline__ void decode_group(const DecodeArgs& A, const HashRows& hp, TileBits& T, uint32_t tile,
                                             uint32_t group) {
  const uint64_t word0 = (uint64_t)tile * kTileWords;
  uint64_t wd[kWordsPerThread];
  read_tile_words<kBlock>(wd, A.bitmap, A.nwords, word0);      // in flight together with the two prefix loads
  const uint64_t base = A.prefix[tile];
  const uint32_t total = (uint32_t)(A.prefix[tile + 1] - base);

  // dense output: group 0 owns the tile's elements; it clears them, and the estimates are
  // written over the zeros after the barrier in scan_tile_words
  if (group == 0 && A.dense_out != nullptr) {
    const uint64_t e0 = word0 * 64;
    const uint64_t e1 = min(A.n, e0 + (uint64_t)kTileElems);
    float4* p4 = reinterpret_cast<float4*>(A.dense_out + e0);     // e0 is a multiple of 64 elements
    const uint64_t n4 = (e1 - e0) / 4;
    for (uint64_t q = threadIdx.x; q < n4; q += kBlock) p4[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    const uint64_t r = e0 + n4 * 4 + threadIdx.x;
    if (r < e1) A.dense_out[r] = 0.0f;
  }
  const uint32_t first = group * kGroupSlots;
  if (first >= total) return;                      // uniform over the workgroup
  const uint32_t last = total - first > (uint32_t)kGroupSlots ? first + kGroupSlots : total;
  scan_tile_words<kBlock>(T, wd);
  // two list positions per thread and trip: 2 D bucket reads in flight
  constexpr int kSlots = 2;
  for (uint32_t t0 = first + threadIdx.x; t0 < last; t0 += kBlock * kSlots) {
    uint32_t i[kSlots];
    float g[kSlots];
#pragma unroll
    for (int u = 0; u < kSlots; ++u) {
      const uint32_t t = t0 + u * kBlock;
      i[u] = t < last ? (uint32_t)(word0 * 64 + locate_set_bit(T, t)) : 0u;
    }
#pragma unroll
    for (int u = 0; u < kSlots; ++u) g[u] = t0 + u * kBlock < last ? query<D>(A, hp, i[u]) : 0.0f;
#pragma unroll
    for (int u = 0; u < kSlots; ++u) {
      const uint32_t t = t0 + u * kBlock;
      if (t >= last) continue;
      const uint64_t pos = base + t;
      if (A.idx_out != nullptr && pos < A.cap) {
        A.idx_out[pos] = i[u];
        A.val_out[pos] = g[u];
      }
      if (A.dense_out != nullptr) A.dense_out[i[u]] = g[u];
      if (A.params != nullptr) A.params[i[u]] = fmaf(A.scale, g[u], A.params[i[u]]);   // union indices are distinct
    }
  }
}

// Workgroups below `helpers` take the further groups of the tiles in the
// dense-tile list (A.dense: the entry count, 64 words later the entries), one
// entry per trip; workgroup helpers + t takes group 0 of tile t.  With a dense output the two kinds must
// not share a launch (group 0 clears the tile's part of it): the host then
// launches the tiles alone (helpers = 0) and afterwards the helpers alone
// (tiles = 0).
template <int D>
__global__ __launch_bounds__(kBlock) void decode_kernel(const DecodeArgs A, const HashRows hp, uint32_t helpers) {
  __shared__ TileBits T;
  if (blockIdx.x >= helpers) {
    decode_group<D>(A, hp, T, blockIdx.x - helpers, 0u);
    return;
  }
  const uint32_t entries = A.dense[0];
  for (uint32_t e = blockIdx.x; e < entries; e += helpers) {
    const uint32_t entry = A.dense[64 + e];
    __syncthreads();                                     // T may still be read by the previous trip
    decode_group<D>(A, hp, T, entry & 0xFFFFFu, entry >> 20);
  }
}

// Block-granular decode by gathers: list position t is element t mod block of
// the (t / block)-th listed block; every position gets its d bucket reads and
// their median (0 for positions of the last block beyond the gradient).  One
// thread per position and trip, kBlock * 4 positions per workgroup.
template <int D>
__global__ __launch_bounds__(kBlock) void decode_blocks_kernel(const DecodeArgs A, const HashRows hp, uint32_t block,
                                                               const uint32_t* __restrict__ blk_list,
                                                               const uint64_t* __restrict__ count) {
  constexpr int kPer = 4;
  const uint64_t total = *count;
  const uint64_t have = (total < A.cap ? total : A.cap) * block;
  // (the grid is sized for the capacity of the list, capped; the listed blocks are usually fewer)
  for (uint64_t wg = blockIdx.x; wg * (kBlock * kPer) < have; wg += gridDim.x) {
    const uint64_t t0 = wg * (kBlock * kPer) + threadIdx.x;
    float g[kPer];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const uint64_t t = t0 + (uint64_t)u * kBlock;
      g[u] = 0.0f;
      if (t < have) {
        const uint64_t q = t / block;
        const uint64_t e = (uint64_t)blk_list[q] * block + (t - q * block);
        if (e < A.n) {
          g[u] = query<D>(A, hp, (uint32_t)e);
          if (A.params != nullptr) A.params[e] = fmaf(A.scale, g[u], A.params[e]);
        }
      }
    }
    if (A.val_out != nullptr) {
#pragma unroll
      for (int u = 0; u < kPer; ++u) {
        const uint64_t t = t0 + (uint64_t)u * kBlock;
        if (t < have) A.val_out[t] = g[u];
      }
    }
  }
}

// ------------------------------------------------------------------ decode, every sketch row on its own XCDs
// The bucket reads of the gather kernels above miss the L2 when the sketch is a few times larger than one
// (4 MB per XCD, eight XCDs that do not share theirs): every thread reads all d rows, so every XCD works on the
// whole sketch.  Here a workgroup reads ONE row, and workgroups are given rows by the XCD they run on
// (workgroups go to the XCDs round robin: workgroup index modulo 8): XCD x serves row x mod d, so that a row of
// up to 4 MB stays in the L2s of the XCDs that serve it.  The estimates meet in memory, est[j * stride + list
// position], written and read as whole lines, and decode_rows_median_kernel takes the medians.  Where the
// assumption about the placement does not hold the results are the same, only slower.  Measured on MI355X
// (1.1 M indices, d = 3, w = 2^20): 27 us + 4 us for the medians against 50 us for decode_kernel<3>.
// Needs d <= 8 (eight XCDs).
//
// Row j and unit of work (a tile or a dense-tile helper; a chunk of list positions in the block codec) of this
// workgroup; false when it has none.  Row j is served by the m XCDs j, j + d, ...: unit u of row j goes to the
// (u mod m)-th of them.  The grid is 8 * ceil(units / floor(8 / d)) workgroups.
__device__ __forceinline__ bool rows_assignment(uint32_t d, uint32_t units, uint32_t& j, uint32_t& unit) {
  const uint32_t x = blockIdx.x & 7u, g = blockIdx.x >> 3;
  j = x % d;
  const uint32_t m = (8u - j + d - 1u) / d;
  unit = g * m + x / d;
  return unit < units;
}

// decode_group for one sketch row: the estimates of row j for the list positions of one group of a tile; the
// workgroups of row 0 also write the indices.
__device__ __forceinline__ void rows_group(const DecodeArgs& A, const HashRows& hp, TileBits& T, uint32_t tile,
                                           uint32_t group, uint32_t j, float* __restrict__ est, uint64_t stride) {
  const uint64_t word0 = (uint64_t)tile * kTileWords;
  uint64_t wd[kWordsPerThread];
  read_tile_words<kBlock>(wd, A.bitmap, A.nwords, word0);      // in flight together with the two prefix loads
  const uint64_t base = A.prefix[tile];
  const uint32_t total = (uint32_t)(A.prefix[tile + 1] - base);
  const uint32_t first = group * kGroupSlots;
  if (first >= total || base + first >= A.cap) return;         // uniform over the workgroup
  const uint32_t last = total - first > (uint32_t)kGroupSlots ? first + kGroupSlots : total;
  scan_tile_words<kBlock>(T, wd);
  constexpr int kSlots = kGroupSlots / kBlock;                 // the whole group in one trip: 8 reads in flight per thread
  uint32_t i[kSlots], raw[kSlots];
  bool live[kSlots];
#pragma unroll
  for (int u = 0; u < kSlots; ++u) {
    const uint32_t t = first + threadIdx.x + u * kBlock;
    live[u] = t < last && base + t < A.cap;
    i[u] = live[u] ? (uint32_t)(word0 * 64 + locate_set_bit(T, t)) : 0u;
  }
  const uint64_t a = hp.a[j], b = hp.b[j], c = hp.c[j], e = hp.e[j];
  const float* __restrict__ row = A.sketch + ((uint64_t)j << A.log2w);
#pragma unroll
  for (int u = 0; u < kSlots; ++u) raw[u] = __float_as_uint(row[bucket_of(i[u], a, b, A.log2w)]);
#pragma unroll
  for (int u = 0; u < kSlots; ++u) {
    if (!live[u]) continue;
    const uint64_t pos = base + first + threadIdx.x + u * kBlock;
    est[j * stride + pos] = __uint_as_float(raw[u] ^ signbit_of(i[u], c, e));
    if (j == 0) A.idx_out[pos] = i[u];
  }
}

// Units [0, ntiles): group 0 of tile `unit`; units [ntiles, ntiles + helpers): the further groups of the tiles
// in the dense-tile list, one entry per trip.
__global__ __launch_bounds__(kBlock) void decode_rows_kernel(const DecodeArgs A, const HashRows hp, float* __restrict__ est,
                                                             uint64_t stride, uint32_t ntiles, uint32_t helpers) {
  __shared__ TileBits T;
  uint32_t j, unit;
  if (!rows_assignment(A.d, ntiles + helpers, j, unit)) return;       // uniform over the workgroup
  if (unit < ntiles) {
    rows_group(A, hp, T, unit, 0u, j, est, stride);
    return;
  }
  const uint32_t entries = A.dense[0];
  for (uint32_t q = unit - ntiles; q < entries; q += helpers) {
    const uint32_t entry = A.dense[64 + q];
    __syncthreads();                                     // T may still be read by the previous trip
    rows_group(A, hp, T, entry & 0xFFFFFu, entry >> 20, j, est, stride);
  }
}

// The same for the block codec: list position t is element t mod block of the (t / block)-th listed block; a
// unit is a chunk of kBlock * kRowsBlockPer positions, and the units beyond the grid's are taken in further trips.
constexpr int kRowsBlockPer = 8;
__global__ __launch_bounds__(kBlock) void decode_rows_blocks_kernel(const DecodeArgs A, const HashRows hp, uint32_t block,
                                                                    const uint32_t* __restrict__ blk_list,
                                                                    const uint64_t* __restrict__ count,
                                                                    float* __restrict__ est, uint64_t stride, uint32_t units) {
  uint32_t j, unit;
  if (!rows_assignment(A.d, units, j, unit)) return;
  const uint64_t total = *count;
  const uint64_t have = (total < A.cap ? total : A.cap) * block;
  const uint64_t a = hp.a[j], b = hp.b[j], c = hp.c[j], e = hp.e[j];
  const float* __restrict__ row = A.sketch + ((uint64_t)j << A.log2w);
  for (uint64_t chunk = unit; chunk * (kBlock * kRowsBlockPer) < have; chunk += units) {
    const uint64_t t0 = chunk * (kBlock * kRowsBlockPer) + threadIdx.x;
    uint32_t i[kRowsBlockPer], raw[kRowsBlockPer];
#pragma unroll
    for (int u = 0; u < kRowsBlockPer; ++u) {
      const uint64_t t = t0 + (uint64_t)u * kBlock;
      uint64_t el = A.n;                                   // (not an element)
      if (t < have) {
        const uint64_t q = t / block;
        el = (uint64_t)blk_list[q] * block + (t - q * block);
      }
      i[u] = el < A.n ? (uint32_t)el : 0u;                 // (positions beyond the gradient read a bucket too; the medians drop them)
    }
#pragma unroll
    for (int u = 0; u < kRowsBlockPer; ++u) raw[u] = __float_as_uint(row[bucket_of(i[u], a, b, A.log2w)]);
#pragma unroll
    for (int u = 0; u < kRowsBlockPer; ++u) {
      const uint64_t t = t0 + (uint64_t)u * kBlock;
      if (t < have) est[j * stride + t] = __uint_as_float(raw[u] ^ signbit_of(i[u], c, e));
    }
  }
}

// The medians of the row route: one thread per list position, d coalesced reads.  In the block codec the
// positions of the last block beyond the gradient get 0.
template <int D>
__global__ __launch_bounds__(kBlock) void decode_rows_median_kernel(const float* __restrict__ est, uint64_t stride,
                                                                    const uint64_t* __restrict__ count, uint64_t cap,
                                                                    float* __restrict__ val_out, uint32_t block, uint64_t n,
                                                                    const uint32_t* __restrict__ blk_list) {
  const uint64_t total = *count;
  const uint64_t listed = total < cap ? total : cap;
  const uint64_t have = block != 0 ? listed * block : listed;
  for (uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x; t < have; t += (uint64_t)gridDim.x * kBlock) {
    float x[D];
#pragma unroll
    for (int j = 0; j < D; ++j) x[j] = est[j * stride + t];
    float g = median_fixed<D>(x);
    if (block != 0) {
      const uint64_t q = t / block;
      if ((uint64_t)blk_list[q] * block + (t - q * block) >= n) g = 0.0f;
    }
    val_out[t] = g;
  }
}

// ------------------------------------------------------------------ decode by sketch slices
// The bucket reads of decode_kernel each fetch a 128-byte line for 4 useful
// bytes.  When the union list is long, s2r_decode instead sorts the (list
// position, row) queries of every chunk of kBinChunk list positions by sketch
// slice with the kernel of the encode's slice strategy (bin_sort_kernel; a record
// is one word that carries the position in the chunk instead of a value) and
//   decode_slice_kernel   workgroup (j, s) loads slice s of row j into LDS with
//                         coalesced loads and answers its bin's queries, chunk by
//                         chunk: the answer to the query at record r of a chunk's
//                         region is the signed estimate at the same place r of the
//                         answers (4 bytes each way: the query says whose it is).  Every item of a chunk has a query in
//                         every row, so row j's answers of chunk c are the count(c)
//                         entries that start at c * kBinChunk * d + j * count(c)
//   decode_median_kernel  workgroup = chunk: row by row, the answers (with their
//                         queries, for the positions) go through LDS into the
//                         registers of the thread that owns the list position; then
//                         the medians, stored coalesced
struct DecodeSliceArgs {
  const float* sketch;
  const uint32_t* rec;       // queries, chunk by chunk, sorted by bin: cell in slice | position in chunk << slice_log2 | sign bit
  uint32_t* answers;         // same shape as rec: the signed estimates (float32 bits)
  const uint32_t* seg;       // [nchunks][nbins + 1]: the bins' segments in a chunk's region
  const uint64_t* count;     // the union count (device)
  uint64_t cap;
  float* val_out;
  uint32_t nbins;
  uint32_t slice_log2;
  uint32_t d;
  uint32_t block;            // block-granular codec: list positions are elements of listed blocks
  uint64_t n;                //   (positions whose element is not below n get 0)
  const uint32_t* blk_list;
};

// The bin's chunks are shared out between the gridDim.y workgroups of the bin (each loads the slice), a
// workgroup's chunks between its waves, a wave's chunks between groups of its lanes (seg_lanes), eight
// chunks or fewer to a pass; the first pass's queries are asked for before the slice is loaded, a pass's
// segment places during the pass before.
__global__ __launch_bounds__(kSliceBlock) void decode_slice_kernel(const DecodeSliceArgs A) {
  extern __shared__ float s_cells[];
  constexpr int kWaves = kSliceBlock / kWave;
  constexpr int kAhead = 8;
  constexpr int kSets = 8;                                // chunks of a lane in a pass, at most
  const uint32_t bin = blockIdx.x;                        // = (j << log2(slices per row)) + s
  const uint64_t total = *A.count;
  const uint64_t listed = total < A.cap ? total : A.cap;
  const uint64_t have = A.block != 0 ? listed * A.block : listed;
  const uint32_t nchunks = (uint32_t)((have + kBinChunk - 1) / kBinChunk);
  const uint32_t share = (nchunks + gridDim.y - 1) / gridDim.y;
  const uint32_t c_begin = blockIdx.y * share;
  if (c_begin >= nchunks) return;                         // uniform over the workgroup
  const uint32_t c_end = c_begin + share < nchunks ? c_begin + share : nchunks;
  const uint64_t stride = (uint64_t)kBinChunk * A.d;
  const uint32_t row_len = A.nbins + 1;                   // of the segment table
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  // the workgroup's chunks are shared out between its waves in consecutive ranges
  const uint32_t cpw = (c_end - c_begin + kWaves - 1) / kWaves;
  const uint32_t w_begin = c_begin + wv * cpw < c_end ? c_begin + wv * cpw : c_end;
  const uint32_t w_end = w_begin + cpw < c_end ? w_begin + cpw : c_end;
  // a group's lanes: about a quarter of a full chunk's queries per bin, so that a pass has most segments
  // in flight whole (kAhead times as many queries), and 16 at least (64 contiguous bytes)
  const uint32_t quarter = (uint32_t)kBinChunk * A.d / A.nbins / 4u;
  uint32_t min_width = 16u;
  while (min_width < quarter && min_width < (uint32_t)kWave) min_width <<= 1;
  const SegLanes sl = seg_lanes(cpw, lane, min_width);
  // A pass: sets * groups chunks, the lane's are chunks cb + g + t * groups (t < sets).  The more segments a
  // wave has in flight the better (measured with 4, 6 and 8 chunks per lane: config 4 78, 66, 70 us, config 5
  // 208, 190, 182 us), and a last pass with little in it costs as much as a full one: so as few passes as
  // kSets allows, all equally full (config 4: 33 chunks per wave, 4 groups: passes of 5 + 4, not 8 + 1).
  const uint32_t all_sets = (cpw + sl.groups - 1) / sl.groups;
  const uint32_t passes = (all_sets + kSets - 1) / kSets;
  const uint32_t sets = passes != 0 ? (all_sets + passes - 1) / passes : 1u;     // uniform over the workgroup
  auto places = [&](uint32_t cb, uint32_t (&f)[kSets], uint32_t (&l)[kSets]) {
#pragma unroll
    for (int t = 0; t < kSets; ++t) {
      const uint32_t c = cb + sl.g + t * sl.groups;
      f[t] = l[t] = 0u;
      if ((uint32_t)t < sets && c < w_end) {
        f[t] = A.seg[(uint64_t)c * row_len + bin];
        l[t] = A.seg[(uint64_t)c * row_len + bin + 1];
      }
    }
  };
  auto fetch = [&](uint32_t cb, const uint32_t (&f)[kSets], const uint32_t (&l)[kSets], uint32_t (&x)[kSets][kAhead]) {
#pragma unroll
    for (int t = 0; t < kSets; ++t) seg_fetch<true, kAhead>(A.rec + (uint64_t)(cb + sl.g + t * sl.groups) * stride, f[t], l[t], sl, x[t]);
  };
  uint32_t cb = w_begin, f[kSets], l[kSets];
  places(cb, f, l);
  const uint32_t cells = 1u << A.slice_log2;
  const float* src = A.sketch + (uint64_t)bin * cells;    // row-major sketch: slice s of row j starts at bin * cells
  if (cells >= 4u * kSliceBlock) {                        // (the sketch and every slice of 4 cells or more are 16-byte aligned)
    for (uint32_t c = threadIdx.x; c < cells / 4; c += kSliceBlock)
      reinterpret_cast<float4*>(s_cells)[c] = reinterpret_cast<const float4*>(src)[c];
  } else {
    for (uint32_t c = threadIdx.x; c < cells; c += kSliceBlock) s_cells[c] = src[c];
  }
  uint32_t x[kSets][kAhead];
  fetch(cb, f, l, x);
  __syncthreads();
  const uint32_t cell_mask = cells - 1u;
  auto put = [&](uint32_t* to, const uint32_t q) {        // the answer goes where the query is
    *to = __float_as_uint(s_cells[q & cell_mask]) ^ (q & 0x80000000u);
  };
  while (true) {                                          // uniform over the wave
    const uint32_t nb = cb + sets * sl.groups;
    uint32_t fn[kSets], ln[kSets];
    if (nb < w_end) places(nb, fn, ln);
#pragma unroll
    for (int t = 0; t < kSets; ++t) {
      const uint64_t region = (uint64_t)(cb + sl.g + t * sl.groups) * stride;
      const uint32_t start = seg_start(f[t], sl);
#pragma unroll
      for (int u = 0; u < kAhead; ++u) {
        const uint32_t i = start + u * sl.width;
        if (i >= f[t] && i < l[t]) put(A.answers + region + i, x[t][u]);
      }
      for (uint32_t i = start + kAhead * sl.width; i < l[t]; i += sl.width)      // the rest of a longer segment
        put(A.answers + region + i, __builtin_nontemporal_load(A.rec + region + i));
    }
    if (nb >= w_end) break;
    cb = nb;
#pragma unroll
    for (int t = 0; t < kSets; ++t) {
      f[t] = fn[t];
      l[t] = ln[t];
    }
    fetch(cb, f, l, x);
  }
}

// The medians of one chunk of list positions (all threads of the workgroup call it with the same arguments).
template <int D>
__device__ __forceinline__ void median_chunk(const DecodeSliceArgs& A, uint32_t chunk, uint64_t have, float* s_est) {
  const uint64_t t0 = (uint64_t)chunk * kBinChunk;
  const uint32_t count = have - t0 < (uint64_t)kBinChunk ? (uint32_t)(have - t0) : (uint32_t)kBinChunk;
  float est[kBinItems][D];
  uint2 cur[kBinItems];                                   // row j's (answer, query)
  const uint32_t* rows = A.answers + t0 * D;
  const uint32_t* asked = A.rec + t0 * D;                 // the query at the same place says whose answer it is
#pragma unroll
  for (int j = 0; j < D; ++j) {
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      const uint32_t t = u * kBinBlock + threadIdx.x;
      cur[u] = t < count ? make_uint2(rows[(uint64_t)j * count + t], asked[(uint64_t)j * count + t]) : make_uint2(0u, 0u);
    }
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      if (u * kBinBlock + threadIdx.x < count) s_est[cur[u].y >> A.slice_log2 & (kBinChunk - 1)] = __uint_as_float(cur[u].x);
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      const uint32_t t = u * kBinBlock + threadIdx.x;
      est[u][j] = t < count ? s_est[t] : 0.0f;
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < kBinItems; ++u) {
    const uint32_t t = u * kBinBlock + threadIdx.x;
    if (t >= count) continue;
    float g = median_fixed<D>(est[u]);
    if (A.block != 0) {                                   // the tail of the last block lies beyond the gradient
      const uint64_t q = (t0 + t) / A.block;
      if ((uint64_t)A.blk_list[q] * A.block + (t0 + t - q * A.block) >= A.n) g = 0.0f;
    }
    A.val_out[t0 + t] = g;
  }
}

// The grid is sized for the number of positions expected, which is normally all there are: a workgroup takes
// chunk blockIdx.x, and only if the list holds more, the chunks blockIdx.x + gridDim.x, ... after it.
template <int D>
__global__ __launch_bounds__(kBinBlock, D <= 5 ? 8 : 4) void decode_median_kernel(const DecodeSliceArgs A) {
  __shared__ float s_est[kBinChunk];
  const uint64_t total = *A.count;
  const uint64_t listed = total < A.cap ? total : A.cap;
  const uint64_t have = A.block != 0 ? listed * A.block : listed;
  uint32_t chunk = blockIdx.x;
  if ((uint64_t)chunk * kBinChunk >= have) return;        // uniform over the workgroup
  median_chunk<D>(A, chunk, have, s_est);
  for (chunk += gridDim.x; (uint64_t)chunk * kBinChunk < have; chunk += gridDim.x) {      // uniform
    __syncthreads();                                      // s_est is rewritten
    median_chunk<D>(A, chunk, have, s_est);
  }
}

}  // namespace s2r
