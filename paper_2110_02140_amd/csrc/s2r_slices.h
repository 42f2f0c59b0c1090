// The insertions of Algorithm 1 without global atomics: a counting sort of
// (item, row) records by sketch slice and the workgroups that own a slice in LDS.
// Included by s2r_kernels.hip only (one translation unit).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/s2r.h"
#include "s2r_tiles.h"
#include "s2r_scan.h"

namespace s2r {

// ------------------------------------------------------------------ encode: sketch by LDS slices
// The insertions S[j, h_j(i)] += s_j(i) g(i) without global atomics.  Row j of the
// sketch is cut into slices of 2^slice_log2 cells (float64 accumulators in LDS); bin (j, s)
// collects the pairs (item, row j) whose bucket falls in slice s.  The listed items are
// cut into chunks of kBinChunk and every chunk is sorted by bin on its own:
//   bin_sort_kernel     a chunk's records (cell in the slice | sign bit, value), counting-sorted by
//                       bin inside LDS and stored in the chunk's own region, with the offsets of
//                       the bins' segments in that region
//   sketch_slice_kernel workgroup (j, s) clears its slice in LDS, adds its bin's segments of
//                       all chunks with LDS float64 atomics and stores the slice as float32
// No kernel needs an offset that depends on other chunks: a histogram kernel, a scan over the chunks
// and a scan over the bins, which an earlier form of this sort needed to give every bin one
// contiguous run, are gone, and the sort's stores are whole contiguous rows of a chunk.
// Work is O(items x rows), whatever the number of slices, and every cell of the
// sketch is written exactly once, by coalesced stores.
constexpr int kBinBlock = 1024;
constexpr int kBinItems = 8;                           // list items per thread
constexpr int kBinChunk = kBinBlock * kBinItems;       // 8192 items per workgroup
constexpr int kMaxBins = 8192;                         // d * slices per row that the LDS histograms hold
constexpr size_t kSliceLdsMax = sizeof(double) << kSliceLog2Max;
constexpr int kDecodeSliceLog2Max = 15;               // decode holds float32 cells: 2^15 of them are 128 KiB of LDS
static_assert(kSliceLog2Max <= 15 && kDecodeSliceLog2Max <= 15, "a slice is at most 128 KiB of LDS");
static_assert(sizeof(uint2) * kBinChunk + sizeof(uint32_t) * kMaxBins <= 160 * 1024, "bin_sort_kernel's LDS");

// The items of the counting sort: the entries of the worker's list, or, in the
// block-granular codec, the elements of the listed blocks (block by block).
__device__ __forceinline__ uint64_t listed_items(const EncodeBatch& B, uint32_t k) {
  const uint64_t nnz = B.nnz_out[k];
  const uint64_t listed = nnz < B.sort_cap ? nnz : B.sort_cap;
  return B.block != 0 ? listed * B.block : listed;
}

// What the items of a sort are, fixed at compile time so that the element codec's kernels carry none of the
// block codec's branches: BLOCKS (the items are the elements of the listed blocks) and QUERY (the payload of
// a record is the item's position, for s2r_decode's queries, instead of its value).
constexpr int kItemsElements = 0, kItemsBlocks = 1, kItemsQuery = 2;      // MODE = blocks | query
__host__ __device__ constexpr bool mode_blocks(int mode) { return (mode & kItemsBlocks) != 0; }
__host__ __device__ constexpr bool mode_query(int mode) { return (mode & kItemsQuery) != 0; }
static inline int items_mode(const EncodeBatch& B) {
  return (B.block != 0 ? kItemsBlocks : 0) | (B.payload_slot != 0 ? kItemsQuery : 0);
}

// Item t (t < listed_items): its element index i and its payload v (the value's
// bits, or the item's position t in a query run).  Returns whether
// the item takes part: with blocks, elements beyond n never do, and elements
// whose value is zero only when the payload is the position (a query), not when
// it is the value (an insertion: zeros are inert).  An item that does not take
// part in a query run is still given d answers (of element 0), which the median
// kernel discards, so that every chunk holds the same number of answers per row.
template <int MODE>
__device__ __forceinline__ bool load_item(const EncodeBatch& B, const WorkerPtrs& P, uint64_t t, uint32_t& i, uint32_t& v) {
  if constexpr (!mode_blocks(MODE)) {
    i = P.nz_idx[t];
    if constexpr (mode_query(MODE)) v = (uint32_t)t; else v = P.nz_val[t];
    return true;
  } else {
    const uint32_t q = (uint32_t)t / B.block;              // (the sort's items are fewer than 2^32)
    const uint64_t e = (uint64_t)P.nz_idx[q] * B.block + ((uint32_t)t - q * B.block);
    const bool inside = e < B.n;
    if constexpr (mode_query(MODE)) {
      i = inside ? (uint32_t)e : 0u;
      v = (uint32_t)t;
      return true;
    } else {
      i = (uint32_t)e;
      v = inside ? P.grad[e] : 0u;
      return inside && (v << 1) != 0u;
    }
  }
}

// The counting sort of one chunk, all inside the workgroup: nothing in it depends on another chunk.
//   1. LDS counters count the chunk's records per bin (d hashes per item, rows outermost: a row's hash
//      parameters are fetched once for a thread's eight items);
//   2. wave j turns row j's counters into their exclusive prefix (64 at a time), which is where each slice's
//      run starts among the chunk's records of that row; with T = the chunk's items that take part (the same
//      in every row), row j's records start at j * T in the chunk's region: seg[chunk][b] = j * T + prefix is
//      stored for the kernels that read the records (seg[chunk][nbins] = d * T);
//   3. per row: every record takes its place in LDS with a fetch-and-add on its slice's counter, and the
//      row's T sorted records are copied out as one contiguous, coalesced run.
// The hashes are computed in both sweeps rather than kept (registers).  Dynamic LDS: kBinChunk records, then
// nbins counters.
// A query's record (MODE with kItemsQuery) is one word: cell in the slice | position in the chunk <<
// slice_log2 | sign bit; its answer will lie at the same place of an array of the same shape, so the
// position inside the chunk (13 bits) is all that has to travel.  An insertion's record is (cell | sign bit,
// value).
template <int MODE>
__global__ __launch_bounds__(kBinBlock, 8) void bin_sort_kernel(const EncodeBatch B, const HashRows hp) {
  extern __shared__ uint2 s_stage[];
  __shared__ uint32_t s_total;
  constexpr int kWaves = kBinBlock / kWave;
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;
  const uint64_t have = listed_items(B, k);
  const uint32_t spr_log2 = B.log2w - B.slice_log2;      // log2 of the slices per row
  const uint32_t spr = 1u << spr_log2;
  uint32_t* s_next = reinterpret_cast<uint32_t*>(s_stage + kBinChunk);
  const WorkerPtrs P = B.w[k];
  const uint32_t mask = (1u << B.slice_log2) - 1u;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  // The grid is sized for the number of items expected; a workgroup takes the chunks blockIdx.x,
  // blockIdx.x + gridDim.x, ... that hold listed items.
  for (uint32_t chunk = blockIdx.x; (uint64_t)chunk * kBinChunk < have; chunk += gridDim.x) {   // uniform
    const uint64_t t0 = (uint64_t)chunk * kBinChunk;
    const uint32_t count = have - t0 < (uint64_t)kBinChunk ? (uint32_t)(have - t0) : (uint32_t)kBinChunk;
    for (uint32_t e = threadIdx.x; e < B.nbins; e += kBinBlock) s_next[e] = 0u;
    if (threadIdx.x == 0) s_total = 0u;
    uint32_t i[kBinItems], v[kBinItems];
    uint32_t ok = 0;                                      // bit u: item u exists and takes part (see load_item)
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      const uint32_t t = u * kBinBlock + threadIdx.x;
      i[u] = 0u;
      v[u] = 0u;
      if (t < count && load_item<MODE>(B, P, t0 + t, i[u], v[u])) ok |= 1u << u;
    }
    __syncthreads();                                      // the counters are zero
    {
      uint32_t mine = __popc(ok);
#pragma unroll
      for (int m = kWave / 2; m >= 1; m >>= 1) mine += __shfl_xor(mine, m, kWave);
      if (lane == 0) __hip_atomic_fetch_add(&s_total, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    for (uint32_t j = 0; j < B.d; ++j) {
      const uint64_t a = hp.a[j], b = hp.b[j];
      uint32_t* row = s_next + (j << spr_log2);
#pragma unroll
      for (int u = 0; u < kBinItems; ++u) {
        if (ok >> u & 1u)
          __hip_atomic_fetch_add(&row[bucket_of(i[u], a, b, B.log2w) >> B.slice_log2], 1u, __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
    __syncthreads();
    const uint32_t T = s_total;
    uint32_t* seg = ws_seg(B, k) + (uint64_t)chunk * (B.nbins + 1);
    for (uint32_t j = threadIdx.x / kWave; j < B.d; j += kWaves) {                // uniform over the wave
      uint32_t carry = 0;
      for (uint32_t s0 = 0; s0 < spr; s0 += kWave) {
        const uint32_t e = s0 + lane;
        const uint32_t x = e < spr ? s_next[(j << spr_log2) + e] : 0u;
        const uint32_t incl = wave_inclusive_scan_u32(x, lane);
        if (e < spr) {
          const uint32_t start = carry + incl - x;
          s_next[(j << spr_log2) + e] = start;            // the next free place of slice e's run
          seg[(j << spr_log2) + e] = j * T + start;
        }
        carry += __shfl(incl, kWave - 1, kWave);
      }
    }
    if (threadIdx.x == 0) seg[B.nbins] = B.d * T;
    __syncthreads();
    uint2* __restrict__ out = ws_records(B, k) + (uint64_t)chunk * kBinChunk * B.d;
    uint32_t* __restrict__ out_q = reinterpret_cast<uint32_t*>(ws_records(B, k)) + (uint64_t)chunk * kBinChunk * B.d;
    uint32_t* s_stage_q = reinterpret_cast<uint32_t*>(s_stage);
    for (uint32_t j = 0; j < B.d; ++j) {
      const uint64_t a = hp.a[j], b = hp.b[j], c = hp.c[j], e = hp.e[j];
      uint32_t* next = s_next + (j << spr_log2);
#pragma unroll
      for (int u = 0; u < kBinItems; ++u) {
        if (ok >> u & 1u) {
          const uint32_t h = bucket_of(i[u], a, b, B.log2w);
          const uint32_t place = __hip_atomic_fetch_add(&next[h >> B.slice_log2], 1u, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_WORKGROUP);
          const uint32_t word = (h & mask) | signbit_of(i[u], c, e);
          if constexpr (mode_query(MODE)) s_stage_q[place] = word | ((u * kBinBlock + threadIdx.x) << B.slice_log2);
          else s_stage[place] = make_uint2(word, v[u]);
        }
      }
      __syncthreads();
      if constexpr (mode_query(MODE)) {
        for (uint32_t p = threadIdx.x; p < T; p += kBinBlock) out_q[(uint64_t)j * T + p] = s_stage_q[p];
      } else {
        for (uint32_t p = threadIdx.x; p < T; p += kBinBlock) out[(uint64_t)j * T + p] = s_stage[p];
      }
      __syncthreads();                                    // s_stage is free again (after the last row: the counters too)
    }
  }
}

// A workgroup takes `per` consecutive bins (j, s) of one worker, one after the
// other.  A slice is accumulated in float64: the LDS float64 atomic add runs at
// full LDS rate on this chip (about 1.7e12 per second over the chip at random
// addresses) while the float32 one takes a slow path (0.2e12 per second,
// whatever the addresses); each cell is rounded to float32 once, when the slice
// is stored.  A bin's records lie in one segment per chunk (bin_sort_kernel): the
// 16 waves share out the chunks, and groups of a wave's lanes its chunks (seg_lanes).
// Segment places are asked for two bins ahead and a segment's first records one bin ahead,
// both before the current slice is read out.  The read-out leaves zeros behind (no
// separate clearing pass).
// STREAM_OUT: the slices leave with streaming stores.  Measured on MI355X: when the sketches of the launch
// add up to more than the memory-side cache keeps (config 5: 1.3 GB), streaming stores are the faster ones;
// when they do not (config 4: 336 MB; config 2: 25 MB), plain stores are, and the merge that reads the
// sketches next gains a little too.  STREAM_IN: the records are read with streaming loads; the same kind of
// threshold from the other side.  (Both are compile-time: as run-time flags inside the unrolled loops they
// cost the kernel 6 to 10 %.)
template <bool STREAM_IN, class REC>
__device__ __forceinline__ REC load_record(const REC* p) {
  if constexpr (STREAM_IN) return __builtin_nontemporal_load(p);
  else return *p;
}

__device__ __forceinline__ void add_record(double* s_slice, const u32x2 x) {
  __hip_atomic_fetch_add(&s_slice[x.x & 0x7FFFFFFFu], (double)__uint_as_float(x.y ^ (x.x & 0x80000000u)),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// How a wave reads segments: its 64 lanes form `groups` groups of `width` lanes, a group reads one chunk's
// segment (the group's lane p reads records p, p + width, ...), so one load instruction serves up to eight
// short segments and every address is the lane's own arithmetic.  A wave with c chunks uses the smallest
// power of two >= c as its number of groups, as long as a group keeps `min_width` lanes (a power of two, 8
// or more: a group's lanes then read 64 contiguous bytes or more); further chunks take further passes.
struct SegLanes {
  uint32_t groups;          // uniform
  uint32_t width;           // lanes per group = 64 / groups
  uint32_t g, p;            // the lane's group and place in it
};
__device__ __forceinline__ SegLanes seg_lanes(uint32_t chunks_per_wave, uint32_t lane, uint32_t min_width) {
  uint32_t log_groups = 0;
  while ((1u << log_groups) < chunks_per_wave && ((uint32_t)kWave >> (log_groups + 1)) >= min_width) ++log_groups;
  SegLanes s;
  s.groups = 1u << log_groups;
  s.width = (uint32_t)kWave >> log_groups;
  s.g = lane >> (6u - log_groups);
  s.p = lane & (s.width - 1u);
  return s;
}

// The lane's records of the segment [first, last) of the region `at` (its start is aligned to 256 bytes or
// more): those at start + p + u * width, start = first rounded down to a multiple of width, so that a trip
// of a group reads one aligned piece of memory (8 lanes: the 64 bytes of one memory request).
__device__ __forceinline__ uint32_t seg_start(uint32_t first, const SegLanes& s) { return (first & ~(s.width - 1u)) + s.p; }

// Trips u < AHEAD: AHEAD loads of a lane in flight.  REC: u32x2 (an insertion's record) or uint32_t (a query's).
template <bool STREAM_IN, int AHEAD, class REC>
__device__ __forceinline__ void seg_fetch(const REC* __restrict__ at, uint32_t first, uint32_t last, const SegLanes& s,
                                          REC (&x)[AHEAD]) {
  const uint32_t start = seg_start(first, s);
#pragma unroll
  for (int u = 0; u < AHEAD; ++u) {
    const uint32_t i = start + u * s.width;
    x[u] = i >= first && i < last ? load_record<STREAM_IN>(at + i) : REC{};
  }
}

// Adds what seg_fetch brought, then the rest of a longer segment.
template <bool STREAM_IN, int AHEAD>
__device__ __forceinline__ void seg_add(const u32x2* __restrict__ at, uint32_t first, uint32_t last, const SegLanes& s,
                                        const u32x2 (&x)[AHEAD], double* s_slice) {
  const uint32_t start = seg_start(first, s);
#pragma unroll
  for (int u = 0; u < AHEAD; ++u) {
    const uint32_t i = start + u * s.width;
    if (i >= first && i < last) add_record(s_slice, x[u]);
  }
  for (uint32_t i0 = start + AHEAD * s.width; i0 < last; i0 += AHEAD * s.width) {   // AHEAD loads in flight here too
    u32x2 y[AHEAD];
#pragma unroll
    for (int u = 0; u < AHEAD; ++u) {
      const uint32_t i = i0 + u * s.width;
      y[u] = i < last ? load_record<STREAM_IN>(at + i) : u32x2{0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < AHEAD; ++u)
      if (i0 + u * s.width < last) add_record(s_slice, y[u]);
  }
}

// The slice goes to `out` as float32, and every cell a thread reads it also clears (no separate clearing pass).
template <bool STREAM_OUT>
__device__ __forceinline__ void read_out_four(double* s_slice, float* out, uint32_t c) {
  double2* cell = reinterpret_cast<double2*>(s_slice) + 2 * c;
  const double2 lo = cell[0], hi = cell[1];
  cell[0] = make_double2(0.0, 0.0);
  cell[1] = make_double2(0.0, 0.0);
  f32x4 o;
  o.x = (float)lo.x; o.y = (float)lo.y; o.z = (float)hi.x; o.w = (float)hi.y;
  if constexpr (STREAM_OUT) __builtin_nontemporal_store(o, &reinterpret_cast<f32x4*>(out)[c]);
  else reinterpret_cast<f32x4*>(out)[c] = o;
}

template <bool STREAM_IN, bool STREAM_OUT>
__global__ __launch_bounds__(kSliceBlock) void sketch_slice_kernel(const EncodeBatch B, uint32_t per) {
  extern __shared__ double s_slice[];
  constexpr int kWaves = kSliceBlock / kWave;
  constexpr int kAhead = 12;                              // with groups of 8 lanes: 96 records of a segment in flight
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;                           // uniform over the workgroup
  const uint32_t bin0 = blockIdx.x * per;                 // bin = (j << log2(slices per row)) + s
  if (bin0 >= B.nbins) return;                            // uniform over the workgroup
  const uint32_t bin1 = bin0 + per < B.nbins ? bin0 + per : B.nbins;
  const uint32_t cells = 1u << B.slice_log2;
  const uint32_t* __restrict__ seg = ws_seg(B, k);
  const u32x2* __restrict__ rec = reinterpret_cast<const u32x2*>(ws_records(B, k));
  const uint64_t have = listed_items(B, k);
  const uint32_t nchunks = (uint32_t)((have + kBinChunk - 1) / kBinChunk);       // the chunks that hold listed items
  const uint64_t stride = (uint64_t)kBinChunk * B.d;      // records of a chunk's region
  const uint32_t row_len = B.nbins + 1;                   // of the segment table
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  // the chunks are shared out between the waves in consecutive ranges
  const uint32_t cpw = (nchunks + kWaves - 1) / kWaves;
  const uint32_t c_begin = wv * cpw < nchunks ? wv * cpw : nchunks;
  const uint32_t c_end = c_begin + cpw < nchunks ? c_begin + cpw : nchunks;
  // a group's lanes: enough that kAhead trips take a segment of one and a half times a full chunk's share
  // of a bin (a longer one goes on with loads that wait one for the other)
  const uint32_t reach = (uint32_t)kBinChunk * B.d / B.nbins * 3u / 2u;
  uint32_t min_width = 8u;
  while (min_width * kAhead < reach && min_width < (uint32_t)kWave) min_width <<= 1;
  const SegLanes sl = seg_lanes(cpw, lane, min_width);
  // The lane's chunk of the first pass.  Ahead of the bin whose records are being added: where that chunk
  // keeps the segments of the next two bins (fa, la and fb, lb take turns), and the next bin's first records
  // (x), asked for before the current bin's slice is read out.
  const uint32_t c0 = c_begin + sl.g;
  const bool mine = c0 < c_end;
  const uint32_t* __restrict__ seg0 = seg + (uint64_t)c0 * row_len;
  const u32x2* __restrict__ rec0 = rec + (uint64_t)c0 * stride;
  auto places = [&](uint32_t bin, uint32_t& f, uint32_t& l) {
    f = l = 0u;
    if (mine) {
      f = seg0[bin];
      l = seg0[bin + 1];
    }
  };
  uint32_t fa, la, fb = 0u, lb = 0u;
  places(bin0, fa, la);
  if (bin0 + 1 < bin1) places(bin0 + 1, fb, lb);
  u32x2 x[kAhead];
  seg_fetch<STREAM_IN, kAhead>(rec0, fa, la, sl, x);
  if (cells >= 2u * kSliceBlock) {                        // (the LDS array is 16-byte aligned)
    for (uint32_t c = threadIdx.x; c < cells / 2; c += kSliceBlock)
      reinterpret_cast<double2*>(s_slice)[c] = make_double2(0.0, 0.0);
  } else {
    for (uint32_t c = threadIdx.x; c < cells; c += kSliceBlock) s_slice[c] = 0.0;
  }
  __syncthreads();                                        // the slice is all zero
  // One bin: [f, l) = its segment in the lane's first chunk (x: that segment's first records), [fn, ln) = the
  // next bin's.
  auto one_bin = [&](uint32_t bin, uint32_t& f, uint32_t& l, const uint32_t fn, const uint32_t ln) {
    seg_add<STREAM_IN, kAhead>(rec0, f, l, sl, x, s_slice);
    for (uint32_t cb = c_begin + sl.groups; cb < c_end; cb += sl.groups) {       // uniform: a wave with more than 8 chunks
      const uint32_t c = cb + sl.g;
      uint32_t f2 = 0u, l2 = 0u;
      if (c < c_end) {
        f2 = seg[(uint64_t)c * row_len + bin];
        l2 = seg[(uint64_t)c * row_len + bin + 1];
      }
      const u32x2* at = rec + (uint64_t)c * stride;
      seg_fetch<STREAM_IN, kAhead>(at, f2, l2, sl, x);
      seg_add<STREAM_IN, kAhead>(at, f2, l2, sl, x, s_slice);
    }
    if (bin + 1 < bin1) {                                 // uniform
      if (bin + 2 < bin1) places(bin + 2, f, l);
      seg_fetch<STREAM_IN, kAhead>(rec0, fn, ln, sl, x);
    }
    __syncthreads();                                      // every record of the bin is in the slice
    // The next bin's records are waited for here, before the read-out's stores are issued: the same wait
    // after the read-out would also wait until those stores have reached memory.
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0)
    float* out = B.w[k].sketch + (uint64_t)bin * cells;   // the slice starts at cell bin * cells of the row-major sketch
    if (cells == 16u * kSliceBlock) {                     // the usual size
#pragma unroll
      for (uint32_t i = 0; i < 4; ++i) read_out_four<STREAM_OUT>(s_slice, out, threadIdx.x + i * kSliceBlock);
    } else if (cells >= 4u * kSliceBlock) {               // (every slice of 4 cells or more is 16-byte aligned)
      for (uint32_t c = threadIdx.x; c < cells / 4; c += kSliceBlock) read_out_four<STREAM_OUT>(s_slice, out, c);
    } else {
      for (uint32_t c = threadIdx.x; c < cells; c += kSliceBlock) {
        out[c] = (float)s_slice[c];
        s_slice[c] = 0.0;
      }
    }
    __syncthreads();                                      // the slice is all zero again
  };
  for (uint32_t bin = bin0; bin < bin1; bin += 2) {       // uniform
    one_bin(bin, fa, la, fb, lb);
    if (bin + 1 < bin1) one_bin(bin + 1, fb, lb, fa, la);
  }
}

// Non-zeros at list positions >= sort_cap (beyond the caller's lists, or beyond
// what the workspace's record area holds) took no part in the counting sort; this
// kernel finds them in the bitmap and inserts them with atomics after the slices
// were stored, so the sketch is complete whatever the capacities are.  Normally there are none:
// each thread checks one tile's range of list positions and the workgroup leaves
// unless one of its kBlock tiles reaches beyond cap.
__global__ __launch_bounds__(kBlock) void sketch_overflow_kernel(const EncodeBatch B, const HashRows hp) {
  __shared__ TileBits T;
  __shared__ uint32_t s_any;
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;                           // uniform over the workgroup
  const WorkerPtrs P = B.w[k];
  const uint64_t* prefix = ws_prefix(B, k);
  const uint32_t tile0 = blockIdx.x * kBlock;
  if (threadIdx.x == 0) s_any = 0u;
  __syncthreads();
  const uint32_t mine = tile0 + threadIdx.x;
  if (mine < B.ntiles && prefix[mine + 1] > B.sort_cap) s_any = 1u;
  __syncthreads();
  if (s_any == 0u) return;                               // uniform over the workgroup
  for (uint32_t tile = tile0; tile < tile0 + kBlock && tile < B.ntiles; ++tile) {
    const uint64_t base = prefix[tile];
    const uint32_t total = (uint32_t)(prefix[tile + 1] - base);
    if (base + total <= B.sort_cap) continue;            // uniform over the workgroup
    const uint64_t word0 = (uint64_t)tile * kTileWords;
    uint64_t wd[kWordsPerThread];
    read_tile_words<kBlock>(wd, P.bitmap, B.nwords, word0);
    __syncthreads();                                     // T may still be read by the previous tile's loop
    scan_tile_words<kBlock>(T, wd);
    const uint32_t first = base >= B.sort_cap ? 0u : (uint32_t)(B.sort_cap - base);
    for (uint32_t t = first + threadIdx.x; t < total; t += kBlock) {
      const uint32_t i = (uint32_t)(word0 * 64 + locate_set_bit(T, t));
      if (B.block == 0) {
        sketch_insert(P.sketch, B.d, B.log2w, hp, i, P.grad[i]);
      } else {                                           // an unlisted block: its non-zero elements
        for (uint32_t o = 0; o < B.block; ++o) {
          const uint64_t e = (uint64_t)i * B.block + o;
          if (e >= B.n) break;
          const uint32_t v = P.grad[e];
          if ((v << 1) != 0u) sketch_insert(P.sketch, B.d, B.log2w, hp, (uint32_t)e, v);
        }
      }
    }
  }
}

}  // namespace s2r
