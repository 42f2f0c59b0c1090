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
// collects the pairs (item, row j) whose bucket falls in slice s.  A counting sort
// over the listed items brings each bin's records together:
//   bin_hist_kernel     per chunk of kBinChunk items, a histogram over the bins and, row by
//                       row, its exclusive prefix over the row's slices
//   bin_colscan_kernel  offsets of every (chunk, bin) run and of every bin
//   bin_scatter_kernel  writes each record (cell in the slice | sign bit, value)
//                       into its run (order inside a run is arbitrary)
//   sketch_slice_kernel workgroup (j, s) clears its slice in LDS, adds its bin's
//                       records with LDS float64 atomics and stores the slice as float32
// Work is O(items x rows), whatever the number of slices, and every cell of the
// sketch is written exactly once, by coalesced stores.
constexpr int kBinBlock = 1024;
constexpr int kBinItems = 8;                           // list items per thread
constexpr int kBinChunk = kBinBlock * kBinItems;       // 8192 items per workgroup
constexpr int kMaxBins = 8192;                         // d * slices per row that the LDS histograms hold
constexpr size_t kSliceLdsMax = sizeof(double) << kSliceLog2Max;
constexpr int kDecodeSliceLog2Max = 15;               // decode holds float32 cells: 2^15 of them are 128 KiB of LDS
static_assert(kMaxBins <= (1 << 13) && kSliceLog2Max <= 15 && kDecodeSliceLog2Max <= 15,
              "bin_scatter_kernel packs slice (bits 16..28) and cell (bits 0..14) into one word");

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

// The histogram of one chunk (all threads of the workgroup call it with the same arguments).  The rows are
// the outer loop: a row's hash parameters are fetched once (they are uniform) for the eight items of a thread.
template <int MODE>
__device__ __forceinline__ void hist_chunk(const EncodeBatch& B, const HashRows& hp, uint32_t k, uint32_t chunk,
                                           uint64_t have, uint32_t* s_hist, uint32_t* s_total) {
  for (uint32_t b = threadIdx.x; b < B.nbins; b += kBinBlock) s_hist[b] = 0u;
  if (threadIdx.x == 0) *s_total = 0u;
  const WorkerPtrs P = B.w[k];
  const uint32_t spr_log2 = B.log2w - B.slice_log2;
  uint32_t i[kBinItems];
  uint32_t ok = 0;                                        // bit u: item u exists and takes part (see load_item)
#pragma unroll
  for (int u = 0; u < kBinItems; ++u) {
    const uint64_t t = (uint64_t)chunk * kBinChunk + u * kBinBlock + threadIdx.x;
    uint32_t v;
    i[u] = 0u;
    if (t < have && load_item<MODE>(B, P, t, i[u], v)) ok |= 1u << u;
  }
  __syncthreads();                                        // s_hist is zero
  {                                                       // the chunk's items that take part (the same in every row)
    uint32_t mine = __popc(ok);
#pragma unroll
    for (int m = kWave / 2; m >= 1; m >>= 1) mine += __shfl_xor(mine, m, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) __hip_atomic_fetch_add(s_total, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  for (uint32_t j = 0; j < B.d; ++j) {
    const uint64_t a = hp.a[j], b = hp.b[j];
    uint32_t* row = s_hist + (j << spr_log2);
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      if (ok >> u & 1u)
        __hip_atomic_fetch_add(&row[bucket_of(i[u], a, b, B.log2w) >> B.slice_log2], 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_WORKGROUP);
    }
  }
  __syncthreads();
  uint32_t* hist = ws_bin_hist(B, k) + (uint64_t)chunk * B.nbins;
  for (uint32_t b = threadIdx.x; b < B.nbins; b += kBinBlock) hist[b] = s_hist[b];
  if (threadIdx.x == 0) ws_chunk_total(B, k)[chunk] = *s_total;
  // row by row, the exclusive prefix of the chunk's counts over the row's slices: where, among the chunk's
  // records of that row sorted by slice, each slice's run starts.  Wave wv takes the rows wv, wv + 16, ...
  // 64 slices at a time.
  constexpr int kWaves = kBinBlock / kWave;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t spr = 1u << spr_log2;
  uint32_t* pre = ws_slice_pre(B, k) + (uint64_t)chunk * B.nbins;
  for (uint32_t j = threadIdx.x / kWave; j < B.d; j += kWaves) {                // uniform over the wave
    uint32_t carry = 0;
    for (uint32_t seg = 0; seg < spr; seg += kWave) {
      const uint32_t e = seg + lane;
      const uint32_t x = e < spr ? s_hist[(j << spr_log2) + e] : 0u;
      const uint32_t incl = wave_inclusive_scan_u32(x, lane);
      if (e < spr) pre[(j << spr_log2) + e] = carry + incl - x;
      carry += __shfl(incl, kWave - 1, kWave);
    }
  }
}

// The grid is sized for the number of items expected, which is normally all there are: a workgroup takes
// chunk blockIdx.x, and only if the lists hold more, the chunks blockIdx.x + gridDim.x, ... after it.  No
// kernel reads the histogram rows of chunks without listed items.
template <int MODE>
__global__ __launch_bounds__(kBinBlock) void bin_hist_kernel(const EncodeBatch B, const HashRows hp) {
  __shared__ uint32_t s_hist[kMaxBins];
  __shared__ uint32_t s_total;
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;                           // uniform over the workgroup
  const uint64_t have = listed_items(B, k);
  uint32_t chunk = blockIdx.x;
  if ((uint64_t)chunk * kBinChunk >= have) return;       // uniform over the workgroup
  hist_chunk<MODE>(B, hp, k, chunk, have, s_hist, &s_total);
  for (chunk += gridDim.x; (uint64_t)chunk * kBinChunk < have; chunk += gridDim.x) {      // uniform
    __syncthreads();                                     // s_hist and s_total are rewritten
    hist_chunk<MODE>(B, hp, k, chunk, have, s_hist, &s_total);
  }
}

// Offsets of the counting sort.
// bin_colscan_kernel: workgroup = 64 adjacent bins of one worker (lane = bin, so a
// chunk's counters are read as one 256-byte row); its 16 waves split the chunks
// into 16 consecutive ranges.  In place, hist[c][b] becomes the number of records
// of bin b in chunks before c: every wave sums its range, the waves' sums are
// exchanged through LDS, then every wave walks its range again with its running
// offset.  Where bin b = (row j, slice s) starts among the worker's records needs no
// scan over the bins and so no kernel of its own: it is the records of the rows
// before j, j times the items that take part (the sum of the chunks' totals), plus
// the records of row j's earlier slices, the sum over the chunks of the slice prefix
// at (chunk, b): two more column sums of the same walk.  bin_start[nbins] = all records.
__global__ __launch_bounds__(kBinBlock) void bin_colscan_kernel(const EncodeBatch B) {
  constexpr int kWaves = kBinBlock / kWave;              // 16
  constexpr uint32_t kAhead = 8;                         // counters in flight per thread
  __shared__ uint32_t s_part[kWaves][kWave];
  __shared__ uint32_t s_before[kWaves][kWave];
  __shared__ uint32_t s_items[kWaves];
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  const uint32_t b = blockIdx.x * kWave + lane;
  const bool live = b < B.nbins;
  uint32_t* hist = ws_bin_hist(B, k);
  const uint32_t* spre = ws_slice_pre(B, k);
  // the chunks that hold listed items (the others' rows were not written)
  const uint64_t filled = (listed_items(B, k) + kBinChunk - 1) / kBinChunk;
  const uint32_t nchunks = filled < B.nchunks ? (uint32_t)filled : B.nchunks;
  const uint32_t per = (nchunks + kWaves - 1) / kWaves;
  const uint32_t c_begin = wv * per < nchunks ? wv * per : nchunks;
  const uint32_t c_end = c_begin + per < nchunks ? c_begin + per : nchunks;
  uint32_t sum = 0, before = 0;
  for (uint32_t c0 = c_begin; c0 < c_end; c0 += kAhead) {
    uint32_t v[kAhead], p[kAhead];
#pragma unroll
    for (uint32_t q = 0; q < kAhead; ++q) {
      const bool in = live && c0 + q < c_end;
      v[q] = in ? hist[(uint64_t)(c0 + q) * B.nbins + b] : 0u;
      p[q] = in ? spre[(uint64_t)(c0 + q) * B.nbins + b] : 0u;
    }
#pragma unroll
    for (uint32_t q = 0; q < kAhead; ++q) { sum += v[q]; before += p[q]; }
  }
  uint32_t items = 0;                                     // the items of this wave's chunks that take part
  for (uint32_t c = c_begin + lane; c < c_end; c += kWave) items += ws_chunk_total(B, k)[c];
#pragma unroll
  for (int m = kWave / 2; m >= 1; m >>= 1) items += __shfl_xor(items, m, kWave);
  s_part[wv][lane] = sum;
  s_before[wv][lane] = before;
  if (lane == 0) s_items[wv] = items;
  __syncthreads();
  uint32_t run = 0, earlier_slices = 0, all_items = 0;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) {
    const uint32_t x = s_part[q][lane];
    if ((uint32_t)q < wv) run += x;
    earlier_slices += s_before[q][lane];
    all_items += s_items[q];
  }
  // decode: what decode_slice_kernel adds to a query's rank in its bin to get the place of its answer: the
  // start of chunk c's answers, plus the chunk's queries in the rows before the bin's row j (every item of a
  // chunk has a query in every row) and in the row's earlier slices, minus the bin's queries in earlier
  // chunks (modulo 2^32; the places themselves are below 2^32)
  uint32_t* place = B.place_off != 0 ? reinterpret_cast<uint32_t*>(B.workspace + k * B.ws_stride + B.place_off) : nullptr;
  const uint64_t have = listed_items(B, k);
  const uint32_t j = b >> (B.log2w - B.slice_log2);
  for (uint32_t c0 = c_begin; c0 < c_end; c0 += kAhead) {
    uint32_t v[kAhead], rp[kAhead];
#pragma unroll
    for (uint32_t q = 0; q < kAhead; ++q) {
      const bool in = live && c0 + q < c_end;
      v[q] = in ? hist[(uint64_t)(c0 + q) * B.nbins + b] : 0u;
      rp[q] = in && place != nullptr ? spre[(uint64_t)(c0 + q) * B.nbins + b] : 0u;
    }
#pragma unroll
    for (uint32_t q = 0; q < kAhead; ++q) {
      if (live && c0 + q < c_end) {
        hist[(uint64_t)(c0 + q) * B.nbins + b] = run;
        if (place != nullptr) {
          const uint64_t t0 = (uint64_t)(c0 + q) * kBinChunk;
          const uint32_t items = have - t0 < (uint64_t)kBinChunk ? (uint32_t)(have - t0) : (uint32_t)kBinChunk;
          place[(uint64_t)(c0 + q) * B.nbins + b] = (c0 + q) * (uint32_t)kBinChunk * B.d + j * items + rp[q] - run;
        }
      }
      run += v[q];
    }
  }
  if (wv == 0 && live) ws_bin_start(B, k)[b] = j * all_items + earlier_slices;
  if (blockIdx.x == 0 && threadIdx.x == 0) ws_bin_start(B, k)[B.nbins] = B.d * all_items;
}

// One workgroup per chunk of kBinChunk list items, one pass per sketch row j.  The
// chunk's records for row j are first sorted by slice inside LDS (the histogram
// pass left, for every row, where each slice's run starts among the chunk's
// records of that row: a record takes its place in the run with a fetch-and-add)
// and then copied out in sorted order, so that consecutive lanes write
// consecutive records of the (chunk, bin) run that the histogram pass reserved.
// In LDS a record carries its slice number in bits 16..28 of its first word (the
// cell takes bits 0..14, the sign bit 31).  Dynamic LDS: kBinChunk records, then
// two arrays of nbins counters: the next free place of every bin's run in the
// sorted order of its row, and what turns such a place into the record's position
// in the worker's records.
template <int MODE>
__global__ __launch_bounds__(kBinBlock, 8) void bin_scatter_kernel(const EncodeBatch B, const HashRows hp) {
  extern __shared__ uint2 s_stage[];
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;
  const uint64_t have = listed_items(B, k);
  const uint32_t spr_log2 = B.log2w - B.slice_log2;      // log2 of the slices per row
  uint32_t* s_next = reinterpret_cast<uint32_t*>(s_stage + kBinChunk);
  uint32_t* s_delta = s_next + B.nbins;
  const WorkerPtrs P = B.w[k];
  const uint32_t* bin_start = ws_bin_start(B, k);
  uint2* __restrict__ rec = ws_records(B, k);
  const uint32_t mask = (1u << B.slice_log2) - 1u;
  // The grid is sized for the number of items expected; a workgroup takes the chunks blockIdx.x,
  // blockIdx.x + gridDim.x, ... that hold listed items.
  for (uint32_t chunk = blockIdx.x; (uint64_t)chunk * kBinChunk < have; chunk += gridDim.x) {   // uniform
    const uint64_t t0 = (uint64_t)chunk * kBinChunk;
    const uint32_t count = have - t0 < (uint64_t)kBinChunk ? (uint32_t)(have - t0) : (uint32_t)kBinChunk;
    const uint32_t* hist = ws_bin_hist(B, k) + (uint64_t)chunk * B.nbins;      // the bin's records in earlier chunks
    const uint32_t* pre = ws_slice_pre(B, k) + (uint64_t)chunk * B.nbins;

    uint32_t i[kBinItems], v[kBinItems];
    uint32_t ok = 0;                                      // bit u: item u exists and takes part (see load_item)
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      const uint32_t t = u * kBinBlock + threadIdx.x;
      if (t < count && load_item<MODE>(B, P, t0 + t, i[u], v[u])) ok |= 1u << u;
    }
    for (uint32_t e = threadIdx.x; e < B.nbins; e += kBinBlock) {
      const uint32_t at = pre[e];
      s_next[e] = at;
      s_delta[e] = bin_start[e] + hist[e] - at;
    }
    __syncthreads();

    for (uint32_t j = 0; j < B.d; ++j) {
      const uint64_t a = hp.a[j], b = hp.b[j], c = hp.c[j], e = hp.e[j];
      uint32_t* next = s_next + (j << spr_log2);
#pragma unroll
      for (int u = 0; u < kBinItems; ++u) {
        if (ok >> u & 1u) {
          const uint32_t h = bucket_of(i[u], a, b, B.log2w);
          const uint32_t sl = h >> B.slice_log2;
          const uint32_t key = (h & mask) | signbit_of(i[u], c, e) | (sl << 16);
          const uint32_t place = __hip_atomic_fetch_add(&next[sl], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          s_stage[place] = make_uint2(key, v[u]);
        }
      }
      __syncthreads();
      // the last slice's run ends where the row's records end
      const uint32_t records = s_next[((j + 1) << spr_log2) - 1];
      const uint32_t* delta = s_delta + (j << spr_log2);
      for (uint32_t p = threadIdx.x; p < records; p += kBinBlock) {
        const uint2 r = s_stage[p];
        rec[p + delta[(r.x >> 16) & 0x1FFFu]] = make_uint2(r.x & 0x80007FFFu, r.y);
      }
      __syncthreads();                                    // s_stage is free again (and, after the last row, the counters)
    }
  }
}

// A workgroup takes `per` consecutive bins (j, s) of one worker, one after the
// other.  A slice is accumulated in float64: the LDS float64 atomic add runs at
// full LDS rate on this chip (about 1.7e12 per second over the chip at random
// addresses) while the float32 one takes a slow path (0.2e12 per second,
// whatever the addresses); each cell is rounded to float32 once, when the slice
// is stored.  With 128 KiB of accumulators a compute unit holds one workgroup,
// and a workgroup that handled a single bin spent its life waiting: for its
// launch, for its first records, for its stores to drain.  Walking several bins
// hides all three: the first records of the next bin are requested before the
// current slice is read out, the read-out leaves zeros behind (no separate
// clearing pass), and the streaming stores of one slice drain while the next
// is being accumulated.
// STREAM_OUT: the slices leave with streaming stores.  Measured on MI355X: when the sketches of the launch
// add up to more than the memory-side cache keeps (config 5: 1.3 GB), streaming stores are the faster ones
// (410 against 442 us); when they do not (config 4: 336 MB; config 2: 25 MB), plain stores are (122 against
// 136 us, 58 against 62 us) and the merge that reads the sketches next gains a little too (86 -> 83 us).
// STREAM_IN: the records are read with streaming loads; the same kind of threshold from the other side: 49 MB
// of records (config 3) are read faster with plain loads (26 against 30 us: the scatter kernel has just
// written them), 253 MB (config 4) with streaming ones (123 against 136 us).
// (Both are compile-time: as run-time flags inside the unrolled loops they cost the kernel 6 to 10 %.)
template <bool STREAM_IN>
__device__ __forceinline__ u32x2 load_record(const u32x2* p) {
  if constexpr (STREAM_IN) return __builtin_nontemporal_load(p);
  else return *p;
}

template <bool STREAM_IN, bool STREAM_OUT>
__global__ __launch_bounds__(kSliceBlock) void sketch_slice_kernel(const EncodeBatch B, uint32_t per) {
  extern __shared__ double s_slice[];
  constexpr int kAhead = 4;                               // 8-byte record loads per thread and batch
  constexpr uint32_t kBatch = kSliceBlock * kAhead;       // records per batch; two batches are in flight
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;                           // uniform over the workgroup
  const uint32_t bin0 = blockIdx.x * per;                 // bin = (j << log2(slices per row)) + s
  if (bin0 >= B.nbins) return;                            // uniform over the workgroup
  const uint32_t bin1 = bin0 + per < B.nbins ? bin0 + per : B.nbins;
  const uint32_t cells = 1u << B.slice_log2;
  const uint32_t* bin_start = ws_bin_start(B, k);
  const u32x2* __restrict__ rec = reinterpret_cast<const u32x2*>(ws_records(B, k));
  const u32x2 none = {0u, 0u};
  // The records of consecutive bins are consecutive in memory: the workgroup streams through those of its
  // bins, batch after batch, whatever the bins' boundaries are; `base` is the position of the batch in x.
  const uint64_t end = bin_start[bin1];                   // 64 bits: positions near 2^32 must not wrap
  uint64_t base = bin_start[bin0];
  u32x2 x[kAhead], y[kAhead];
#pragma unroll
  for (int u = 0; u < kAhead; ++u) {
    const uint64_t r = base + threadIdx.x + u * kSliceBlock;
    x[u] = r < end ? load_record<STREAM_IN>(&rec[r]) : none;
    y[u] = r + kBatch < end ? load_record<STREAM_IN>(&rec[r + kBatch]) : none;
  }
  if (cells >= 2u * kSliceBlock) {                        // (the LDS array is 16-byte aligned)
    for (uint32_t c = threadIdx.x; c < cells / 2; c += kSliceBlock)
      reinterpret_cast<double2*>(s_slice)[c] = make_double2(0.0, 0.0);
  } else {
    for (uint32_t c = threadIdx.x; c < cells; c += kSliceBlock) s_slice[c] = 0.0;
  }
  uint32_t bin = bin0;
  uint64_t first = base, last = bin_start[bin0 + 1];      // the current bin's records are [first, last)
  uint64_t next_last = bin0 + 1 < bin1 ? bin_start[bin0 + 2] : last;
  __syncthreads();                                        // the slice is all zero
  while (true) {
    // the part of the batch that belongs to the current bin
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const uint64_t r = base + threadIdx.x + u * kSliceBlock;
      if (r >= first && r < last)
        __hip_atomic_fetch_add(&s_slice[x[u].x & 0x7FFFFFFFu],
                               (double)__uint_as_float(x[u].y ^ (x[u].x & 0x80000000u)),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    if (base + kBatch < last) {                           // uniform: the bin goes on beyond this batch
      base += kBatch;
#pragma unroll
      for (int u = 0; u < kAhead; ++u) {
        x[u] = y[u];
        const uint64_t r = base + kBatch + threadIdx.x + u * kSliceBlock;
        y[u] = r < end ? load_record<STREAM_IN>(&rec[r]) : none;
      }
      continue;
    }
    __syncthreads();                                      // every record of the bin is in the slice
    // the slice starts at cell bin * cells of the row-major sketch; every cell a thread reads it also clears
    float* out = B.w[k].sketch + (uint64_t)bin * cells;
    if (cells >= 4u * kSliceBlock) {                      // (every slice of 4 cells or more is 16-byte aligned)
      for (uint32_t c = threadIdx.x; c < cells / 4; c += kSliceBlock) {
        double2* cell = reinterpret_cast<double2*>(s_slice) + 2 * c;
        const double2 lo = cell[0], hi = cell[1];
        cell[0] = make_double2(0.0, 0.0);
        cell[1] = make_double2(0.0, 0.0);
        f32x4 o;
        o.x = (float)lo.x; o.y = (float)lo.y; o.z = (float)hi.x; o.w = (float)hi.y;
        if constexpr (STREAM_OUT) __builtin_nontemporal_store(o, &reinterpret_cast<f32x4*>(out)[c]);
        else reinterpret_cast<f32x4*>(out)[c] = o;
      }
    } else {
      for (uint32_t c = threadIdx.x; c < cells; c += kSliceBlock) {
        out[c] = (float)s_slice[c];
        s_slice[c] = 0.0;
      }
    }
    if (++bin == bin1) break;                             // uniform
    first = last;
    last = next_last;
    next_last = bin + 1 < bin1 ? bin_start[bin + 2] : last;
    if (first >= base + kBatch) {                         // uniform: the bin ended with the batch
      base += kBatch;
#pragma unroll
      for (int u = 0; u < kAhead; ++u) {
        x[u] = y[u];
        const uint64_t r = base + kBatch + threadIdx.x + u * kSliceBlock;
        y[u] = r < end ? load_record<STREAM_IN>(&rec[r]) : none;
      }
    }
    __syncthreads();                                      // the slice is all zero again
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
