// Host side and C ABI of the sparse-sketch gradient codec for gfx950
// (S2 Reducer, Algorithm 1 and Section 3.1).  See include/s2r.h for the
// contract of every entry point.  The kernels are in the headers included
// below, one per stage (s2r_scan.h, s2r_tiles.h, s2r_slices.h, s2r_merge.h,
// s2r_decode.h; s2r_layout.h holds their shared constants and argument
// structs); the Top-K sparsifier is a translation unit of its own (s2r_topk.hip).
//
// The gradient, the bitmaps and the index lists are cut into tiles of
// kTileWords bitmap words (= 64 * kTileWords elements), a tile into kScansPerTile
// pieces of kScanWords words.  No kernel waits for another workgroup and none
// shares a counter with another: ascending index lists come from per-piece counts
// (one 16-bit store per scan workgroup), a small prefix kernel over the tiles,
// and a second kernel that expands the bitmap at known offsets.
//
//   s2r_encode : zero_kernel           (atomic variant) zero the sketch
//                encode_scan_kernel    the one pass over the dense gradient:
//                                      bitmap words from wave ballots, per-piece
//                                      non-zero counts, and (INSERT variant) the
//                                      insertions S[j, h_j(i)] += s_j(i) g(i) as
//                                      float32 atomics
//                tile_prefix_kernel    tile counts from the piece counts, their
//                                      exclusive prefix, total
//                encode_compact_kernel Sparse(g): expands the bitmap (n/8 bytes)
//                                      and gathers the values at the set bits; tiles
//                                      with more than kGroupSlots set bits get
//                                      extra workgroups through a dense-tile list
//                bin_sort_kernel       (slice variant) Sparse(g) x rows, chunk by chunk, sorted by
//                                      sketch slice inside LDS into (cell, signed value) records
//                sketch_slice_kernel   (slice variant) every workgroup owns a slice of
//                                      one sketch row in LDS, adds the records of its
//                                      bin and stores the slice: no global atomics, no
//                                      zeroing of the sketch
//                sketch_overflow_kernel (slice variant) inserts, with atomics, the
//                                      non-zeros that did not fit the caller's list
//   s2r_merge  : merge_kernel          S = sum_k S_k (ascending k), C = OR_k C_k
//   s2r_decode : bitmap_count_kernel   per-piece popcounts of the aggregated bitmap
//                tile_prefix_kernel
//                decode_kernel         (gather variant) expands the bitmap; per index
//                                      the d signed bucket reads and their median
//                encode_compact_kernel, bin_sort_kernel, decode_slice_kernel,
//                decode_median_kernel  (slice variant) the union list, its queries
//                                      sorted by sketch slice chunk by chunk, answered
//                                      from LDS in place, medians per chunk
//                decode_rows_kernel, decode_rows_median_kernel
//                                      (rows variant) one sketch row per XCD: the
//                                      estimates row by row, then their medians
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include <atomic>

#include "../../include/s2r.h"
#include "s2r_device.h"
#include "s2r_internal.h"
#include "s2r_layout.h"
#include "s2r_scan.h"
#include "s2r_tiles.h"
#include "s2r_slices.h"
#include "s2r_merge.h"
#include "s2r_decode.h"

namespace s2r {

// ------------------------------------------------------------------ host side
// The library keeps no state between calls: strategies, the second stream and the
// measurement hooks of a call arrive in its s2r_options (resolved into an Exec).
static inline uint64_t splitmix_next(uint64_t& state) {
  state += 0x9E3779B97F4A7C15ull;
  uint64_t z = state;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static void make_hash_rows(uint64_t seed, uint32_t d, HashRows* hp) {
  uint64_t state = seed;
  for (uint32_t j = 0; j < (uint32_t)kMaxRows; ++j) {
    if (j < d) {
      hp->a[j] = splitmix_next(state) | 1ull;
      hp->b[j] = splitmix_next(state);
      hp->c[j] = splitmix_next(state) | 1ull;
      hp->e[j] = splitmix_next(state);
    } else {
      hp->a[j] = hp->b[j] = hp->c[j] = hp->e[j] = 0;
    }
  }
}

static inline bool is_pow2(uint32_t w) { return w != 0 && (w & (w - 1)) == 0; }
static inline uint32_t log2_of(uint32_t w) { uint32_t l = 0; while ((1u << l) < w) ++l; return l; }
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static s2r_status check_sizes(uint64_t n, uint32_t d, uint32_t w) {
  if (n == 0 || n > (1ull << 32)) return S2R_ERR_SIZE;
  if (d == 0 || d > S2R_MAX_ROWS) return S2R_ERR_SIZE;
  if (w == 0) return S2R_ERR_SIZE;
  if (!is_pow2(w)) return S2R_ERR_WIDTH;
  if (w > (1u << 31)) return S2R_ERR_SIZE;
  if ((uint64_t)d * w > (1ull << 32)) return S2R_ERR_SIZE;
  return S2R_OK;
}

static inline uint32_t tiles_of(uint64_t n) { return (uint32_t)ceil_div(ceil_div(n, 64), kTileWords); }

// workspace of one worker: [piece counts u16[ntiles * 16]] [tile prefix u64[ntiles + 1]]
// [dense-tile list: count u32, at +256 bytes entries u32[ntiles * 16]], and for the slice
// strategy [segment table u32[nchunks][nbins + 1]] [records 8 B x d*cap, a region of d * kBinChunk per chunk];
// each part 256-byte aligned.  The slice parts exist only when the caller's workspace is large enough for its cap.
static inline size_t workspace_prefix_off(uint64_t n) {
  return align256((size_t)tiles_of(n) * kScansPerTile * sizeof(uint16_t));
}
static inline size_t workspace_dense_off(uint64_t n) {
  return workspace_prefix_off(n) + align256(((size_t)tiles_of(n) + 1) * sizeof(uint64_t));
}
static inline size_t workspace_base(uint64_t n) {
  return workspace_dense_off(n) + 256 + align256((size_t)tiles_of(n) * kGroupsPerTile * sizeof(uint32_t));
}
// Workgroups of the kernels that take the dense-tile list (per problem); each loops over the entries.  An
// entry stands for kGroupSlots list positions beyond a tile's first kGroupSlots, so `positions` expected list
// positions make at most positions / kGroupSlots entries: launching more helpers than that only fills the
// chip with workgroups that read the entry count and leave (with 8 workers and 2048 helpers each, eight rounds
// of them before the first tile was touched).
static inline uint32_t dense_grid(uint32_t ntiles, uint64_t positions, uint32_t most) {
  uint64_t entries = (uint64_t)ntiles * (kGroupsPerTile - 1);
  const uint64_t expected = positions / kGroupSlots + 8;
  if (entries > expected) entries = expected;
  return (uint32_t)(entries < most ? (entries > 0 ? entries : 1) : most);
}
struct SliceLayout {
  bool possible;             // the bins fit the LDS histograms and record positions fit 32 bits
  uint32_t slice_log2, nbins, nchunks;
  size_t seg_off, rec_off, total;
};
static SliceLayout slice_layout(uint64_t n, uint32_t d, uint32_t w, uint64_t cap) {
  SliceLayout L;
  const uint32_t log2w = log2_of(w);
  L.slice_log2 = log2w < (uint32_t)kSliceLog2Max ? log2w : (uint32_t)kSliceLog2Max;
  const uint64_t nbins = (uint64_t)d << (log2w - L.slice_log2);
  L.possible = nbins <= (uint64_t)kMaxBins && (uint64_t)d * cap < (1ull << 32) && cap > 0;
  L.nbins = (uint32_t)(L.possible ? nbins : 0);
  L.nchunks = (uint32_t)(L.possible ? ceil_div(cap, kBinChunk) : 0);
  // the segment offsets u32[nchunks][nbins + 1], then the records: a chunk's region holds kBinChunk * d of them
  // (the last chunk's, d * what is left of cap)
  L.seg_off = workspace_base(n);
  L.rec_off = L.seg_off + align256((size_t)L.nchunks * ((size_t)L.nbins + 1) * sizeof(uint32_t));
  L.total = L.rec_off + align256((size_t)(L.possible ? d * cap : 0) * 8);
  return L;
}

// How s2r_encode forms the sketch.  Cost models fitted to measurements on MI355X
// (W = 4..16, n = 2^20..1e9, d = 3..5, w = 2^14..2^22):
//  - atomics: the sketch is zeroed first (about 4.5e12 bytes per second); scattered
//    float32 atomics retire at about 21e9 per second over the whole chip whatever
//    their scope, and when the dense scan issues them it hides about 40 % of that
//    time (less when the non-zeros are clustered in few workgroups);
//  - slices: three more kernels, about 13 us of launches; 4 us per round of 256
//    slice workgroups (each clears and stores 128 KiB of LDS); sort and slice
//    kernels together pass about 200e9 records per second.
// `sort_cap` is the number of list items whose counting sort the workspace holds (at most the lists'
// capacity), `expect` the number of items expected (the caller's estimate, or the lists' capacity when
// there is none); `asked` the caller's wish.
// The largest number of list items (<= cap) whose counting sort fits a workspace share of `bytes`; 0 if none.
static uint64_t sort_capacity(uint64_t n, uint32_t d, uint32_t w, uint64_t cap, size_t bytes) {
  if (cap == 0) return 0;
  uint64_t hi = cap;                                       // (record positions are 32-bit)
  const uint64_t most = ((1ull << 32) - 1) / d;
  if (hi > most) hi = most;
  {
    const SliceLayout L = slice_layout(n, d, w, hi);
    if (!L.possible) return 0;
    if (L.total <= bytes) return hi;
  }
  uint64_t lo = 0;                                         // total(lo) fits (or lo = 0), total(hi) does not
  while (hi - lo > 1) {
    const uint64_t mid = lo + (hi - lo) / 2;
    if (slice_layout(n, d, w, mid).total <= bytes) lo = mid; else hi = mid;
  }
  return lo;
}

static int32_t choose_strategy(uint32_t W, uint64_t n, uint32_t d, uint32_t w, bool have_lists, uint64_t sort_cap,
                               uint64_t expect, int32_t asked) {
  if (!have_lists || sort_cap == 0) return S2R_INSERT_ATOMIC;     // the slice strategy reads Sparse(g)
  if (asked != S2R_INSERT_AUTO) return asked;
  if (sort_cap < expect) return S2R_INSERT_ATOMIC;           // most items would be inserted with atomics after all
  const SliceLayout L = slice_layout(n, d, w, sort_cap);
  const double records = (double)expect * d;
  const double rounds = (double)ceil_div((uint64_t)W * L.nbins, 256);       // all workers' slices share the CUs
  const double t_slice = 20e-6 + rounds * 4e-6 + W * records / 180e9;
  const double t_atomic = W * (4.0 * d * w / 4.5e12 + 0.6 * records / 21e9);
  return t_slice < t_atomic ? S2R_INSERT_SLICE : S2R_INSERT_ATOMIC;
}

// Workspace of s2r_decode when it partitions its queries by sketch slice: the base parts, then
// [segment offsets u32[nchunks][nbins + 1]] [queries, chunk by chunk, sorted by bin, 4 B x d * nchunks * kBinChunk]
// [answers, same shape].
constexpr int kDecodeSliceMaxRows = 8;                   // decode_median_kernel keeps 8 x d estimates per thread
struct DecodeLayout {
  bool possible;
  uint32_t slice_log2, nbins, nchunks;
  size_t seg_off, rec_off, answers_off, total;
};
static DecodeLayout decode_layout(uint64_t n, uint32_t d, uint32_t w, uint64_t cap) {
  DecodeLayout L;
  const uint32_t log2w = log2_of(w);
  L.slice_log2 = log2w < (uint32_t)kDecodeSliceLog2Max ? log2w : (uint32_t)kDecodeSliceLog2Max;
  const uint64_t nbins = (uint64_t)d << (log2w - L.slice_log2);
  L.possible = nbins <= (uint64_t)kMaxBins && (uint64_t)d * (cap + kBinChunk) < (1ull << 32) && cap > 0 &&
               d <= (uint32_t)kDecodeSliceMaxRows;                 // (places of answers are 32-bit)
  L.nbins = (uint32_t)(L.possible ? nbins : 0);
  L.nchunks = (uint32_t)(L.possible ? ceil_div(cap, kBinChunk) : 0);
  L.seg_off = workspace_base(n);
  L.rec_off = L.seg_off + align256((size_t)L.nchunks * ((size_t)L.nbins + 1) * sizeof(uint32_t));
  L.answers_off = L.rec_off + align256((size_t)L.nchunks * kBinChunk * d * 4);
  L.total = L.answers_off + align256((size_t)L.nchunks * kBinChunk * d * 4);
  return L;
}

// Workspace of s2r_decode's row route: the base parts, then the estimates, float32[d][stride], stride = the
// list's capacity rounded up to 64 entries.
constexpr uint32_t kRowsMaxRows = 8;                     // eight XCDs
struct RowsLayout {
  bool possible;
  uint64_t stride;
  size_t est_off, total;
};
static RowsLayout rows_layout(uint64_t n, uint32_t d, uint64_t cap) {
  RowsLayout L;
  L.possible = d <= kRowsMaxRows && cap > 0;
  L.stride = ceil_div(cap, 64) * 64;
  L.est_off = workspace_base(n);
  L.total = L.est_off + (L.possible ? align256((size_t)d * L.stride * sizeof(float)) : 0);
  return L;
}

// How s2r_decode reads the buckets.  Measured on MI355X: gathers from a sketch far larger than the L2
// (4 MB per XCD) run at about 56e9 per second (each fetches a 128-byte line), from one of a few L2 sizes at
// about 70e9, from one that fits at about 200e9; the slice route costs about 80 us of launches and latency
// and passes about 110e9 queries per second.
// `cap` is the capacity of the caller's lists, `expect` the number of union indices expected (the caller's
// estimate, or cap when there is none: only the device knows the true number); `asked` the caller's wish.
static int32_t choose_decode(uint64_t n, uint32_t d, uint32_t w, bool have_lists, bool dense_out, uint64_t cap,
                             uint64_t expect, size_t workspace_bytes, int32_t asked) {
  if (!have_lists || dense_out || cap == 0) return S2R_DECODE_GATHER;
  const DecodeLayout L = decode_layout(n, d, w, cap);
  const RowsLayout R = rows_layout(n, d, cap);
  const bool slice_ok = L.possible && workspace_bytes >= L.total;
  const bool rows_ok = R.possible && workspace_bytes >= R.total;
  if (asked == S2R_DECODE_SLICE) return slice_ok ? S2R_DECODE_SLICE : S2R_DECODE_GATHER;
  if (asked == S2R_DECODE_ROWS) return rows_ok ? S2R_DECODE_ROWS : S2R_DECODE_GATHER;
  if (asked == S2R_DECODE_GATHER) return S2R_DECODE_GATHER;
  const double queries = (double)expect * d;
  const double sketch_bytes = 4.0 * d * w;
  double best = queries / (sketch_bytes > 16e6 ? 56e9 : sketch_bytes > 4e6 ? 70e9 : 200e9);
  int32_t choice = S2R_DECODE_GATHER;
  // a row per XCD pays when a row fits an L2 (4 MB) and the whole sketch does not; it costs one more launch and
  // a pass over the estimates
  if (rows_ok && 4.0 * w <= 4.2e6 && sketch_bytes > 4.2e6 && 8e-6 + queries / 125e9 < best) {
    best = 8e-6 + queries / 125e9;
    choice = S2R_DECODE_ROWS;
  }
  if (slice_ok && 80e-6 + queries / 110e9 < best) choice = S2R_DECODE_SLICE;
  return choice;
}

// The slice kernels use more dynamic LDS than the default limit allows; the limit is a property of the
// loaded kernel, raised once per device (asking again is harmless).
static bool raise_scatter_lds(const void* kernel) {
  return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)(kBinChunk * sizeof(uint2) + sizeof(uint32_t) * kMaxBins)) == hipSuccess;
}
static bool raise_slice_lds(const void* kernel) {
  return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSliceLdsMax) == hipSuccess;
}
static bool raise_lds_limits() {
  constexpr int kMaxDevices = 64;
  static std::atomic<bool> raised[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) return false;
  if (dev < kMaxDevices && raised[dev].load(std::memory_order_acquire)) return true;
  if (!raise_slice_lds(reinterpret_cast<const void*>(sketch_slice_kernel<true, true>)) ||
      !raise_slice_lds(reinterpret_cast<const void*>(sketch_slice_kernel<true, false>)) ||
      !raise_slice_lds(reinterpret_cast<const void*>(sketch_slice_kernel<false, true>)) ||
      !raise_slice_lds(reinterpret_cast<const void*>(sketch_slice_kernel<false, false>)) ||
      !raise_scatter_lds(reinterpret_cast<const void*>(bin_sort_kernel<0>)) ||
      !raise_scatter_lds(reinterpret_cast<const void*>(bin_sort_kernel<1>)) ||
      !raise_scatter_lds(reinterpret_cast<const void*>(bin_sort_kernel<2>)) ||
      !raise_scatter_lds(reinterpret_cast<const void*>(bin_sort_kernel<3>)) ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(decode_slice_kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)(sizeof(float) << kDecodeSliceLog2Max)) != hipSuccess)
    return false;
  if (dev < kMaxDevices) raised[dev].store(true, std::memory_order_release);
  return true;
}

static inline void record(const Exec& X, int slot, bool end, hipStream_t st) {
  if (X.trace == nullptr) return;
  hipEvent_t ev = (hipEvent_t)(end ? X.trace->end[slot] : X.trace->begin[slot]);
  if (ev != nullptr) (void)hipEventRecord(ev, st);
}

static inline bool launch_ok() { return hipGetLastError() == hipSuccess; }

static void launch_rows_median(uint32_t d, const float* est, uint64_t stride, const uint64_t* count, uint64_t cap,
                               float* val_out, uint32_t block, uint64_t n, const uint32_t* blk_list, uint64_t expect,
                               hipStream_t st) {
  const uint64_t wgs = ceil_div(expect > 0 ? expect : 1, (uint64_t)kBlock * 2);        // (the threads loop)
  const dim3 grid((uint32_t)(wgs < 16384 ? wgs : 16384)), blk(kBlock);
  switch (d) {
    case 1: hipLaunchKernelGGL(decode_rows_median_kernel<1>, grid, blk, 0, st, est, stride, count, cap, val_out, block, n, blk_list); break;
    case 2: hipLaunchKernelGGL(decode_rows_median_kernel<2>, grid, blk, 0, st, est, stride, count, cap, val_out, block, n, blk_list); break;
    case 3: hipLaunchKernelGGL(decode_rows_median_kernel<3>, grid, blk, 0, st, est, stride, count, cap, val_out, block, n, blk_list); break;
    case 4: hipLaunchKernelGGL(decode_rows_median_kernel<4>, grid, blk, 0, st, est, stride, count, cap, val_out, block, n, blk_list); break;
    case 5: hipLaunchKernelGGL(decode_rows_median_kernel<5>, grid, blk, 0, st, est, stride, count, cap, val_out, block, n, blk_list); break;
    case 6: hipLaunchKernelGGL(decode_rows_median_kernel<6>, grid, blk, 0, st, est, stride, count, cap, val_out, block, n, blk_list); break;
    case 7: hipLaunchKernelGGL(decode_rows_median_kernel<7>, grid, blk, 0, st, est, stride, count, cap, val_out, block, n, blk_list); break;
    default: hipLaunchKernelGGL(decode_rows_median_kernel<8>, grid, blk, 0, st, est, stride, count, cap, val_out, block, n, blk_list); break;
  }
}

template <int D>
static void launch_decode(uint32_t ntiles, uint32_t helpers, hipStream_t st, const DecodeArgs& A, const HashRows& hp) {
  if (A.dense_out == nullptr) {
    hipLaunchKernelGGL(decode_kernel<D>, dim3(helpers + ntiles), dim3(kBlock), 0, st, A, hp, helpers);
  } else {                                               // group 0 of every tile first: it clears the dense output
    hipLaunchKernelGGL(decode_kernel<D>, dim3(ntiles), dim3(kBlock), 0, st, A, hp, 0u);
    hipLaunchKernelGGL(decode_kernel<D>, dim3(helpers), dim3(kBlock), 0, st, A, hp, helpers);
  }
}

}  // namespace s2r

using namespace s2r;

extern "C" {

int32_t s2r_version(void) { return 510; }

const char* s2r_status_string(s2r_status status) {
  switch (status) {
    case S2R_OK: return "ok";
    case S2R_ERR_NULL: return "a required pointer is NULL";
    case S2R_ERR_SIZE: return "n, d, w, W or cap outside the supported range";
    case S2R_ERR_WIDTH: return "sketch width w is not a power of two";
    case S2R_ERR_WORKSPACE: return "workspace is NULL, misaligned or too small";
    case S2R_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    case S2R_ERR_ALIGN: return "a buffer is not aligned as documented";
    default: return "unknown status";
  }
}

size_t s2r_workspace_bytes(uint64_t n, uint32_t d, uint32_t w) {
  if (check_sizes(n, d, w) != S2R_OK) return 0;
  return workspace_base(n);
}

size_t s2r_encode_workspace_bytes(uint64_t n, uint32_t d, uint32_t w, uint64_t cap) {
  if (check_sizes(n, d, w) != S2R_OK || cap > n) return 0;
  const SliceLayout L = slice_layout(n, d, w, cap);
  return L.possible ? L.total : workspace_base(n);
}

s2r_status s2r_hash_params(uint64_t seed, uint32_t d, uint64_t* params_out) {
  if (params_out == nullptr) return S2R_ERR_NULL;
  if (d == 0 || d > S2R_MAX_ROWS) return S2R_ERR_SIZE;
  HashRows hp;
  make_hash_rows(seed, d, &hp);
  for (uint32_t j = 0; j < d; ++j) {
    params_out[4 * j + 0] = hp.a[j];
    params_out[4 * j + 1] = hp.b[j];
    params_out[4 * j + 2] = hp.c[j];
    params_out[4 * j + 3] = hp.e[j];
  }
  return S2R_OK;
}

size_t s2r_decode_workspace_bytes(uint64_t n, uint32_t d, uint32_t w, uint64_t cap) {
  if (check_sizes(n, d, w) != S2R_OK || cap > n) return 0;
  const DecodeLayout L = decode_layout(n, d, w, cap);
  const RowsLayout R = rows_layout(n, d, cap);
  return L.possible && L.total > R.total ? L.total : R.total;
}

s2r_status s2r_probe_read(const void* src, size_t bytes, uint64_t* sink, void* stream) {
  if (src == nullptr || sink == nullptr) return S2R_ERR_NULL;
  if (bytes < 16 || bytes / 16 > (1ull << 40)) return S2R_ERR_SIZE;
  if (((uintptr_t)src & 15u) || ((uintptr_t)sink & 7u)) return S2R_ERR_ALIGN;
  const uint64_t nvec = bytes / 16;
  const uint64_t blocks = ceil_div(nvec, (uint64_t)kBlock * kProbePer);
  if (blocks > 0x7FFFFFFFull) return S2R_ERR_SIZE;
  hipLaunchKernelGGL(probe_read_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0, (hipStream_t)stream,
                     reinterpret_cast<const u32x4*>(src), nvec, sink, 0xA5C3F00Du);
  return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
}

// The encode of W workers (W = 1 for s2r_encode): every kernel takes a group of
// workers, the worker in first_worker + blockIdx.y.  workspace_bytes is the size of
// the whole workspace, split evenly between the workers.
// block = 0: the element codec (bitmaps of n bits, lists of non-zero elements with their values).
// block >= 1: the block-granular codec (bitmaps of ceil(n / block) bits, lists of non-zero blocks, nz_val
// unused, cap counted in blocks).
// The chunk-local counting sort, in the variant for what the items are.
static void launch_bin_sort(const EncodeBatch& E, const HashRows& hp, dim3 grid, hipStream_t st) {
  const size_t lds = (size_t)kBinChunk * sizeof(uint2) + sizeof(uint32_t) * E.nbins;
  switch (items_mode(E)) {
    case 0: hipLaunchKernelGGL(bin_sort_kernel<0>, grid, dim3(kBinBlock), lds, st, E, hp); break;
    case 1: hipLaunchKernelGGL(bin_sort_kernel<1>, grid, dim3(kBinBlock), lds, st, E, hp); break;
    case 2: hipLaunchKernelGGL(bin_sort_kernel<2>, grid, dim3(kBinBlock), lds, st, E, hp); break;
    default: hipLaunchKernelGGL(bin_sort_kernel<3>, grid, dim3(kBinBlock), lds, st, E, hp); break;
  }
}

struct EncodeLaunch {                      // what the launches of one call share
  uint32_t ntiles, scan_blocks, scan_group;
  uint32_t chunk_grid;                     // workgroups per worker of the kernels that walk the list chunks
  uint64_t expect_bits;                    // set bits expected in a worker's bitmap
  uint64_t expect_items;                   // items expected in a worker's counting sort
  uint64_t nvec, zb;
  uint32_t ntail;
  int32_t strategy;
  bool lists, marked;
  uint32_t log2w;
};

// Zeroing and the dense scan of workers first .. first + count - 1 on st (gradients of 1 GiB and more are
// scanned worker by worker, smaller ones with one launch over the group).
static s2r_status launch_scans(EncodeBatch& E, const HashRows& hp, const EncodeLaunch& L, uint32_t first,
                               uint32_t count, bool traced, const Exec& X, hipStream_t st, uint32_t* last_launch) {
  const bool atomics = L.strategy == S2R_INSERT_ATOMIC;
  const uint32_t step = L.scan_group < count ? L.scan_group : count;
  for (uint32_t k0 = first; k0 < first + count; k0 += step) {
    const uint32_t gy = first + count - k0 < step ? first + count - k0 : step;
    const bool last = traced && k0 + gy == first + count;    // the events bracket the call's last scan launch
    E.first_worker = k0;
    if (atomics || E.block != 0) {                            // the block bitmap is set bit by bit: zero it first
      hipLaunchKernelGGL(zero_kernel, dim3((uint32_t)L.zb, gy), dim3(kBlock), 0, st, E, atomics ? L.nvec : (uint64_t)0,
                         atomics ? L.ntail : 0u, E.block != 0 ? E.nwords : (uint64_t)0);
      if (!launch_ok()) return S2R_ERR_LAUNCH;
    }
    if (last) record(X, S2R_KERNEL_ENCODE_SCAN, false, st);
    const dim3 sgrid(L.scan_blocks, gy), sblock(kBlock);
    if (E.block != 0 && atomics)
      hipLaunchKernelGGL((encode_scan_kernel<kScanEPL, true, true>), sgrid, sblock, 0, st, E, hp);
    else if (E.block != 0)
      hipLaunchKernelGGL((encode_scan_kernel<kScanEPL, false, true>), sgrid, sblock, 0, st, E, hp);
    else if (atomics)
      hipLaunchKernelGGL((encode_scan_kernel<kScanEPL, true, false>), sgrid, sblock, 0, st, E, hp);
    else
      hipLaunchKernelGGL((encode_scan_kernel<kScanEPL, false, false>), sgrid, sblock, 0, st, E, hp);
    if (last) record(X, S2R_KERNEL_ENCODE_SCAN, true, st);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    *last_launch = gy;
  }
  return S2R_OK;
}

// Everything after the scan for workers first .. first + count - 1, on st: counts of the block bitmap,
// tile prefix, the lists, and the sketch by slices (or, for marked blocks under the atomic strategy, by the
// overflow kernel from list position 0).
static s2r_status launch_after_scan(EncodeBatch& E, const HashRows& hp, const EncodeLaunch& L, uint32_t first,
                                    uint32_t count, bool traced, const Exec& X, hipStream_t st) {
  E.first_worker = first;
  const uint32_t ntiles = L.ntiles;
  if (E.block != 0) {                                        // the counts of the block bitmap's pieces
    hipLaunchKernelGGL(bitmap_count_batch_kernel, dim3((uint32_t)ceil_div(ntiles, kWavesPerBlock), count), dim3(kBlock),
                       0, st, E);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(tile_prefix_kernel, dim3(1, count), dim3(kPrefixBlock), 0, st, E.workspace + first * E.ws_stride,
                     E.ws_stride, E.prefix_off, E.dense_off, ntiles, E.nnz_out + first);
  if (!launch_ok()) return S2R_ERR_LAUNCH;

  if (L.lists && E.cap > 0) {
    const uint32_t helpers = dense_grid(ntiles, L.expect_bits, 512);
    if (E.w[first].nz_val != nullptr)          // (all workers of a call have value lists, or none has)
      hipLaunchKernelGGL(encode_compact_kernel<true>, dim3(helpers + ntiles, count), dim3(kBlock), 0, st, E, helpers);
    else
      hipLaunchKernelGGL(encode_compact_kernel<false>, dim3(helpers + ntiles, count), dim3(kBlock), 0, st, E, helpers);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }

  if (L.strategy == S2R_INSERT_SLICE) {
    const size_t lds = sizeof(double) << E.slice_log2;
    launch_bin_sort(E, hp, dim3(L.chunk_grid, count), st);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    if (traced) record(X, S2R_KERNEL_ENCODE_SLICE, false, st);
    // about one workgroup per compute unit, each walking `per` consecutive bins of one worker
    // One workgroup is resident per compute unit (its slice fills the LDS).  Two rounds of workgroups with half
    // the bins each beat one round when a workgroup still walks enough bins to spread its start-up (clearing
    // 128 KiB of LDS, the first loads), or when one round would leave units idle anyway.  Measured (us): 5120
    // (bin, worker) pairs 135 -> 129, 384 pairs of 67 K records 66 -> 57, 20480 pairs 465 -> 467; 1536 pairs
    // (6 or 3 bins per workgroup) 27.5 -> 29, which therefore stay one round.
    const uint64_t pairs = (uint64_t)E.nbins * count;
    uint32_t per = (uint32_t)ceil_div(pairs, 2 * kSliceWorkgroups);
    if (per < 4 && ceil_div(pairs, kSliceWorkgroups) > 2) per = (uint32_t)ceil_div(pairs, kSliceWorkgroups);
    // (streaming stores only when the call's sketches are more than the memory-side cache keeps)
    const bool stream_out = ((uint64_t)E.nworkers * E.d << E.log2w) * sizeof(float) > (512ull << 20);
    const bool stream_in = (uint64_t)E.nworkers * L.expect_items * E.d * 8 > (128ull << 20);
    const dim3 sgrid((uint32_t)ceil_div(E.nbins, per), count), sblock(kSliceBlock);
    if (stream_in && stream_out) hipLaunchKernelGGL((sketch_slice_kernel<true, true>), sgrid, sblock, lds, st, E, per);
    else if (stream_in) hipLaunchKernelGGL((sketch_slice_kernel<true, false>), sgrid, sblock, lds, st, E, per);
    else if (stream_out) hipLaunchKernelGGL((sketch_slice_kernel<false, true>), sgrid, sblock, lds, st, E, per);
    else hipLaunchKernelGGL((sketch_slice_kernel<false, false>), sgrid, sblock, lds, st, E, per);
    if (traced) record(X, S2R_KERNEL_ENCODE_SLICE, true, st);
    if (!launch_ok()) return S2R_ERR_LAUNCH;

    hipLaunchKernelGGL(sketch_overflow_kernel, dim3((uint32_t)ceil_div(ntiles, kBlock), count), dim3(kBlock), 0, st, E, hp);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  } else if (L.marked) {
    // no scan has inserted anything: every set block goes the way of the blocks beyond the lists
    EncodeBatch A = E;
    A.sort_cap = 0;
    hipLaunchKernelGGL(sketch_overflow_kernel, dim3((uint32_t)ceil_div(ntiles, kBlock), count), dim3(kBlock), 0, st, A, hp);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }
  return S2R_OK;
}

static s2r_status encode_workers(const float* const* grads, uint32_t W, uint64_t n, uint32_t block, uint32_t d,
                                 uint32_t w, uint64_t seed, float* const* sketches, uint64_t* const* bitmaps,
                                 uint32_t* const* nz_idx, float* const* nz_val, uint64_t cap, uint64_t* nnz_out,
                                 void* workspace, size_t workspace_bytes, hipStream_t st, const Exec& X,
                                 bool marked = false) {
  // marked: the (block) bitmaps are given; there is no scan, and grads[k] is read inside the set blocks only
  if (grads == nullptr || sketches == nullptr || bitmaps == nullptr || nnz_out == nullptr) return S2R_ERR_NULL;
  if (W == 0 || W > S2R_MAX_WORKERS || (marked && block == 0)) return S2R_ERR_SIZE;
  const s2r_status sz = check_sizes(n, d, w);
  if (sz != S2R_OK) return sz;
  const bool lists = nz_idx != nullptr && nz_idx[0] != nullptr;
  if (block == 0 && (nz_idx == nullptr) != (nz_val == nullptr)) return S2R_ERR_NULL;
  if (((uintptr_t)nnz_out & 7u) != 0) return S2R_ERR_ALIGN;
  const uint64_t nbits = block != 0 ? ceil_div(n, block) : n;      // bits of a worker's bitmap

  EncodeBatch E;
  for (uint32_t k = 0; k < W; ++k) {
    if (grads[k] == nullptr || sketches[k] == nullptr || bitmaps[k] == nullptr) return S2R_ERR_NULL;
    uint32_t* ik = nz_idx ? nz_idx[k] : nullptr;
    float* vk = nz_val ? nz_val[k] : nullptr;
    if ((block == 0 && (ik == nullptr) != (vk == nullptr)) || (ik != nullptr) != lists) return S2R_ERR_NULL;
    if (((uintptr_t)grads[k] & 3u) || ((uintptr_t)sketches[k] & 15u) || ((uintptr_t)bitmaps[k] & 7u) ||
        ((uintptr_t)ik & 3u) || ((uintptr_t)vk & 3u)) return S2R_ERR_ALIGN;
    E.w[k].grad = reinterpret_cast<const uint32_t*>(grads[k]);
    E.w[k].sketch = sketches[k];
    E.w[k].bitmap = bitmaps[k];
    E.w[k].nz_idx = ik;
    E.w[k].nz_val = reinterpret_cast<uint32_t*>(vk);
  }
  if (!lists) cap = 0;
  if (cap > nbits) cap = nbits;                               // there cannot be more list entries than bits
  const uint64_t cap_items = block != 0 ? cap * block : cap;  // elements the lists stand for, at most
  uint64_t expect = X.expected_nnz != 0 && X.expected_nnz < cap ? X.expected_nnz : cap;
  if (block != 0) expect *= block;                            // items the sort is expected to see
  const size_t ws_each = (workspace_bytes / W) & ~(size_t)255;
  if (workspace == nullptr || ((uintptr_t)workspace & 255u) != 0 || ws_each < workspace_base(nbits))
    return S2R_ERR_WORKSPACE;

  HashRows hp;
  make_hash_rows(seed, d, &hp);
  EncodeLaunch L;
  L.ntiles = tiles_of(nbits);
  L.log2w = log2_of(w);
  // what the counting sort can take: list items (elements of listed blocks in the block codec), whole list
  // entries only
  uint64_t sort_items = lists ? sort_capacity(nbits, d, w, cap_items, ws_each) : 0;
  if (block != 0) sort_items -= sort_items % block;
  L.strategy = choose_strategy(W, nbits, d, w, lists, sort_items, expect, X.insert_strategy);
  if (L.strategy != S2R_INSERT_SLICE) sort_items = 0;
  L.lists = lists;
  L.marked = marked;
  // (the chunk kernels loop: a grid sized for the expected items serves any number of them)
  L.chunk_grid = (uint32_t)ceil_div(expect > 0 ? expect : 1, kBinChunk);
  L.expect_bits = block != 0 ? expect / block : expect;
  L.expect_items = expect;

  E.nworkers = W;
  E.payload_slot = 0;
  E.nnz_out = nnz_out;
  E.workspace = reinterpret_cast<char*>(workspace);
  E.ws_stride = ws_each;
  E.block = block;
  E.prefix_off = workspace_prefix_off(nbits);
  E.dense_off = workspace_dense_off(nbits);
  const SliceLayout SL = slice_layout(nbits, d, w, sort_items);
  E.seg_off = SL.seg_off;
  E.rec_off = SL.rec_off;
  E.nbins = SL.nbins;
  E.nchunks = SL.nchunks;
  E.n = n;
  E.nwords = ceil_div(nbits, 64);
  E.cap = cap;
  E.sort_cap = block != 0 ? sort_items / block : sort_items;
  E.ntiles = L.ntiles;
  E.d = d;
  E.log2w = L.log2w;
  E.slice_log2 = SL.slice_log2;
  E.first_worker = 0;

  // The scan, preceded by the zeroing of the sketch when the scan inserts into it with atomics.  Gradients
  // of 1 GiB and more are scanned worker by worker, smaller ones with one launch over a whole group.
  // Measured on config 5 (4 GB per worker, 84 MB sketches): one launch per worker takes 632 us per worker,
  // one launch over all workers 649 us; with atomics, a scan whose sketch was zeroed just before it takes
  // 760 us against 820 us when all 16 sketches were zeroed first.  Below 1 GiB the launches saved count more.
  const uint64_t cells = (uint64_t)d * w;
  const bool atomics = L.strategy == S2R_INSERT_ATOMIC;
  L.nvec = cells / 4;
  L.ntail = (uint32_t)(cells - L.nvec * 4);
  L.zb = ceil_div(L.nvec > 0 ? L.nvec : 1, kBlock);
  if (L.zb > 2048) L.zb = 2048;
  L.scan_group = n * sizeof(float) >= (1ull << 30) ? 1u : W;
  // element codec: every piece of every tile gets its count; block codec: the pieces that hold elements
  L.scan_blocks = block != 0 ? (uint32_t)ceil_div(ceil_div(n, 64), kScanWords) : L.ntiles * kScansPerTile;
  if (L.strategy == S2R_INSERT_SLICE && !raise_lds_limits()) return S2R_ERR_LAUNCH;

  if (X.report != nullptr) X.report->insert_strategy = L.strategy;
  uint32_t last_launch = 0;
  if (marked) {
    if (atomics) {                                            // the sketches only: the bitmaps are the caller's
      hipLaunchKernelGGL(zero_kernel, dim3((uint32_t)L.zb, W), dim3(kBlock), 0, st, E, L.nvec, L.ntail, (uint64_t)0);
      if (!launch_ok()) return S2R_ERR_LAUNCH;
    }
    return launch_after_scan(E, hp, L, 0, W, true, X, st);
  }

  s2r_status rc = launch_scans(E, hp, L, 0, W, true, X, st, &last_launch);
  if (rc != S2R_OK) return rc;
  rc = launch_after_scan(E, hp, L, 0, W, true, X, st);
  if (rc != S2R_OK) return rc;
  if (X.report != nullptr) X.report->scan_launch_workers = last_launch;
  return S2R_OK;
}

s2r_status s2r_encode_batch_ex(const float* const* grads, uint32_t W, uint64_t n, uint32_t d, uint32_t w,
                               uint64_t seed, float* const* sketches, uint64_t* const* bitmaps,
                               uint32_t* const* nz_idx, float* const* nz_val, uint64_t cap, uint64_t* nnz_out,
                               void* workspace, size_t workspace_bytes, void* stream, const s2r_options* options) {
  Exec X;
  const s2r_status rc = resolve_options(options, &X);
  if (rc != S2R_OK) return rc;
  return encode_workers(grads, W, n, 0u, d, w, seed, sketches, bitmaps, nz_idx, nz_val, cap, nnz_out, workspace,
                        workspace_bytes, (hipStream_t)stream, X);
}

s2r_status s2r_encode_ex(const float* grad, uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                         float* sketch, uint64_t* bitmap, uint32_t* nz_idx, float* nz_val, uint64_t cap,
                         uint64_t* nnz_out, void* workspace, size_t workspace_bytes, void* stream,
                         const s2r_options* options) {
  if ((nz_idx == nullptr) != (nz_val == nullptr)) return S2R_ERR_NULL;
  return s2r_encode_batch_ex(&grad, 1, n, d, w, seed, &sketch, &bitmap, nz_idx ? &nz_idx : nullptr,
                             nz_val ? &nz_val : nullptr, cap, nnz_out, workspace, workspace_bytes, stream, options);
}

s2r_status s2r_encode(const float* grad, uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                      float* sketch, uint64_t* bitmap, uint32_t* nz_idx, float* nz_val, uint64_t cap,
                      uint64_t* nnz_out, void* workspace, size_t workspace_bytes, void* stream) {
  return s2r_encode_ex(grad, n, d, w, seed, sketch, bitmap, nz_idx, nz_val, cap, nnz_out, workspace, workspace_bytes,
                       stream, nullptr);
}

s2r_status s2r_encode_batch(const float* const* grads, uint32_t W, uint64_t n, uint32_t d, uint32_t w,
                            uint64_t seed, float* const* sketches, uint64_t* const* bitmaps,
                            uint32_t* const* nz_idx, float* const* nz_val, uint64_t cap, uint64_t* nnz_out,
                            void* workspace, size_t workspace_bytes, void* stream) {
  return s2r_encode_batch_ex(grads, W, n, d, w, seed, sketches, bitmaps, nz_idx, nz_val, cap, nnz_out, workspace,
                             workspace_bytes, stream, nullptr);
}

// piece_count: NULL, or where the aggregated bitmap's set-bit counts per piece go (uint16[16 * tiles]: the
// first part of a decode workspace).  launch = false only checks the arguments.
static s2r_status merge_impl(const float* const* sketches, const uint64_t* const* bitmaps, uint32_t W, uint64_t n,
                             uint32_t d, uint32_t w, float* sketch_out, uint64_t* bitmap_out, uint16_t* piece_count,
                             void* stream, const Exec& X, bool launch = true) {
  if (sketches == nullptr || bitmaps == nullptr || sketch_out == nullptr || bitmap_out == nullptr) return S2R_ERR_NULL;
  const s2r_status sz = check_sizes(n, d, w);
  if (sz != S2R_OK) return sz;
  if (W == 0 || W > S2R_MAX_WORKERS) return S2R_ERR_SIZE;
  MergeArgs A;
  for (uint32_t k = 0; k < S2R_MAX_WORKERS; ++k) {
    A.sketch[k] = k < W ? sketches[k] : nullptr;
    A.bitmap[k] = k < W ? bitmaps[k] : nullptr;
    if (k < W) {
      if (sketches[k] == nullptr || bitmaps[k] == nullptr) return S2R_ERR_NULL;
      if (((uintptr_t)sketches[k] & 15u) || ((uintptr_t)bitmaps[k] & 7u)) return S2R_ERR_ALIGN;
    }
  }
  if (((uintptr_t)sketch_out & 15u) || ((uintptr_t)bitmap_out & 7u)) return S2R_ERR_ALIGN;
  if (!launch) return S2R_OK;
  A.sketch_out = sketch_out;
  A.bitmap_out = bitmap_out;
  A.ncells = (uint64_t)d * w;
  A.ncell4 = A.ncells / 4;
  A.nwords = ceil_div(n, 64);
  A.W = W;
  A.piece_count = piece_count;
  A.count_words = piece_count != nullptr ? (uint64_t)tiles_of(n) * kTileWords : 0;
  // one thread per 16 bytes of sketch / 8 bytes of bitmap (d*w <= 2^32 and n <= 2^32 keep the grid below 2^23);
  // with counts, the bitmap part covers every piece of every tile
  const uint64_t sb = ceil_div(A.ncell4 > 0 ? A.ncell4 : 1, kBlock);
  const uint64_t bb = ceil_div(piece_count != nullptr ? A.count_words : A.nwords, kBlock);
  A.sketch_blocks = (uint32_t)sb;
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid((uint32_t)(sb + bb)), block(kBlock);
  record(X, S2R_KERNEL_MERGE, false, st);
  if (W >= 16) {
    if (piece_count != nullptr) hipLaunchKernelGGL((merge_kernel<8, true>), grid, block, 0, st, A);
    else hipLaunchKernelGGL((merge_kernel<8, false>), grid, block, 0, st, A);
  } else {
    if (piece_count != nullptr) hipLaunchKernelGGL((merge_kernel<4, true>), grid, block, 0, st, A);
    else hipLaunchKernelGGL((merge_kernel<4, false>), grid, block, 0, st, A);
  }
  record(X, S2R_KERNEL_MERGE, true, st);
  return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
}

s2r_status s2r_merge(const float* const* sketches, const uint64_t* const* bitmaps, uint32_t W, uint64_t n,
                     uint32_t d, uint32_t w, uint64_t seed, float* sketch_out, uint64_t* bitmap_out,
                     void* stream) {
  (void)seed;
  return merge_impl(sketches, bitmaps, W, n, d, w, sketch_out, bitmap_out, nullptr, stream, Exec());
}

// Where decode_impl takes the piece counts of the bitmap from: its own counting kernel, or the workspace, where
// merge_impl has just put them; kCheckOnly: check the arguments and launch nothing.
constexpr int kCountsFromBitmap = 0, kCountsInWorkspace = 1, kCheckOnly = 2;

// block = 0: the element codec.  block >= 1: the block-granular codec: the bitmap has ceil(n / block) bits,
// idx_out lists the set blocks (cap of them at most), val_out holds block values per listed block, and there
// is no dense output.
static s2r_status decode_impl(const float* sketch, const uint64_t* bitmap, uint64_t n, uint32_t block, uint32_t d,
                              uint32_t w, uint64_t seed, uint32_t* idx_out, float* val_out, uint64_t cap,
                              uint64_t* count_out, float* dense_out, void* workspace, size_t workspace_bytes,
                              void* stream, const Exec& X, float* params = nullptr, float scale = 0.0f,
                              int counts = kCountsFromBitmap) {
  if (sketch == nullptr || bitmap == nullptr || count_out == nullptr) return S2R_ERR_NULL;
  // (a block-granular parameter update lists the blocks but returns no values)
  if ((idx_out == nullptr) != (val_out == nullptr) && !(block != 0 && params != nullptr && val_out == nullptr))
    return S2R_ERR_NULL;
  const s2r_status sz = check_sizes(n, d, w);
  if (sz != S2R_OK) return sz;
  const uint64_t elements = n;
  if (block != 0) n = ceil_div(n, block);                  // from here on n counts the bits of the bitmap
  if (workspace == nullptr || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < workspace_base(n))
    return S2R_ERR_WORKSPACE;
  if (((uintptr_t)sketch & 15u) || ((uintptr_t)bitmap & 7u) || ((uintptr_t)idx_out & 3u) ||
      ((uintptr_t)val_out & 3u) || ((uintptr_t)count_out & 7u) || ((uintptr_t)dense_out & 15u)) return S2R_ERR_ALIGN;
  if (counts == kCheckOnly) return S2R_OK;

  hipStream_t st = (hipStream_t)stream;
  HashRows hp;
  make_hash_rows(seed, d, &hp);
  const uint32_t ntiles = tiles_of(n);
  const uint64_t nwords = ceil_div(n, 64);

  uint16_t* piece_count = reinterpret_cast<uint16_t*>(workspace);
  uint64_t* tile_prefix = reinterpret_cast<uint64_t*>((char*)workspace + workspace_prefix_off(n));
  if (counts == kCountsFromBitmap) {
    hipLaunchKernelGGL(bitmap_count_kernel, dim3((uint32_t)ceil_div(ntiles, kWavesPerBlock)), dim3(kBlock), 0, st,
                       bitmap, nwords, ntiles, piece_count);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(tile_prefix_kernel, dim3(1), dim3(kPrefixBlock), 0, st, (char*)workspace, (uint64_t)0,
                     (uint64_t)workspace_prefix_off(n), (uint64_t)workspace_dense_off(n), ntiles, count_out);
  if (!launch_ok()) return S2R_ERR_LAUNCH;
  if ((idx_out == nullptr || cap == 0) && dense_out == nullptr && params == nullptr) return S2R_OK;   // only the count was asked for

  if (cap > n) cap = n;
  const uint64_t cap_items = block != 0 ? cap * block : cap;    // list positions that get a value, at most
  // (an update of parameters, like a dense output, must reach the union indices beyond the lists' capacity too)
  uint64_t expect = X.expected_nnz != 0 && X.expected_nnz < cap ? X.expected_nnz : cap;
  if (block != 0) expect *= block;
  const int32_t strategy = choose_decode(n, d, w, idx_out != nullptr, dense_out != nullptr || params != nullptr,
                                         idx_out ? cap_items : 0, expect, workspace_bytes, X.decode_strategy);
  if (X.report != nullptr) X.report->decode_strategy = strategy;
  if (strategy == S2R_DECODE_SLICE) {
    const DecodeLayout L = decode_layout(n, d, w, cap_items);
    if (!raise_lds_limits()) return S2R_ERR_LAUNCH;
    // the kernels of the encode's slice strategy, on one "worker" whose list is the union list
    EncodeBatch B;
    B.w[0].grad = nullptr;                                 // expansion without values
    B.w[0].sketch = nullptr;
    B.w[0].bitmap = const_cast<uint64_t*>(bitmap);        // only read
    B.w[0].nz_idx = idx_out;
    B.w[0].nz_val = nullptr;
    B.nnz_out = count_out;
    B.workspace = reinterpret_cast<char*>(workspace);
    B.ws_stride = 0;
    B.prefix_off = workspace_prefix_off(n);
    B.dense_off = workspace_dense_off(n);
    B.seg_off = L.seg_off;
    B.rec_off = L.rec_off;
    B.payload_slot = 1;
    B.block = block;
    B.n = elements;
    B.nwords = nwords;
    B.cap = cap;
    B.sort_cap = cap;
    B.ntiles = ntiles;
    B.d = d;
    B.log2w = log2_of(w);
    B.slice_log2 = L.slice_log2;
    B.nbins = L.nbins;
    B.nchunks = L.nchunks;
    B.first_worker = 0;
    B.nworkers = 1;
    char* ws = reinterpret_cast<char*>(workspace);
    DecodeSliceArgs Q;
    Q.sketch = sketch;
    Q.rec = reinterpret_cast<const uint32_t*>(ws + L.rec_off);
    Q.answers = reinterpret_cast<uint32_t*>(ws + L.answers_off);
    Q.seg = reinterpret_cast<const uint32_t*>(ws + L.seg_off);
    Q.count = count_out;
    Q.cap = cap;
    Q.val_out = val_out;
    Q.nbins = L.nbins;
    Q.slice_log2 = L.slice_log2;
    Q.d = d;
    Q.block = block;
    Q.n = elements;
    Q.blk_list = idx_out;

    record(X, S2R_KERNEL_DECODE, false, st);
    const uint32_t helpers = dense_grid(ntiles, block != 0 ? expect / block : expect, 2048);
    hipLaunchKernelGGL(encode_compact_kernel<false>, dim3(helpers + ntiles, 1), dim3(kBlock), 0, st, B, helpers);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    const uint32_t chunk_grid = (uint32_t)ceil_div(expect > 0 ? expect : 1, kBinChunk);   // (the chunk kernels loop)
    launch_bin_sort(B, hp, dim3(chunk_grid, 1), st);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    // one workgroup per compute unit at a time (the slice fills its LDS): with few bins, several workgroups
    // share a bin's queries so that the last round of workgroups is not mostly idle units
    const uint64_t per_bin = expect * d / L.nbins;         // expected, on average
    uint32_t parts = L.nbins >= 512 ? 1u : (uint32_t)ceil_div(768, L.nbins);   // (two rounds and more: no gain measured)
    while (parts > 1 && per_bin / parts < 16384) --parts;
    if (parts > 8) parts = 8;
    hipLaunchKernelGGL(decode_slice_kernel, dim3(L.nbins, parts), dim3(kSliceBlock), sizeof(float) << L.slice_log2, st, Q);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    const dim3 mgrid(chunk_grid), mblock(kBinBlock);
    switch (d) {
      case 1: hipLaunchKernelGGL(decode_median_kernel<1>, mgrid, mblock, 0, st, Q); break;
      case 2: hipLaunchKernelGGL(decode_median_kernel<2>, mgrid, mblock, 0, st, Q); break;
      case 3: hipLaunchKernelGGL(decode_median_kernel<3>, mgrid, mblock, 0, st, Q); break;
      case 4: hipLaunchKernelGGL(decode_median_kernel<4>, mgrid, mblock, 0, st, Q); break;
      case 5: hipLaunchKernelGGL(decode_median_kernel<5>, mgrid, mblock, 0, st, Q); break;
      case 6: hipLaunchKernelGGL(decode_median_kernel<6>, mgrid, mblock, 0, st, Q); break;
      case 7: hipLaunchKernelGGL(decode_median_kernel<7>, mgrid, mblock, 0, st, Q); break;
      default: hipLaunchKernelGGL(decode_median_kernel<8>, mgrid, mblock, 0, st, Q); break;
    }
    record(X, S2R_KERNEL_DECODE, true, st);
    return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
  }

  DecodeArgs A;
  A.sketch = sketch;
  A.bitmap = bitmap;
  A.n = block != 0 ? elements : n;
  A.nwords = nwords;
  A.d = d;
  A.log2w = log2_of(w);
  A.prefix = tile_prefix;
  A.dense = reinterpret_cast<const uint32_t*>((char*)workspace + workspace_dense_off(n));
  A.idx_out = idx_out;
  A.val_out = val_out;
  A.cap = idx_out ? cap : 0;
  A.dense_out = dense_out;
  A.params = params;
  A.scale = scale;

  if (block != 0) {                                        // the block list, then one thread per element of a listed block
    EncodeBatch B;
    B.w[0].grad = nullptr;
    B.w[0].sketch = nullptr;
    B.w[0].bitmap = const_cast<uint64_t*>(bitmap);        // only read
    B.w[0].nz_idx = idx_out;
    B.w[0].nz_val = nullptr;
    B.nnz_out = count_out;
    B.workspace = reinterpret_cast<char*>(workspace);
    B.ws_stride = 0;
    B.prefix_off = workspace_prefix_off(n);
    B.dense_off = workspace_dense_off(n);

    B.payload_slot = 0;
    B.block = block;
    B.n = elements;
    B.nwords = nwords;
    B.cap = cap;
    B.sort_cap = cap;
    B.ntiles = ntiles;
    B.d = d;
    B.log2w = A.log2w;
    B.first_worker = 0;
    B.nworkers = 1;
    record(X, S2R_KERNEL_DECODE, false, st);
    const uint32_t helpers = dense_grid(ntiles, block != 0 ? expect / block : expect, 2048);
    hipLaunchKernelGGL(encode_compact_kernel<false>, dim3(helpers + ntiles, 1), dim3(kBlock), 0, st, B, helpers);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    if (strategy == S2R_DECODE_ROWS) {
      const RowsLayout R = rows_layout(n, d, cap_items);
      float* est = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + R.est_off);
      uint64_t units = ceil_div(expect > 0 ? expect : 1, (uint64_t)kBlock * kRowsBlockPer);   // (the units loop)
      if (units > 16384) units = 16384;
      const uint32_t groups = (uint32_t)ceil_div(units, 8u / d);
      hipLaunchKernelGGL(decode_rows_blocks_kernel, dim3(8u * groups), dim3(kBlock), 0, st, A, hp, block, idx_out,
                         count_out, est, R.stride, (uint32_t)units);
      if (!launch_ok()) return S2R_ERR_LAUNCH;
      launch_rows_median(d, est, R.stride, count_out, cap, val_out, block, elements, idx_out, expect, st);
      record(X, S2R_KERNEL_DECODE, true, st);
      return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
    }
    const uint64_t bwgs = ceil_div(cap_items, (uint64_t)kBlock * 4);
    const dim3 bgrid((uint32_t)(bwgs < 8192 ? bwgs : 8192)), bblock(kBlock);      // (the workgroups loop)
    switch (d) {
      case 1: hipLaunchKernelGGL(decode_blocks_kernel<1>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 2: hipLaunchKernelGGL(decode_blocks_kernel<2>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 3: hipLaunchKernelGGL(decode_blocks_kernel<3>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 4: hipLaunchKernelGGL(decode_blocks_kernel<4>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 5: hipLaunchKernelGGL(decode_blocks_kernel<5>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 6: hipLaunchKernelGGL(decode_blocks_kernel<6>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 7: hipLaunchKernelGGL(decode_blocks_kernel<7>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 8: hipLaunchKernelGGL(decode_blocks_kernel<8>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 9: hipLaunchKernelGGL(decode_blocks_kernel<9>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 10: hipLaunchKernelGGL(decode_blocks_kernel<10>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 11: hipLaunchKernelGGL(decode_blocks_kernel<11>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 12: hipLaunchKernelGGL(decode_blocks_kernel<12>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 13: hipLaunchKernelGGL(decode_blocks_kernel<13>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 14: hipLaunchKernelGGL(decode_blocks_kernel<14>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      case 15: hipLaunchKernelGGL(decode_blocks_kernel<15>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
      default: hipLaunchKernelGGL(decode_blocks_kernel<16>, bgrid, bblock, 0, st, A, hp, block, idx_out, count_out); break;
    }
    record(X, S2R_KERNEL_DECODE, true, st);
    return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
  }

  record(X, S2R_KERNEL_DECODE, false, st);
  const uint32_t helpers = dense_grid(ntiles, block != 0 ? expect / block : expect, 2048);
  if (strategy == S2R_DECODE_ROWS) {
    const RowsLayout R = rows_layout(n, d, cap_items);
    float* est = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + R.est_off);
    const uint32_t groups = (uint32_t)ceil_div((uint64_t)ntiles + helpers, 8u / d);
    hipLaunchKernelGGL(decode_rows_kernel, dim3(8u * groups), dim3(kBlock), 0, st, A, hp, est, R.stride, ntiles, helpers);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    launch_rows_median(d, est, R.stride, count_out, cap, val_out, 0u, elements, nullptr, expect, st);
    record(X, S2R_KERNEL_DECODE, true, st);
    return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
  }
  switch (d) {
    case 1: launch_decode<1>(ntiles, helpers, st, A, hp); break;
    case 2: launch_decode<2>(ntiles, helpers, st, A, hp); break;
    case 3: launch_decode<3>(ntiles, helpers, st, A, hp); break;
    case 4: launch_decode<4>(ntiles, helpers, st, A, hp); break;
    case 5: launch_decode<5>(ntiles, helpers, st, A, hp); break;
    case 6: launch_decode<6>(ntiles, helpers, st, A, hp); break;
    case 7: launch_decode<7>(ntiles, helpers, st, A, hp); break;
    case 8: launch_decode<8>(ntiles, helpers, st, A, hp); break;
    case 9: launch_decode<9>(ntiles, helpers, st, A, hp); break;
    case 10: launch_decode<10>(ntiles, helpers, st, A, hp); break;
    case 11: launch_decode<11>(ntiles, helpers, st, A, hp); break;
    case 12: launch_decode<12>(ntiles, helpers, st, A, hp); break;
    case 13: launch_decode<13>(ntiles, helpers, st, A, hp); break;
    case 14: launch_decode<14>(ntiles, helpers, st, A, hp); break;
    case 15: launch_decode<15>(ntiles, helpers, st, A, hp); break;
    default: launch_decode<16>(ntiles, helpers, st, A, hp); break;
  }
  record(X, S2R_KERNEL_DECODE, true, st);
  return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
}


s2r_status s2r_decode_ex(const float* sketch, const uint64_t* bitmap, uint64_t n, uint32_t d, uint32_t w,
                         uint64_t seed, uint32_t* idx_out, float* val_out, uint64_t cap, uint64_t* count_out,
                         float* dense_out, void* workspace, size_t workspace_bytes, void* stream,
                         const s2r_options* options) {
  Exec X;
  const s2r_status rc = resolve_options(options, &X);
  if (rc != S2R_OK) return rc;
  return decode_impl(sketch, bitmap, n, 0u, d, w, seed, idx_out, val_out, cap, count_out, dense_out, workspace,
                     workspace_bytes, stream, X);
}

s2r_status s2r_decode(const float* sketch, const uint64_t* bitmap, uint64_t n, uint32_t d, uint32_t w,
                      uint64_t seed, uint32_t* idx_out, float* val_out, uint64_t cap, uint64_t* count_out,
                      float* dense_out, void* workspace, size_t workspace_bytes, void* stream) {
  return s2r_decode_ex(sketch, bitmap, n, d, w, seed, idx_out, val_out, cap, count_out, dense_out, workspace,
                       workspace_bytes, stream, nullptr);
}

// merge and decode in one call: the merge kernel counts the aggregated bitmap while it forms it
static s2r_status merge_decode_impl(const float* const* sketches, const uint64_t* const* bitmaps, uint32_t W,
                                    uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t seed,
                                    float* sketch_out, uint64_t* bitmap_out, uint32_t* idx_out, float* val_out,
                                    uint64_t cap, uint64_t* count_out, float* dense_out, void* workspace,
                                    size_t workspace_bytes, void* stream, const s2r_options* options) {
  Exec X;
  s2r_status rc = resolve_options(options, &X);
  if (rc != S2R_OK) return rc;
  const s2r_status sz = check_sizes(n, d, w);
  if (sz != S2R_OK) return sz;
  const uint64_t nbits = block != 0 ? ceil_div(n, block) : n;
  // both halves' arguments are checked before anything is launched
  rc = merge_impl(sketches, bitmaps, W, nbits, d, w, sketch_out, bitmap_out, nullptr, stream, X, false);
  if (rc != S2R_OK) return rc;
  rc = decode_impl(sketch_out, bitmap_out, n, block, d, w, seed, idx_out, val_out, cap, count_out, dense_out,
                   workspace, workspace_bytes, stream, X, nullptr, 0.0f, kCheckOnly);
  if (rc != S2R_OK) return rc;
  rc = merge_impl(sketches, bitmaps, W, nbits, d, w, sketch_out, bitmap_out, reinterpret_cast<uint16_t*>(workspace),
                  stream, X);
  if (rc != S2R_OK) return rc;
  return decode_impl(sketch_out, bitmap_out, n, block, d, w, seed, idx_out, val_out, cap, count_out, dense_out,
                     workspace, workspace_bytes, stream, X, nullptr, 0.0f, kCountsInWorkspace);
}

s2r_status s2r_merge_decode_ex(const float* const* sketches, const uint64_t* const* bitmaps, uint32_t W, uint64_t n,
                               uint32_t d, uint32_t w, uint64_t seed, float* sketch_out, uint64_t* bitmap_out,
                               uint32_t* idx_out, float* val_out, uint64_t cap, uint64_t* count_out,
                               float* dense_out, void* workspace, size_t workspace_bytes, void* stream,
                               const s2r_options* options) {
  return merge_decode_impl(sketches, bitmaps, W, n, 0u, d, w, seed, sketch_out, bitmap_out, idx_out, val_out, cap,
                           count_out, dense_out, workspace, workspace_bytes, stream, options);
}

s2r_status s2r_merge_decode(const float* const* sketches, const uint64_t* const* bitmaps, uint32_t W, uint64_t n,
                            uint32_t d, uint32_t w, uint64_t seed, float* sketch_out, uint64_t* bitmap_out,
                            uint32_t* idx_out, float* val_out, uint64_t cap, uint64_t* count_out, float* dense_out,
                            void* workspace, size_t workspace_bytes, void* stream) {
  return merge_decode_impl(sketches, bitmaps, W, n, 0u, d, w, seed, sketch_out, bitmap_out, idx_out, val_out, cap,
                           count_out, dense_out, workspace, workspace_bytes, stream, nullptr);
}

s2r_status s2r_decode_update(const float* sketch, const uint64_t* bitmap, uint64_t n, uint32_t d, uint32_t w,
                             uint64_t seed, float* params, float scale, uint32_t* idx_out, float* val_out, uint64_t cap,
                             uint64_t* count_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (params == nullptr) return S2R_ERR_NULL;
  if (((uintptr_t)params & 3u) != 0) return S2R_ERR_ALIGN;
  return decode_impl(sketch, bitmap, n, 0u, d, w, seed, idx_out, val_out, cap, count_out, nullptr, workspace,
                     workspace_bytes, stream, Exec(), params, scale);
}

// ---- block-granular codec
static inline bool block_ok(uint64_t n, uint32_t block) { return block >= 1 && n >= 1 && (uint64_t)block <= (1ull << 31); }

size_t s2r_blocks_workspace_bytes(uint64_t n, uint32_t block, uint32_t d, uint32_t w) {
  if (check_sizes(n, d, w) != S2R_OK || !block_ok(n, block)) return 0;
  return workspace_base(ceil_div(n, block));
}

size_t s2r_encode_blocks_workspace_bytes(uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t blk_cap) {
  if (check_sizes(n, d, w) != S2R_OK || !block_ok(n, block) || blk_cap > ceil_div(n, block)) return 0;
  const uint64_t nb = ceil_div(n, block);
  const SliceLayout L = slice_layout(nb, d, w, blk_cap * block);
  return L.possible ? L.total : workspace_base(nb);
}

size_t s2r_decode_blocks_workspace_bytes(uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t blk_cap) {
  if (check_sizes(n, d, w) != S2R_OK || !block_ok(n, block) || blk_cap > ceil_div(n, block)) return 0;
  const uint64_t nb = ceil_div(n, block);
  const DecodeLayout L = decode_layout(nb, d, w, blk_cap * block);
  const RowsLayout R = rows_layout(nb, d, blk_cap * block);
  return L.possible && L.total > R.total ? L.total : R.total;
}

s2r_status s2r_encode_blocks_batch_ex(const float* const* grads, uint32_t W, uint64_t n, uint32_t block, uint32_t d,
                                      uint32_t w, uint64_t seed, float* const* sketches,
                                      uint64_t* const* block_bitmaps, uint32_t* const* blk_idx, uint64_t blk_cap,
                                      uint64_t* nblk_out, void* workspace, size_t workspace_bytes, void* stream,
                                      const s2r_options* options) {
  if (!block_ok(n, block)) return S2R_ERR_SIZE;
  Exec X;
  const s2r_status rc = resolve_options(options, &X);
  if (rc != S2R_OK) return rc;
  return encode_workers(grads, W, n, block, d, w, seed, sketches, block_bitmaps, blk_idx, nullptr, blk_cap, nblk_out,
                        workspace, workspace_bytes, (hipStream_t)stream, X);
}

s2r_status s2r_encode_blocks_ex(const float* grad, uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t seed,
                                float* sketch, uint64_t* block_bitmap, uint32_t* blk_idx, uint64_t blk_cap,
                                uint64_t* nblk_out, void* workspace, size_t workspace_bytes, void* stream,
                                const s2r_options* options) {
  return s2r_encode_blocks_batch_ex(&grad, 1, n, block, d, w, seed, &sketch, &block_bitmap,
                                    blk_idx ? &blk_idx : nullptr, blk_cap, nblk_out, workspace, workspace_bytes,
                                    stream, options);
}

s2r_status s2r_encode_blocks_batch(const float* const* grads, uint32_t W, uint64_t n, uint32_t block, uint32_t d,
                                   uint32_t w, uint64_t seed, float* const* sketches, uint64_t* const* block_bitmaps,
                                   uint32_t* const* blk_idx, uint64_t blk_cap, uint64_t* nblk_out, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  return s2r_encode_blocks_batch_ex(grads, W, n, block, d, w, seed, sketches, block_bitmaps, blk_idx, blk_cap,
                                    nblk_out, workspace, workspace_bytes, stream, nullptr);
}

s2r_status s2r_encode_blocks(const float* grad, uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t seed,
                             float* sketch, uint64_t* block_bitmap, uint32_t* blk_idx, uint64_t blk_cap,
                             uint64_t* nblk_out, void* workspace, size_t workspace_bytes, void* stream) {
  return s2r_encode_blocks_ex(grad, n, block, d, w, seed, sketch, block_bitmap, blk_idx, blk_cap, nblk_out, workspace,
                              workspace_bytes, stream, nullptr);
}

}  // extern "C"

void s2r::record_kernel_event(const Exec& X, int slot, bool end, void* stream) {
  record(X, slot, end, (hipStream_t)stream);
}

s2r_status s2r::resolve_options(const s2r_options* options, Exec* X) {
  *X = Exec();
  if (options == nullptr) return S2R_OK;
  if (options->struct_bytes != sizeof(s2r_options) || options->flags != 0) return S2R_ERR_SIZE;
  if (options->insert_strategy != S2R_INSERT_AUTO && options->insert_strategy != S2R_INSERT_ATOMIC &&
      options->insert_strategy != S2R_INSERT_SLICE)
    return S2R_ERR_SIZE;
  if (options->decode_strategy != S2R_DECODE_AUTO && options->decode_strategy != S2R_DECODE_GATHER &&
      options->decode_strategy != S2R_DECODE_SLICE && options->decode_strategy != S2R_DECODE_ROWS)
    return S2R_ERR_SIZE;
  if (options->trace != nullptr) {
    for (int slot = 0; slot < S2R_KERNEL_SLOTS; ++slot)
      if ((options->trace->begin[slot] == nullptr) != (options->trace->end[slot] == nullptr)) return S2R_ERR_NULL;
  }
  X->insert_strategy = options->insert_strategy;
  X->decode_strategy = options->decode_strategy;
  X->expected_nnz = options->expected_nnz;
  X->report = options->report;
  X->trace = options->trace;
  if (X->report != nullptr) {
    X->report->insert_strategy = S2R_INSERT_AUTO;
    X->report->decode_strategy = S2R_DECODE_AUTO;
    X->report->scan_launch_workers = 0;
    X->report->reserved = 0;
  }
  return S2R_OK;
}

s2r_status s2r::encode_marked_blocks(const float* const* values, uint32_t W, uint64_t n, uint32_t block, uint32_t d,
                                     uint32_t w, uint64_t seed, float* const* sketches, uint64_t* const* block_bitmaps,
                                     uint32_t* const* blk_idx, uint64_t cap, uint64_t* nblk_out, void* workspace,
                                     size_t workspace_bytes, void* stream, const Exec& X) {
  if (!block_ok(n, block)) return S2R_ERR_SIZE;
  return encode_workers(values, W, n, block, d, w, seed, sketches, block_bitmaps, blk_idx, nullptr, cap, nblk_out,
                        workspace, workspace_bytes, (hipStream_t)stream, X, true);
}

extern "C" {

size_t s2r_decode_blocks_update_workspace_bytes(uint64_t n, uint32_t block, uint32_t d, uint32_t w) {
  if (check_sizes(n, d, w) != S2R_OK || !block_ok(n, block)) return 0;
  const uint64_t nb = ceil_div(n, block);
  return workspace_base(nb) + align256((size_t)nb * sizeof(uint32_t));
}

s2r_status s2r_decode_blocks_update(const float* sketch, const uint64_t* block_bitmap, uint64_t n, uint32_t block,
                                    uint32_t d, uint32_t w, uint64_t seed, float* params, float scale,
                                    uint64_t* nblk_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (params == nullptr) return S2R_ERR_NULL;
  if (((uintptr_t)params & 3u) != 0) return S2R_ERR_ALIGN;
  if (!block_ok(n, block)) return S2R_ERR_SIZE;
  const s2r_status sz = check_sizes(n, d, w);
  if (sz != S2R_OK) return sz;
  const uint64_t nb = ceil_div(n, block);
  if (workspace == nullptr || workspace_bytes < workspace_base(nb) + align256((size_t)nb * sizeof(uint32_t)))
    return S2R_ERR_WORKSPACE;
  // the complete list of set blocks goes to the workspace, behind the parts every decode uses
  uint32_t* list = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(workspace) + workspace_base(nb));
  return decode_impl(sketch, block_bitmap, n, block, d, w, seed, list, nullptr, nb, nblk_out, nullptr, workspace,
                     workspace_bytes, stream, Exec(), params, scale);
}

s2r_status s2r_decode_blocks_ex(const float* sketch, const uint64_t* block_bitmap, uint64_t n, uint32_t block,
                                uint32_t d, uint32_t w, uint64_t seed, uint32_t* blk_idx_out, float* val_out,
                                uint64_t blk_cap, uint64_t* nblk_out, void* workspace, size_t workspace_bytes,
                                void* stream, const s2r_options* options) {
  if (!block_ok(n, block)) return S2R_ERR_SIZE;
  Exec X;
  const s2r_status rc = resolve_options(options, &X);
  if (rc != S2R_OK) return rc;
  return decode_impl(sketch, block_bitmap, n, block, d, w, seed, blk_idx_out, val_out, blk_cap, nblk_out, nullptr,
                     workspace, workspace_bytes, stream, X);
}

s2r_status s2r_merge_decode_blocks_ex(const float* const* sketches, const uint64_t* const* block_bitmaps, uint32_t W,
                                      uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t seed,
                                      float* sketch_out, uint64_t* bitmap_out, uint32_t* blk_idx_out, float* val_out,
                                      uint64_t blk_cap, uint64_t* nblk_out, void* workspace, size_t workspace_bytes,
                                      void* stream, const s2r_options* options) {
  if (!block_ok(n, block)) return S2R_ERR_SIZE;
  return merge_decode_impl(sketches, block_bitmaps, W, n, block, d, w, seed, sketch_out, bitmap_out, blk_idx_out,
                           val_out, blk_cap, nblk_out, nullptr, workspace, workspace_bytes, stream, options);
}

s2r_status s2r_merge_decode_blocks(const float* const* sketches, const uint64_t* const* block_bitmaps, uint32_t W,
                                   uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t seed,
                                   float* sketch_out, uint64_t* bitmap_out, uint32_t* blk_idx_out, float* val_out,
                                   uint64_t blk_cap, uint64_t* nblk_out, void* workspace, size_t workspace_bytes,
                                   void* stream) {
  return s2r_merge_decode_blocks_ex(sketches, block_bitmaps, W, n, block, d, w, seed, sketch_out, bitmap_out,
                                    blk_idx_out, val_out, blk_cap, nblk_out, workspace, workspace_bytes, stream,
                                    nullptr);
}

s2r_status s2r_decode_blocks(const float* sketch, const uint64_t* block_bitmap, uint64_t n, uint32_t block, uint32_t d,
                             uint32_t w, uint64_t seed, uint32_t* blk_idx_out, float* val_out, uint64_t blk_cap,
                             uint64_t* nblk_out, void* workspace, size_t workspace_bytes, void* stream) {
  return s2r_decode_blocks_ex(sketch, block_bitmap, n, block, d, w, seed, blk_idx_out, val_out, blk_cap, nblk_out,
                              workspace, workspace_bytes, stream, nullptr);
}

// ---- s2r_decode without a workspace argument and without any allocation
// The scratch that s2r_decode takes from its caller (piece counts, tile prefix, dense-tile list) lives in a
// file-scope device array instead; every GPU the library runs on holds its own copy until the process ends.
// Host code never uses the array's name as an address: the device address is asked for once per device.
constexpr uint64_t kNoAllocMaxN = S2R_DECODE_NOALLOC_MAX_N;
constexpr size_t kNoAllocScratchBytes = 448 * 1024;          // >= workspace_base(kNoAllocMaxN), checked at run time
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

static void* noalloc_scratch_ptr() {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> ptr_of[kMaxDevices];              // zero-initialised; one address per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = ptr_of[dev].load(std::memory_order_acquire);
  if (p != nullptr) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
    (void)hipGetLastError();
    return nullptr;
  }
  ptr_of[dev].store(p, std::memory_order_release);            // (two threads may both ask: same answer)
  return p;
}

s2r_status s2r_decode_noalloc(const float* sketch, const uint64_t* bitmap, uint64_t n, uint32_t d, uint32_t w,
                              uint64_t seed, uint32_t* idx_out, float* val_out, uint64_t cap, uint64_t* count_out,
                              float* dense_out, void* stream) {
  const s2r_status sz = check_sizes(n, d, w);
  if (sz != S2R_OK) return sz;
  if (n > kNoAllocMaxN || workspace_base(n) > kNoAllocScratchBytes) return S2R_ERR_SIZE;
  void* ws = noalloc_scratch_ptr();
  if (ws == nullptr) return S2R_ERR_LAUNCH;
  Exec X;
  X.decode_strategy = S2R_DECODE_GATHER;     // (the slice route would want a workspace that grows with cap)
  return decode_impl(sketch, bitmap, n, 0u, d, w, seed, idx_out, val_out, cap, count_out, dense_out, ws,
                     kNoAllocScratchBytes, stream, X);
}

}  // extern "C"
