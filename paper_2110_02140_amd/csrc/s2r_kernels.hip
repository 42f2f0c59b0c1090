// gfx950 kernels and C ABI of the sparse-sketch gradient codec
// (S2 Reducer, Algorithm 1 and Section 3.1).  See include/s2r.h for the
// contract of every entry point.
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
//                bin_hist_kernel,      (slice variant) Sparse(g) x rows is partitioned by
//                bin_colscan_kernel,   sketch slice (counting sort: histogram per chunk,
//                bin_start_kernel,     offsets, scatter of (cell, signed value) records
//                bin_scatter_kernel    sorted by slice inside LDS first)
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
//                encode_compact_kernel, bin_*_kernel, decode_slice_kernel,
//                decode_median_kernel  (slice variant) the union list, its queries
//                                      partitioned by sketch slice, answered from
//                                      LDS, brought back to list order, medians
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/s2r.h"
#include "s2r_device.h"
#include "s2r_internal.h"

namespace s2r {

constexpr int kBlock = 256;                       // threads per workgroup (4 waves)
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kTileWords = 512;                   // bitmap words per tile
constexpr int kTileElems = kTileWords * 64;       // 32768 gradient elements per tile
constexpr int kWordsPerThread = kTileWords / kBlock;         // 2
constexpr int kScanEPL = 8;                       // dense scan: bitmap words (loads in flight) per wave
constexpr int kScanWords = kWavesPerBlock * kScanEPL;        // 32 words = 2048 elements per scan workgroup
constexpr int kScansPerTile = kTileWords / kScanWords;       // 16
constexpr int kGroupSlots = 2048;                 // list positions one expansion workgroup handles; a tile with more
                                                  // set bits gets extra workgroups through the dense-tile list
constexpr int kGroupsPerTile = kTileElems / kGroupSlots;     // 16
constexpr int kPrefixBlock = 1024;                // threads of the single prefix workgroup
constexpr int kPrefixPer = 8;                     // tiles per thread per round
constexpr int kSliceBlock = 1024;                 // threads of a sketch-slice workgroup
constexpr int kSliceLog2Max = 14;                 // 2^14 cells = 128 KiB of float64 accumulators in LDS (smaller slices
                                                  // with smaller workgroups measured slower in total: more bins)
static_assert(kTileWords % kScanWords == 0, "scan workgroups must not straddle tiles");
static_assert(kScanWords * 64 <= 0xFFFF, "a piece count must fit 16 bits");
static_assert(kScansPerTile == 16, "tile_prefix_kernel reads a tile's piece counts as two 16-byte loads");

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));      // a 16-byte vector the nontemporal builtins accept

static inline __host__ __device__ uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// ------------------------------------------------------------------ encode: arguments
// s2r_encode is a batch of one: every encode kernel takes the whole batch and
// blockIdx.y is the worker.  The per-worker pointers travel in the kernel
// arguments and are read with scalar loads.
struct WorkerPtrs {
  const uint32_t* grad;      // dense gradient as bit patterns
  float* sketch;
  uint64_t* bitmap;
  uint32_t* nz_idx;          // may be null
  uint32_t* nz_val;          // float bit patterns; may be null
};

struct EncodeBatch {
  WorkerPtrs w[S2R_MAX_WORKERS];
  uint64_t* nnz_out;         // [W]
  char* workspace;           // W chunks of ws_stride bytes: piece counts | tile prefix | slice parts
  uint64_t ws_stride;
  uint64_t prefix_off;       // byte offset of the tile prefix inside a chunk
  uint64_t dense_off;        // byte offset of the dense-tile list (count, then entries 256 bytes later)
  uint64_t hist_off;         // slice variant: byte offsets inside a chunk of the per-chunk bin histogram
  uint64_t binstart_off;     //   [nchunks][nbins] u32, the bin starts [nbins + 1] u32,
  uint64_t rec_off;          //   and the binned records [d * cap] of 8 bytes
  uint64_t rowpre_off;       // decode by slices: per chunk, the exclusive prefix of its histogram over the
                             //   bins, [nchunks][nbins] u32; 0 when not wanted
  uint32_t payload_slot;     // non-zero: a record carries its item's list position instead of nz_val
  uint32_t block;            // block-granular codec: elements per bitmap bit; nz_idx then lists blocks, and
                             //   bitmap / nwords / ntiles / cap describe the block bitmap.  0: one bit per element
  uint64_t n;
  uint64_t nwords;
  uint64_t cap;
  uint32_t ntiles;
  uint32_t d;
  uint32_t log2w;
  uint32_t slice_log2;       // log2 of cells per LDS slice (<= log2w)
  uint32_t nbins;            // d * slices per row
  uint32_t nchunks;          // list chunks of kBinChunk items
  uint32_t first_worker;     // zero and scan kernels: worker = first_worker + blockIdx.y
  uint32_t nworkers;         // W; a workgroup whose worker is not below it leaves at once
};

__device__ __forceinline__ uint16_t* ws_piece_count(const EncodeBatch& B, uint32_t k) {
  return reinterpret_cast<uint16_t*>(B.workspace + k * B.ws_stride);
}
__device__ __forceinline__ uint64_t* ws_prefix(const EncodeBatch& B, uint32_t k) {
  return reinterpret_cast<uint64_t*>(B.workspace + k * B.ws_stride + B.prefix_off);
}
__device__ __forceinline__ const uint32_t* ws_dense_list(const EncodeBatch& B, uint32_t k) {
  return reinterpret_cast<const uint32_t*>(B.workspace + k * B.ws_stride + B.dense_off);
}
__device__ __forceinline__ uint32_t* ws_bin_hist(const EncodeBatch& B, uint32_t k) {
  return reinterpret_cast<uint32_t*>(B.workspace + k * B.ws_stride + B.hist_off);
}
__device__ __forceinline__ uint32_t* ws_bin_start(const EncodeBatch& B, uint32_t k) {
  return reinterpret_cast<uint32_t*>(B.workspace + k * B.ws_stride + B.binstart_off);
}
__device__ __forceinline__ uint2* ws_records(const EncodeBatch& B, uint32_t k) {
  return reinterpret_cast<uint2*>(B.workspace + k * B.ws_stride + B.rec_off);
}

// ------------------------------------------------------------------ zero
// Per worker: zeroes the sketch (nvec 16-byte units plus ntail trailing floats)
// and, with bitmap_words, the (block) bitmap that the scan then sets bit by bit.
__global__ __launch_bounds__(kBlock) void zero_kernel(const EncodeBatch B, uint64_t nvec, uint32_t ntail,
                                                      uint64_t bitmap_words) {
  const uint32_t k = B.first_worker + blockIdx.y;
  if (k >= B.nworkers) return;
  const uint64_t tid = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  uint4* p16 = reinterpret_cast<uint4*>(B.w[k].sketch);
  for (uint64_t i = tid; i < nvec; i += stride) p16[i] = make_uint4(0u, 0u, 0u, 0u);
  if (tid < ntail) B.w[k].sketch[nvec * 4 + tid] = 0.0f;
  for (uint64_t i = tid; i < bitmap_words; i += stride) B.w[k].bitmap[i] = 0ull;
}

// ------------------------------------------------------------------ encode: dense scan
__device__ __forceinline__ void sketch_insert(float* sketch, uint32_t d, uint32_t log2w, const HashRows& hp,
                                              uint32_t i, uint32_t vbits) {
  for (uint32_t j = 0; j < d; ++j) {
    const uint32_t h = bucket_of(i, hp.a[j], hp.b[j], log2w);
    const uint32_t sv = vbits ^ signbit_of(i, hp.c[j], hp.e[j]);
    __hip_atomic_fetch_add(&sketch[((uint64_t)j << log2w) + h], __uint_as_float(sv),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// One workgroup scans kScanWords bitmap words (2048 elements), each wave EPL of
// them in one shot.  Lane l reads element 64k + l of the wave's chunk for
// k = 0..EPL-1: every load instruction is one coalesced 256-byte row and its
// ballot is bitmap word k.  Consecutive workgroups read consecutive 8 KiB, so the
// workgroups resident at any time sweep one compact window of memory.  The
// workgroup's non-zero count (at most 2048) is stored as piece blockIdx.x of the
// worker's 16-bit piece counts; the grid covers every piece of every tile, so
// the pieces past the end of the gradient are written too (as zero).
// Sets bit x of a block bitmap.  Atomics on one address retire one at a time, and many waves meet in the
// 64 blocks of a word, so the bit is only written when it is not yet seen set.
__device__ __forceinline__ void set_block_bit(uint64_t* bitmap, uint32_t x) {
  unsigned long long* word = reinterpret_cast<unsigned long long*>(&bitmap[x >> 6]);
  const unsigned long long bit = 1ull << (x & 63u);
  if ((__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit) == 0) atomicOr(word, bit);
}

// BLOCKS: the block-granular codec.  No element bitmap and no counts are written;
// instead every non-zero element sets the bit of its block B.block in the worker's
// (zeroed) block bitmap with an atomic OR, once per run of non-zero lanes of a
// word that fall in the same block.
template <int EPL, bool INSERT, bool BLOCKS>
__global__ __launch_bounds__(kBlock) void encode_scan_kernel(const EncodeBatch B, const HashRows hp) {
  __shared__ uint32_t s_wave_count[kWavesPerBlock];
  __shared__ unsigned long long s_block_bits[2];         // BLOCKS: the workgroup's bits of two bitmap words

  const uint32_t worker = B.first_worker + blockIdx.y;
  if (worker >= B.nworkers) return;                      // uniform over the workgroup
  const WorkerPtrs P = B.w[worker];
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  if (BLOCKS && B.block >= (uint32_t)kWave) {            // uniform over the workgroup
    if (threadIdx.x < 2) s_block_bits[threadIdx.x] = 0ull;
    __syncthreads();
  }
  const uint64_t word0 = (uint64_t)blockIdx.x * kScanWords + (uint64_t)wv * EPL;   // this wave's first word
  const uint64_t e0 = word0 * 64;

  uint32_t v[EPL];
  if (e0 + (uint64_t)EPL * kWave <= B.n) {               // uniform over the wave
#pragma unroll
    for (int k = 0; k < EPL; ++k) v[k] = __builtin_nontemporal_load(&P.grad[e0 + k * kWave + lane]);
  } else {
#pragma unroll
    for (int k = 0; k < EPL; ++k) {
      const uint64_t i = e0 + k * kWave + lane;
      v[k] = i < B.n ? P.grad[i] : 0u;
    }
  }

  uint32_t count = 0;          // non-zeros seen by this wave (uniform)
  uint64_t parked = 0;         // lane k keeps word k until the store below
  uint64_t bal[EPL] = {};      // BLOCKS: the ballots (uniform)
#pragma unroll
  for (int k = 0; k < EPL; ++k) {
    const bool nz = (v[k] << 1) != 0u;                   // anything but +0.0 / -0.0
    const uint64_t b = __ballot(nz);
    if (!BLOCKS && lane == (uint32_t)k) parked = b;
    if (b != 0) {                                        // uniform: most words are empty
      count += (uint32_t)__popcll(b);
      const uint32_t i = (uint32_t)(e0 + k * kWave + lane);       // < 2^32 wherever nz holds
      if (INSERT && nz) sketch_insert(P.sketch, B.d, B.log2w, hp, i, v[k]);
      if (BLOCKS) {
        bal[k] = b;
        if (B.block < (uint32_t)kWave) {
          // small blocks: one atomic per run of non-zero lanes of this word that share a block
          const uint32_t x = i / B.block;
          const uint64_t below = b & ((1ull << lane) - 1ull);     // non-zero lanes before this one
          const uint32_t prev = below != 0 ? 63u - (uint32_t)__clzll((long long)below) : lane;
          const uint32_t xp = (uint32_t)__shfl((int)x, (int)prev, kWave);
          if (nz && (below == 0 || xp != x)) set_block_bit(P.bitmap, x);
        }
      }
    }
  }
  if (BLOCKS) {
    // blocks of 64 elements and more: the wave's EPL * 64 elements meet at most EPL + 1 blocks; lane j takes
    // the j-th of them and tests the ballots (which every lane holds) against the block's range of bits.
    // The workgroup's 2048 elements meet at most 33 blocks, whose bits lie in two adjacent bitmap words:
    // they are collected in LDS and go out as at most two atomics per workgroup.
    if (B.block >= (uint32_t)kWave) {
      const uint64_t g0 = (uint64_t)blockIdx.x * kScanWords * 64;   // the workgroup's first element
      const uint64_t wbase = (g0 / B.block) >> 6;                   // bitmap word of its first block (uniform)
      if (count != 0) {
        const uint64_t c1 = e0 + (uint64_t)EPL * kWave;             // the wave's elements are [e0, c1)
        const uint64_t x = (uint32_t)e0 / B.block + lane;           // (a wave that saw a non-zero starts below 2^32)
        const uint64_t lo = x * B.block, hi = lo + B.block;         // the block's elements are [lo, hi)
        if (lo < c1 && hi > e0) {
          const uint32_t r0 = lo > e0 ? (uint32_t)(lo - e0) : 0u;
          const uint32_t r1 = hi < c1 ? (uint32_t)(hi - e0) : (uint32_t)(EPL * kWave);
          bool any = false;
#pragma unroll
          for (int k = 0; k < EPL; ++k) {
            const uint32_t a = r0 > (uint32_t)(k * kWave) ? r0 - k * kWave : 0u;          // bits [a, z) of word k
            const uint32_t z = r1 < (uint32_t)((k + 1) * kWave) ? (r1 > (uint32_t)(k * kWave) ? r1 - k * kWave : 0u) : (uint32_t)kWave;
            if (a < z) {
              const uint64_t upto = z == (uint32_t)kWave ? ~0ull : (1ull << z) - 1ull;
              any |= (bal[k] & upto & ~((1ull << a) - 1ull)) != 0;
            }
          }
          if (any)
            __hip_atomic_fetch_or(&s_block_bits[(x >> 6) - wbase], 1ull << (x & 63u), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_WORKGROUP);
        }
      }
      __syncthreads();
      if (threadIdx.x < 2 && wbase + threadIdx.x < B.nwords) {
        const unsigned long long bits = s_block_bits[threadIdx.x];
        unsigned long long* word = reinterpret_cast<unsigned long long*>(&P.bitmap[wbase + threadIdx.x]);
        if (bits != 0 && (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bits) != bits)
          atomicOr(word, bits);
      }
    }
    return;
  }
  // streaming store: the words are not read again by this kernel, and keeping them out of the L2 leaves it
  // to the gradient stream (measured: 8 % shorter scans at 4 GB per gradient)
  if (lane < (uint32_t)EPL && word0 + lane < B.nwords) __builtin_nontemporal_store(parked, &P.bitmap[word0 + lane]);

  if (lane == 0) s_wave_count[wv] = count;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0;
#pragma unroll
    for (int q = 0; q < kWavesPerBlock; ++q) t += s_wave_count[q];
    ws_piece_count(B, worker)[blockIdx.x] = (uint16_t)t;
  }
}

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
  const uint32_t k = blockIdx.y;
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
    const bool values = P.nz_val != nullptr;             // expansions of aggregated or block bitmaps carry no values
#pragma unroll
    for (int u = 0; u < kSlots; ++u) v[u] = live[u] && values ? P.grad[i[u]] : 0u;
#pragma unroll
    for (int u = 0; u < kSlots; ++u) {
      if (!live[u]) continue;
      const uint64_t pos = base + t0 + u * kBlock;
      P.nz_idx[pos] = i[u];
      if (values) P.nz_val[pos] = v[u];
    }
  }
}

// The first `helpers` workgroups of a worker take the further groups of the tiles
// in the dense-tile list, one entry per trip (they start first: theirs is the
// longest work); workgroup helpers + t takes the first kGroupSlots list positions
// of tile t.
__global__ __launch_bounds__(kBlock) void encode_compact_kernel(const EncodeBatch B, uint32_t helpers) {
  __shared__ TileBits T;
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;                           // uniform over the workgroup
  if (blockIdx.x >= helpers) {
    compact_group(B, B.w[k], ws_prefix(B, k), T, blockIdx.x - helpers, 0u);
    return;
  }
  const uint32_t* dense = ws_dense_list(B, k);
  const uint32_t entries = dense[0];
  for (uint32_t e = blockIdx.x; e < entries; e += helpers) {
    const uint32_t entry = dense[64 + e];
    __syncthreads();                                     // T may still be read by the previous trip
    compact_group(B, B.w[k], ws_prefix(B, k), T, entry & 0xFFFFFu, entry >> 20);
  }
}

// ------------------------------------------------------------------ encode: sketch by LDS slices
// The insertions S[j, h_j(i)] += s_j(i) g(i) without global atomics.  Row j of the
// sketch is cut into slices of 2^slice_log2 cells (float64 accumulators in LDS); bin (j, s)
// collects the pairs (item, row j) whose bucket falls in slice s.  A counting sort
// over the listed items brings each bin's records together:
//   bin_hist_kernel     per chunk of kBinChunk items, a histogram over the bins
//   bin_colscan_kernel, bin_start_kernel   offsets of every (chunk, bin) run and of every bin
//   bin_scatter_kernel  writes each record (cell in the slice | sign bit, value)
//                       into its run (order inside a run is arbitrary)
//   sketch_slice_kernel workgroup (j, s) clears its slice in LDS, adds its bin's
//                       records with LDS float64 atomics and stores the slice as float32
// Work is O(items x rows), whatever the number of slices, and every cell of the
// sketch is written exactly once by plain coalesced stores.
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
  const uint64_t listed = nnz < B.cap ? nnz : B.cap;
  return B.block != 0 ? listed * B.block : listed;
}

// Item t (t < listed_items): its element index i and its payload v (the value's
// bits, or the item's position t when B.payload_slot is set).  Returns whether
// the item takes part: with blocks, elements beyond n never do, and elements
// whose value is zero only when the payload is the position (a query), not when
// it is the value (an insertion: zeros are inert).  An item that does not take
// part in a query run is still given d answers (of element 0), which the median
// kernel discards, so that every chunk holds the same number of answers per row.
__device__ __forceinline__ bool load_item(const EncodeBatch& B, const WorkerPtrs& P, uint64_t t, uint32_t& i, uint32_t& v) {
  if (B.block == 0) {
    i = P.nz_idx[t];
    v = B.payload_slot != 0 ? (uint32_t)t : P.nz_val[t];
    return true;
  }
  const uint32_t q = (uint32_t)t / B.block;                // (the sort's items are fewer than 2^32)
  const uint64_t e = (uint64_t)P.nz_idx[q] * B.block + ((uint32_t)t - q * B.block);
  const bool inside = e < B.n;
  if (B.payload_slot != 0) {
    i = inside ? (uint32_t)e : 0u;
    v = (uint32_t)t;
    return true;
  }
  i = (uint32_t)e;
  v = inside ? P.grad[e] : 0u;
  return inside && (v << 1) != 0u;
}

__global__ __launch_bounds__(kBinBlock) void bin_hist_kernel(const EncodeBatch B, const HashRows hp) {
  __shared__ uint32_t s_hist[kMaxBins];
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;                           // uniform over the workgroup
  const uint32_t chunk = blockIdx.x;
  for (uint32_t b = threadIdx.x; b < B.nbins; b += kBinBlock) s_hist[b] = 0u;
  __syncthreads();
  const uint64_t have = listed_items(B, k);
  const WorkerPtrs P = B.w[k];
  const uint32_t spr_log2 = B.log2w - B.slice_log2;
  uint32_t i[kBinItems], v[kBinItems];
  bool ok[kBinItems];
#pragma unroll
  for (int u = 0; u < kBinItems; ++u) {
    const uint64_t t = (uint64_t)chunk * kBinChunk + u * kBinBlock + threadIdx.x;
    ok[u] = t < have && load_item(B, P, t, i[u], v[u]);
  }
#pragma unroll
  for (int u = 0; u < kBinItems; ++u) {
    if (ok[u]) {
      for (uint32_t j = 0; j < B.d; ++j) {
        const uint32_t bin = (j << spr_log2) + (bucket_of(i[u], hp.a[j], hp.b[j], B.log2w) >> B.slice_log2);
        __hip_atomic_fetch_add(&s_hist[bin], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
  }
  __syncthreads();
  uint32_t* hist = ws_bin_hist(B, k) + (uint64_t)chunk * B.nbins;
  for (uint32_t b = threadIdx.x; b < B.nbins; b += kBinBlock) hist[b] = s_hist[b];
  if (B.rowpre_off == 0) return;                         // uniform over the workgroup
  // exclusive prefix of this chunk's counts over the bins; thread t owns bins t*per .. t*per + per - 1
  constexpr int kWaves = kBinBlock / kWave;
  constexpr int kMaxPer = kMaxBins / kBinBlock;
  __shared__ uint32_t s_wave[kWaves];
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  const uint32_t per = (B.nbins + kBinBlock - 1) / kBinBlock;
  uint32_t c[kMaxPer], sum = 0;
#pragma unroll
  for (int q = 0; q < kMaxPer; ++q) {
    const uint32_t e = threadIdx.x * per + q;
    c[q] = ((uint32_t)q < per && e < B.nbins) ? s_hist[e] : 0u;
    sum += c[q];
  }
  const uint32_t incl = wave_inclusive_scan_u32(sum, lane);
  if (lane == kWave - 1) s_wave[wv] = incl;
  __syncthreads();
  uint32_t run = incl - sum;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) run += (uint32_t)q < wv ? s_wave[q] : 0u;
  uint32_t* rowpre = reinterpret_cast<uint32_t*>(B.workspace + k * B.ws_stride + B.rowpre_off) + (uint64_t)chunk * B.nbins;
#pragma unroll
  for (int q = 0; q < kMaxPer; ++q) {
    const uint32_t e = threadIdx.x * per + q;
    if ((uint32_t)q < per && e < B.nbins) {
      rowpre[e] = run;
      run += c[q];
    }
  }
}

// Offsets of the counting sort, two kernels.
// bin_colscan_kernel: workgroup = 64 adjacent bins of one worker (lane = bin, so a
// chunk's counters are read as one 256-byte row); its 16 waves split the chunks
// into 16 consecutive ranges.  In place, hist[c][b] becomes the number of records
// of bin b in chunks before c: every wave sums its range, the waves' sums are
// exchanged through LDS, then every wave walks its range again with its running
// offset.  The bin's total goes to bin_start[b].
// bin_start_kernel: one workgroup per worker turns the totals in bin_start[0..nbins)
// into the number of records in bins before b (bin_start[nbins] = all records).
__global__ __launch_bounds__(kBinBlock) void bin_colscan_kernel(const EncodeBatch B) {
  constexpr int kWaves = kBinBlock / kWave;              // 16
  constexpr uint32_t kAhead = 8;                         // counters in flight per thread
  __shared__ uint32_t s_part[kWaves][kWave];
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  const uint32_t b = blockIdx.x * kWave + lane;
  const bool live = b < B.nbins;
  uint32_t* hist = ws_bin_hist(B, k);
  const uint32_t per = (B.nchunks + kWaves - 1) / kWaves;
  const uint32_t c_begin = wv * per < B.nchunks ? wv * per : B.nchunks;
  const uint32_t c_end = c_begin + per < B.nchunks ? c_begin + per : B.nchunks;
  uint32_t sum = 0;
  for (uint32_t c0 = c_begin; c0 < c_end; c0 += kAhead) {
    uint32_t v[kAhead];
#pragma unroll
    for (uint32_t q = 0; q < kAhead; ++q) v[q] = (live && c0 + q < c_end) ? hist[(uint64_t)(c0 + q) * B.nbins + b] : 0u;
#pragma unroll
    for (uint32_t q = 0; q < kAhead; ++q) sum += v[q];
  }
  s_part[wv][lane] = sum;
  __syncthreads();
  uint32_t run = 0, total = 0;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) {
    const uint32_t x = s_part[q][lane];
    if ((uint32_t)q < wv) run += x;
    total += x;
  }
  for (uint32_t c0 = c_begin; c0 < c_end; c0 += kAhead) {
    uint32_t v[kAhead];
#pragma unroll
    for (uint32_t q = 0; q < kAhead; ++q) v[q] = (live && c0 + q < c_end) ? hist[(uint64_t)(c0 + q) * B.nbins + b] : 0u;
#pragma unroll
    for (uint32_t q = 0; q < kAhead; ++q) {
      if (live && c0 + q < c_end) hist[(uint64_t)(c0 + q) * B.nbins + b] = run;
      run += v[q];
    }
  }
  if (wv == 0 && live) ws_bin_start(B, k)[b] = total;
}

__global__ __launch_bounds__(kBinBlock) void bin_start_kernel(const EncodeBatch B) {
  constexpr int kWaves = kBinBlock / kWave;
  constexpr int kMaxPer = kMaxBins / kBinBlock;           // 8
  __shared__ uint32_t s_wave[kWaves];
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  uint32_t* bin_start = ws_bin_start(B, k);
  const uint32_t per = (B.nbins + kBinBlock - 1) / kBinBlock;   // thread t owns bins t*per .. t*per + per - 1
  uint32_t c[kMaxPer], sum = 0;
#pragma unroll
  for (int q = 0; q < kMaxPer; ++q) {
    const uint32_t e = threadIdx.x * per + q;
    c[q] = ((uint32_t)q < per && e < B.nbins) ? bin_start[e] : 0u;
    sum += c[q];
  }
  const uint32_t incl = wave_inclusive_scan_u32(sum, lane);
  if (lane == kWave - 1) s_wave[wv] = incl;
  __syncthreads();
  uint32_t run = incl - sum, all = 0;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) {
    const uint32_t x = s_wave[q];
    if ((uint32_t)q < wv) run += x;
    all += x;
  }
#pragma unroll
  for (int q = 0; q < kMaxPer; ++q) {
    const uint32_t e = threadIdx.x * per + q;
    if ((uint32_t)q < per && e < B.nbins) {
      bin_start[e] = run;
      run += c[q];
    }
  }
  if (threadIdx.x == 0) bin_start[B.nbins] = all;
}

// One workgroup per chunk of kBinChunk list items, one pass per sketch row j.  The
// chunk's records for row j are first sorted by slice inside LDS (a counting
// sort: LDS counters give every record its rank in its slice, a scan of the
// counters gives the start of every slice's run) and then copied out in sorted
// order, so that consecutive lanes write consecutive records of the (chunk, bin)
// run that the histogram pass reserved.  In LDS a record carries its slice number
// in bits 16..28 of its first word (the cell takes bits 0..14, the sign bit 31).
// Dynamic LDS: kBinChunk records, then two arrays of (slices per row) counters.
__global__ __launch_bounds__(kBinBlock) void bin_scatter_kernel(const EncodeBatch B, const HashRows hp) {
  extern __shared__ uint2 s_stage[];
  constexpr int kWaves = kBinBlock / kWave;
  constexpr int kMaxPer = kMaxBins / kBinBlock;           // counters per thread in the scan, at most
  __shared__ uint32_t s_wave[kWaves];
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;
  const uint32_t chunk = blockIdx.x;
  const uint64_t have = listed_items(B, k);
  const uint64_t t0 = (uint64_t)chunk * kBinChunk;
  if (t0 >= have) return;                                 // uniform over the workgroup
  const uint32_t count = have - t0 < (uint64_t)kBinChunk ? (uint32_t)(have - t0) : (uint32_t)kBinChunk;
  const uint32_t spr_log2 = B.log2w - B.slice_log2;
  const uint32_t spr = 1u << spr_log2;                    // slices per row
  uint32_t* s_loc = reinterpret_cast<uint32_t*>(s_stage + kBinChunk);
  uint32_t* s_delta = s_loc + spr;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  const WorkerPtrs P = B.w[k];
  const uint32_t* hist = ws_bin_hist(B, k) + (uint64_t)chunk * B.nbins;
  const uint32_t* bin_start = ws_bin_start(B, k);
  uint2* __restrict__ rec = ws_records(B, k);
  const uint32_t mask = (1u << B.slice_log2) - 1u;
  const uint32_t per = (spr + kBinBlock - 1) / kBinBlock; // counters per thread in the scan (<= kMaxPer)

  uint32_t i[kBinItems], v[kBinItems];
  bool ok[kBinItems];                                     // the item exists and takes part (see load_item)
#pragma unroll
  for (int u = 0; u < kBinItems; ++u) {
    const uint32_t t = u * kBinBlock + threadIdx.x;
    ok[u] = t < count && load_item(B, P, t0 + t, i[u], v[u]);
  }
  for (uint32_t e = threadIdx.x; e < spr; e += kBinBlock) s_loc[e] = 0u;

  for (uint32_t j = 0; j < B.d; ++j) {
    // where the runs of this (chunk, row) start in the worker's records; needed after the scan
    uint32_t gpos[kMaxPer];
#pragma unroll
    for (int q = 0; q < kMaxPer; ++q) {
      const uint32_t e = threadIdx.x * per + q;
      gpos[q] = ((uint32_t)q < per && e < spr) ? bin_start[(j << spr_log2) + e] + hist[(j << spr_log2) + e] : 0u;
    }
    __syncthreads();                                      // s_loc is zero, s_stage is free
    uint32_t key[kBinItems], rank[kBinItems];
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      if (ok[u]) {
        const uint32_t h = bucket_of(i[u], hp.a[j], hp.b[j], B.log2w);
        const uint32_t sl = h >> B.slice_log2;
        key[u] = (h & mask) | signbit_of(i[u], hp.c[j], hp.e[j]) | (sl << 16);
        rank[u] = __hip_atomic_fetch_add(&s_loc[sl], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
    __syncthreads();
    // exclusive scan of the counters; thread t owns counters t*per .. t*per + per - 1
    uint32_t c[kMaxPer], sum = 0;
#pragma unroll
    for (int q = 0; q < kMaxPer; ++q) {
      const uint32_t e = threadIdx.x * per + q;
      c[q] = ((uint32_t)q < per && e < spr) ? s_loc[e] : 0u;
      sum += c[q];
    }
    const uint32_t incl = wave_inclusive_scan_u32(sum, lane);
    if (lane == kWave - 1) s_wave[wv] = incl;
    __syncthreads();
    uint32_t run = incl - sum, records = 0;               // records: the chunk's items that take part
#pragma unroll
    for (int q = 0; q < kWaves; ++q) {
      const uint32_t x = s_wave[q];
      if ((uint32_t)q < wv) run += x;
      records += x;
    }
#pragma unroll
    for (int q = 0; q < kMaxPer; ++q) {
      const uint32_t e = threadIdx.x * per + q;
      if ((uint32_t)q < per && e < spr) {
        s_loc[e] = run;
        s_delta[e] = gpos[q] - run;                       // sorted position p of slice e goes to record p + delta
        run += c[q];
      }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      if (ok[u]) s_stage[s_loc[(key[u] >> 16) & 0x1FFFu] + rank[u]] = make_uint2(key[u], v[u]);
    }
    __syncthreads();
    for (uint32_t p = threadIdx.x; p < records; p += kBinBlock) {
      const uint2 r = s_stage[p];
      rec[p + s_delta[(r.x >> 16) & 0x1FFFu]] = make_uint2(r.x & 0x80007FFFu, r.y);
    }
    for (uint32_t e = threadIdx.x; e < spr; e += kBinBlock) s_loc[e] = 0u;      // for the next row; not read above
  }
}

// Workgroup = bin (j, s) of worker blockIdx.y.  The slice is accumulated in
// float64: the LDS float64 atomic add runs at full LDS rate on this chip (about
// 1.7e12 per second over the chip at random addresses) while the float32 one
// takes a slow path (0.2e12 per second, whatever the addresses); each cell is
// rounded to float32 once, when the slice is stored.  The first records are
// requested before the slice is cleared, and each later batch while the previous
// one is added.
__global__ __launch_bounds__(kSliceBlock) void sketch_slice_kernel(const EncodeBatch B) {
  extern __shared__ double s_slice[];
  constexpr int kAhead = 4;                               // 8-byte record loads in flight per thread
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;                           // uniform over the workgroup
  const uint32_t bin = blockIdx.x;                        // = (j << log2(slices per row)) + s
  const uint32_t cells = 1u << B.slice_log2;
  const uint32_t* bin_start = ws_bin_start(B, k);
  const uint32_t first = bin_start[bin], last = bin_start[bin + 1];
  const u32x2* __restrict__ rec = reinterpret_cast<const u32x2*>(ws_records(B, k));
  const u32x2 none = {0u, 0u};
  u32x2 x[kAhead];
  uint64_t r0 = (uint64_t)first + threadIdx.x;            // 64 bits: positions near 2^32 must not wrap
#pragma unroll
  for (int u = 0; u < kAhead; ++u)
    x[u] = r0 + u * kSliceBlock < last ? __builtin_nontemporal_load(&rec[r0 + u * kSliceBlock]) : none;

  if (cells >= 2u * kSliceBlock) {                        // (the LDS array is 16-byte aligned)
    for (uint32_t c = threadIdx.x; c < cells / 2; c += kSliceBlock)
      reinterpret_cast<double2*>(s_slice)[c] = make_double2(0.0, 0.0);
  } else {
    for (uint32_t c = threadIdx.x; c < cells; c += kSliceBlock) s_slice[c] = 0.0;
  }
  __syncthreads();

  while (r0 < last) {                                     // x holds the records r0 + u * kSliceBlock
    const uint64_t r1 = r0 + kSliceBlock * kAhead;
    u32x2 y[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u)
      y[u] = r1 + u * kSliceBlock < last ? __builtin_nontemporal_load(&rec[r1 + u * kSliceBlock]) : none;
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      if (r0 + u * kSliceBlock < last)
        __hip_atomic_fetch_add(&s_slice[x[u].x & 0x7FFFFFFFu],
                               (double)__uint_as_float(x[u].y ^ (x[u].x & 0x80000000u)),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u) x[u] = y[u];
    r0 = r1;
  }
  __syncthreads();
  // bin = j * slices-per-row + s, so the slice starts at cell bin * cells of the row-major sketch
  float* out = B.w[k].sketch + (uint64_t)bin * cells;
  if (cells >= 4u * kSliceBlock) {                        // (every slice of 4 cells or more is 16-byte aligned)
    for (uint32_t c = threadIdx.x; c < cells / 4; c += kSliceBlock) {
      const double2 lo = reinterpret_cast<const double2*>(s_slice)[2 * c];
      const double2 hi = reinterpret_cast<const double2*>(s_slice)[2 * c + 1];
      f32x4 o;
      o.x = (float)lo.x; o.y = (float)lo.y; o.z = (float)hi.x; o.w = (float)hi.y;
      __builtin_nontemporal_store(o, &reinterpret_cast<f32x4*>(out)[c]);
    }
  } else {
    for (uint32_t c = threadIdx.x; c < cells; c += kSliceBlock) out[c] = (float)s_slice[c];
  }
}

// Non-zeros at list positions >= cap are not in the caller's lists; this kernel
// finds them in the bitmap and inserts them with atomics after the slices were
// stored, so the sketch is complete whatever cap is.  Normally there are none:
// each thread checks one tile's range of list positions and the workgroup leaves
// unless one of its kBlock tiles reaches beyond cap.
__global__ __launch_bounds__(kBlock) void sketch_overflow_kernel(const EncodeBatch B, const HashRows hp) {
  __shared__ TileBits T;
  __shared__ uint32_t s_any;
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;                           // uniform over the workgroup
  const WorkerPtrs P = B.w[k];
  const uint64_t* prefix = ws_prefix(B, k);
  const uint32_t tile0 = blockIdx.x * kBlock;
  if (threadIdx.x == 0) s_any = 0u;
  __syncthreads();
  const uint32_t mine = tile0 + threadIdx.x;
  if (mine < B.ntiles && prefix[mine + 1] > B.cap) s_any = 1u;
  __syncthreads();
  if (s_any == 0u) return;                               // uniform over the workgroup
  for (uint32_t tile = tile0; tile < tile0 + kBlock && tile < B.ntiles; ++tile) {
    const uint64_t base = prefix[tile];
    const uint32_t total = (uint32_t)(prefix[tile + 1] - base);
    if (base + total <= B.cap) continue;                 // uniform over the workgroup
    const uint64_t word0 = (uint64_t)tile * kTileWords;
    uint64_t wd[kWordsPerThread];
    read_tile_words<kBlock>(wd, P.bitmap, B.nwords, word0);
    __syncthreads();                                     // T may still be read by the previous tile's loop
    scan_tile_words<kBlock>(T, wd);
    const uint32_t first = base >= B.cap ? 0u : (uint32_t)(B.cap - base);
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

// ------------------------------------------------------------------ merge
struct MergeArgs {
  const float* sketch[S2R_MAX_WORKERS];
  const uint64_t* bitmap[S2R_MAX_WORKERS];
  float* sketch_out;
  uint64_t* bitmap_out;
  uint64_t ncell4;          // number of 4-cell groups
  uint64_t ncells;          // d*w
  uint64_t nwords;
  uint32_t W;
  uint32_t sketch_blocks;   // blocks [0, sketch_blocks) sum the sketch, the rest OR the bitmap
};

// One thread per 16 bytes of sketch (blocks [0, sketch_blocks)) or per bitmap word
// (the remaining blocks).  The W inputs of a position are independent streams:
// they are read eight at a time so that eight loads are in flight per thread, and
// added in ascending worker order.
__global__ __launch_bounds__(kBlock) void merge_kernel(const MergeArgs A) {
  constexpr uint32_t kDepth = 8;
  if (blockIdx.x < A.sketch_blocks) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < A.ncell4) {
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      for (uint32_t k0 = 0; k0 < A.W; k0 += kDepth) {
        f32x4 x[kDepth];
#pragma unroll
        for (uint32_t u = 0; u < kDepth; ++u)
          if (k0 + u < A.W) x[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(A.sketch[k0 + u]) + i);
#pragma unroll
        for (uint32_t u = 0; u < kDepth; ++u) {
          if (k0 + u < A.W) acc = (k0 + u == 0) ? x[0] : acc + x[u];      // worker 0 starts the sum: no 0 + x
        }
      }
      reinterpret_cast<f32x4*>(A.sketch_out)[i] = acc;
    }
    // cells beyond the last full group of four (only when d*w is not a multiple of 4)
    const uint64_t t = A.ncell4 * 4 + i;
    if (t < A.ncells) {
      float acc = A.sketch[0][t];
      for (uint32_t k = 1; k < A.W; ++k) acc += A.sketch[k][t];
      A.sketch_out[t] = acc;
    }
  } else {
    const uint64_t i = (uint64_t)(blockIdx.x - A.sketch_blocks) * kBlock + threadIdx.x;
    if (i < A.nwords) {
      uint64_t acc = 0;
      for (uint32_t k0 = 0; k0 < A.W; k0 += kDepth) {
        uint64_t x[kDepth];
#pragma unroll
        for (uint32_t u = 0; u < kDepth; ++u) x[u] = k0 + u < A.W ? __builtin_nontemporal_load(A.bitmap[k0 + u] + i) : 0ull;
#pragma unroll
        for (uint32_t u = 0; u < kDepth; ++u) acc |= x[u];
      }
      A.bitmap_out[i] = acc;
    }
  }
}

// ------------------------------------------------------------------ streaming-read probe
// A plain read of nvec 16-byte words, shaped like the dense scan (each wave reads
// kProbePer consecutive 1 KiB rows with streaming loads): what the memory system
// delivers to a kernel that only reads.  The XOR of the words keeps the loads alive;
// it is stored only if it equals a value the host chooses.
constexpr int kProbePer = 8;
__global__ __launch_bounds__(kBlock) void probe_read_kernel(const u32x4* __restrict__ src, uint64_t nvec,
                                                            uint64_t* __restrict__ sink, uint32_t magic) {
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint64_t wave = (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  const uint64_t v0 = wave * (kProbePer * kWave) + lane;
  u32x4 x[kProbePer];
#pragma unroll
  for (int q = 0; q < kProbePer; ++q) {
    const uint64_t v = v0 + (uint64_t)q * kWave;
    x[q] = v < nvec ? __builtin_nontemporal_load(&src[v]) : u32x4{0u, 0u, 0u, 0u};
  }
  uint32_t acc = 0;
#pragma unroll
  for (int q = 0; q < kProbePer; ++q) acc ^= x[q].x ^ x[q].y ^ x[q].z ^ x[q].w;
  if (acc == magic) *sink = acc;
}

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
// of the inputs (odd D); even D averages the two middle ones in float32.
template <int D>
__device__ __forceinline__ float median_fixed(float (&x)[D]) {
#pragma unroll
  for (int a = 0; a < D - 1; ++a) {
#pragma unroll
    for (int b = 0; b < D - 1 - a; ++b) {
      const float lo = fminf(x[b], x[b + 1]);
      const float hi = fmaxf(x[b], x[b + 1]);
      x[b] = lo;
      x[b + 1] = hi;
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

// ------------------------------------------------------------------ decode by sketch slices
// The bucket reads of decode_kernel each fetch a 128-byte line for 4 useful
// bytes.  When the union list is long, s2r_decode instead partitions the
// (list position, row) queries by sketch slice with the kernels of the encode's
// slice strategy (records carry the list position instead of a value) and
//   decode_slice_kernel   workgroup (j, s) loads slice s of row j into LDS with
//                         coalesced loads, answers its bin's queries from LDS
//                         and writes (estimate, position in chunk) into the
//                         region of the query's chunk of kBinChunk list
//                         positions: row j's answers of chunk c start at
//                         (c * kBinChunk * d) + j * (items in c), and inside
//                         them bin (j, s) starts where the prefix of the
//                         chunk's histogram over the bins says
//   decode_median_kernel  workgroup = chunk: row by row, the answers go through
//                         LDS into the registers of the thread that owns the
//                         list position; then the medians, stored coalesced
struct DecodeSliceArgs {
  const float* sketch;
  const u32x2* rec;          // queries sorted by bin: (cell in slice | sign bit, list position)
  uint2* answers;            // [nchunks][d][kBinChunk]-shaped regions, see above
  const uint32_t* bin_start; // [nbins + 1]
  const uint32_t* colpre;    // [nchunks][nbins]: queries of the bin in earlier chunks
  const uint32_t* rowpre;    // [nchunks][nbins]: queries of the chunk in earlier bins
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

constexpr int kBinChunkLog2 = 13;
static_assert((1 << kBinChunkLog2) == kBinChunk, "list positions are split into chunk and offset by shifts");

__global__ __launch_bounds__(kSliceBlock) void decode_slice_kernel(const DecodeSliceArgs A) {
  extern __shared__ float s_cells[];
  constexpr int kAhead = 4;
  const uint32_t bin = blockIdx.x;                        // = (j << log2(slices per row)) + s
  const uint32_t first = A.bin_start[bin], last = A.bin_start[bin + 1];
  if (first == last) return;                              // uniform over the workgroup
  const u32x2 none = {0u, 0u};
  u32x2 x[kAhead];                                        // the first queries are requested together with the slice
  uint64_t r0 = (uint64_t)first + threadIdx.x;
#pragma unroll
  for (int u = 0; u < kAhead; ++u)
    x[u] = r0 + u * kSliceBlock < last ? __builtin_nontemporal_load(&A.rec[r0 + u * kSliceBlock]) : none;
  const uint32_t cells = 1u << A.slice_log2;
  const float* src = A.sketch + (uint64_t)bin * cells;    // row-major sketch: slice s of row j starts at bin * cells
  if (cells >= 4u * kSliceBlock) {                        // (the sketch and every slice of 4 cells or more are 16-byte aligned)
    for (uint32_t c = threadIdx.x; c < cells / 4; c += kSliceBlock)
      reinterpret_cast<float4*>(s_cells)[c] = reinterpret_cast<const float4*>(src)[c];
  } else {
    for (uint32_t c = threadIdx.x; c < cells; c += kSliceBlock) s_cells[c] = src[c];
  }
  __syncthreads();
  while (r0 < last) {                                     // x holds the queries r0 + u * kSliceBlock
    const uint64_t r1 = r0 + kSliceBlock * kAhead;
    u32x2 y[kAhead];
    uint32_t colp[kAhead], rowp[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u)
      y[u] = r1 + u * kSliceBlock < last ? __builtin_nontemporal_load(&A.rec[r1 + u * kSliceBlock]) : none;
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const uint64_t at = (uint64_t)(x[u].y >> kBinChunkLog2) * A.nbins + bin;
      const bool live = r0 + u * kSliceBlock < last;
      colp[u] = live ? A.colpre[at] : 0u;
      rowp[u] = live ? A.rowpre[at] : 0u;
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const uint64_t r = r0 + u * kSliceBlock;
      if (r >= last) continue;
      const uint32_t est = __float_as_uint(s_cells[x[u].x & 0x7FFFFFFFu]) ^ (x[u].x & 0x80000000u);
      const uint64_t chunk = x[u].y >> kBinChunkLog2;
      const uint64_t at = chunk * kBinChunk * A.d + rowp[u] + (uint32_t)(r - first - colp[u]);
      A.answers[at] = make_uint2(est, x[u].y & (kBinChunk - 1));
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u) x[u] = y[u];
    r0 = r1;
  }
}

template <int D>
__global__ __launch_bounds__(kBinBlock) void decode_median_kernel(const DecodeSliceArgs A) {
  __shared__ float s_est[kBinChunk];
  const uint32_t chunk = blockIdx.x;
  const uint64_t total = *A.count;
  const uint64_t listed = total < A.cap ? total : A.cap;
  const uint64_t have = A.block != 0 ? listed * A.block : listed;
  const uint64_t t0 = (uint64_t)chunk * kBinChunk;
  if (t0 >= have) return;                                 // uniform over the workgroup
  const uint32_t count = have - t0 < (uint64_t)kBinChunk ? (uint32_t)(have - t0) : (uint32_t)kBinChunk;
  float est[kBinItems][D];
  uint2 cur[kBinItems], nxt[kBinItems];                   // row j's answers, and row j + 1's on their way
  const uint2* rows = A.answers + t0 * D;
#pragma unroll
  for (int u = 0; u < kBinItems; ++u) {
    const uint32_t t = u * kBinBlock + threadIdx.x;
    cur[u] = t < count ? rows[t] : make_uint2(0u, 0u);
  }
#pragma unroll
  for (int j = 0; j < D; ++j) {
    if (j + 1 < D) {
#pragma unroll
      for (int u = 0; u < kBinItems; ++u) {
        const uint32_t t = u * kBinBlock + threadIdx.x;
        nxt[u] = t < count ? rows[(uint64_t)(j + 1) * count + t] : make_uint2(0u, 0u);
      }
    }
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      if (u * kBinBlock + threadIdx.x < count) s_est[cur[u].y] = __uint_as_float(cur[u].x);
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) {
      const uint32_t t = u * kBinBlock + threadIdx.x;
      est[u][j] = t < count ? s_est[t] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kBinItems; ++u) cur[u] = nxt[u];
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

// ------------------------------------------------------------------ host side
struct EventPair { hipEvent_t begin, end; };
static thread_local EventPair g_events[S2R_KERNEL_SLOTS] = {};
static thread_local int32_t g_strategy = S2R_INSERT_AUTO;
static thread_local int32_t g_last_strategy = S2R_INSERT_AUTO;   // what the last encode call used
static thread_local int32_t g_decode_strategy = S2R_DECODE_AUTO;
static thread_local int32_t g_last_decode_strategy = S2R_DECODE_AUTO;   // what the last decode call used
static thread_local uint32_t g_scan_launch_workers = 0;     // workers covered by the scan launch the events bracket

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
// strategy [bin histogram u32[nchunks][nbins]] [bin starts u32[nbins + 1]] [records 8 B x d*cap]; each part
// 256-byte aligned.  The slice parts exist only when the caller's workspace is large enough for its cap.
static inline size_t workspace_prefix_off(uint64_t n) {
  return align256((size_t)tiles_of(n) * kScansPerTile * sizeof(uint16_t));
}
static inline size_t workspace_dense_off(uint64_t n) {
  return workspace_prefix_off(n) + align256(((size_t)tiles_of(n) + 1) * sizeof(uint64_t));
}
static inline size_t workspace_base(uint64_t n) {
  return workspace_dense_off(n) + 256 + align256((size_t)tiles_of(n) * kGroupsPerTile * sizeof(uint32_t));
}
// workgroups of the kernels that take the dense-tile list (per problem); each loops over the entries
static inline uint32_t dense_grid(uint32_t ntiles, uint32_t most) {
  const uint64_t entries = (uint64_t)ntiles * (kGroupsPerTile - 1);
  return (uint32_t)(entries < most ? (entries > 0 ? entries : 1) : most);
}
struct SliceLayout {
  bool possible;             // the bins fit the LDS histograms and record positions fit 32 bits
  uint32_t slice_log2, nbins, nchunks;
  size_t hist_off, binstart_off, rec_off, total;
};
static SliceLayout slice_layout(uint64_t n, uint32_t d, uint32_t w, uint64_t cap) {
  SliceLayout L;
  const uint32_t log2w = log2_of(w);
  L.slice_log2 = log2w < (uint32_t)kSliceLog2Max ? log2w : (uint32_t)kSliceLog2Max;
  const uint64_t nbins = (uint64_t)d << (log2w - L.slice_log2);
  L.possible = nbins <= (uint64_t)kMaxBins && (uint64_t)d * cap < (1ull << 32) && cap > 0;
  L.nbins = (uint32_t)(L.possible ? nbins : 0);
  L.nchunks = (uint32_t)(L.possible ? ceil_div(cap, kBinChunk) : 0);
  L.hist_off = workspace_base(n);
  L.binstart_off = L.hist_off + align256((size_t)L.nchunks * L.nbins * sizeof(uint32_t));
  L.rec_off = L.binstart_off + align256(((size_t)L.nbins + 1) * sizeof(uint32_t));
  L.total = L.rec_off + align256((size_t)(L.possible ? d * cap : 0) * 8);
  return L;
}

// How s2r_encode forms the sketch.  Cost models fitted to measurements on MI355X
// (W = 4..16, n = 2^20..1e9, d = 3..5, w = 2^14..2^22):
//  - atomics: the sketch is zeroed first (about 4.5e12 bytes per second); scattered
//    float32 atomics retire at about 21e9 per second over the whole chip whatever
//    their scope, and when the dense scan issues them it hides about 40 % of that
//    time (less when the non-zeros are clustered in few workgroups);
//  - slices: five more kernels, about 20 us of launches; 4 us per round of 256
//    slice workgroups (each clears and stores 128 KiB of LDS); histogram, scatter
//    and slice kernels together pass about 180e9 records per second.
// `cap` is the caller's bound on the number of non-zeros.
static int32_t choose_strategy(uint32_t W, uint64_t n, uint32_t d, uint32_t w, bool have_lists, uint64_t cap,
                               size_t workspace_bytes) {
  (void)n;
  if (!have_lists || cap == 0) return S2R_INSERT_ATOMIC;     // the slice strategy reads Sparse(g)
  const SliceLayout L = slice_layout(n, d, w, cap);
  if (!L.possible || workspace_bytes < L.total) return S2R_INSERT_ATOMIC;
  if (g_strategy != S2R_INSERT_AUTO) return g_strategy;
  const double records = (double)cap * d;
  const double rounds = (double)ceil_div((uint64_t)W * L.nbins, 256);       // all workers' slices share the CUs
  const double t_slice = 20e-6 + rounds * 4e-6 + W * records / 180e9;
  const double t_atomic = W * (4.0 * d * w / 4.5e12 + 0.6 * records / 21e9);
  return t_slice < t_atomic ? S2R_INSERT_SLICE : S2R_INSERT_ATOMIC;
}

// Workspace of s2r_decode when it partitions its queries by sketch slice: the base parts, then
// [bin histogram u32[nchunks][nbins]] [its per-chunk prefix over the bins, same shape] [bin starts u32[nbins + 1]]
// [queries sorted by bin, 8 B x d*cap] [answers grouped by chunk, 8 B x d * nchunks * kBinChunk].
constexpr int kDecodeSliceMaxRows = 8;                   // decode_median_kernel keeps 8 x d estimates per thread
struct DecodeLayout {
  bool possible;
  uint32_t slice_log2, nbins, nchunks;
  size_t hist_off, rowpre_off, binstart_off, rec_off, answers_off, total;
};
static DecodeLayout decode_layout(uint64_t n, uint32_t d, uint32_t w, uint64_t cap) {
  DecodeLayout L;
  const uint32_t log2w = log2_of(w);
  L.slice_log2 = log2w < (uint32_t)kDecodeSliceLog2Max ? log2w : (uint32_t)kDecodeSliceLog2Max;
  const uint64_t nbins = (uint64_t)d << (log2w - L.slice_log2);
  L.possible = nbins <= (uint64_t)kMaxBins && (uint64_t)d * cap < (1ull << 32) && cap > 0 &&
               d <= (uint32_t)kDecodeSliceMaxRows;
  L.nbins = (uint32_t)(L.possible ? nbins : 0);
  L.nchunks = (uint32_t)(L.possible ? ceil_div(cap, kBinChunk) : 0);
  const size_t matrix = align256((size_t)L.nchunks * L.nbins * sizeof(uint32_t));
  L.hist_off = workspace_base(n);
  L.rowpre_off = L.hist_off + matrix;
  L.binstart_off = L.rowpre_off + matrix;
  L.rec_off = L.binstart_off + align256(((size_t)L.nbins + 1) * sizeof(uint32_t));
  L.answers_off = L.rec_off + align256((size_t)(L.possible ? d * cap : 0) * 8);
  L.total = L.answers_off + align256((size_t)L.nchunks * kBinChunk * d * 8);
  return L;
}

// How s2r_decode reads the buckets.  Measured on MI355X: gathers from a sketch far larger than the L2
// (4 MB per XCD) run at about 56e9 per second (each fetches a 128-byte line), from one of a few L2 sizes at
// about 70e9, from one that fits at about 200e9; the slice route costs about 80 us of launches and latency
// and passes about 110e9 queries per second.
// `cap` (the capacity of the caller's lists) stands in for the number of union indices, which only the
// device knows.
static int32_t choose_decode(uint64_t n, uint32_t d, uint32_t w, bool have_lists, bool dense_out, uint64_t cap,
                             size_t workspace_bytes) {
  if (!have_lists || dense_out || cap == 0) return S2R_DECODE_GATHER;
  const DecodeLayout L = decode_layout(n, d, w, cap);
  if (!L.possible || workspace_bytes < L.total) return S2R_DECODE_GATHER;
  if (g_decode_strategy != S2R_DECODE_AUTO) return g_decode_strategy;
  const double queries = (double)cap * d;
  const double sketch_bytes = 4.0 * d * w;
  const double t_gather = queries / (sketch_bytes > 16e6 ? 56e9 : sketch_bytes > 4e6 ? 70e9 : 200e9);
  const double t_slice = 80e-6 + queries / 110e9;
  return t_slice < t_gather ? S2R_DECODE_SLICE : S2R_DECODE_GATHER;
}

// The slice kernels use more dynamic LDS than the default limit allows; raised once per host thread and device.
static bool raise_lds_limits() {
  constexpr int kMaxDevices = 64;
  static thread_local bool raised[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) return false;
  if (dev < kMaxDevices && raised[dev]) return true;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(sketch_slice_kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSliceLdsMax) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(bin_scatter_kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)(kBinChunk * sizeof(uint2) + 2 * sizeof(uint32_t) * kMaxBins)) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(decode_slice_kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)(sizeof(float) << kDecodeSliceLog2Max)) != hipSuccess)
    return false;
  if (dev < kMaxDevices) raised[dev] = true;
  return true;
}

static inline void record(int slot, bool end, hipStream_t st) {
  hipEvent_t ev = end ? g_events[slot].end : g_events[slot].begin;
  if (ev != nullptr) (void)hipEventRecord(ev, st);
}

static inline bool launch_ok() { return hipGetLastError() == hipSuccess; }

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

int32_t s2r_version(void) { return 300; }

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

s2r_status s2r_set_insert_strategy(int32_t strategy) {
  if (strategy != S2R_INSERT_AUTO && strategy != S2R_INSERT_ATOMIC && strategy != S2R_INSERT_SLICE) return S2R_ERR_SIZE;
  g_strategy = strategy;
  return S2R_OK;
}

s2r_status s2r_set_decode_strategy(int32_t strategy) {
  if (strategy != S2R_DECODE_AUTO && strategy != S2R_DECODE_GATHER && strategy != S2R_DECODE_SLICE) return S2R_ERR_SIZE;
  g_decode_strategy = strategy;
  return S2R_OK;
}

int32_t s2r_last_decode_strategy(void) { return g_last_decode_strategy; }

size_t s2r_decode_workspace_bytes(uint64_t n, uint32_t d, uint32_t w, uint64_t cap) {
  if (check_sizes(n, d, w) != S2R_OK || cap > n) return 0;
  const DecodeLayout L = decode_layout(n, d, w, cap);
  return L.possible ? L.total : workspace_base(n);
}

uint32_t s2r_scan_launch_workers(void) { return g_scan_launch_workers; }

int32_t s2r_last_insert_strategy(void) { return g_last_strategy; }

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

s2r_status s2r_set_kernel_events(int32_t slot, void* ev_begin, void* ev_end) {
  if (slot < 0 || slot >= S2R_KERNEL_SLOTS) return S2R_ERR_SIZE;
  if ((ev_begin == nullptr) != (ev_end == nullptr)) return S2R_ERR_NULL;
  g_events[slot].begin = (hipEvent_t)ev_begin;
  g_events[slot].end = (hipEvent_t)ev_end;
  return S2R_OK;
}

// The encode of W workers (W = 1 for s2r_encode): every kernel is launched once
// with the worker in blockIdx.y.  workspace_bytes is the size of the whole
// workspace, split evenly between the workers.
// block = 0: the element codec (bitmaps of n bits, lists of non-zero elements with their values).
// block >= 1: the block-granular codec (bitmaps of ceil(n / block) bits, lists of non-zero blocks, nz_val
// unused, cap counted in blocks).
static s2r_status encode_workers(const float* const* grads, uint32_t W, uint64_t n, uint32_t block, uint32_t d,
                                 uint32_t w, uint64_t seed, float* const* sketches, uint64_t* const* bitmaps,
                                 uint32_t* const* nz_idx, float* const* nz_val, uint64_t cap, uint64_t* nnz_out,
                                 void* workspace, size_t workspace_bytes, hipStream_t st, bool marked = false) {
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
  const size_t ws_each = (workspace_bytes / W) & ~(size_t)255;
  if (workspace == nullptr || ((uintptr_t)workspace & 255u) != 0 || ws_each < workspace_base(nbits))
    return S2R_ERR_WORKSPACE;

  HashRows hp;
  make_hash_rows(seed, d, &hp);
  const uint32_t ntiles = tiles_of(nbits);
  const uint32_t log2w = log2_of(w);
  const int32_t strategy = choose_strategy(W, nbits, d, w, lists, cap_items, ws_each);
  g_last_strategy = strategy;

  E.nworkers = W;
  E.rowpre_off = 0;
  E.payload_slot = 0;
  E.nnz_out = nnz_out;
  E.workspace = reinterpret_cast<char*>(workspace);
  E.ws_stride = ws_each;
  E.block = block;
  E.prefix_off = workspace_prefix_off(nbits);
  E.dense_off = workspace_dense_off(nbits);
  const SliceLayout L = slice_layout(nbits, d, w, cap_items);
  E.hist_off = L.hist_off;
  E.binstart_off = L.binstart_off;
  E.rec_off = L.rec_off;
  E.nbins = L.nbins;
  E.nchunks = L.nchunks;
  E.n = n;
  E.nwords = ceil_div(nbits, 64);
  E.cap = cap;
  E.ntiles = ntiles;
  E.d = d;
  E.log2w = log2w;
  E.slice_log2 = L.slice_log2;

  // The scan, preceded by the zeroing of the sketch when the scan inserts into it with atomics.  Gradients
  // of 1 GiB and more are scanned worker by worker, smaller ones with one launch over the whole batch.
  // Measured on config 5 (4 GB per worker, 84 MB sketches): one launch per worker takes 632 us per worker,
  // one launch over all workers 649 us; with atomics, a scan whose sketch was zeroed just before it takes
  // 760 us against 820 us when all 16 sketches were zeroed first.  Below 1 GiB the launches saved count more.
  const uint64_t cells = (uint64_t)d * w;
  const bool atomics = strategy == S2R_INSERT_ATOMIC;
  const uint64_t nvec = cells / 4;
  const uint32_t ntail = (uint32_t)(cells - nvec * 4);
  uint64_t zb = ceil_div(nvec > 0 ? nvec : 1, kBlock);
  if (zb > 2048) zb = 2048;
  const uint32_t group = n * sizeof(float) >= (1ull << 30) ? 1u : W;
  // element codec: every piece of every tile gets its count; block codec: the pieces that hold elements
  const uint32_t scan_blocks = block != 0 ? (uint32_t)ceil_div(ceil_div(n, 64), kScanWords) : ntiles * kScansPerTile;
  uint32_t last_group = 0;
  if (marked && atomics) {                                    // the sketches only: the bitmaps are the caller's
    E.first_worker = 0;
    hipLaunchKernelGGL(zero_kernel, dim3((uint32_t)zb, W), dim3(kBlock), 0, st, E, nvec, ntail, (uint64_t)0);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }
  for (uint32_t k0 = 0; k0 < W && !marked; k0 += group) {
    const uint32_t gy = W - k0 < group ? W - k0 : group;      // workers k0 .. k0 + gy - 1, all < W
    const bool last = k0 + gy == W;                           // the events bracket the last scan launch
    E.first_worker = k0;
    if (atomics || block != 0) {                              // the block bitmap is set bit by bit: zero it first
      hipLaunchKernelGGL(zero_kernel, dim3((uint32_t)zb, gy), dim3(kBlock), 0, st, E, atomics ? nvec : (uint64_t)0,
                         atomics ? ntail : 0u, block != 0 ? E.nwords : (uint64_t)0);
      if (!launch_ok()) return S2R_ERR_LAUNCH;
    }
    if (last) record(S2R_KERNEL_ENCODE_SCAN, false, st);
    const dim3 sgrid(scan_blocks, gy), sblock(kBlock);
    if (block != 0 && atomics)
      hipLaunchKernelGGL((encode_scan_kernel<kScanEPL, true, true>), sgrid, sblock, 0, st, E, hp);
    else if (block != 0)
      hipLaunchKernelGGL((encode_scan_kernel<kScanEPL, false, true>), sgrid, sblock, 0, st, E, hp);
    else if (atomics)
      hipLaunchKernelGGL((encode_scan_kernel<kScanEPL, true, false>), sgrid, sblock, 0, st, E, hp);
    else
      hipLaunchKernelGGL((encode_scan_kernel<kScanEPL, false, false>), sgrid, sblock, 0, st, E, hp);
    if (last) record(S2R_KERNEL_ENCODE_SCAN, true, st);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    last_group = gy;
  }
  g_scan_launch_workers = last_group;
  E.first_worker = 0;

  if (block != 0) {                                          // the counts of the block bitmap's pieces
    hipLaunchKernelGGL(bitmap_count_batch_kernel, dim3((uint32_t)ceil_div(ntiles, kWavesPerBlock), W), dim3(kBlock), 0,
                       st, E);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(tile_prefix_kernel, dim3(1, W), dim3(kPrefixBlock), 0, st, E.workspace, E.ws_stride,
                     E.prefix_off, E.dense_off, ntiles, nnz_out);
  if (!launch_ok()) return S2R_ERR_LAUNCH;

  if (lists && cap > 0) {
    const uint32_t helpers = dense_grid(ntiles, 512);
    hipLaunchKernelGGL(encode_compact_kernel, dim3(helpers + ntiles, W), dim3(kBlock), 0, st, E, helpers);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }

  if (strategy == S2R_INSERT_SLICE) {
    const size_t lds = sizeof(double) << E.slice_log2;
    if (!raise_lds_limits()) return S2R_ERR_LAUNCH;
    hipLaunchKernelGGL(bin_hist_kernel, dim3(E.nchunks, W), dim3(kBinBlock), 0, st, E, hp);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    hipLaunchKernelGGL(bin_colscan_kernel, dim3((uint32_t)ceil_div(E.nbins, kWave), W), dim3(kBinBlock), 0, st, E);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    hipLaunchKernelGGL(bin_start_kernel, dim3(1, W), dim3(kBinBlock), 0, st, E);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    const size_t scatter_lds = (size_t)kBinChunk * sizeof(uint2) + 2 * sizeof(uint32_t) * ((size_t)1 << (log2w - E.slice_log2));
    hipLaunchKernelGGL(bin_scatter_kernel, dim3(E.nchunks, W), dim3(kBinBlock), scatter_lds, st, E, hp);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    record(S2R_KERNEL_ENCODE_SLICE, false, st);
    hipLaunchKernelGGL(sketch_slice_kernel, dim3(E.nbins, W), dim3(kSliceBlock), lds, st, E);
    record(S2R_KERNEL_ENCODE_SLICE, true, st);
    if (!launch_ok()) return S2R_ERR_LAUNCH;

    hipLaunchKernelGGL(sketch_overflow_kernel, dim3((uint32_t)ceil_div(ntiles, kBlock), W), dim3(kBlock), 0, st, E, hp);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  } else if (marked) {
    // no scan has inserted anything: every set block goes the way of the blocks beyond the lists
    EncodeBatch A = E;
    A.cap = 0;
    hipLaunchKernelGGL(sketch_overflow_kernel, dim3((uint32_t)ceil_div(ntiles, kBlock), W), dim3(kBlock), 0, st, A, hp);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }
  return S2R_OK;
}

s2r_status s2r_encode(const float* grad, uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                      float* sketch, uint64_t* bitmap, uint32_t* nz_idx, float* nz_val, uint64_t cap,
                      uint64_t* nnz_out, void* workspace, size_t workspace_bytes, void* stream) {
  if ((nz_idx == nullptr) != (nz_val == nullptr)) return S2R_ERR_NULL;
  return encode_workers(&grad, 1, n, 0u, d, w, seed, &sketch, &bitmap, nz_idx ? &nz_idx : nullptr,
                        nz_val ? &nz_val : nullptr, cap, nnz_out, workspace, workspace_bytes, (hipStream_t)stream);
}

s2r_status s2r_encode_batch(const float* const* grads, uint32_t W, uint64_t n, uint32_t d, uint32_t w,
                            uint64_t seed, float* const* sketches, uint64_t* const* bitmaps,
                            uint32_t* const* nz_idx, float* const* nz_val, uint64_t cap, uint64_t* nnz_out,
                            void* workspace, size_t workspace_bytes, void* stream) {
  return encode_workers(grads, W, n, 0u, d, w, seed, sketches, bitmaps, nz_idx, nz_val, cap, nnz_out, workspace,
                        workspace_bytes, (hipStream_t)stream);
}

s2r_status s2r_merge(const float* const* sketches, const uint64_t* const* bitmaps, uint32_t W, uint64_t n,
                     uint32_t d, uint32_t w, uint64_t seed, float* sketch_out, uint64_t* bitmap_out,
                     void* stream) {
  (void)seed;
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
  A.sketch_out = sketch_out;
  A.bitmap_out = bitmap_out;
  A.ncells = (uint64_t)d * w;
  A.ncell4 = A.ncells / 4;
  A.nwords = ceil_div(n, 64);
  A.W = W;
  // one thread per 16 bytes of sketch / 8 bytes of bitmap (d*w <= 2^32 and n <= 2^32 keep the grid below 2^23)
  const uint64_t sb = ceil_div(A.ncell4 > 0 ? A.ncell4 : 1, kBlock);
  const uint64_t bb = ceil_div(A.nwords, kBlock);
  A.sketch_blocks = (uint32_t)sb;
  hipStream_t st = (hipStream_t)stream;
  record(S2R_KERNEL_MERGE, false, st);
  hipLaunchKernelGGL(merge_kernel, dim3((uint32_t)(sb + bb)), dim3(kBlock), 0, st, A);
  record(S2R_KERNEL_MERGE, true, st);
  return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
}

// block = 0: the element codec.  block >= 1: the block-granular codec: the bitmap has ceil(n / block) bits,
// idx_out lists the set blocks (cap of them at most), val_out holds block values per listed block, and there
// is no dense output.
static s2r_status decode_impl(const float* sketch, const uint64_t* bitmap, uint64_t n, uint32_t block, uint32_t d,
                              uint32_t w, uint64_t seed, uint32_t* idx_out, float* val_out, uint64_t cap,
                              uint64_t* count_out, float* dense_out, void* workspace, size_t workspace_bytes,
                              void* stream, float* params = nullptr, float scale = 0.0f) {
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

  hipStream_t st = (hipStream_t)stream;
  HashRows hp;
  make_hash_rows(seed, d, &hp);
  const uint32_t ntiles = tiles_of(n);
  const uint64_t nwords = ceil_div(n, 64);

  uint16_t* piece_count = reinterpret_cast<uint16_t*>(workspace);
  uint64_t* tile_prefix = reinterpret_cast<uint64_t*>((char*)workspace + workspace_prefix_off(n));
  hipLaunchKernelGGL(bitmap_count_kernel, dim3((uint32_t)ceil_div(ntiles, kWavesPerBlock)), dim3(kBlock), 0, st,
                     bitmap, nwords, ntiles, piece_count);
  if (!launch_ok()) return S2R_ERR_LAUNCH;
  hipLaunchKernelGGL(tile_prefix_kernel, dim3(1), dim3(kPrefixBlock), 0, st, (char*)workspace, (uint64_t)0,
                     (uint64_t)workspace_prefix_off(n), (uint64_t)workspace_dense_off(n), ntiles, count_out);
  if (!launch_ok()) return S2R_ERR_LAUNCH;
  if ((idx_out == nullptr || cap == 0) && dense_out == nullptr && params == nullptr) return S2R_OK;   // only the count was asked for

  if (cap > n) cap = n;
  const uint64_t cap_items = block != 0 ? cap * block : cap;    // list positions that get a value, at most
  // (an update of parameters, like a dense output, must reach the union indices beyond the lists' capacity too)
  const int32_t strategy = choose_decode(n, d, w, idx_out != nullptr, dense_out != nullptr || params != nullptr, idx_out ? cap_items : 0,
                                         workspace_bytes);
  g_last_decode_strategy = strategy;
  if (strategy == S2R_DECODE_SLICE) {
    const DecodeLayout L = decode_layout(n, d, w, cap_items);
    if (!raise_lds_limits()) return S2R_ERR_LAUNCH;
    // the kernels of the encode's slice strategy, on one "worker" whose list is the union list
    static thread_local EncodeBatch X;                     // (2.6 KB: not on the stack of every call)
    X.w[0].grad = nullptr;                                 // expansion without values
    X.w[0].sketch = nullptr;
    X.w[0].bitmap = const_cast<uint64_t*>(bitmap);        // only read
    X.w[0].nz_idx = idx_out;
    X.w[0].nz_val = nullptr;
    X.nnz_out = count_out;
    X.workspace = reinterpret_cast<char*>(workspace);
    X.ws_stride = 0;
    X.prefix_off = workspace_prefix_off(n);
    X.dense_off = workspace_dense_off(n);
    X.hist_off = L.hist_off;
    X.binstart_off = L.binstart_off;
    X.rec_off = L.rec_off;
    X.rowpre_off = L.rowpre_off;
    X.payload_slot = 1;
    X.block = block;
    X.n = elements;
    X.nwords = nwords;
    X.cap = cap;
    X.ntiles = ntiles;
    X.d = d;
    X.log2w = log2_of(w);
    X.slice_log2 = L.slice_log2;
    X.nbins = L.nbins;
    X.nchunks = L.nchunks;
    X.first_worker = 0;
    X.nworkers = 1;
    char* ws = reinterpret_cast<char*>(workspace);
    DecodeSliceArgs Q;
    Q.sketch = sketch;
    Q.rec = reinterpret_cast<const u32x2*>(ws + L.rec_off);
    Q.answers = reinterpret_cast<uint2*>(ws + L.answers_off);
    Q.bin_start = reinterpret_cast<const uint32_t*>(ws + L.binstart_off);
    Q.colpre = reinterpret_cast<const uint32_t*>(ws + L.hist_off);
    Q.rowpre = reinterpret_cast<const uint32_t*>(ws + L.rowpre_off);
    Q.count = count_out;
    Q.cap = cap;
    Q.val_out = val_out;
    Q.nbins = L.nbins;
    Q.slice_log2 = L.slice_log2;
    Q.d = d;
    Q.block = block;
    Q.n = elements;
    Q.blk_list = idx_out;

    record(S2R_KERNEL_DECODE, false, st);
    const uint32_t helpers = dense_grid(ntiles, 2048);
    hipLaunchKernelGGL(encode_compact_kernel, dim3(helpers + ntiles, 1), dim3(kBlock), 0, st, X, helpers);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    hipLaunchKernelGGL(bin_hist_kernel, dim3(L.nchunks, 1), dim3(kBinBlock), 0, st, X, hp);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    hipLaunchKernelGGL(bin_colscan_kernel, dim3((uint32_t)ceil_div(L.nbins, kWave), 1), dim3(kBinBlock), 0, st, X);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    hipLaunchKernelGGL(bin_start_kernel, dim3(1, 1), dim3(kBinBlock), 0, st, X);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    const size_t scatter_lds = (size_t)kBinChunk * sizeof(uint2) + 2 * sizeof(uint32_t) * ((size_t)1 << (X.log2w - X.slice_log2));
    hipLaunchKernelGGL(bin_scatter_kernel, dim3(L.nchunks, 1), dim3(kBinBlock), scatter_lds, st, X, hp);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    hipLaunchKernelGGL(decode_slice_kernel, dim3(L.nbins), dim3(kSliceBlock), sizeof(float) << L.slice_log2, st, Q);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
    const dim3 mgrid(L.nchunks), mblock(kBinBlock);
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
    record(S2R_KERNEL_DECODE, true, st);
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
    static thread_local EncodeBatch X;
    X.w[0].grad = nullptr;
    X.w[0].sketch = nullptr;
    X.w[0].bitmap = const_cast<uint64_t*>(bitmap);        // only read
    X.w[0].nz_idx = idx_out;
    X.w[0].nz_val = nullptr;
    X.nnz_out = count_out;
    X.workspace = reinterpret_cast<char*>(workspace);
    X.ws_stride = 0;
    X.prefix_off = workspace_prefix_off(n);
    X.dense_off = workspace_dense_off(n);
    X.rowpre_off = 0;
    X.payload_slot = 0;
    X.block = block;
    X.n = elements;
    X.nwords = nwords;
    X.cap = cap;
    X.ntiles = ntiles;
    X.d = d;
    X.log2w = A.log2w;
    X.first_worker = 0;
    X.nworkers = 1;
    record(S2R_KERNEL_DECODE, false, st);
    const uint32_t helpers = dense_grid(ntiles, 2048);
    hipLaunchKernelGGL(encode_compact_kernel, dim3(helpers + ntiles, 1), dim3(kBlock), 0, st, X, helpers);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
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
    record(S2R_KERNEL_DECODE, true, st);
    return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
  }

  record(S2R_KERNEL_DECODE, false, st);
  const uint32_t helpers = dense_grid(ntiles, 2048);
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
  record(S2R_KERNEL_DECODE, true, st);
  return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
}


s2r_status s2r_decode(const float* sketch, const uint64_t* bitmap, uint64_t n, uint32_t d, uint32_t w,
                      uint64_t seed, uint32_t* idx_out, float* val_out, uint64_t cap, uint64_t* count_out,
                      float* dense_out, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_impl(sketch, bitmap, n, 0u, d, w, seed, idx_out, val_out, cap, count_out, dense_out, workspace,
                     workspace_bytes, stream);
}

s2r_status s2r_decode_update(const float* sketch, const uint64_t* bitmap, uint64_t n, uint32_t d, uint32_t w,
                             uint64_t seed, float* params, float scale, uint32_t* idx_out, float* val_out, uint64_t cap,
                             uint64_t* count_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (params == nullptr) return S2R_ERR_NULL;
  if (((uintptr_t)params & 3u) != 0) return S2R_ERR_ALIGN;
  return decode_impl(sketch, bitmap, n, 0u, d, w, seed, idx_out, val_out, cap, count_out, nullptr, workspace,
                     workspace_bytes, stream, params, scale);
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
  return L.possible ? L.total : workspace_base(nb);
}

s2r_status s2r_encode_blocks_batch(const float* const* grads, uint32_t W, uint64_t n, uint32_t block, uint32_t d,
                                   uint32_t w, uint64_t seed, float* const* sketches, uint64_t* const* block_bitmaps,
                                   uint32_t* const* blk_idx, uint64_t blk_cap, uint64_t* nblk_out, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  if (!block_ok(n, block)) return S2R_ERR_SIZE;
  return encode_workers(grads, W, n, block, d, w, seed, sketches, block_bitmaps, blk_idx, nullptr, blk_cap, nblk_out,
                        workspace, workspace_bytes, (hipStream_t)stream);
}

s2r_status s2r_encode_blocks(const float* grad, uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t seed,
                             float* sketch, uint64_t* block_bitmap, uint32_t* blk_idx, uint64_t blk_cap,
                             uint64_t* nblk_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!block_ok(n, block)) return S2R_ERR_SIZE;
  return encode_workers(&grad, 1, n, block, d, w, seed, &sketch, &block_bitmap, blk_idx ? &blk_idx : nullptr, nullptr,
                        blk_cap, nblk_out, workspace, workspace_bytes, (hipStream_t)stream);
}

}  // extern "C"

void s2r::record_kernel_event(int slot, bool end, void* stream) { record(slot, end, (hipStream_t)stream); }

s2r_status s2r::encode_marked_blocks(const float* const* values, uint32_t W, uint64_t n, uint32_t block, uint32_t d,
                                     uint32_t w, uint64_t seed, float* const* sketches, uint64_t* const* block_bitmaps,
                                     uint32_t* const* blk_idx, uint64_t cap, uint64_t* nblk_out, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  if (!block_ok(n, block)) return S2R_ERR_SIZE;
  return encode_workers(values, W, n, block, d, w, seed, sketches, block_bitmaps, blk_idx, nullptr, cap, nblk_out,
                        workspace, workspace_bytes, (hipStream_t)stream, true);
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
                     workspace_bytes, stream, params, scale);
}

s2r_status s2r_decode_blocks(const float* sketch, const uint64_t* block_bitmap, uint64_t n, uint32_t block, uint32_t d,
                             uint32_t w, uint64_t seed, uint32_t* blk_idx_out, float* val_out, uint64_t blk_cap,
                             uint64_t* nblk_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!block_ok(n, block)) return S2R_ERR_SIZE;
  return decode_impl(sketch, block_bitmap, n, block, d, w, seed, blk_idx_out, val_out, blk_cap, nblk_out, nullptr,
                     workspace, workspace_bytes, stream);
}

}  // extern "C"
