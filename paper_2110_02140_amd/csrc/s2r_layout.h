// Constants, vector types and kernel-argument structs shared by the codec's kernels:
// the tiling of gradient, bitmaps and lists, the batch of workers an encode kernel
// takes, and where each part of a worker's workspace share lies.
// Included by s2r_kernels.hip only (one translation unit).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/s2r.h"
#include "s2r_device.h"

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
constexpr int kSliceWorkgroups = 256;             // slice workgroups that are resident at a time: one per compute unit
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
  uint64_t seg_off;          // slice variant: byte offsets inside a chunk of the segment offsets u32[nchunks][nbins + 1]
  uint64_t rec_off;          //   and of the sorted records, 8 bytes each, kBinChunk * d per chunk of list items
  uint32_t payload_slot;     // non-zero: a record carries its item's list position instead of nz_val
  uint32_t block;            // block-granular codec: elements per bitmap bit; nz_idx then lists blocks, and
                             //   bitmap / nwords / ntiles / cap describe the block bitmap.  0: one bit per element
  uint64_t n;
  uint64_t nwords;
  uint64_t cap;              // capacity of the caller's lists (entries; blocks in the block codec)
  uint64_t sort_cap;         // list entries that take part in the counting sort (<= cap; 0: none): what the
                             //   workspace's record area holds; entries beyond it are inserted with atomics
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
__device__ __forceinline__ uint32_t* ws_seg(const EncodeBatch& B, uint32_t k) {
  return reinterpret_cast<uint32_t*>(B.workspace + k * B.ws_stride + B.seg_off);
}
__device__ __forceinline__ uint2* ws_records(const EncodeBatch& B, uint32_t k) {
  return reinterpret_cast<uint2*>(B.workspace + k * B.ws_stride + B.rec_off);
}

}  // namespace s2r
