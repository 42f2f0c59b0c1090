// The aggregation AllReduce(S, C) of Algorithm 1 on one GPU, and the streaming-read
// probe used by the benchmark.
// Included by s2r_kernels.hip only (one translation unit).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/s2r.h"
#include "s2r_layout.h"

namespace s2r {

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
  uint16_t* piece_count;    // COUNTS: the aggregated bitmap's set bits per piece of kScanWords words, for every
  uint64_t count_words;     //   piece of every tile: count_words = tiles * kTileWords words are covered
};

// One thread per 16 bytes of sketch (blocks [0, sketch_blocks)) or per bitmap word
// (the remaining blocks).  The W inputs of a position are independent streams,
// read DEPTH at a time with streaming loads and added in ascending worker order;
// the outputs leave with streaming stores.  Measured on MI355X (sketches of 12 to
// 84 MB): with up to 8 workers 2 or 4 loads in flight per thread reach 5.9 to
// 6.1 TB/s and 8 only 4.7 to 5.1; with 16 workers 8 in flight are the best
// (6.1 against 5.7 TB/s): the host picks DEPTH = 4 below 16 workers, else 8.
// COUNTS: the bitmap part also leaves what the decompression step reads first, the
// set-bit counts of the aggregated bitmap per piece (the pieces the dense scan
// counts for a worker's bitmap): a piece is kScanWords = 32 consecutive words,
// that is 32 consecutive lanes, whose popcounts meet in a butterfly.
template <int DEPTH, bool COUNTS>
__global__ __launch_bounds__(kBlock) void merge_kernel(const MergeArgs A) {
  constexpr uint32_t kDepth = DEPTH;
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
      __builtin_nontemporal_store(acc, reinterpret_cast<f32x4*>(A.sketch_out) + i);
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
    uint64_t acc = 0;
    if (i < A.nwords) {
      for (uint32_t k0 = 0; k0 < A.W; k0 += kDepth) {
        uint64_t x[kDepth];
#pragma unroll
        for (uint32_t u = 0; u < kDepth; ++u) x[u] = k0 + u < A.W ? __builtin_nontemporal_load(A.bitmap[k0 + u] + i) : 0ull;
#pragma unroll
        for (uint32_t u = 0; u < kDepth; ++u) acc |= x[u];
      }
      __builtin_nontemporal_store(acc, A.bitmap_out + i);
    }
    if (COUNTS) {                                          // (every lane of the wave is here: words beyond the end count 0)
      static_assert(kScanWords == 32 && kBlock % kScanWords == 0, "a piece is one half of a wave");
      uint32_t c = (uint32_t)__popcll(acc);
#pragma unroll
      for (int m = kScanWords / 2; m >= 1; m >>= 1) c += __shfl_xor(c, m, kWave);
      if ((threadIdx.x & (kScanWords - 1)) == 0 && i < A.count_words) A.piece_count[i / kScanWords] = (uint16_t)c;
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

}  // namespace s2r
