// Encode, first pass (Algorithm 1, the bitmap line and, in the atomic variant, the
// insertion loops): zeroing of sketches and block bitmaps, and the one pass over
// the dense gradient.
// Included by s2r_kernels.hip only (one translation unit).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/s2r.h"
#include "s2r_layout.h"

namespace s2r {

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

}  // namespace s2r
