// gfx950 kernels and C ABI of the block-wise Top-K sparsifier with error
// feedback that the paper puts in front of the codec for dense layers
// (Section 2.2: the l2 norm of every block, the K largest blocks are kept;
// Theorem 2: what is not sent stays in an error sequence added to the next
// gradient).  See include/s2r.h for the contract.
//
//   topk_score_kernel,  acc = g + e per element; per block the sum of squares
//   topk_score_vec_kernel (float64 accumulation, one rounding to float32) packed
//                       with the block index into a 64-bit key, larger key =
//                       kept first (higher score, then lower block).  STORE: acc
//                       is written back over e on the way
//   topk_hist_kernel,   radix select of the K-th largest key: six digits of 11
//   topk_pick_kernel    or 10 bits from the top; per digit a histogram of the
//                       keys that share the digits found so far.  The digit is
//                       picked from the complete histogram by every workgroup of
//                       the next pass (and by one last small launch).  Keys are
//                       distinct, so the result is the exact threshold
//   topk_apply_kernel   second pass: kept blocks go to the sparse gradient, the
//                       rest to the new residual
//   topk_bitmap_kernel  bitmap of the kept blocks, a wave ballot per word
//   topk_clear_kept_kernel  (one-call sparsify + compress) the residual of the
//                       kept blocks becomes zero once the codec has read acc there
// No kernel waits for another workgroup.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/s2r.h"
#include "s2r_device.h"
#include "s2r_internal.h"

namespace s2r_topk {
using s2r::kWave;
using s2r::wave_inclusive_scan_u32;

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kHistBlock = 1024;
constexpr int kHistPer = 8;                       // keys per thread of a histogram workgroup
constexpr int kBins = 2048;                       // 11-bit digits (the last two digits have 10 bits)
constexpr int kPasses = 6;
__constant__ const uint32_t kShift[kPasses] = {53, 42, 31, 20, 10, 0};
__constant__ const uint32_t kWidth[kPasses] = {11, 11, 11, 11, 10, 10};
constexpr int kScorePer = 4;                      // blocks per wave of the score kernel
constexpr int kScoreLoads = 4;                    // rows of 64 elements per block and trip
constexpr int kApplyPer = 4;                      // elements per thread of the apply kernel (one 16-byte access)

static inline __host__ __device__ uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct TopkState {          // per worker, in the workspace
  uint64_t prefix;          // the digits of the K-th largest key found so far; after the last pass, the key itself
  uint64_t remaining;       // how many keys still to take among those that share the prefix
};

struct TopkWorker {
  const float* grad;
  float* residual;           // may be null: no error feedback
  float* sparse;
  uint64_t* kept_bitmap;     // may be null
};

struct TopkBatch {
  TopkWorker w[S2R_MAX_WORKERS];
  char* workspace;           // W chunks of ws_stride bytes: keys u64[nb] | histograms u32[kPasses][kBins] | TopkState[kPasses + 1]
  uint64_t ws_stride;
  uint64_t hist_off, state_off;
  uint64_t n;
  uint64_t nb;
  uint64_t K;
  uint32_t block;
  uint32_t nworkers;
};

__device__ __forceinline__ uint64_t* ws_keys(const TopkBatch& B, uint32_t k) {
  return reinterpret_cast<uint64_t*>(B.workspace + k * B.ws_stride);
}
__device__ __forceinline__ uint32_t* ws_hist(const TopkBatch& B, uint32_t k) {
  return reinterpret_cast<uint32_t*>(B.workspace + k * B.ws_stride + B.hist_off);
}
__device__ __forceinline__ TopkState* ws_state(const TopkBatch& B, uint32_t k) {
  return reinterpret_cast<TopkState*>(B.workspace + k * B.ws_stride + B.state_off);
}

__device__ __forceinline__ uint64_t make_key(double sum_sq, uint64_t x) {
  const uint32_t bits = __float_as_uint((float)sum_sq) & 0x7FFFFFFFu;      // a sum of squares has no sign
  return ((uint64_t)bits << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)x);
}

// One wave per block (blocks of 32 elements and more) or one thread per block.
// Workgroup 0 of every worker also resets the histogram and the selection state.
// STORE: acc = g + e is also written back over e (the caller wants the residual
// updated in place and reads acc from there afterwards); needs a residual.
template <bool STORE>
__global__ __launch_bounds__(kBlock) void topk_score_kernel(const TopkBatch B) {
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;
  const TopkWorker P = B.w[k];
  uint64_t* keys = ws_keys(B, k);
  if (blockIdx.x == 0) {
    uint32_t* hist = ws_hist(B, k);                         // one histogram per pass of the select
    for (uint32_t b = threadIdx.x; b < kPasses * kBins; b += kBlock) hist[b] = 0u;
    if (threadIdx.x == 0) {
      TopkState* st = ws_state(B, k);                       // state[p]: after the digits of passes 0 .. p-1
      st->prefix = 0ull;
      st->remaining = B.K;
    }
  }
  const uint32_t lane = threadIdx.x & (kWave - 1);
  if (B.block >= 32u) {
    // a wave takes kScorePer consecutive blocks and walks them together, kScoreLoads rows of 64 elements of
    // each per trip: 2 * kScorePer * kScoreLoads streaming loads in flight per lane
    const uint64_t x0 = ((uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave) * kScorePer;
    if (x0 >= B.nb) return;                                // uniform over the wave
    double sum[kScorePer];
#pragma unroll
    for (int q = 0; q < kScorePer; ++q) sum[q] = 0.0;
    for (uint32_t o = lane; o < B.block; o += kScoreLoads * kWave) {
      float a[kScorePer][kScoreLoads];
#pragma unroll
      for (int q = 0; q < kScorePer; ++q) {
#pragma unroll
        for (int u = 0; u < kScoreLoads; ++u) {
          const uint64_t i = (x0 + q) * B.block + o + (uint64_t)u * kWave;
          const bool in = x0 + q < B.nb && o + u * kWave < B.block && i < B.n;
          a[q][u] = in ? __builtin_nontemporal_load(&P.grad[i]) : 0.0f;
          if (in && P.residual != nullptr) a[q][u] += __builtin_nontemporal_load(&P.residual[i]);
        }
      }
      if (STORE) {
#pragma unroll
        for (int q = 0; q < kScorePer; ++q) {
#pragma unroll
          for (int u = 0; u < kScoreLoads; ++u) {
            const uint64_t i = (x0 + q) * B.block + o + (uint64_t)u * kWave;
            const bool in = x0 + q < B.nb && o + u * kWave < B.block && i < B.n;
            if (in) P.residual[i] = a[q][u];
          }
        }
      }
#pragma unroll
      for (int q = 0; q < kScorePer; ++q) {
#pragma unroll
        for (int u = 0; u < kScoreLoads; ++u) sum[q] += (double)a[q][u] * (double)a[q][u];
      }
    }
#pragma unroll
    for (int q = 0; q < kScorePer; ++q) {
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) sum[q] += __shfl_xor(sum[q], off, kWave);
      if (lane == 0 && x0 + q < B.nb) keys[x0 + q] = make_key(sum[q], x0 + q);
    }
  } else {
    const uint64_t x = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (x >= B.nb) return;
    double sum = 0.0;
    for (uint32_t o = 0; o < B.block; ++o) {
      const uint64_t i = x * B.block + o;
      if (i >= B.n) break;
      float a = P.grad[i];
      if (P.residual != nullptr) a += P.residual[i];
      if (STORE) P.residual[i] = a;
      sum += (double)a * (double)a;
    }
    keys[x] = make_key(sum, x);
  }
}

// The same for blocks of a multiple of 4 elements (32 and more): 16-byte accesses.
// A wave takes kScorePer consecutive blocks; lane l owns the 4-element chunks
// l, l + 64, ... of each, kVecTrips of them per block and trip.  The last block
// of a gradient whose length is not a multiple of 4 ends in a chunk that is read
// and written element by element.
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kVecTrips = 1;

template <bool STORE>
__global__ __launch_bounds__(kBlock) void topk_score_vec_kernel(const TopkBatch B) {
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;
  const TopkWorker P = B.w[k];
  uint64_t* keys = ws_keys(B, k);
  if (blockIdx.x == 0) {
    uint32_t* hist = ws_hist(B, k);                         // one histogram per pass of the select
    for (uint32_t b = threadIdx.x; b < kPasses * kBins; b += kBlock) hist[b] = 0u;
    if (threadIdx.x == 0) {
      TopkState* st = ws_state(B, k);                       // state[p]: after the digits of passes 0 .. p-1
      st->prefix = 0ull;
      st->remaining = B.K;
    }
  }
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint64_t x0 = ((uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave) * kScorePer;
  if (x0 >= B.nb) return;                                  // uniform over the wave
  const uint32_t chunks = B.block / 4;
  double sum[kScorePer];
#pragma unroll
  for (int q = 0; q < kScorePer; ++q) sum[q] = 0.0;
  for (uint32_t c = lane; c < chunks; c += kVecTrips * kWave) {
    f32x4 a[kScorePer][kVecTrips];
#pragma unroll
    for (int q = 0; q < kScorePer; ++q) {
#pragma unroll
      for (int u = 0; u < kVecTrips; ++u) {
        const uint32_t cc = c + (uint32_t)u * kWave;
        const uint64_t i = (x0 + q) * B.block + 4ull * cc;
        const bool in = x0 + q < B.nb && cc < chunks && i < B.n;
        a[q][u] = (f32x4)(0.0f);
        if (in && i + 4 <= B.n) {
          a[q][u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(P.grad + i));
          if (P.residual != nullptr) a[q][u] += __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(P.residual + i));
        } else if (in) {
          for (int j = 0; j < 4; ++j) {
            if (i + j < B.n) {
              float v = P.grad[i + j];
              if (P.residual != nullptr) v += P.residual[i + j];
              a[q][u][j] = v;
            }
          }
        }
      }
    }
    if (STORE) {
#pragma unroll
      for (int q = 0; q < kScorePer; ++q) {
#pragma unroll
        for (int u = 0; u < kVecTrips; ++u) {
          const uint32_t cc = c + (uint32_t)u * kWave;
          const uint64_t i = (x0 + q) * B.block + 4ull * cc;
          const bool in = x0 + q < B.nb && cc < chunks && i < B.n;
          if (in && i + 4 <= B.n) {
            __builtin_nontemporal_store(a[q][u], reinterpret_cast<f32x4*>(P.residual + i));
          } else if (in) {
            for (int j = 0; j < 4; ++j)
              if (i + j < B.n) P.residual[i + j] = a[q][u][j];
          }
        }
      }
    }
#pragma unroll
    for (int q = 0; q < kScorePer; ++q) {
#pragma unroll
      for (int u = 0; u < kVecTrips; ++u) {
#pragma unroll
        for (int j = 0; j < 4; ++j) sum[q] += (double)a[q][u][j] * (double)a[q][u][j];
      }
    }
  }
#pragma unroll
  for (int q = 0; q < kScorePer; ++q) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum[q] += __shfl_xor(sum[q], off, kWave);
    if (lane == 0 && x0 + q < B.nb) keys[x0 + q] = make_key(sum[q], x0 + q);
  }
}

// The digit of pass `pass` from that pass's complete histogram: the digit d with
// (keys above d) < remaining <= (keys above d) + (keys in d), appended to the
// state before the pass.  All kHistBlock threads of a workgroup call it (thread
// t looks at bins 2t and 2t + 1); every thread gets the new state.  Keys are
// distinct and remaining <= number of keys, so exactly one bin qualifies.
__device__ __forceinline__ TopkState pick_digit(const uint32_t* __restrict__ hist, const TopkState prev, uint32_t pass,
                                                uint32_t* s_wave, TopkState* s_out) {
  constexpr int kWaves = kHistBlock / kWave;
  const uint32_t lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
  const uint32_t c0 = hist[2 * threadIdx.x], c1 = hist[2 * threadIdx.x + 1];   // bins 2t, 2t + 1
  const uint32_t sum = c0 + c1;
  const uint32_t incl = wave_inclusive_scan_u32(sum, lane);
  if (lane == kWave - 1) s_wave[wv] = incl;
  if (threadIdx.x == 0) *s_out = prev;                     // stays if there is nothing to find
  __syncthreads();
  uint32_t before = incl - sum, total = 0;                 // keys in bins below 2t; all keys counted
#pragma unroll
  for (int q = 0; q < kWaves; ++q) {
    const uint32_t x = s_wave[q];
    if ((uint32_t)q < wv) before += x;
    total += x;
  }
  if (prev.remaining != 0 && prev.remaining <= total) {
    const uint64_t above1 = total - before - sum;          // keys in bins above 2t + 1
    const uint64_t above0 = above1 + c1;                   // keys in bins above 2t
    if (above1 < prev.remaining && prev.remaining <= above1 + c1) {
      s_out->prefix = prev.prefix | ((uint64_t)(2 * threadIdx.x + 1) << kShift[pass]);
      s_out->remaining = prev.remaining - above1;
    } else if (above0 < prev.remaining && prev.remaining <= above0 + c0) {
      s_out->prefix = prev.prefix | ((uint64_t)(2 * threadIdx.x) << kShift[pass]);
      s_out->remaining = prev.remaining - above0;
    }
  }
  __syncthreads();
  return *s_out;
}

// Histogram of digit `pass` over the keys that share the digits found so far.
// Every workgroup first works out the digit of the pass before from that pass's
// histogram (complete: it was another launch), which spares a launch per pass;
// workgroup 0 also records the state for the next launch.
__global__ __launch_bounds__(kHistBlock) void topk_hist_kernel(const TopkBatch B, uint32_t pass) {
  __shared__ uint32_t s_hist[kBins];
  __shared__ uint32_t s_wave[kHistBlock / kWave];
  __shared__ TopkState s_state;
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;
  for (uint32_t b = threadIdx.x; b < kBins; b += kHistBlock) s_hist[b] = 0u;
  TopkState* state = ws_state(B, k);
  TopkState st = state[0];
  if (pass > 0) {
    st = pick_digit(ws_hist(B, k) + (size_t)(pass - 1) * kBins, state[pass - 1], pass - 1, s_wave, &s_state);
    if (blockIdx.x == 0 && threadIdx.x == 0) state[pass] = st;
  }
  __syncthreads();
  const uint64_t* __restrict__ keys = ws_keys(B, k);
  const uint64_t prefix = st.prefix;
  const uint32_t shift = kShift[pass], above = shift + kWidth[pass];
  const uint32_t mask = (1u << kWidth[pass]) - 1u;
  uint64_t key[kHistPer];
#pragma unroll
  for (int u = 0; u < kHistPer; ++u) {
    const uint64_t x = ((uint64_t)blockIdx.x * kHistPer + u) * kHistBlock + threadIdx.x;
    key[u] = x < B.nb ? keys[x] : ~0ull;                   // ~0 is no key (bit 63 of a key is clear)
  }
#pragma unroll
  for (int u = 0; u < kHistPer; ++u) {
    const bool same = above >= 64u || (key[u] >> above) == (prefix >> above);
    if (key[u] != ~0ull && same)
      __hip_atomic_fetch_add(&s_hist[(uint32_t)(key[u] >> shift) & mask], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  __syncthreads();
  uint32_t* hist = ws_hist(B, k) + (size_t)pass * kBins;
  for (uint32_t b = threadIdx.x; b < kBins; b += kHistBlock)
    if (s_hist[b] != 0u) atomicAdd(&hist[b], s_hist[b]);
}

// One workgroup per worker, after the last pass: its digit completes the K-th
// largest key, state[kPasses].prefix, the threshold the later kernels compare with.
__global__ __launch_bounds__(kHistBlock) void topk_pick_kernel(const TopkBatch B) {
  __shared__ uint32_t s_wave[kHistBlock / kWave];
  __shared__ TopkState s_state;
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;
  TopkState* state = ws_state(B, k);
  const TopkState st = pick_digit(ws_hist(B, k) + (size_t)(kPasses - 1) * kBins, state[kPasses - 1], kPasses - 1, s_wave,
                                  &s_state);
  if (threadIdx.x == 0) state[kPasses] = st;
}

// Four consecutive elements per thread.  `all` / `none` bypass the threshold
// (K >= number of blocks, K = 0).  ACC_IN_E: the scores' pass has left acc in the
// residual; the gradient is not read again and the residual is only written where
// a block is kept.
template <bool ACC_IN_E>
__global__ __launch_bounds__(kBlock) void topk_apply_kernel(const TopkBatch B, uint32_t all, uint32_t none) {
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers) return;
  const TopkWorker P = B.w[k];
  const uint64_t* __restrict__ keys = ws_keys(B, k);
  const uint64_t T = all ? 0ull : none ? ~0ull : ws_state(B, k)[kPasses].prefix;
  const uint64_t i0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * kApplyPer;
  if (i0 >= B.n) return;
  float a[kApplyPer];
  const bool whole = i0 + kApplyPer <= B.n;
  if (whole) {
    const float4 g4 = *reinterpret_cast<const float4*>((ACC_IN_E ? P.residual : P.grad) + i0);
    a[0] = g4.x; a[1] = g4.y; a[2] = g4.z; a[3] = g4.w;
    if (!ACC_IN_E && P.residual != nullptr) {
      const float4 e4 = *reinterpret_cast<const float4*>(P.residual + i0);
      a[0] += e4.x; a[1] += e4.y; a[2] += e4.z; a[3] += e4.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < kApplyPer; ++j) {
      a[j] = 0.0f;
      if (i0 + j < B.n) {
        a[j] = ACC_IN_E ? P.residual[i0 + j] : P.grad[i0 + j];
        if (!ACC_IN_E && P.residual != nullptr) a[j] += P.residual[i0 + j];
      }
    }
  }
  uint64_t x = i0 / B.block;
  uint32_t r = (uint32_t)(i0 - x * B.block);
  float s[kApplyPer], e[kApplyPer];
  bool any_kept = false;
#pragma unroll
  for (int j = 0; j < kApplyPer; ++j) {
    const bool kept = x < B.nb && keys[x] >= T;
    any_kept |= kept;
    s[j] = kept ? a[j] : 0.0f;
    e[j] = kept ? 0.0f : a[j];
    if (++r == B.block) { r = 0; ++x; }
  }
  const bool store_e = P.residual != nullptr && (!ACC_IN_E || any_kept);     // (elsewhere e already holds acc)
  if (whole) {
    *reinterpret_cast<float4*>(P.sparse + i0) = make_float4(s[0], s[1], s[2], s[3]);
    if (store_e) *reinterpret_cast<float4*>(P.residual + i0) = make_float4(e[0], e[1], e[2], e[3]);
  } else {
#pragma unroll
    for (int j = 0; j < kApplyPer; ++j) {
      if (i0 + j < B.n) {
        P.sparse[i0 + j] = s[j];
        if (store_e) P.residual[i0 + j] = e[j];
      }
    }
  }
}

// One wave per word of the kept-block bitmap: lane l tests block 64 * word + l,
// and the ballot is the word.
__device__ __forceinline__ uint64_t kept_word(const TopkBatch& B, uint32_t k, uint64_t wd, uint32_t all, uint32_t none) {
  const uint64_t* __restrict__ keys = ws_keys(B, k);
  const uint64_t T = all ? 0ull : none ? ~0ull : ws_state(B, k)[kPasses].prefix;
  const uint64_t x = wd * 64 + (threadIdx.x & (kWave - 1));
  return __ballot(x < B.nb && keys[x] >= T);
}

__global__ __launch_bounds__(kBlock) void topk_bitmap_kernel(const TopkBatch B, uint32_t all, uint32_t none) {
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers || B.w[k].kept_bitmap == nullptr) return;
  const uint64_t wd = (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  if (wd >= ceil_div(B.nb, 64)) return;                    // uniform over the wave
  const uint64_t bits = kept_word(B, k, wd, all, none);
  if ((threadIdx.x & (kWave - 1)) == 0) B.w[k].kept_bitmap[wd] = bits;
}

// The residual of every kept block becomes +0.0 (the block has been sent).  A
// wave finds the kept blocks among its 64 and clears them one after the other.
__global__ __launch_bounds__(kBlock) void topk_clear_kept_kernel(const TopkBatch B, uint32_t all, uint32_t none) {
  const uint32_t k = blockIdx.y;
  if (k >= B.nworkers || B.w[k].residual == nullptr) return;
  float* __restrict__ e = B.w[k].residual;
  const uint64_t wd = (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  if (wd >= ceil_div(B.nb, 64)) return;                    // uniform over the wave
  const uint32_t lane = threadIdx.x & (kWave - 1);
  uint64_t bits = kept_word(B, k, wd, all, none);          // the same in every lane
  while (bits != 0) {
    const uint64_t x = wd * 64 + (uint32_t)__builtin_ctzll(bits);
    bits &= bits - 1;
    const uint64_t i0 = x * B.block;                       // < n: block x exists
    const uint64_t len = B.n - i0 < (uint64_t)B.block ? B.n - i0 : (uint64_t)B.block;
    if (B.block % 4u == 0u) {                              // 16-byte aligned block starts
      for (uint64_t c = lane; 4 * c < len; c += kWave) {
        if (4 * c + 4 <= len) {
          *reinterpret_cast<f32x4*>(e + i0 + 4 * c) = (f32x4)(0.0f);
        } else {
          for (uint64_t o = 4 * c; o < len; ++o) e[i0 + o] = 0.0f;
        }
      }
    } else {
      for (uint64_t o = lane; o < len; o += kWave) e[i0 + o] = 0.0f;
    }
  }
}

static inline size_t keys_bytes(uint64_t nb) { return align256((size_t)nb * sizeof(uint64_t)); }
static inline size_t hist_bytes() { return align256((size_t)kPasses * kBins * sizeof(uint32_t)); }
static inline size_t workspace_each(uint64_t nb) { return keys_bytes(nb) + hist_bytes() + 256; }
static_assert((kPasses + 1) * sizeof(TopkState) <= 256, "the states share one 256-byte part of the workspace");
static inline bool sizes_ok(uint64_t n, uint32_t block) {
  return n >= 1 && n <= (1ull << 32) && block >= 1 && (uint64_t)block <= (1ull << 31);
}
static inline bool launch_ok() { return hipGetLastError() == hipSuccess; }

// Fills B for W workers and checks the arguments that every entry point shares.
static s2r_status fill_batch(TopkBatch& B, const float* const* grads, float* const* residuals, uint32_t W, uint64_t n,
                             uint32_t block, uint64_t K, float* const* sparse_out, uint64_t* const* kept_bitmaps,
                             void* workspace, size_t workspace_bytes) {
  if (grads == nullptr) return S2R_ERR_NULL;
  if (W == 0 || W > S2R_MAX_WORKERS || !sizes_ok(n, block)) return S2R_ERR_SIZE;
  const uint64_t nb = ceil_div(n, block);
  for (uint32_t k = 0; k < W; ++k) {
    float* ek = residuals ? residuals[k] : nullptr;
    float* sk = sparse_out ? sparse_out[k] : nullptr;
    uint64_t* bk = kept_bitmaps ? kept_bitmaps[k] : nullptr;
    if (grads[k] == nullptr || (sparse_out && sk == nullptr) || (residuals && ek == nullptr) ||
        (kept_bitmaps && bk == nullptr))
      return S2R_ERR_NULL;
    if (((uintptr_t)grads[k] & 15u) || ((uintptr_t)sk & 15u) || ((uintptr_t)ek & 15u) || ((uintptr_t)bk & 7u))
      return S2R_ERR_ALIGN;
    B.w[k].grad = grads[k];
    B.w[k].residual = ek;
    B.w[k].sparse = sk;
    B.w[k].kept_bitmap = bk;
  }
  const size_t ws_each = (workspace_bytes / W) & ~(size_t)255;
  if (workspace == nullptr || ((uintptr_t)workspace & 255u) != 0 || ws_each < workspace_each(nb)) return S2R_ERR_WORKSPACE;
  B.workspace = reinterpret_cast<char*>(workspace);
  B.ws_stride = ws_each;
  B.hist_off = keys_bytes(nb);
  B.state_off = B.hist_off + hist_bytes();
  B.n = n;
  B.nb = nb;
  B.K = K > nb ? nb : K;
  B.block = block;
  B.nworkers = W;
  return S2R_OK;
}

// Scores (with acc written over the residuals if store_acc) and the radix select
// of the K-th largest key; afterwards block x is kept iff keys[x] >= state.prefix.
static s2r_status launch_selection(const TopkBatch& B, bool store_acc, hipStream_t st, const s2r::Exec& X) {
  const uint32_t W = B.nworkers;
  const uint64_t score_blocks =
      B.block >= 32u ? ceil_div(B.nb, (uint64_t)kWavesPerBlock * kScorePer) : ceil_div(B.nb, kBlock);
  const bool vec = B.block >= 32u && B.block % 4u == 0u;   // (gradients and residuals are 16-byte aligned)
  s2r::record_kernel_event(X, S2R_KERNEL_TOPK_SCORES, false, st);
  if (vec && store_acc)
    hipLaunchKernelGGL(topk_score_vec_kernel<true>, dim3((uint32_t)score_blocks, W), dim3(kBlock), 0, st, B);
  else if (vec)
    hipLaunchKernelGGL(topk_score_vec_kernel<false>, dim3((uint32_t)score_blocks, W), dim3(kBlock), 0, st, B);
  else if (store_acc)
    hipLaunchKernelGGL(topk_score_kernel<true>, dim3((uint32_t)score_blocks, W), dim3(kBlock), 0, st, B);
  else
    hipLaunchKernelGGL(topk_score_kernel<false>, dim3((uint32_t)score_blocks, W), dim3(kBlock), 0, st, B);
  s2r::record_kernel_event(X, S2R_KERNEL_TOPK_SCORES, true, st);
  if (!launch_ok()) return S2R_ERR_LAUNCH;
  if (B.K != B.nb && B.K != 0) {
    const uint32_t hist_blocks = (uint32_t)ceil_div(B.nb, (uint64_t)kHistBlock * kHistPer);
    for (uint32_t pass = 0; pass < (uint32_t)kPasses; ++pass) {
      hipLaunchKernelGGL(topk_hist_kernel, dim3(hist_blocks, W), dim3(kHistBlock), 0, st, B, pass);
      if (!launch_ok()) return S2R_ERR_LAUNCH;
    }
    hipLaunchKernelGGL(topk_pick_kernel, dim3(1, W), dim3(kHistBlock), 0, st, B);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }
  return S2R_OK;
}

static s2r_status launch_bitmaps(const TopkBatch& B, hipStream_t st) {
  const uint32_t all = B.K == B.nb ? 1u : 0u, none = B.K == 0 ? 1u : 0u;
  hipLaunchKernelGGL(topk_bitmap_kernel, dim3((uint32_t)ceil_div(ceil_div(B.nb, 64), kWavesPerBlock), B.nworkers),
                     dim3(kBlock), 0, st, B, all, none);
  return launch_ok() ? S2R_OK : S2R_ERR_LAUNCH;
}

}  // namespace s2r_topk

using namespace s2r_topk;

extern "C" {

size_t s2r_topk_workspace_bytes(uint64_t n, uint32_t block) {
  if (!sizes_ok(n, block)) return 0;
  return workspace_each(ceil_div(n, block));
}

s2r_status s2r_topk_blocks_batch(const float* const* grads, float* const* residuals, uint32_t W, uint64_t n,
                                 uint32_t block, uint64_t K, float* const* sparse_out, uint64_t* const* kept_bitmaps,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  if (sparse_out == nullptr) return S2R_ERR_NULL;
  TopkBatch B = {};
  s2r_status rc = fill_batch(B, grads, residuals, W, n, block, K, sparse_out, kept_bitmaps, workspace, workspace_bytes);
  if (rc != S2R_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  // with residuals the scores' pass leaves acc = g + e in them, and the second pass reads 4 bytes per element, not 8
  const bool acc_in_e = residuals != nullptr;
  if ((rc = launch_selection(B, acc_in_e, st, s2r::Exec())) != S2R_OK) return rc;
  const uint32_t all = B.K == B.nb ? 1u : 0u, none = B.K == 0 ? 1u : 0u;
  const dim3 agrid((uint32_t)ceil_div(n, (uint64_t)kBlock * kApplyPer), W);
  if (acc_in_e)
    hipLaunchKernelGGL(topk_apply_kernel<true>, agrid, dim3(kBlock), 0, st, B, all, none);
  else
    hipLaunchKernelGGL(topk_apply_kernel<false>, agrid, dim3(kBlock), 0, st, B, all, none);
  if (!launch_ok()) return S2R_ERR_LAUNCH;
  return kept_bitmaps != nullptr ? launch_bitmaps(B, st) : S2R_OK;
}

s2r_status s2r_topk_blocks(const float* grad, float* residual, uint64_t n, uint32_t block, uint64_t K,
                           float* sparse_out, uint64_t* kept_bitmap, void* workspace, size_t workspace_bytes,
                           void* stream) {
  return s2r_topk_blocks_batch(&grad, residual ? &residual : nullptr, 1, n, block, K, &sparse_out,
                               kept_bitmap ? &kept_bitmap : nullptr, workspace, workspace_bytes, stream);
}

size_t s2r_topk_encode_blocks_workspace_bytes(uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t blk_cap) {
  const size_t select = s2r_topk_workspace_bytes(n, block);
  const size_t codec = s2r_encode_blocks_workspace_bytes(n, block, d, w, blk_cap);
  return select == 0 || codec == 0 ? 0 : select + codec;          // both are multiples of 256
}

s2r_status s2r_topk_encode_blocks_batch_ex(const float* const* grads, float* const* residuals, uint32_t W, uint64_t n,
                                           uint32_t block, uint64_t K, uint32_t d, uint32_t w, uint64_t seed,
                                           float* const* sketches, uint64_t* const* block_bitmaps,
                                           uint32_t* const* blk_idx, uint64_t blk_cap, uint64_t* nblk_out,
                                           void* workspace, size_t workspace_bytes, void* stream,
                                           const s2r_options* options) {
  s2r::Exec X;
  const s2r_status orc = s2r::resolve_options(options, &X);
  if (orc != S2R_OK) return orc;
  if (block_bitmaps == nullptr || sketches == nullptr || nblk_out == nullptr) return S2R_ERR_NULL;
  if (W == 0 || W > S2R_MAX_WORKERS || !sizes_ok(n, block)) return S2R_ERR_SIZE;
  // everything the compress step would refuse is refused here, before the residuals are touched
  if (((uintptr_t)nblk_out & 7u) != 0) return S2R_ERR_ALIGN;
  for (uint32_t k = 0; k < W; ++k) {
    if (sketches[k] == nullptr || (blk_idx != nullptr && blk_idx[k] == nullptr)) return S2R_ERR_NULL;
    if (((uintptr_t)sketches[k] & 15u) || (blk_idx != nullptr && ((uintptr_t)blk_idx[k] & 3u))) return S2R_ERR_ALIGN;
  }
  if (blk_idx == nullptr) blk_cap = 0;
  if (blk_cap > ceil_div(n, block)) blk_cap = ceil_div(n, block);    // there cannot be more list entries than blocks
  const size_t select_each = s2r_topk_workspace_bytes(n, block);
  const size_t codec_each = s2r_encode_blocks_workspace_bytes(n, block, d, w, blk_cap);
  if (select_each == 0 || codec_each == 0) return S2R_ERR_SIZE;
  if (workspace == nullptr || ((uintptr_t)workspace & 255u) != 0 ||
      workspace_bytes / W < select_each + codec_each)
    return S2R_ERR_WORKSPACE;
  // the workspace: W selection shares, then W codec shares
  char* select_ws = reinterpret_cast<char*>(workspace);
  char* codec_ws = select_ws + (size_t)W * select_each;
  const size_t codec_bytes = workspace_bytes - (size_t)W * select_each;
  TopkBatch B = {};
  s2r_status rc = fill_batch(B, grads, residuals, W, n, block, K, nullptr, block_bitmaps, select_ws,
                             (size_t)W * select_each);
  if (rc != S2R_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  // acc = g + e replaces e during the scores' pass; the kept blocks are read from there and cleared at the end
  if ((rc = launch_selection(B, residuals != nullptr, st, X)) != S2R_OK) return rc;
  if ((rc = launch_bitmaps(B, st)) != S2R_OK) return rc;
  const float* values[S2R_MAX_WORKERS];
  for (uint32_t k = 0; k < W; ++k) values[k] = residuals != nullptr ? residuals[k] : grads[k];
  rc = s2r::encode_marked_blocks(values, W, n, block, d, w, seed, sketches, block_bitmaps, blk_idx, blk_cap, nblk_out,
                                 codec_ws, codec_bytes, stream, X);
  if (rc != S2R_OK) return rc;
  if (residuals != nullptr) {
    const uint32_t all = B.K == B.nb ? 1u : 0u, none = B.K == 0 ? 1u : 0u;
    const uint64_t blocks = ceil_div(ceil_div(B.nb, 64), kWavesPerBlock);
    hipLaunchKernelGGL(topk_clear_kept_kernel, dim3((uint32_t)blocks, W), dim3(kBlock), 0, st, B, all, none);
    if (!launch_ok()) return S2R_ERR_LAUNCH;
  }
  return S2R_OK;
}

s2r_status s2r_topk_encode_blocks_batch(const float* const* grads, float* const* residuals, uint32_t W, uint64_t n,
                                        uint32_t block, uint64_t K, uint32_t d, uint32_t w, uint64_t seed,
                                        float* const* sketches, uint64_t* const* block_bitmaps,
                                        uint32_t* const* blk_idx, uint64_t blk_cap, uint64_t* nblk_out,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  return s2r_topk_encode_blocks_batch_ex(grads, residuals, W, n, block, K, d, w, seed, sketches, block_bitmaps, blk_idx,
                                         blk_cap, nblk_out, workspace, workspace_bytes, stream, nullptr);
}

}  // extern "C"
