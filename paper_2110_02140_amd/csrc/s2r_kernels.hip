// gfx950 kernels and C ABI of the sparse-sketch gradient codec
// (S2 Reducer, Algorithm 1 and Section 3.1).  See include/s2r.h for the
// contract of every entry point.
//
// Kernels
//   prep_kernel          zero the sketch, the tile status words and the counters
//   encode_scan_kernel   one pass over the dense gradient: bitmap words from
//                        wave ballots, ascending Sparse(g) through a chained
//                        tile prefix, and the sketch insertions
//                        S[j, h_j(i)] += s_j(i) g(i) as float32 atomics
//   merge_kernel         S = sum_k S_k (ascending k), C = OR_k C_k
//   decode_kernel        one pass over the aggregated bitmap: ascending index
//                        list through the same chained prefix, per index the
//                        d signed bucket reads and their median
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/s2r.h"
#include "s2r_device.h"

namespace s2r {

constexpr int kBlock = 256;                 // threads per workgroup (4 waves)
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kEncodeEPL = 8;               // elements per lane in the dense scan
constexpr int kEncodeTile = kBlock * kEncodeEPL;
constexpr int kDecodeWordsPerThread = 2;
constexpr int kDecodeTileWords = kBlock * kDecodeWordsPerThread;
constexpr size_t kHeaderBytes = 256;

struct WorkHeader {
  uint32_t tile_counter;
  uint32_t pad[63];
};
static_assert(sizeof(WorkHeader) == kHeaderBytes, "header is one 256-byte block");

// ------------------------------------------------------------------ prep
// Zeroes `nvec` 16-byte units at `sketch16` (may be 0), `nstatus` status words,
// the header, and the 8-byte count output.
__global__ __launch_bounds__(kBlock) void prep_kernel(uint4* __restrict__ sketch16, uint64_t nvec,
                                                      float* __restrict__ sketch_tail, uint32_t ntail,
                                                      uint64_t* __restrict__ status, uint64_t nstatus,
                                                      WorkHeader* __restrict__ hdr,
                                                      uint64_t* __restrict__ count_out) {
  const uint64_t tid = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = tid; i < nvec; i += stride) sketch16[i] = make_uint4(0u, 0u, 0u, 0u);
  for (uint64_t i = tid; i < nstatus; i += stride) status[i] = 0ull;
  if (tid < ntail) sketch_tail[tid] = 0.0f;
  if (tid < 64) reinterpret_cast<uint32_t*>(hdr)[tid] = 0u;
  if (tid == 0) *count_out = 0ull;
}

// ------------------------------------------------------------------ encode
struct EncodeArgs {
  const uint32_t* grad;      // dense gradient as bit patterns
  uint64_t n;
  uint64_t nwords;
  uint32_t d;
  uint32_t log2w;
  float* sketch;
  uint64_t* bitmap;
  uint32_t* nz_idx;          // may be null
  float* nz_val;             // may be null
  uint64_t cap;
  uint64_t* nnz_out;
  WorkHeader* hdr;
  uint64_t* status;
  uint32_t ntiles;
};

template <int EPL>
__global__ __launch_bounds__(kBlock) void encode_scan_kernel(const EncodeArgs A, const HashRows hp) {
  constexpr int TILE = kBlock * EPL;
  __shared__ uint32_t s_tile;
  __shared__ uint32_t s_wave_count[kWavesPerBlock];
  __shared__ uint64_t s_base;

  if (threadIdx.x == 0) s_tile = atomicAdd(&A.hdr->tile_counter, 1u);
  __syncthreads();
  const uint32_t tile = s_tile;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  // first element of the 64*EPL-element chunk this wave scans
  const uint64_t chunk0 = (uint64_t)tile * TILE + (uint64_t)wv * (kWave * EPL);

  // Lane l reads element chunk0 + 64k + l for k = 0..EPL-1: each load is one
  // fully coalesced 256-byte row, and the ballot of load k is bitmap word k.
  uint32_t v[EPL];
  if (chunk0 + (uint64_t)kWave * EPL <= A.n) {
#pragma unroll
    for (int k = 0; k < EPL; ++k) v[k] = __builtin_nontemporal_load(&A.grad[chunk0 + k * kWave + lane]);
  } else {
#pragma unroll
    for (int k = 0; k < EPL; ++k) {
      const uint64_t i = chunk0 + k * kWave + lane;
      v[k] = i < A.n ? A.grad[i] : 0u;
    }
  }

  uint64_t myword = 0;                 // lane k (< EPL) keeps word k of this wave's chunk
#pragma unroll
  for (int k = 0; k < EPL; ++k) {
    const uint64_t b = __ballot((v[k] << 1) != 0u);     // non-zero: anything but +-0.0
    if (lane == (uint32_t)k) myword = b;
  }
  const uint64_t word0 = chunk0 >> 6;
  if (lane < (uint32_t)EPL && word0 + lane < A.nwords) A.bitmap[word0 + lane] = myword;

  // non-zeros in the words before word k of this wave, and in the whole wave
  const uint32_t cnt = (uint32_t)__popcll(myword);
  uint32_t incl = cnt;
#pragma unroll
  for (int off = 1; off < EPL; off <<= 1) {
    const uint32_t t = __shfl_up(incl, off, kWave);
    if (lane >= (uint32_t)off) incl += t;
  }
  const uint32_t word_excl = incl - cnt;
  const uint32_t wave_total = __shfl(incl, EPL - 1, kWave);
  if (lane == 0) s_wave_count[wv] = wave_total;
  __syncthreads();

  uint32_t tile_total = 0, wave_off = 0;
#pragma unroll
  for (int q = 0; q < kWavesPerBlock; ++q) {
    const uint32_t c = s_wave_count[q];
    if ((uint32_t)q < wv) wave_off += c;
    tile_total += c;
  }

  if (wv == 0) {
    bool timed_out = false;
    const uint64_t excl = chained_exclusive_prefix(A.status, tile, tile_total, &timed_out);
    if (lane == 0) {
      s_base = excl;
      if (tile == A.ntiles - 1) atomicMax((unsigned long long*)A.nnz_out, (unsigned long long)(excl + tile_total));
      if (timed_out) atomicMax((unsigned long long*)A.nnz_out, (unsigned long long)S2R_COUNT_POISON);
    }
  }
  __syncthreads();
  if (tile_total == 0) return;         // uniform over the workgroup

  const uint64_t base = s_base + wave_off;
  const uint32_t d = A.d;
#pragma unroll
  for (int k = 0; k < EPL; ++k) {
    // (readlane returns a signed int: go through uint32_t so that bit 31 does not sign-extend)
    const uint64_t wk = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)(myword >> 32), k) << 32) |
                        (uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)myword, k);
    if (wk == 0) continue;             // uniform over the wave
    const uint32_t pk = (uint32_t)__builtin_amdgcn_readlane(word_excl, k);
    if ((v[k] << 1) != 0u) {
      const uint64_t pos = base + pk + bits_below_lane(wk);
      const uint32_t i = (uint32_t)(chunk0 + k * kWave + lane);
      if (A.nz_idx != nullptr && pos < A.cap) {
        A.nz_idx[pos] = i;
        A.nz_val[pos] = __uint_as_float(v[k]);
      }
      for (uint32_t j = 0; j < d; ++j) {
        const uint32_t h = bucket_of(i, hp.a[j], hp.b[j], A.log2w);
        const uint32_t sv = v[k] ^ signbit_of(i, hp.c[j], hp.e[j]);
        __hip_atomic_fetch_add(&A.sketch[((uint64_t)j << A.log2w) + h], __uint_as_float(sv),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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

__global__ __launch_bounds__(kBlock) void merge_kernel(const MergeArgs A) {
  if (blockIdx.x < A.sketch_blocks) {
    const uint64_t stride = (uint64_t)A.sketch_blocks * kBlock;
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < A.ncell4; i += stride) {
      float4 acc = reinterpret_cast<const float4*>(A.sketch[0])[i];
      for (uint32_t k = 1; k < A.W; ++k) {
        const float4 x = reinterpret_cast<const float4*>(A.sketch[k])[i];
        acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
      }
      reinterpret_cast<float4*>(A.sketch_out)[i] = acc;
    }
    // cells beyond the last full group of four (only when d*w is not a multiple of 4)
    const uint64_t t = A.ncell4 * 4 + (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (t < A.ncells) {
      float acc = A.sketch[0][t];
      for (uint32_t k = 1; k < A.W; ++k) acc += A.sketch[k][t];
      A.sketch_out[t] = acc;
    }
  } else {
    const uint64_t nb = gridDim.x - A.sketch_blocks;
    const uint64_t stride = nb * kBlock;
    for (uint64_t i = (uint64_t)(blockIdx.x - A.sketch_blocks) * kBlock + threadIdx.x; i < A.nwords; i += stride) {
      uint64_t acc = A.bitmap[0][i];
      for (uint32_t k = 1; k < A.W; ++k) acc |= A.bitmap[k][i];
      A.bitmap_out[i] = acc;
    }
  }
}

// ------------------------------------------------------------------ decode
struct DecodeArgs {
  const float* sketch;
  const uint64_t* bitmap;
  uint64_t n;
  uint64_t nwords;
  uint32_t d;
  uint32_t log2w;
  uint32_t* idx_out;         // may be null
  float* val_out;            // may be null
  uint64_t cap;
  uint64_t* count_out;
  float* dense_out;          // may be null
  WorkHeader* hdr;
  uint64_t* status;
  uint32_t ntiles;
};

template <int D>
__device__ __forceinline__ float median_fixed(float (&x)[D]) {
  // selection by a fully unrolled exchange network; every output is one of the inputs
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
  if (D & 1) return x[D / 2];
  return 0.5f * (x[D / 2 - 1] + x[D / 2]);
}

template <int D>
__device__ __forceinline__ float query_fixed(const DecodeArgs& A, const HashRows& hp, uint32_t i) {
  float est[D];
#pragma unroll
  for (int j = 0; j < D; ++j) {
    const uint32_t h = bucket_of(i, hp.a[j], hp.b[j], A.log2w);
    const uint32_t raw = __float_as_uint(A.sketch[((uint64_t)j << A.log2w) + h]);
    est[j] = __uint_as_float(raw ^ signbit_of(i, hp.c[j], hp.e[j]));
  }
  return median_fixed<D>(est);
}

// any d up to kMaxRows: estimates kept in a local array, insertion sort
__device__ __noinline__ float query_any(const DecodeArgs& A, const HashRows& hp, uint32_t i) {
  float est[kMaxRows];
  const uint32_t d = A.d;
  for (uint32_t j = 0; j < d; ++j) {
    const uint32_t h = bucket_of(i, hp.a[j], hp.b[j], A.log2w);
    const uint32_t raw = __float_as_uint(A.sketch[((uint64_t)j << A.log2w) + h]);
    const float x = __uint_as_float(raw ^ signbit_of(i, hp.c[j], hp.e[j]));
    uint32_t p = j;
    while (p > 0 && est[p - 1] > x) { est[p] = est[p - 1]; --p; }
    est[p] = x;
  }
  if (d & 1u) return est[d / 2];
  return 0.5f * (est[d / 2 - 1] + est[d / 2]);
}

template <int D>   // D == 0: runtime d
__global__ __launch_bounds__(kBlock) void decode_kernel(const DecodeArgs A, const HashRows hp) {
  __shared__ uint32_t s_tile;
  __shared__ uint64_t s_words[kDecodeTileWords];
  __shared__ uint32_t s_prefix[kDecodeTileWords + 1];   // exclusive prefix of popcounts, [last] = total
  __shared__ uint32_t s_wave_count[kWavesPerBlock];
  __shared__ uint64_t s_base;

  if (threadIdx.x == 0) s_tile = atomicAdd(&A.hdr->tile_counter, 1u);
  __syncthreads();
  const uint32_t tile = s_tile;
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const uint32_t wv = threadIdx.x / kWave;
  const uint64_t word0 = (uint64_t)tile * kDecodeTileWords;

  // thread t owns words 2t and 2t+1 of the tile
  uint64_t wd[kDecodeWordsPerThread];
  uint32_t pc[kDecodeWordsPerThread];
  uint32_t cnt = 0;
#pragma unroll
  for (int q = 0; q < kDecodeWordsPerThread; ++q) {
    const uint64_t wi = word0 + (uint64_t)threadIdx.x * kDecodeWordsPerThread + q;
    wd[q] = wi < A.nwords ? A.bitmap[wi] : 0ull;
    pc[q] = (uint32_t)__popcll(wd[q]);
    cnt += pc[q];
  }
  uint32_t incl = cnt;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint32_t t = __shfl_up(incl, off, kWave);
    if (lane >= (uint32_t)off) incl += t;
  }
  if (lane == kWave - 1) s_wave_count[wv] = incl;
  __syncthreads();
  uint32_t tile_total = 0, wave_off = 0;
#pragma unroll
  for (int q = 0; q < kWavesPerBlock; ++q) {
    const uint32_t c = s_wave_count[q];
    if ((uint32_t)q < wv) wave_off += c;
    tile_total += c;
  }
  {
    uint32_t run = wave_off + incl - cnt;
#pragma unroll
    for (int q = 0; q < kDecodeWordsPerThread; ++q) {
      s_words[threadIdx.x * kDecodeWordsPerThread + q] = wd[q];
      s_prefix[threadIdx.x * kDecodeWordsPerThread + q] = run;
      run += pc[q];
    }
    if (threadIdx.x == kBlock - 1) s_prefix[kDecodeTileWords] = run;
  }

  if (wv == 0) {
    bool timed_out = false;
    const uint64_t excl = chained_exclusive_prefix(A.status, tile, tile_total, &timed_out);
    if (lane == 0) {
      s_base = excl;
      if (tile == A.ntiles - 1) atomicMax((unsigned long long*)A.count_out, (unsigned long long)(excl + tile_total));
      if (timed_out) atomicMax((unsigned long long*)A.count_out, (unsigned long long)S2R_COUNT_POISON);
    }
  }

  // dense output: this workgroup owns elements [64*word0, 64*(word0 + tile words)):
  // clear them first, the estimates are written over the zeros after the barrier
  if (A.dense_out != nullptr) {
    const uint64_t e0 = word0 * 64;
    const uint64_t e1 = min(A.n, e0 + (uint64_t)kDecodeTileWords * 64);
    if (e1 > e0) {
      float4* p4 = reinterpret_cast<float4*>(A.dense_out + e0);   // e0 is a multiple of 64 elements
      const uint64_t n4 = (e1 - e0) / 4;
      for (uint64_t q = threadIdx.x; q < n4; q += kBlock) p4[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      const uint64_t r = e0 + n4 * 4 + threadIdx.x;
      if (r < e1) A.dense_out[r] = 0.0f;
    }
  }
  __syncthreads();
  if (tile_total == 0) return;

  const uint64_t base = s_base;
  for (uint32_t t = threadIdx.x; t < tile_total; t += kBlock) {
    // the word holding the t-th set bit of the tile: last w with prefix[w] <= t
    uint32_t lo = 0, hi = kDecodeTileWords;     // invariant: prefix[lo] <= t < prefix[hi]
#pragma unroll
    for (int step = 0; step < 9; ++step) {      // 2^9 = 512 words per tile
      const uint32_t mid = (lo + hi) >> 1;
      if (s_prefix[mid] <= t) lo = mid; else hi = mid;
    }
    const uint32_t bit = select_bit(s_words[lo], t - s_prefix[lo]);
    const uint32_t i = (uint32_t)((word0 + lo) * 64 + bit);
    float g;
    if (D == 0) g = query_any(A, hp, i);
    else g = query_fixed<(D == 0 ? 1 : D)>(A, hp, i);
    const uint64_t pos = base + t;
    if (A.idx_out != nullptr && pos < A.cap) {
      A.idx_out[pos] = i;
      A.val_out[pos] = g;
    }
    if (A.dense_out != nullptr) A.dense_out[i] = g;
  }
}
static_assert(kDecodeTileWords == 512, "the word search in decode_kernel takes log2(tile words) = 9 steps");

// ------------------------------------------------------------------ host side
struct EventPair { hipEvent_t begin, end; };
static thread_local EventPair g_events[S2R_KERNEL_SLOTS] = {};

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
static inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

static s2r_status check_sizes(uint64_t n, uint32_t d, uint32_t w) {
  if (n == 0 || n > (1ull << 32)) return S2R_ERR_SIZE;
  if (d == 0 || d > S2R_MAX_ROWS) return S2R_ERR_SIZE;
  if (w == 0) return S2R_ERR_SIZE;
  if (!is_pow2(w)) return S2R_ERR_WIDTH;
  if (w > (1u << 31)) return S2R_ERR_SIZE;
  if ((uint64_t)d * w > (1ull << 32)) return S2R_ERR_SIZE;
  return S2R_OK;
}

static inline uint32_t encode_tiles(uint64_t n) { return (uint32_t)ceil_div(n, kEncodeTile); }
static inline uint32_t decode_tiles(uint64_t n) { return (uint32_t)ceil_div(ceil_div(n, 64), kDecodeTileWords); }

static inline void record(int slot, bool end, hipStream_t st) {
  hipEvent_t ev = end ? g_events[slot].end : g_events[slot].begin;
  if (ev != nullptr) (void)hipEventRecord(ev, st);
}

static inline s2r_status launch_status() {
  return hipGetLastError() == hipSuccess ? S2R_OK : S2R_ERR_LAUNCH;
}

}  // namespace s2r

using namespace s2r;

extern "C" {

int32_t s2r_version(void) { return 100; }

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
  const uint64_t tiles = encode_tiles(n) > decode_tiles(n) ? encode_tiles(n) : decode_tiles(n);
  const uint64_t bytes = kHeaderBytes + tiles * sizeof(uint64_t);
  return (size_t)((bytes + 255) & ~(uint64_t)255);
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

s2r_status s2r_set_kernel_events(int32_t slot, void* ev_begin, void* ev_end) {
  if (slot < 0 || slot >= S2R_KERNEL_SLOTS) return S2R_ERR_SIZE;
  if ((ev_begin == nullptr) != (ev_end == nullptr)) return S2R_ERR_NULL;
  g_events[slot].begin = (hipEvent_t)ev_begin;
  g_events[slot].end = (hipEvent_t)ev_end;
  return S2R_OK;
}

s2r_status s2r_encode(const float* grad, uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                      float* sketch, uint64_t* bitmap, uint32_t* nz_idx, float* nz_val, uint64_t cap,
                      uint64_t* nnz_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (grad == nullptr || sketch == nullptr || bitmap == nullptr || nnz_out == nullptr) return S2R_ERR_NULL;
  if ((nz_idx == nullptr) != (nz_val == nullptr)) return S2R_ERR_NULL;
  const s2r_status sz = check_sizes(n, d, w);
  if (sz != S2R_OK) return sz;
  if (workspace == nullptr || ((uintptr_t)workspace & 255u) != 0 ||
      workspace_bytes < s2r_workspace_bytes(n, d, w)) return S2R_ERR_WORKSPACE;
  if (((uintptr_t)grad & 3u) || ((uintptr_t)sketch & 15u) || ((uintptr_t)bitmap & 7u) ||
      ((uintptr_t)nz_idx & 3u) || ((uintptr_t)nz_val & 3u) || ((uintptr_t)nnz_out & 7u)) return S2R_ERR_ALIGN;

  hipStream_t st = (hipStream_t)stream;
  HashRows hp;
  make_hash_rows(seed, d, &hp);

  EncodeArgs A;
  A.grad = reinterpret_cast<const uint32_t*>(grad);
  A.n = n;
  A.nwords = ceil_div(n, 64);
  A.d = d;
  A.log2w = log2_of(w);
  A.sketch = sketch;
  A.bitmap = bitmap;
  A.nz_idx = nz_idx;
  A.nz_val = nz_val;
  A.cap = nz_idx ? cap : 0;
  A.nnz_out = nnz_out;
  A.hdr = reinterpret_cast<WorkHeader*>(workspace);
  A.status = reinterpret_cast<uint64_t*>((char*)workspace + kHeaderBytes);
  A.ntiles = encode_tiles(n);

  const uint64_t cells = (uint64_t)d * w;
  const uint64_t nvec = cells / 4;
  const uint32_t ntail = (uint32_t)(cells - nvec * 4);
  uint64_t work = nvec > A.ntiles ? nvec : A.ntiles;
  uint32_t pblocks = (uint32_t)(ceil_div(work, kBlock) < 2048 ? ceil_div(work, kBlock) : 2048);
  if (pblocks == 0) pblocks = 1;
  hipLaunchKernelGGL(prep_kernel, dim3(pblocks), dim3(kBlock), 0, st, reinterpret_cast<uint4*>(sketch), nvec,
                     sketch + nvec * 4, ntail, A.status, (uint64_t)A.ntiles, A.hdr, nnz_out);
  if (launch_status() != S2R_OK) return S2R_ERR_LAUNCH;

  record(S2R_KERNEL_ENCODE_SCAN, false, st);
  hipLaunchKernelGGL(encode_scan_kernel<kEncodeEPL>, dim3(A.ntiles), dim3(kBlock), 0, st, A, hp);
  record(S2R_KERNEL_ENCODE_SCAN, true, st);
  return launch_status();
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
  // one thread per 16 bytes of sketch / 8 bytes of bitmap, capped so that the grid stays a few waves deep
  uint64_t sb = ceil_div(A.ncell4 > 0 ? A.ncell4 : 1, kBlock);
  uint64_t bb = ceil_div(A.nwords, kBlock);
  if (sb > 4096) sb = 4096;
  if (bb > 4096) bb = 4096;
  A.sketch_blocks = (uint32_t)sb;
  hipStream_t st = (hipStream_t)stream;
  record(S2R_KERNEL_MERGE, false, st);
  hipLaunchKernelGGL(merge_kernel, dim3((uint32_t)(sb + bb)), dim3(kBlock), 0, st, A);
  record(S2R_KERNEL_MERGE, true, st);
  return launch_status();
}

s2r_status s2r_decode(const float* sketch, const uint64_t* bitmap, uint64_t n, uint32_t d, uint32_t w,
                      uint64_t seed, uint32_t* idx_out, float* val_out, uint64_t cap, uint64_t* count_out,
                      float* dense_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (sketch == nullptr || bitmap == nullptr || count_out == nullptr) return S2R_ERR_NULL;
  if ((idx_out == nullptr) != (val_out == nullptr)) return S2R_ERR_NULL;
  const s2r_status sz = check_sizes(n, d, w);
  if (sz != S2R_OK) return sz;
  if (workspace == nullptr || ((uintptr_t)workspace & 255u) != 0 ||
      workspace_bytes < s2r_workspace_bytes(n, d, w)) return S2R_ERR_WORKSPACE;
  if (((uintptr_t)sketch & 15u) || ((uintptr_t)bitmap & 7u) || ((uintptr_t)idx_out & 3u) ||
      ((uintptr_t)val_out & 3u) || ((uintptr_t)count_out & 7u) || ((uintptr_t)dense_out & 15u)) return S2R_ERR_ALIGN;

  hipStream_t st = (hipStream_t)stream;
  HashRows hp;
  make_hash_rows(seed, d, &hp);

  DecodeArgs A;
  A.sketch = sketch;
  A.bitmap = bitmap;
  A.n = n;
  A.nwords = ceil_div(n, 64);
  A.d = d;
  A.log2w = log2_of(w);
  A.idx_out = idx_out;
  A.val_out = val_out;
  A.cap = idx_out ? cap : 0;
  A.count_out = count_out;
  A.dense_out = dense_out;
  A.hdr = reinterpret_cast<WorkHeader*>(workspace);
  A.status = reinterpret_cast<uint64_t*>((char*)workspace + kHeaderBytes);
  A.ntiles = decode_tiles(n);

  uint32_t pblocks = (uint32_t)(ceil_div(A.ntiles, kBlock) < 2048 ? ceil_div(A.ntiles, kBlock) : 2048);
  hipLaunchKernelGGL(prep_kernel, dim3(pblocks), dim3(kBlock), 0, st, (uint4*)nullptr, (uint64_t)0, (float*)nullptr,
                     0u, A.status, (uint64_t)A.ntiles, A.hdr, count_out);
  if (launch_status() != S2R_OK) return S2R_ERR_LAUNCH;

  record(S2R_KERNEL_DECODE, false, st);
  const dim3 grid(A.ntiles), block(kBlock);
  switch (d) {
    case 1: hipLaunchKernelGGL(decode_kernel<1>, grid, block, 0, st, A, hp); break;
    case 2: hipLaunchKernelGGL(decode_kernel<2>, grid, block, 0, st, A, hp); break;
    case 3: hipLaunchKernelGGL(decode_kernel<3>, grid, block, 0, st, A, hp); break;
    case 4: hipLaunchKernelGGL(decode_kernel<4>, grid, block, 0, st, A, hp); break;
    case 5: hipLaunchKernelGGL(decode_kernel<5>, grid, block, 0, st, A, hp); break;
    case 6: hipLaunchKernelGGL(decode_kernel<6>, grid, block, 0, st, A, hp); break;
    case 7: hipLaunchKernelGGL(decode_kernel<7>, grid, block, 0, st, A, hp); break;
    default: hipLaunchKernelGGL(decode_kernel<0>, grid, block, 0, st, A, hp); break;
  }
  record(S2R_KERNEL_DECODE, true, st);
  return launch_status();
}

}  // extern "C"
