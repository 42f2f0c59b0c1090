/*
 * s2r.h -- C ABI of the MI355X (gfx950) sparse-sketch gradient codec.
 *
 * The library implements the data-parallel hot path of the Sparse-Sketch
 * Reducer (S2 Reducer, Algorithm 1 and Section 3.1):
 *
 *   s2r_encode   one worker's compress step: non-zero bitmap C, Sparse(g), and
 *                the count-sketch S of the non-zero values
 *   s2r_merge    the aggregation AllReduce(S, C), carried out on one GPU over W
 *                workers' buffers: S = sum_k S_k, C = OR_k C_k
 *   s2r_decode   the decompress step: indices from the aggregated bitmap and,
 *                at each, the median over rows of s_j(i) * S[j, h_j(i)]
 * and, around it, the paper's block-granular bitmap (s2r_encode_blocks,
 * s2r_decode_blocks) and its block-wise Top-K sparsifier with error feedback
 * (s2r_topk_blocks; s2r_topk_encode_blocks_batch fuses it with the compress step).
 *
 * Notation.  n = gradient length (the paper's d in Section 3.1), d = sketch rows
 * (the paper's r), w = sketch columns (the paper's c, m in Section 3.1), W =
 * number of workers.
 *
 * Conventions common to all calls
 *   - Every pointer named "dev" is a device pointer on the current HIP device;
 *     the caller owns all memory.  The library allocates nothing, keeps no
 *     pointer after the call returns and performs no host synchronisation: a
 *     call validates its arguments on the host, enqueues kernels on `stream`
 *     (a hipStream_t passed as void*; NULL is the default stream) and returns.
 *     Results, including counts, are written to device memory in stream order.
 *   - Return value: S2R_OK or a negative s2r_status.  Argument errors are
 *     reported before anything is enqueued.  A launch failure reported by the
 *     runtime gives S2R_ERR_LAUNCH.
 *   - Bitmap layout: ceil(n/64) 64-bit little-endian words; element i is bit
 *     (i mod 64), least significant first, of word floor(i/64); the unused high
 *     bits of the last word are written as 0.  (The paper does not fix a
 *     layout; Section 3.1 only says one flag per block.  A block is one
 *     element in s2r_encode / s2r_decode and `block` elements in the *_blocks
 *     calls.)
 *   - "Non-zero" is decided on the float32 bit pattern: everything except +0.0
 *     and -0.0, i.e. (bits & 0x7fffffff) != 0.
 *   - Sketch layout: d rows of w float32 cells, row-major, S[j*w + b].
 *   - Hash family (the paper names none; Section 3.1, Algorithm 1
 *     initialisation): row j has 64-bit parameters a_j, b_j, c_j, e_j, the
 *     outputs number 4j .. 4j+3 of a SplitMix64 generator whose state starts at
 *     `seed`, with a_j and c_j made odd.  Arithmetic mod 2^64:
 *         h_j(i) = (a_j * i + b_j) >> (64 - log2 w)        (0 when w == 1)
 *         s_j(i) = +1 if bit 63 of (c_j * i + e_j) is 0, else -1
 *   - Limits: 1 <= n <= 2^32 (indices are uint32), 1 <= d <= S2R_MAX_ROWS,
 *     w a power of two with 1 <= w <= 2^31 and d*w <= 2^32,
 *     1 <= W <= S2R_MAX_WORKERS.
 *   - Determinism: bitmaps, index lists and counts are bit-exact and identical
 *     from run to run.  A worker's sketch cell is a sum formed by hardware
 *     atomics in arbitrary order: float32 atomics in global memory (which may
 *     flush denormal operands and results to zero), or float64 atomics in LDS
 *     rounded to float32 once (see s2r_options.insert_strategy).  Cells, and the
 *     decoded values that read them, are therefore reproducible only up to
 *     the summation order.
 *   - Workspace: s2r_encode and s2r_decode need a device scratch buffer of at
 *     least s2r_workspace_bytes(n, d, w) bytes, 256-byte aligned (counts per
 *     2048 elements, their prefix sums per 32768 elements, and the list of
 *     the 32768-element tiles that hold more than 2048 non-zeros).  Its
 *     contents on entry are irrelevant and on exit unspecified.  Two calls
 *     that overlap in time (different streams) must not share a workspace.
 *   - No kernel of the library waits for another workgroup: every launch
 *     finishes whatever the order in which the hardware schedules workgroups.
 */
#ifndef S2R_H
#define S2R_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t s2r_status;

#define S2R_OK               0
#define S2R_ERR_NULL        -1   /* a required pointer is NULL                         */
#define S2R_ERR_SIZE        -2   /* n, d, w, W or cap outside the documented limits     */
#define S2R_ERR_WIDTH       -3   /* w is not a power of two                            */
#define S2R_ERR_WORKSPACE   -4   /* workspace NULL, misaligned or too small            */
#define S2R_ERR_LAUNCH      -5   /* the HIP runtime refused a kernel launch            */
#define S2R_ERR_ALIGN       -6   /* a buffer is not aligned as documented              */

#define S2R_MAX_ROWS        16
#define S2R_MAX_WORKERS     64

/* Library version as major*10000 + minor*100 + patch.  Host only. */
int32_t s2r_version(void);

/* Static, NUL-terminated description of a status code.  Host only. */
const char* s2r_status_string(s2r_status status);

/* Bytes of device scratch s2r_encode / s2r_decode need for these sizes (the
 * larger of the two).  Host only; returns 0 for sizes outside the limits. */
size_t s2r_workspace_bytes(uint64_t n, uint32_t d, uint32_t w);

/* Bytes of device scratch with which the LDS-slice strategy of s2r_encode can
 * take cap list entries per worker (s2r_workspace_bytes plus 8*d bytes per
 * entry for the sorted records, plus a table of their segments).  cap need not be the
 * capacity of the lists: with a workspace for fewer entries than a worker lists,
 * the strategy takes as many as fit and the call inserts the rest with atomics
 * (so a caller with long lists sizes the workspace for what it expects, with
 * some margin, and says so in s2r_options.expected_nnz); with no room for any
 * (but at least s2r_workspace_bytes) the call inserts with atomics only.
 * Host only; returns 0 outside the limits or if cap > n. */
size_t s2r_encode_workspace_bytes(uint64_t n, uint32_t d, uint32_t w, uint64_t cap);

/* The four hash parameters of each of the d rows, as the kernels use them:
 * params_out[4*j + 0..3] = a_j, b_j, c_j, e_j.  Host pointer, host only.
 * (Section 3.1 "hash function h", "random sign s"; the family is this
 * library's reading, stated at the top of this file.) */
s2r_status s2r_hash_params(uint64_t seed, uint32_t d, uint64_t* params_out /* host, 4*d */);

/*
 * Compress one worker's gradient (Algorithm 1: the bitmap line and the two
 * insertion loops; Section 3.1 "Compressing Sparse Gradient").
 *
 *   grad     dev, in : n float32, dense-stored, mostly zero; 4-byte aligned
 *   sketch   dev, out: d*w float32, OVERWRITTEN (zeroed, then
 *                      S[j, h_j(i)] += s_j(i) * g(i) for every non-zero i);
 *                      16-byte aligned
 *   bitmap   dev, out: ceil(n/64) uint64, OVERWRITTEN; 8-byte aligned
 *   nz_idx   dev, out: Sparse(g): the non-zero indices in ascending order,
 *   nz_val   dev, out: and the values at them; capacity `cap` entries each.
 *                      Both NULL (then cap is ignored) or both non-NULL.
 *                      Entries at positions >= cap are not written.
 *   nnz_out  dev, out: one uint64, the true number of non-zeros (also when it
 *                      exceeds cap: the caller compares).  Required.
 */
s2r_status s2r_encode(const float* grad, uint64_t n,
                      uint32_t d, uint32_t w, uint64_t seed,
                      float* sketch, uint64_t* bitmap,
                      uint32_t* nz_idx, float* nz_val, uint64_t cap,
                      uint64_t* nnz_out,
                      void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * s2r_encode for W workers in one call: the same kernels, each launched once over
 * all workers, which spares small gradients the per-worker launch overheads.
 * Worker k's outputs are exactly those of s2r_encode on grads[k].
 *
 *   grads, sketches, bitmaps   HOST arrays of W dev pointers (as in s2r_encode)
 *   nz_idx, nz_val             HOST arrays of W dev pointers, capacity cap each; both
 *                              arrays NULL (no lists for any worker), or all 2W
 *                              pointers non-NULL
 *   nnz_out                    dev, out: W uint64
 *   workspace                  dev scratch, 256-byte aligned, split evenly between
 *                              the workers: at least W * s2r_workspace_bytes(n,d,w),
 *                              or W * s2r_encode_workspace_bytes(n,d,w,cap) to
 *                              allow the LDS-slice strategy
 * The host arrays are read before the call returns.  1 <= W <= S2R_MAX_WORKERS.
 */
s2r_status s2r_encode_batch(const float* const* grads, uint32_t W, uint64_t n,
                            uint32_t d, uint32_t w, uint64_t seed,
                            float* const* sketches, uint64_t* const* bitmaps,
                            uint32_t* const* nz_idx, float* const* nz_val, uint64_t cap,
                            uint64_t* nnz_out,
                            void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * Aggregate W workers' sketches and bitmaps (Algorithm 1: AllReduce(S, C);
 * Section 3.1 "Collecting Sparse-Sketch with AllReduce": sketches add, and the
 * set bits of the aggregated bitmap mark the union of the non-zero blocks).
 * On one GPU the collective is an elementwise float32 sum taken in ascending
 * worker order and a bitwise OR.
 *
 *   sketches   HOST array of W dev pointers, each d*w float32, 16-byte aligned
 *   bitmaps    HOST array of W dev pointers, each ceil(n/64) uint64
 *   sketch_out dev, out: d*w float32; may be the same buffer as sketches[k]
 *   bitmap_out dev, out: ceil(n/64) uint64; may be the same as bitmaps[k]
 *   seed       accepted for uniformity of the three signatures; unused (the
 *              aggregation does not depend on the hashes)
 * The host arrays are read before the call returns.
 */
s2r_status s2r_merge(const float* const* sketches, const uint64_t* const* bitmaps,
                     uint32_t W, uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                     float* sketch_out, uint64_t* bitmap_out,
                     void* stream);

/*
 * Decompress (Algorithm 1: "Recover Sparse(g) from aggregated bitmap", the
 * estimates loop and the median; Section 3.1 "Decompressing Sparse Gradient").
 *
 *   sketch    dev, in : d*w float32 (aggregated)
 *   bitmap    dev, in : ceil(n/64) uint64 (aggregated); bits at positions >= n
 *                       in the last word must be 0
 *   idx_out   dev, out: ascending indices of the set bits, capacity cap
 *   val_out   dev, out: g^(i) = median_j s_j(i) * S[j, h_j(i)] at each of them
 *                       (middle order statistic for odd d; mean of the two
 *                       middle ones, in float32, for even d).  idx_out and
 *                       val_out are both NULL or both non-NULL.
 *   count_out dev, out: one uint64, the number of set bits.  Required.
 *   dense_out dev, out: NULL, or n float32 that are fully written: the
 *                       estimate at set bits, +0.0 elsewhere.  16-byte aligned.
 * The estimate is of the SUM over workers (Algorithm 1 does not divide by W).
 */
s2r_status s2r_decode(const float* sketch, const uint64_t* bitmap,
                      uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                      uint32_t* idx_out, float* val_out, uint64_t cap,
                      uint64_t* count_out,
                      float* dense_out,
                      void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * Aggregate and decompress in one call (Algorithm 1 from AllReduce(S, C) to the
 * median, on one GPU): exactly s2r_merge followed by s2r_decode of its outputs,
 * arguments as for those two.  The aggregation kernel counts the set bits of the
 * aggregated bitmap while it forms it, so the decompression starts without a
 * pass of its own over that bitmap: one kernel launch fewer.  sketch_out and
 * bitmap_out are written as by s2r_merge and are the sketch and bitmap the
 * decompression reads.  All arguments are checked before anything is enqueued.
 */
s2r_status s2r_merge_decode(const float* const* sketches, const uint64_t* const* bitmaps,
                            uint32_t W, uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                            float* sketch_out, uint64_t* bitmap_out,
                            uint32_t* idx_out, float* val_out, uint64_t cap,
                            uint64_t* count_out,
                            float* dense_out,
                            void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * s2r_decode for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and errors as s2r_decode, without the
 * workspace: the scratch (counts per 2048 bitmap bits, their prefix sums, the
 * dense-tile list; under 448 KiB) is a static array in device memory that every
 * GPU the library runs on holds until the process ends.  The call allocates
 * nothing and frees nothing.  The bucket reads are gathers (S2R_DECODE_GATHER).
 *   - n <= S2R_DECODE_NOALLOC_MAX_N, else S2R_ERR_SIZE (nothing is enqueued).
 *   - All calls on one GPU share the one array: calls that overlap in time on one
 *     GPU (different streams, or different host threads) race and must be
 *     serialised by the caller.  Nothing in it has to be cleared between calls:
 *     every call writes all the entries it later reads.
 *   - S2R_ERR_LAUNCH if the runtime cannot give the array's device address.
 */
#define S2R_DECODE_NOALLOC_MAX_N (1ull << 27)
s2r_status s2r_decode_noalloc(const float* sketch, const uint64_t* bitmap,
                              uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                              uint32_t* idx_out, float* val_out, uint64_t cap,
                              uint64_t* count_out,
                              float* dense_out,
                              void* stream);

/*
 * Block-granular codec: the bitmap as Section 3.1 sizes it, one bit per word
 * vector or gradient block that tells whether the block holds a non-zero
 * gradient (the bitmap line of Algorithm 1 is written per block).  Block x is
 * the elements x*block .. x*block + block - 1 (the last block may be shorter);
 * the bitmap has nb = ceil(n / block) bits in the layout described at the top of
 * this file.  The sketch is the one s2r_encode builds: only non-zero elements
 * are inserted (Section 3.1: zeros do not change a bucket), so it does not
 * depend on block, and block = 1 is the element codec.  Aggregation is s2r_merge with n = nb.
 * Decompression queries every element of every block whose aggregated bit is
 * set.  Limits: as above, and 1 <= block <= 2^31.
 *
 * s2r_blocks_workspace_bytes: the least scratch for s2r_encode_blocks* and
 * s2r_decode_blocks; the other two: what lets them also use S2R_INSERT_SLICE /
 * S2R_DECODE_SLICE (needs d * (blk_cap * block + 8192) < 2^32) / S2R_DECODE_ROWS for
 * lists of blk_cap blocks.
 * Host only; 0 outside the limits or if blk_cap > nb.
 */
size_t s2r_blocks_workspace_bytes(uint64_t n, uint32_t block, uint32_t d, uint32_t w);
size_t s2r_encode_blocks_workspace_bytes(uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t blk_cap);
size_t s2r_decode_blocks_workspace_bytes(uint64_t n, uint32_t block, uint32_t d, uint32_t w, uint64_t blk_cap);

/*
 * Compress with a block bitmap (Algorithm 1: the bitmap line as printed, and the
 * two insertion loops).  Arguments as s2r_encode / s2r_encode_batch except:
 *   block          elements per bitmap bit
 *   block_bitmap   dev, out: ceil(nb/64) uint64, OVERWRITTEN; 8-byte aligned
 *   blk_idx        dev, out: the non-zero blocks in ascending order, capacity
 *                  blk_cap entries; may be NULL (then blk_cap is ignored and the
 *                  insertions are atomics).  Entries at positions >= blk_cap are
 *                  not written.
 *   nblk_out       dev, out: uint64 (one per worker), the true number of non-zero
 *                  blocks.  Required.
 * The sketch is complete whatever blk_cap is.  The batch form takes host arrays of
 * W device pointers, blk_idx NULL or an array of W non-NULL pointers, and splits
 * the workspace evenly between the workers.
 */
s2r_status s2r_encode_blocks(const float* grad, uint64_t n, uint32_t block,
                             uint32_t d, uint32_t w, uint64_t seed,
                             float* sketch, uint64_t* block_bitmap,
                             uint32_t* blk_idx, uint64_t blk_cap,
                             uint64_t* nblk_out,
                             void* workspace, size_t workspace_bytes,
                             void* stream);

s2r_status s2r_encode_blocks_batch(const float* const* grads /* host array */, uint32_t W,
                                   uint64_t n, uint32_t block,
                                   uint32_t d, uint32_t w, uint64_t seed,
                                   float* const* sketches /* host array */,
                                   uint64_t* const* block_bitmaps /* host array */,
                                   uint32_t* const* blk_idx /* host array or NULL */, uint64_t blk_cap,
                                   uint64_t* nblk_out /* dev, W entries */,
                                   void* workspace, size_t workspace_bytes,
                                   void* stream);

/*
 * Decompress with a block bitmap (Algorithm 1: the recovery line and the query
 * loops over every element of the recovered blocks).
 *   sketch, block_bitmap   dev, in : the aggregated sketch and block bitmap
 *   blk_idx_out  dev, out: the set blocks in ascending order, blk_cap entries
 *   val_out      dev, out: blk_cap * block float32; entry p*block + o is the
 *                median-of-rows estimate of element blk_idx_out[p]*block + o, or
 *                +0.0 where that element is not below n.  Both NULL (count only)
 *                or both non-NULL; nothing is written for list positions
 *                >= blk_cap.
 *   nblk_out     dev, out: one uint64, the true number of set blocks.  Required.
 * Routes and their conditions as for s2r_decode (s2r_options.decode_strategy), with
 * cap = blk_cap * block; there is no dense output.
 */
s2r_status s2r_decode_blocks(const float* sketch, const uint64_t* block_bitmap,
                             uint64_t n, uint32_t block,
                             uint32_t d, uint32_t w, uint64_t seed,
                             uint32_t* blk_idx_out, float* val_out, uint64_t blk_cap,
                             uint64_t* nblk_out,
                             void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * s2r_merge followed by s2r_decode_blocks in one call, as s2r_merge_decode; the
 * W inputs and bitmap_out are block bitmaps of ceil(ceil(n / block) / 64) words.
 */
s2r_status s2r_merge_decode_blocks(const float* const* sketches, const uint64_t* const* block_bitmaps,
                                   uint32_t W, uint64_t n, uint32_t block,
                                   uint32_t d, uint32_t w, uint64_t seed,
                                   float* sketch_out, uint64_t* bitmap_out,
                                   uint32_t* blk_idx_out, float* val_out, uint64_t blk_cap,
                                   uint64_t* nblk_out,
                                   void* workspace, size_t workspace_bytes,
                                   void* stream);

/*
 * Block-wise Top-K sparsifier with error feedback, the step the paper puts in
 * front of the codec for dense layers (Section 2.2: the gradient is cut into
 * blocks, the l2 norm of every block is computed and the K largest blocks are
 * the ones communicated; Theorem 2 and its proof: the part that is not sent is
 * kept as an error sequence and added to the next gradient).
 *
 *   acc[i]   = grad[i] + residual[i]                    (float32; grad[i] alone without a residual)
 *   score[x] = sum of acc[i]^2 over block x, accumulated in float64 and rounded
 *              once to float32 (the same order as the l2 norm)
 *   kept     = the K blocks that come first when ordered by (score descending,
 *              block index ascending); all blocks if K >= ceil(n / block)
 *   sparse_out[i] = acc[i] in kept blocks, +0.0 elsewhere
 *   residual[i]   = +0.0 in kept blocks, acc[i] elsewhere         (updated in place)
 *
 *   grad         dev, in    : n float32; 16-byte aligned
 *   residual     dev, in/out: n float32, 16-byte aligned, or NULL (plain Top-K:
 *                             what is not kept is dropped)
 *   sparse_out   dev, out   : n float32, 16-byte aligned; may be grad itself
 *   kept_bitmap  dev, out   : ceil(ceil(n/block)/64) uint64 in the bitmap layout
 *                             of this file, bit x set iff block x is kept; or NULL
 *   workspace    dev scratch, 256-byte aligned, W * s2r_topk_workspace_bytes
 * A score is the float64 sum rounded once to float32; equal scores are ordered by
 * lower block index.  The float64 sum is formed in an order of the library's
 * choosing, so against another summation order a score can differ by one
 * float32 rounding where the sum lies at a rounding boundary: only a kept and
 * a dropped block whose scores are within one float32 rounding of each other
 * may swap; everything else is bit-exact.  Inputs are expected to be finite.  Limits: 1 <= n <= 2^32, 1 <= block <= 2^31 (blocks of
 * more than a few thousand elements are served by one wave each).  The batch
 * form takes host arrays of W device pointers (residuals and kept_bitmaps may be
 * NULL as a whole).  Enqueues on stream and returns; errors as for s2r_encode.
 */
size_t s2r_topk_workspace_bytes(uint64_t n, uint32_t block);

s2r_status s2r_topk_blocks(const float* grad, float* residual, uint64_t n,
                           uint32_t block, uint64_t K,
                           float* sparse_out, uint64_t* kept_bitmap,
                           void* workspace, size_t workspace_bytes,
                           void* stream);

s2r_status s2r_topk_blocks_batch(const float* const* grads /* host array */,
                                 float* const* residuals /* host array or NULL */, uint32_t W,
                                 uint64_t n, uint32_t block, uint64_t K,
                                 float* const* sparse_out /* host array */,
                                 uint64_t* const* kept_bitmaps /* host array or NULL */,
                                 void* workspace, size_t workspace_bytes,
                                 void* stream);

/*
 * The sparsifier and the compress step as one call, for W workers: what
 * s2r_topk_blocks_batch followed by s2r_encode_blocks_batch computes, without
 * the sparse gradient in between (Section 2.2 feeding the compress lines of
 * Algorithm 1; Section 3.1: the bitmap has one bit per gradient block).
 *
 *   acc, score, kept  as for s2r_topk_blocks
 *   block_bitmaps[k]  bit x set iff block x of worker k is kept -- the blocks the
 *                     sparsifier chose ARE the communicated blocks; a kept block
 *                     whose elements are all zero is still marked (it differs
 *                     from s2r_encode_blocks of the sparse gradient only there)
 *   blk_idx[k]        the kept blocks, ascending, at most blk_cap; nblk_out[k] =
 *                     min(K, ceil(n / block))
 *   sketches[k]       the count-sketch of the non-zero elements of acc in the kept
 *                     blocks, complete whatever blk_cap is
 *   residuals[k]      updated in place: +0.0 in kept blocks, acc elsewhere
 *
 * residuals may be NULL as a whole (plain Top-K: acc = grad, nothing is written
 * besides the outputs).  Otherwise residuals[k] must not overlap grads[k]; while
 * the call's kernels run it holds acc everywhere.  Every element is read once
 * (grad and residual) and the residual written once: 12 bytes per element
 * against 28 for the two calls.  Pointers, alignment, limits and the float64
 * summation order as for s2r_topk_blocks and s2r_encode_blocks_batch; workspace:
 * W * s2r_topk_encode_blocks_workspace_bytes(n, block, d, w, blk_cap), 256-byte
 * aligned.  Enqueues on stream and returns; errors as for s2r_encode.
 */
size_t s2r_topk_encode_blocks_workspace_bytes(uint64_t n, uint32_t block,
                                              uint32_t d, uint32_t w, uint64_t blk_cap);

s2r_status s2r_topk_encode_blocks_batch(const float* const* grads /* host array */,
                                        float* const* residuals /* host array or NULL */, uint32_t W,
                                        uint64_t n, uint32_t block, uint64_t K,
                                        uint32_t d, uint32_t w, uint64_t seed,
                                        float* const* sketches /* host array */,
                                        uint64_t* const* block_bitmaps /* host array */,
                                        uint32_t* const* blk_idx /* host array or NULL */, uint64_t blk_cap,
                                        uint64_t* nblk_out /* dev, W entries */,
                                        void* workspace, size_t workspace_bytes,
                                        void* stream);

/*
 * s2r_decode that applies the aggregated gradient instead of (or besides)
 * returning it: params[i] <- params[i] + scale * g_hat(i) (one fused
 * multiply-add) at every index i of the aggregated bitmap, also at those beyond
 * the lists' capacity; other entries of params are not touched.  Section 1: the
 * aggregated gradient is what updates the model; Algorithm 1 returns the sum
 * over workers, so scale carries the learning rate, its sign and the 1/W.
 *   params   dev, in/out: n float32, 4-byte aligned.  Required.
 *   idx_out, val_out, cap, count_out, workspace: as s2r_decode (the lists may be
 *   NULL).  The bucket reads are gathers (S2R_DECODE_GATHER).
 */
s2r_status s2r_decode_update(const float* sketch, const uint64_t* bitmap,
                             uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                             float* params, float scale,
                             uint32_t* idx_out, float* val_out, uint64_t cap,
                             uint64_t* count_out,
                             void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * The same with the block-granular bitmap: params[i] <- params[i] + scale *
 * g_hat(i) at every element i < n of every block whose bit is set in
 * block_bitmap (Section 3.1's bitmap over gradient blocks; Algorithm 1's
 * decompress lines), however many blocks that is; other entries of params are
 * not touched.  No values are returned; *nblk_out receives the number of set
 * blocks.  The complete list of set blocks is built in the workspace:
 * s2r_decode_blocks_update_workspace_bytes(n, block, d, w) bytes, 256-byte
 * aligned.  params: dev, n float32, 4-byte aligned.  Other arguments, limits
 * and errors as for s2r_decode_blocks.
 */
size_t s2r_decode_blocks_update_workspace_bytes(uint64_t n, uint32_t block, uint32_t d, uint32_t w);

s2r_status s2r_decode_blocks_update(const float* sketch, const uint64_t* block_bitmap,
                                    uint64_t n, uint32_t block,
                                    uint32_t d, uint32_t w, uint64_t seed,
                                    float* params, float scale,
                                    uint64_t* nblk_out,
                                    void* workspace, size_t workspace_bytes,
                                    void* stream);

/*
 * Size query of s2r_decode's routes that need scratch of their own (see
 * s2r_options.decode_strategy): bytes of device scratch with which s2r_decode can use
 * any of them for lists of capacity cap: s2r_workspace_bytes plus, for
 * S2R_DECODE_SLICE, 8*d bytes per list entry and a table of segments, or, for
 * S2R_DECODE_ROWS alone (where the slice route's limits are not met), 4*d bytes
 * per list entry.  With a smaller workspace (but at least s2r_workspace_bytes) the
 * call gathers.  Host only; returns 0 outside the limits or if cap > n.
 */
size_t s2r_decode_workspace_bytes(uint64_t n, uint32_t d, uint32_t w, uint64_t cap);

/* ------------------------------------------------------------------ per-call options
 *
 * Every entry point above that forms a sketch or reads one has a sibling with the
 * suffix _ex and one more argument, a pointer to s2r_options.  The library keeps
 * no state between calls: what steers a call travels with the call.  A NULL
 * pointer, or a struct that is all zero except struct_bytes, gives exactly the
 * plain entry point.
 *
 * insert_strategy: how the insertion loops of Algorithm 1 (S[j, h_j(i)] += s_j(i) g(i))
 * are carried out; the sketch is the same either way.
 *   S2R_INSERT_ATOMIC  float32 atomics on the sketch in device memory, issued
 *                      from the dense scan (the sketch is zeroed first)
 *   S2R_INSERT_SLICE   workgroups that each own a slice of one sketch row in
 *                      LDS (float64 accumulators, rounded to float32 once) and
 *                      add the entries of Sparse(g), which a counting sort has
 *                      partitioned by slice; needs nz_idx / nz_val, d*w <= 2^27
 *                      and a workspace with room for the sort of at least one
 *                      list entry (s2r_encode_workspace_bytes; otherwise the
 *                      call uses atomics whatever is asked for).  List entries
 *                      beyond what the workspace holds, and beyond (2^32-1)/d,
 *                      are inserted with atomics
 *   S2R_INSERT_AUTO    (0, default) chosen from W, n, d, w and the expected number
 *                      of non-zeros per worker; slices only if the workspace holds
 *                      the sort of that many entries
 *
 * decode_strategy: how the query loops of Algorithm 1 (the d bucket reads per union
 * index) are carried out; the result is the same either way, bit for bit.
 *   S2R_DECODE_GATHER  every list position reads its d buckets from the sketch in
 *                      device memory (one 128-byte line fetched per 4-byte cell)
 *   S2R_DECODE_SLICE   the (position, row) queries are partitioned by sketch
 *                      slice with a counting sort; workgroups that each hold a
 *                      slice of one sketch row in LDS answer them; the answers
 *                      return to list order through LDS and meet in the median.
 *                      Needs idx_out / val_out, no dense_out, d <= 8,
 *                      d*w <= 2^27, d*(cap + 8192) < 2^32 and a workspace of
 *                      s2r_decode_workspace_bytes (otherwise the call gathers
 *                      whatever is asked for)
 *   S2R_DECODE_ROWS    gathers again, but a workgroup reads one sketch row only, and
 *                      the rows are shared out between the chip's eight dies so that
 *                      a row of up to 4 MB stays in the cache of the dies that read
 *                      it; the estimates meet in the workspace and a second kernel
 *                      takes the medians.  Needs idx_out / val_out, no dense_out,
 *                      d <= 8 and a workspace of s2r_decode_workspace_bytes
 *                      (otherwise the call gathers as S2R_DECODE_GATHER does)
 *   S2R_DECODE_AUTO    (0, default) chosen from d, w and the expected number of
 *                      union indices
 *
 * expected_nnz: the caller's estimate of the number of non-zeros per worker (encode
 * calls; non-zero blocks for the block codec) or of set bits of the aggregated bitmap
 * (decode calls).  Only the AUTO choices and the way the work is cut into launches
 * read it; results never depend on it.  0 = no estimate: the capacity of the caller's
 * lists (cap) stands in for it, so a caller whose cap is a loose upper bound should
 * give an estimate.
 *
 * report: NULL, or a host struct the call fills in before it returns: the strategies it
 * used (S2R_INSERT_* / S2R_DECODE_*; AUTO when the call formed no sketch / read none) and
 * the number of workers the last dense-scan launch covered.
 *
 * trace: NULL, or measurement hooks declared in s2r_bench.h.
 *
 * Errors: S2R_ERR_SIZE if struct_bytes is not sizeof(s2r_options), a strategy is not one of
 * its values, or flags is not 0.
 */
#define S2R_INSERT_AUTO   0
#define S2R_INSERT_ATOMIC 1
#define S2R_INSERT_SLICE  2
#define S2R_DECODE_AUTO   0
#define S2R_DECODE_GATHER 1
#define S2R_DECODE_SLICE  2
#define S2R_DECODE_ROWS   3

typedef struct s2r_report {
  int32_t  insert_strategy;
  int32_t  decode_strategy;
  uint32_t scan_launch_workers;
  uint32_t reserved;
} s2r_report;

struct s2r_trace;

typedef struct s2r_options {
  uint32_t struct_bytes;            /* sizeof(s2r_options) */
  int32_t  insert_strategy;
  int32_t  decode_strategy;
  uint32_t flags;                   /* must be 0 */
  uint64_t expected_nnz;
  s2r_report* report;               /* host, out */
  const struct s2r_trace* trace;    /* host, in; see s2r_bench.h */
} s2r_options;

s2r_status s2r_encode_ex(const float* grad, uint64_t n,
                         uint32_t d, uint32_t w, uint64_t seed,
                         float* sketch, uint64_t* bitmap,
                         uint32_t* nz_idx, float* nz_val, uint64_t cap,
                         uint64_t* nnz_out,
                         void* workspace, size_t workspace_bytes,
                         void* stream, const s2r_options* options);

s2r_status s2r_encode_batch_ex(const float* const* grads, uint32_t W, uint64_t n,
                               uint32_t d, uint32_t w, uint64_t seed,
                               float* const* sketches, uint64_t* const* bitmaps,
                               uint32_t* const* nz_idx, float* const* nz_val, uint64_t cap,
                               uint64_t* nnz_out,
                               void* workspace, size_t workspace_bytes,
                               void* stream, const s2r_options* options);

s2r_status s2r_decode_ex(const float* sketch, const uint64_t* bitmap,
                         uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                         uint32_t* idx_out, float* val_out, uint64_t cap,
                         uint64_t* count_out,
                         float* dense_out,
                         void* workspace, size_t workspace_bytes,
                         void* stream, const s2r_options* options);

s2r_status s2r_encode_blocks_ex(const float* grad, uint64_t n, uint32_t block,
                                uint32_t d, uint32_t w, uint64_t seed,
                                float* sketch, uint64_t* block_bitmap,
                                uint32_t* blk_idx, uint64_t blk_cap,
                                uint64_t* nblk_out,
                                void* workspace, size_t workspace_bytes,
                                void* stream, const s2r_options* options);

s2r_status s2r_encode_blocks_batch_ex(const float* const* grads /* host array */, uint32_t W,
                                      uint64_t n, uint32_t block,
                                      uint32_t d, uint32_t w, uint64_t seed,
                                      float* const* sketches /* host array */,
                                      uint64_t* const* block_bitmaps /* host array */,
                                      uint32_t* const* blk_idx /* host array or NULL */, uint64_t blk_cap,
                                      uint64_t* nblk_out /* dev, W entries */,
                                      void* workspace, size_t workspace_bytes,
                                      void* stream, const s2r_options* options);

s2r_status s2r_decode_blocks_ex(const float* sketch, const uint64_t* block_bitmap,
                                uint64_t n, uint32_t block,
                                uint32_t d, uint32_t w, uint64_t seed,
                                uint32_t* blk_idx_out, float* val_out, uint64_t blk_cap,
                                uint64_t* nblk_out,
                                void* workspace, size_t workspace_bytes,
                                void* stream, const s2r_options* options);

s2r_status s2r_merge_decode_ex(const float* const* sketches /* host array */,
                               const uint64_t* const* bitmaps /* host array */,
                               uint32_t W, uint64_t n, uint32_t d, uint32_t w, uint64_t seed,
                               float* sketch_out, uint64_t* bitmap_out,
                               uint32_t* idx_out, float* val_out, uint64_t cap,
                               uint64_t* count_out,
                               float* dense_out,
                               void* workspace, size_t workspace_bytes,
                               void* stream, const s2r_options* options);

s2r_status s2r_merge_decode_blocks_ex(const float* const* sketches /* host array */,
                                      const uint64_t* const* block_bitmaps /* host array */,
                                      uint32_t W, uint64_t n, uint32_t block,
                                      uint32_t d, uint32_t w, uint64_t seed,
                                      float* sketch_out, uint64_t* bitmap_out,
                                      uint32_t* blk_idx_out, float* val_out, uint64_t blk_cap,
                                      uint64_t* nblk_out,
                                      void* workspace, size_t workspace_bytes,
                                      void* stream, const s2r_options* options);

s2r_status s2r_topk_encode_blocks_batch_ex(const float* const* grads /* host array */,
                                           float* const* residuals /* host array or NULL */, uint32_t W,
                                           uint64_t n, uint32_t block, uint64_t K,
                                           uint32_t d, uint32_t w, uint64_t seed,
                                           float* const* sketches /* host array */,
                                           uint64_t* const* block_bitmaps /* host array */,
                                           uint32_t* const* blk_idx /* host array or NULL */, uint64_t blk_cap,
                                           uint64_t* nblk_out /* dev, W entries */,
                                           void* workspace, size_t workspace_bytes,
                                           void* stream, const s2r_options* options);

#ifdef __cplusplus
}
#endif
#endif /* S2R_H */
