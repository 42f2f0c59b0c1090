// Calls between the library's translation units; not part of the C ABI.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "../../include/s2r.h"
#include "../../include/s2r_bench.h"

namespace s2r {

// A call's s2r_options, checked and resolved (a NULL options pointer gives the defaults).
struct Exec {
  int32_t insert_strategy = S2R_INSERT_AUTO;
  int32_t decode_strategy = S2R_DECODE_AUTO;
  uint64_t expected_nnz = 0;
  s2r_report* report = nullptr;
  const s2r_trace* trace = nullptr;
};

// Fills X from options (may be NULL) and zeroes the report, if any.  S2R_ERR_SIZE /
// S2R_ERR_NULL as the header says.
__attribute__((visibility("hidden")))
s2r_status resolve_options(const s2r_options* options, Exec* X);

// The block-granular compress step (Algorithm 1) of W workers whose block bitmaps
// are already filled in on the device: bit x of block_bitmaps[k] set for every block
// that is communicated, bits at and beyond ceil(n / block) clear.  Lists the set
// blocks in blk_idx (ascending, at most cap; may be NULL), counts them in nblk_out
// and forms the sketches from the non-zero elements of values[k] inside the set
// blocks; values[k] is not read anywhere else.  Arguments, workspace size
// (s2r_encode_blocks_workspace_bytes per worker) and errors as for
// s2r_encode_blocks_batch.
__attribute__((visibility("hidden")))
s2r_status encode_marked_blocks(const float* const* values, uint32_t W, uint64_t n, uint32_t block, uint32_t d,
                                uint32_t w, uint64_t seed, float* const* sketches, uint64_t* const* block_bitmaps,
                                uint32_t* const* blk_idx, uint64_t cap, uint64_t* nblk_out, void* workspace,
                                size_t workspace_bytes, void* stream, const Exec& X);

// Records the begin (end = false) or end event of a trace slot on the stream, if the
// call's options carry one.
__attribute__((visibility("hidden")))
void record_kernel_event(const Exec& X, int slot, bool end, void* stream);

}  // namespace s2r
