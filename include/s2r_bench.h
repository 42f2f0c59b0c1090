/*
 * s2r_bench.h -- measurement hooks of the sparse-sketch codec library.  No part
 * of the method (s2r.h holds that): what a benchmark needs to time single
 * kernels inside a call and to find the read rate the device delivers.
 */
#ifndef S2R_BENCH_H
#define S2R_BENCH_H

#include "s2r.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * s2r_options.trace.  While begin[slot] and end[slot] are both non-NULL
 * hipEvent_t, the call brackets the corresponding kernel launch with
 * hipEventRecord(begin[slot]) / hipEventRecord(end[slot]) on the call's
 * stream.  Host struct, read before the call returns; the events are the
 * caller's.  A slot with exactly one of the two events set gives S2R_ERR_NULL.
 *   S2R_KERNEL_ENCODE_SCAN : the dense scan kernel of the encode calls; when the
 *                            batch is scanned in several launches, the last one
 *                            (s2r_report.scan_launch_workers says how many workers
 *                            that launch covered)
 *   S2R_KERNEL_DECODE      : the kernels of the decode calls that follow the counts and
 *                            their prefix (expansion, queries, medians)
 *   S2R_KERNEL_ENCODE_SLICE: the LDS-slice sketch kernel of the encode calls
 *   S2R_KERNEL_TOPK_SCORES : the scores kernel (the pass over gradient and residual)
 *                            of s2r_topk_encode_blocks_batch_ex
 *   S2R_KERNEL_MERGE       : the aggregation kernel of the s2r_merge_decode calls
 */
#define S2R_KERNEL_ENCODE_SCAN  0
#define S2R_KERNEL_DECODE       1
#define S2R_KERNEL_ENCODE_SLICE 2
#define S2R_KERNEL_TOPK_SCORES  3
#define S2R_KERNEL_MERGE        4
#define S2R_KERNEL_SLOTS        5

struct s2r_trace {
  void* begin[S2R_KERNEL_SLOTS];
  void* end[S2R_KERNEL_SLOTS];
};

/*
 * One kernel that only reads the first bytes/16 16-byte words of src with
 * streaming loads, in the access pattern of the dense scan of s2r_encode.  Timed
 * by the caller, it gives the read rate the memory system delivers on this
 * device, the ceiling for the scan.
 *   src    dev, in : at least bytes bytes, 16-byte aligned; bytes >= 16
 *   sink   dev, out: one uint64, 8-byte aligned; written only if the XOR of all
 *                    words read equals an arbitrary constant (it keeps the loads
 *                    alive), so normally left untouched
 * Enqueues on stream and returns; S2R_ERR_NULL / _SIZE / _ALIGN / _LAUNCH as in s2r.h.
 */
s2r_status s2r_probe_read(const void* src, size_t bytes, uint64_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* S2R_BENCH_H */
