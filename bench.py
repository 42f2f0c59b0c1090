#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: W x s2r_encode + s2r_merge +
s2r_decode over one batch of synthetic worker gradients resident in HBM.

Prints ONE JSON line.  `value` is dense-gradient GB/s = W*n*4 bytes per step /
time per step.  `roofline` is for the dominant kernel (the dense scan of
s2r_encode; with --fused-topk the sparsifier's pass over gradient and residual),
timed with HIP events on the launch stream.  `cpu_baseline` is the
CPU oracle timed on a bounded sample of the same workload.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the encode scan kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this file,
# scaled by what the same counters read for a plain 1 GiB copy (profiles/hbm_traffic_<workload>.txt):
# (workload, insert strategy, workers per launch) -> bytes.  Other combinations have not been counted.
MEASURED_SCAN_TRAFFIC = {("cfg5_large_zipf", "atomic", 1): 4.299e9, ("cfg5_large_zipf", "lds_slice", 1): 4.138e9}
# the same for the scores kernel of s2r_topk_encode_blocks_batch: (workload, block, kept fraction) -> bytes per launch
MEASURED_SCORES_TRAFFIC = {("cfg3_block_sparse", 256, 0.01): 2.464e9}


def algorithmic_bytes(wl, nnz, union: int) -> float:
    """What the method itself must move in one step: per worker the dense read
    (4n), the bitmap (n/8), the list (8 nnz) and the sketch written once (4dw);
    the merge reads W sketches and bitmaps and writes one of each; the decode
    reads the bitmap and the sketch and writes the union list (8 bytes each)."""
    cells, words8 = 4.0 * wl.d * wl.w, wl.n / 8.0
    encode = sum(4.0 * wl.n + words8 + 8.0 * float(c) + cells for c in nnz)
    merge = wl.W * (cells + words8) + cells + words8
    decode = words8 + cells + 8.0 * union
    return encode + merge + decode


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg1_lds"],
                    help="which BASELINE config to time (default: the largest single-GPU one); cfg1_lds is "
                         "config 1 with w = 2^13, the only size whose whole sketch fits one compute unit's LDS")
    ap.add_argument("--block", type=int, default=0,
                    help="use the block-granular codec with blocks of this many elements (0: one bitmap bit per "
                         "element); the natural sizes are 650 for cfg2 and 256 for cfg3")
    ap.add_argument("--topk-frac", type=float, default=0.0,
                    help="with --block: start every step from DENSE random gradients of the workload's W and n and "
                         "put the block-wise Top-K sparsifier with error feedback (this fraction of the blocks kept) "
                         "in front of the block codec")
    ap.add_argument("--fused-topk", action="store_true",
                    help="with --topk-frac: sparsifier and compress step through the one call "
                         "s2r_topk_encode_blocks_batch (no sparse gradient in between) instead of two")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph (torch.cuda.CUDAGraph) and time its replays: the same "
                         "kernels without the per-launch host work, which matters for the small configs")
    ap.add_argument("--per-worker-calls", action="store_true",
                    help="encode with W s2r_encode calls instead of one s2r_encode_batch call")
    ap.add_argument("--insert-strategy", default="auto", choices=["auto", "atomic", "slice"],
                    help="how s2r_encode forms the sketch (default: the library's own choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-elems", type=int, default=0, help="override the oracle sample length")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a kernel of known traffic, for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def algorithmic_bytes_blocks(wl, block: int, nnz, nblk, union_blocks: int) -> float:
    """The same count for the block-granular codec: bitmaps of n / block bits, lists
    of 4 bytes per non-zero block, decode writing block values per set block."""
    nb = (wl.n + block - 1) // block
    cells, words8 = 4.0 * wl.d * wl.w, nb / 8.0
    encode = sum(4.0 * wl.n + words8 + 4.0 * float(c) + cells for c in nblk)
    merge = wl.W * (cells + words8) + cells + words8
    decode = words8 + cells + (4.0 + 4.0 * block) * union_blocks
    return encode + merge + decode


def scan_kernel_bytes(n: int, nnz: float, d: int, inserts: bool) -> float:
    """Algorithmic bytes the encode scan kernel moves per worker: the dense read
    (4 B per element), the bitmap (1 bit per element), the compacted index+value
    list (8 B per non-zero) and the sketch insertions (d cells read and written,
    4 B each way, per non-zero) when this kernel makes them; without them (LDS
    slice strategy) the list and the sketch are written by other kernels.  One
    launch covers one or more workers."""
    return 4.0 * n + n / 8.0 + (8.0 * nnz + 8.0 * d * nnz if inserts else 0.0)


def cpu_baseline(wl, first_sample: int, budget_s: float = 12.0):
    """The oracle, as it stands, on the first ns elements of Ws workers: per worker
    the dense scan + insert (one dense buffer in host memory at a time; filling it
    is not timed), then merge and decode.  The sample grows (ns doubles up to the
    whole gradient, then Ws doubles up to W) until the runs so far have used
    `budget_s` seconds; the last, largest run is the one reported."""
    import numpy as np
    from oracle import s2r_oracle as orc
    Ws = min(wl.W, 4)
    ns = min(wl.n, first_sample)
    spent = 0.0
    while True:
        dt = 0.0
        sketches, bitmaps = [], []
        for k in range(Ws):
            cut = int(np.searchsorted(wl.idx[k], ns))
            g = np.zeros(ns, dtype=np.float32)
            g[wl.idx[k][:cut]] = wl.val[k][:cut]
            t0 = time.perf_counter()
            e = orc.encode(g, wl.d, wl.w, wl.seed)
            dt += time.perf_counter() - t0
            sketches.append(e["S"])
            bitmaps.append(e["bitmap"])
            del g, e
        t0 = time.perf_counter()
        S, C = orc.merge(sketches, bitmaps)
        out = orc.decode(S, C, ns, wl.seed)
        dt += time.perf_counter() - t0
        spent += dt
        union = len(out["idx"])
        del sketches, bitmaps, S, C, out
        grow_w = ns >= wl.n and Ws < wl.W
        if spent >= budget_s or spent + 2 * dt > 30.0 or (ns >= wl.n and not grow_w):     # the next run takes about 2 dt
            break
        if grow_w:
            Ws = min(wl.W, Ws * 2)
        else:
            ns = min(wl.n, ns * 2)
    gbs = Ws * ns * 4 / dt / 1e9
    return {"value": round(gbs, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{Ws} workers x first {ns} elements of {wl.name} (dense scan+insert per worker, merge, decode; "
                      f"{union} union indices), {dt:.1f} s on 1 thread"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (W workers are simulated in one GPU's HBM); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2110_02140_amd import binding, pipeline, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the codec has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    binding.load()
    binding.set_insert_strategy({"auto": binding.S2R_INSERT_AUTO, "atomic": binding.S2R_INSERT_ATOMIC,
                                 "slice": binding.S2R_INSERT_SLICE}[args.insert_strategy])

    cfg = int(args.workload[3])
    t_gen = time.perf_counter()
    wl = workloads.make_cfg1_lds() if args.workload == "cfg1_lds" else workloads.make(cfg)
    t_gen = time.perf_counter() - t_gen
    topk = args.topk_frac > 0
    if topk and args.block <= 0:
        print("bench.py: --topk-frac needs --block", file=sys.stderr)
        sys.exit(2)
    batched = not args.per_worker_calls
    stream = torch.cuda.current_stream()
    if topk:
        # dense N(0, 0.01) gradients, one per worker, resident; the sparsifier writes the sparse gradients the
        # block codec then reads, and keeps its residuals from step to step
        nb = (wl.n + args.block - 1) // args.block
        K = max(1, int(round(args.topk_frac * nb)))
        b = pipeline.BlockBuffers(wl.W, wl.n, args.block, wl.d, wl.w, wl.seed, K, wl.W * K)
        gen = torch.Generator(device=b.device).manual_seed(1000 * cfg + 998)
        dense = [torch.empty(wl.n, dtype=torch.float32, device=b.device).normal_(0, 0.01, generator=gen)
                 for _ in range(wl.W)]
        resid = [torch.zeros(wl.n, dtype=torch.float32, device=b.device) for _ in range(wl.W)]
        b.grads = [torch.empty(wl.n, dtype=torch.float32, device=b.device) for _ in range(wl.W)]
        ws_topk = torch.empty(binding.topk_workspace_bytes(wl.n, args.block) * wl.W, dtype=torch.uint8, device=b.device)
        tk_pairs = []

        if args.fused_topk:
            def step():
                b.topk_encode_all(dense, resid, K, stream)
                b.merge(stream)
                b.decode(stream)
        else:
            def step():
                binding.topk_blocks_batch(dense, resid, wl.n, args.block, K, b.grads, None, ws_topk, stream)
                b.step(stream, batched)
    else:
        b = pipeline.block_buffers_for(wl, args.block) if args.block > 0 else pipeline.buffers_for(wl)

        def step():
            b.step(stream, batched)
    torch.cuda.synchronize()

    for _ in range(max(args.warmup, 1) if args.graph else args.warmup):
        step()
    torch.cuda.synchronize()
    timed_step = step
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        eager_stream = stream
        with torch.cuda.graph(graph):
            stream = torch.cuda.current_stream()            # the capture stream
            step()
        stream = eager_stream
        timed_step = graph.replay
        for _ in range(2):
            timed_step()
        torch.cuda.synchronize()
    ev0, ev1 = binding.HipEvent(), binding.HipEvent()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        timed_step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_ms(ev1)
    ms_per_step = wall * 1e3 / args.steps
    value = wl.dense_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel timing, same call sequence, HIP events recorded by the library around its own launches
    reps = max(1, min(args.steps, 10))
    slots = {"scan": binding.S2R_KERNEL_ENCODE_SCAN, "merge": binding.S2R_KERNEL_MERGE,
             "decode": binding.S2R_KERNEL_DECODE}
    timed = {k: [] for k in slots}

    slice_pairs = []

    def bracket(name, call):
        e0, e1 = binding.HipEvent(), binding.HipEvent()
        binding.set_kernel_events(slots[name], e0.handle, e1.handle)
        if name == "scan":          # the LDS-slice kernel, when the encode uses it, is bracketed in the same call
            s0, s1 = binding.HipEvent(), binding.HipEvent()
            binding.set_kernel_events(binding.S2R_KERNEL_ENCODE_SLICE, s0.handle, s1.handle)
        call()
        binding.set_kernel_events(slots[name], None, None)
        timed[name].append((e0, e1))
        if name == "scan":
            binding.set_kernel_events(binding.S2R_KERNEL_ENCODE_SLICE, None, None)
            slice_pairs.append((s0, s1))

    for r in range(reps):
        if topk and args.fused_topk:        # one call; its dominant kernel is the scores' pass over g and e
            t_a, t_b, c0, c1, s0, s1 = (binding.HipEvent() for _ in range(6))
            binding.set_kernel_events(binding.S2R_KERNEL_TOPK_SCORES, c0.handle, c1.handle)
            binding.set_kernel_events(binding.S2R_KERNEL_ENCODE_SLICE, s0.handle, s1.handle)
            t_a.record(stream)
            b.topk_encode_all(dense, resid, K, stream)
            t_b.record(stream)
            binding.set_kernel_events(binding.S2R_KERNEL_TOPK_SCORES, None, None)
            binding.set_kernel_events(binding.S2R_KERNEL_ENCODE_SLICE, None, None)
            tk_pairs.append((t_a, t_b))
            timed["scan"].append((c0, c1))
            slice_pairs.append((s0, s1))
            bracket("merge", lambda: b.merge(stream))
            bracket("decode", lambda: b.decode(stream))
            continue
        if topk:
            t_a, t_b = binding.HipEvent(), binding.HipEvent()
            t_a.record(stream)
            binding.topk_blocks_batch(dense, resid, wl.n, args.block, K, b.grads, None, ws_topk, stream)
            t_b.record(stream)
            tk_pairs.append((t_a, t_b))
        if batched:
            bracket("scan", lambda: b.encode_all(stream))
        else:
            for k in range(wl.W):
                bracket("scan", lambda k=k: b.encode(k, stream))
        bracket("merge", lambda: b.merge(stream))
        bracket("decode", lambda: b.decode(stream))
    torch.cuda.synchronize()
    scan_ms, merge_ms, decode_ms = (float(np.mean([a.elapsed_ms(c) for a, c in timed[k]]))
                                    for k in ("scan", "merge", "decode"))
    fused = topk and args.fused_topk
    workers_per_launch = wl.W if fused else binding.scan_launch_workers()
    atomic = binding.last_insert_strategy() == binding.S2R_INSERT_ATOMIC
    slice_ms = None if atomic else float(np.mean([a.elapsed_ms(c) for a, c in slice_pairs]))

    # ---- the read rate this device delivers to a kernel that only reads (same access pattern as the scan)
    sink = torch.zeros(1, dtype=torch.int64, device=b.device)
    p0, p1 = binding.HipEvent(), binding.HipEvent()
    probe_reps = min(4, wl.W)
    for k in range(probe_reps):
        binding.probe_read(b.grads[k], sink, stream)
    p0.record(stream)
    for k in range(probe_reps):
        binding.probe_read(b.grads[k], sink, stream)
    p1.record(stream)
    torch.cuda.synchronize()
    read_ceiling = probe_reps * wl.n * 4 / (p0.elapsed_ms(p1) * 1e-3) / 1e9

    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 18, dtype=torch.float32, device=b.device)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    union = int(b.out_count.cpu()[0])
    nnz = np.array([len(i) for i in wl.idx], dtype=np.float64)
    topk_ms = float(np.mean([a.elapsed_ms(c) for a, c in tk_pairs])) if topk else None
    if args.block > 0:
        nblk = b.nblk.cpu().numpy()
        if topk:
            assert all(int(x) == K for x in nblk), "every worker must send exactly K blocks"
            nnz = np.full(wl.W, float(K * args.block))
        else:
            assert [int(x) for x in nblk] == [len(np.unique(i // np.uint32(args.block))) for i in wl.idx], \
                "encode's block counts differ from the generator's"
        per_worker = 4.0 * wl.n + ((wl.n + args.block - 1) // args.block) / 8.0 + (8.0 * wl.d * nnz.mean() if atomic else 0.0)
        alg_bytes = workers_per_launch * per_worker
        step_alg_bytes = algorithmic_bytes_blocks(wl, args.block, nnz, nblk, union)
        if fused:       # g and e read once, e written once; no sparse gradient for a codec scan to read
            alg_bytes = wl.W * 12.0 * wl.n
            step_alg_bytes += wl.W * (12.0 - 4.0) * wl.n
        elif topk:      # g and e read and e <- g + e written by the scores' pass; e read and the sparse gradient written by the second
            step_alg_bytes += wl.W * 20.0 * wl.n
    else:
        assert [int(x) for x in b.nnz.cpu().numpy()] == [len(i) for i in wl.idx], "encode counts differ from the generator's"
        alg_bytes = workers_per_launch * scan_kernel_bytes(wl.n, float(nnz.mean()), wl.d, atomic)
        step_alg_bytes = algorithmic_bytes(wl, nnz, union)
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9

    out = {
        "metric": "dense-gradient GB/s for encode+merge+decode on 1 MI355X; % of HBM peak",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "W": wl.W, "n": wl.n, "d": wl.d, "w": wl.w, "seed": wl.seed,
                   "block": args.block, "topk_blocks_kept": K if topk else None,
                   "input": "dense N(0, 0.01) gradients + residuals" if topk else "dense-stored sparse gradients",
                   "nnz_per_worker": int(nnz.mean()),
                   "union_blocks" if args.block > 0 else "union_nnz": union,
                   "dense_bytes_per_step": wl.dense_bytes},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "algorithmic_bytes_per_step": int(step_alg_bytes),
        "algorithmic_frac_of_hbm_peak": round(step_alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "stream_read_GBs": round(read_ceiling, 1),
        "event_ms_per_step": round(ev_ms / args.steps, 4),
        "launch": "hip graph replay" if args.graph else "eager",
        "encode_calls": "s2r_topk_encode_blocks_batch" if fused else
                        ("s2r_encode_blocks_batch" if batched else "s2r_encode_blocks x W") if args.block > 0
                        else ("s2r_encode_batch" if batched else "s2r_encode x W"),
        "decode_route": "slice" if binding.last_decode_strategy() == binding.S2R_DECODE_SLICE else "gather",
        "insert_strategy": "atomic" if atomic else "lds_slice",
        "kernel_ms": {"topk_scores_per_launch" if fused else "encode_scan_per_launch": round(scan_ms, 4),
                      "workers_per_scan_launch": workers_per_launch,
                      "encode_slice_per_launch": None if slice_ms is None else round(slice_ms, 4),
                      "merge": round(merge_ms, 4), "decode": round(decode_ms, 4),
                      "topk_and_compress_call" if fused else "topk_sparsifier":
                          None if topk_ms is None else round(topk_ms, 4)},
        "roofline": {"kernel": "topk_score_kernel" if fused else "encode_scan_kernel", "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_SCORES_TRAFFIC.get((wl.name, args.block, args.topk_frac)) if fused else
                                None if args.block > 0 else
                                MEASURED_SCAN_TRAFFIC.get((wl.name, "atomic" if atomic else "lds_slice", workers_per_launch)),
                     "algorithmic_bytes_per_launch": int(alg_bytes)},
        "setup_s": {"generate": round(t_gen, 1)},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample_elems or 16_000_000)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
