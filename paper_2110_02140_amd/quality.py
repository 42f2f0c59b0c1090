"""Estimation quality of the codec on synthetic gradients: the relative error of
the decoded sum, || g_hat - sum_k g_k || / || sum_k g_k ||, over the union
indices, as a function of the sketch size lambda and of the number of rows d.

This is the kernel-level counterpart of the paper's sensitivity study
(Section 3.1 defines lambda = m / (alpha * d'), buckets per non-zero; Section 4,
"Sensitivity", varies it on real training runs).  Here the inputs are the
seeded recipes of workloads.py, every step runs in the library's kernels, and
the host only forms the true sum and the two norms.  lambda is reported both
ways the paper's text can be read: per row (w / union) and for the whole
table (d * w / union).

    python -m paper_2110_02140_amd.quality [--n 4194304] [--workers 4] [--density 0.01]
"""

from __future__ import annotations

import argparse

import numpy as np


def true_sum(wl):
    """Union indices (ascending) and the float64 sum of the workers' values there."""
    idx = np.concatenate(wl.idx)
    val = np.concatenate(wl.val).astype(np.float64)
    union, inv = np.unique(idx, return_inverse=True)
    total = np.zeros(len(union))
    np.add.at(total, inv, val)
    return union.astype(np.uint32), total


def relative_error(wl) -> dict:
    """One encode + merge + decode on cuda:0; returns the error and the sizes."""
    import torch
    from . import pipeline
    b = pipeline.buffers_for(wl)
    b.step()
    torch.cuda.synchronize()
    cnt = int(b.out_count.cpu()[0])
    union, total = true_sum(wl)
    assert cnt == len(union) and np.array_equal(b.out_idx[:cnt].cpu().numpy().view(np.uint32), union)
    got = b.out_val[:cnt].cpu().numpy().astype(np.float64)
    err = float(np.linalg.norm(got - total) / np.linalg.norm(total))
    return {"d": wl.d, "w": wl.w, "union": cnt, "lambda_row": wl.w / cnt, "lambda_table": wl.d * wl.w / cnt,
            "rel_error": err, "exact_fraction": float(np.mean(got.astype(np.float32) == total.astype(np.float32)))}


def sweep(n: int, W: int, density: float, rows=(1, 3, 5), log2w=range(12, 21)) -> list[dict]:
    from . import workloads
    out = []
    for d in rows:
        for L in log2w:
            out.append(relative_error(workloads.cfg1(W=W, n=n, density=density, d=d, w=1 << L)))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=1 << 22)
    ap.add_argument("--workers", type=int, default=4)
    ap.add_argument("--density", type=float, default=0.01)
    args = ap.parse_args()
    print(f"# uniform recipe: W={args.workers} n={args.n} density={args.density} per worker, values N(0, 0.01)")
    print(f"{'d':>2s} {'w':>8s} {'union':>8s} {'lambda/row':>10s} {'lambda/table':>12s} {'rel. error':>10s} {'exact':>6s}")
    for r in sweep(args.n, args.workers, args.density):
        print(f"{r['d']:2d} {r['w']:8d} {r['union']:8d} {r['lambda_row']:10.3f} {r['lambda_table']:12.3f} "
              f"{r['rel_error']:10.4f} {r['exact_fraction']:6.3f}", flush=True)


if __name__ == "__main__":
    main()
