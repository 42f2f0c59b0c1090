"""Device buffers for one workload and the call sequence of the hot path:
W x s2r_encode -> s2r_merge -> s2r_decode (the last two as one s2r_merge_decode
call by default), all on one stream.

torch is used for device memory only (allocation, host<->device copies of test
data).  Every step of the path itself is a call into libs2r.so.
"""

from __future__ import annotations

import numpy as np
import torch

from . import binding


def words_of(n: int) -> int:
    return (n + 63) // 64


def upload_dense(idx: np.ndarray, val: np.ndarray, n: int, device) -> torch.Tensor:
    """Dense float32[n] on the device with val at idx, zero elsewhere (input
    staging, not part of the timed path)."""
    g = torch.zeros(n, dtype=torch.float32, device=device)
    if idx.shape[0]:
        ti = torch.from_numpy(idx.astype(np.int64)).to(device)
        tv = torch.from_numpy(np.ascontiguousarray(val, dtype=np.float32)).to(device)
        g.index_put_((ti,), tv)
    return g


class Buffers:
    """All device memory the path touches for a (W, n, d, w) problem."""

    def __init__(self, W: int, n: int, d: int, w: int, seed: int, nz_cap: int, union_cap: int,
                 device="cuda:0", dense_out: bool = False, sort_cap: int | None = None):
        """nz_cap / union_cap: capacity of the workers' lists and of the union list.  sort_cap: the
        number of list entries the encode workspace is sized for (default: nz_cap); entries beyond it
        are inserted with atomics."""
        self.W, self.n, self.d, self.w, self.seed = W, n, d, w, seed
        self.device = torch.device(device)
        dev = self.device
        nw = words_of(n)
        self.grads: list[torch.Tensor] = []
        self.sketch = [torch.empty(d * w, dtype=torch.float32, device=dev) for _ in range(W)]
        self.bitmap = [torch.empty(nw, dtype=torch.int64, device=dev) for _ in range(W)]
        self.nz_idx = [torch.empty(max(nz_cap, 1), dtype=torch.int32, device=dev) for _ in range(W)]
        self.nz_val = [torch.empty(max(nz_cap, 1), dtype=torch.float32, device=dev) for _ in range(W)]
        self.nnz = torch.zeros(W, dtype=torch.int64, device=dev)
        self.sketch_sum = torch.empty(d * w, dtype=torch.float32, device=dev)
        self.bitmap_or = torch.empty(nw, dtype=torch.int64, device=dev)
        self.out_idx = torch.empty(max(union_cap, 1), dtype=torch.int32, device=dev)
        self.out_val = torch.empty(max(union_cap, 1), dtype=torch.float32, device=dev)
        self.out_count = torch.zeros(1, dtype=torch.int64, device=dev)
        self.dense_out = torch.empty(n, dtype=torch.float32, device=dev) if dense_out else None
        ws = binding.encode_workspace_bytes(n, d, w, min(max(nz_cap if sort_cap is None else sort_cap, 1), n))
        ws_decode = binding.decode_workspace_bytes(n, d, w, min(max(union_cap, 1), n))
        if ws == 0 or ws_decode == 0:
            raise ValueError("sizes outside the library's limits")
        if sort_cap is None:
            # W shares for encode_batch; the same buffer serves s2r_decode afterwards
            self.workspace = torch.empty(max(ws * W, ws_decode), dtype=torch.uint8, device=dev)
            self.decode_workspace = self.workspace
        else:
            # exactly what was asked for, so that the encode's sort capacity is what the caller chose
            self.workspace = torch.empty(ws * W, dtype=torch.uint8, device=dev)
            self.decode_workspace = torch.empty(ws_decode, dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0 and self.decode_workspace.data_ptr() % 256 == 0

    # ------------------------------------------------------------ the path
    def encode(self, k: int, stream=None):
        binding.encode(self.grads[k], self.d, self.w, self.seed, self.sketch[k], self.bitmap[k],
                       self.nz_idx[k], self.nz_val[k], self.nnz[k:k + 1], self.workspace, stream, n=self.n)

    def encode_all(self, stream=None):
        """All W workers through one s2r_encode_batch call."""
        binding.encode_batch(self.grads, self.n, self.d, self.w, self.seed, self.sketch, self.bitmap,
                             self.nz_idx, self.nz_val, self.nnz, self.workspace, stream)

    def merge(self, stream=None):
        binding.merge(self.sketch, self.bitmap, self.n, self.d, self.w, self.seed,
                      self.sketch_sum, self.bitmap_or, stream)

    def decode(self, stream=None):
        binding.decode(self.sketch_sum, self.bitmap_or, self.n, self.d, self.w, self.seed,
                       self.out_idx, self.out_val, self.out_count, self.dense_out, self.decode_workspace, stream)

    def merge_decode(self, stream=None):
        """merge and decode as one s2r_merge_decode call."""
        binding.merge_decode(self.sketch, self.bitmap, self.n, self.d, self.w, self.seed, self.sketch_sum,
                             self.bitmap_or, self.out_idx, self.out_val, self.out_count, self.dense_out,
                             self.decode_workspace, stream)

    def step(self, stream=None, batched: bool = True, fused_merge_decode: bool = True):
        """One pass of the whole hot path over the resident gradients: the W
        encodes (one s2r_encode_batch call, or W s2r_encode calls), merge, decode."""
        if batched:
            self.encode_all(stream)
        else:
            for k in range(self.W):
                self.encode(k, stream)
        if fused_merge_decode:
            self.merge_decode(stream)
        else:
            self.merge(stream)
            self.decode(stream)


def buffers_for(wl, device="cuda:0", dense_out: bool = False, slack: int = 0, sort_cap: int | None = None) -> Buffers:
    """Buffers sized for a workloads.Workload, with its gradients uploaded."""
    nz_cap = max(len(i) for i in wl.idx) + slack
    union_cap = min(wl.n, sum(len(i) for i in wl.idx)) + slack
    b = Buffers(wl.W, wl.n, wl.d, wl.w, wl.seed, nz_cap, union_cap, device, dense_out, sort_cap)
    for k in range(wl.W):
        b.grads.append(upload_dense(wl.idx[k], wl.val[k], wl.n, b.device))
    return b


class BlockBuffers:
    """Device memory of the block-granular codec for a (W, n, block, d, w) problem."""

    def __init__(self, W: int, n: int, block: int, d: int, w: int, seed: int, blk_cap: int, union_cap: int,
                 device="cuda:0"):
        self.W, self.n, self.block, self.d, self.w, self.seed = W, n, block, d, w, seed
        self.device = torch.device(device)
        dev = self.device
        self.nb = (n + block - 1) // block
        nw = words_of(self.nb)
        blk_cap, union_cap = min(max(blk_cap, 1), self.nb), min(max(union_cap, 1), self.nb)
        self.grads: list[torch.Tensor] = []
        self.sketch = [torch.empty(d * w, dtype=torch.float32, device=dev) for _ in range(W)]
        self.bitmap = [torch.empty(nw, dtype=torch.int64, device=dev) for _ in range(W)]
        self.blk_idx = [torch.empty(blk_cap, dtype=torch.int32, device=dev) for _ in range(W)]
        self.nblk = torch.zeros(W, dtype=torch.int64, device=dev)
        self.sketch_sum = torch.empty(d * w, dtype=torch.float32, device=dev)
        self.bitmap_or = torch.empty(nw, dtype=torch.int64, device=dev)
        self.out_blk = torch.empty(union_cap, dtype=torch.int32, device=dev)
        self.out_val = torch.empty(union_cap * block, dtype=torch.float32, device=dev)
        self.out_count = torch.zeros(1, dtype=torch.int64, device=dev)
        ws = binding.encode_blocks_workspace_bytes(n, block, d, w, blk_cap)
        ws_decode = binding.decode_blocks_workspace_bytes(n, block, d, w, union_cap)
        if ws == 0 or ws_decode == 0:
            raise ValueError("sizes outside the library's limits")
        self.workspace = torch.empty(max(ws * W, ws_decode), dtype=torch.uint8, device=dev)

    def encode(self, k: int, stream=None):
        binding.encode_blocks(self.grads[k], self.block, self.d, self.w, self.seed, self.sketch[k], self.bitmap[k],
                              self.blk_idx[k], self.nblk[k:k + 1], self.workspace, stream, n=self.n)

    def encode_all(self, stream=None):
        binding.encode_blocks_batch(self.grads, self.n, self.block, self.d, self.w, self.seed, self.sketch,
                                    self.bitmap, self.blk_idx, self.nblk, self.workspace, stream)

    def topk_encode_all(self, dense, residuals, K: int, stream=None):
        """Sparsifier and compress step in one call (s2r_topk_encode_blocks_batch) from the
        dense gradients and the residuals; self.grads is not used."""
        need = binding.topk_encode_blocks_workspace_bytes(self.n, self.block, self.d, self.w,
                                                          self.blk_idx[0].numel()) * self.W
        if getattr(self, "fused_ws", None) is None or self.fused_ws.numel() < need:
            self.fused_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        binding.topk_encode_blocks_batch(dense, residuals, self.n, self.block, K, self.d, self.w, self.seed,
                                         self.sketch, self.bitmap, self.blk_idx, self.nblk, self.fused_ws, stream)

    def merge(self, stream=None):
        binding.merge(self.sketch, self.bitmap, self.nb, self.d, self.w, self.seed,
                      self.sketch_sum, self.bitmap_or, stream)

    def decode(self, stream=None):
        binding.decode_blocks(self.sketch_sum, self.bitmap_or, self.n, self.block, self.d, self.w, self.seed,
                              self.out_blk, self.out_val, self.out_count, self.workspace, stream)

    def merge_decode(self, stream=None):
        binding.merge_decode_blocks(self.sketch, self.bitmap, self.n, self.block, self.d, self.w, self.seed,
                                    self.sketch_sum, self.bitmap_or, self.out_blk, self.out_val, self.out_count,
                                    self.workspace, stream)

    def step(self, stream=None, batched: bool = True, fused_merge_decode: bool = True):
        if batched:
            self.encode_all(stream)
        else:
            for k in range(self.W):
                self.encode(k, stream)
        if fused_merge_decode:
            self.merge_decode(stream)
        else:
            self.merge(stream)
            self.decode(stream)


def block_buffers_for(wl, block: int, device="cuda:0", slack: int = 0) -> BlockBuffers:
    """BlockBuffers sized for a workloads.Workload cut into blocks of `block` elements."""
    per_worker = [len(np.unique(i // np.uint32(block))) for i in wl.idx]
    b = BlockBuffers(wl.W, wl.n, block, wl.d, wl.w, wl.seed, max(per_worker) + slack, sum(per_worker) + slack, device)
    for k in range(wl.W):
        b.grads.append(upload_dense(wl.idx[k], wl.val[k], wl.n, b.device))
    return b


def u64(t: torch.Tensor) -> np.ndarray:
    """Device int64 words -> host uint64 array."""
    return t.cpu().numpy().view(np.uint64)


class SparsifiedStep:
    """One data-parallel parameter update of W simulated workers, start to end in
    the library's kernels (Algorithm 1 with the block-wise Top-K sparsifier and
    the error-feedback residual of Section 2.2 / Appendix A.2 in front of it).

    fused (default), block-granular bitmaps:
        dense gradients g_k  ->  s2r_topk_encode_blocks_batch   acc_k = g_k + e_k, keep K blocks, e_k <- rest;
                                                                 bitmap C_k of the kept blocks, sketch S_k
                             ->  s2r_merge                      S = sum_k S_k, C = OR_k C_k  (stands in for AllReduce)
                             ->  s2r_decode_blocks_update       params[i] += scale * median_j(...) in every block of C
    not fused, element bitmaps:
        s2r_topk_blocks_batch (sparse gradients materialised) -> s2r_encode_batch -> s2r_merge -> s2r_decode_update

    The caller owns the gradients and the parameters (float32[n] device tensors);
    this object owns the residuals and every intermediate buffer.
    """

    def __init__(self, W: int, n: int, block: int, K: int, d: int, w: int, seed: int = 0, device="cuda:0",
                 fused: bool = True):
        nb = (n + block - 1) // block
        if not 0 < K <= nb:
            raise ValueError("K must be in 1..number of blocks")
        self.block, self.K, self.fused = block, K, fused
        if fused:
            self.codec = BlockBuffers(W, n, block, d, w, seed, K, 1, device)
            dev = self.codec.device
            self.update_ws = torch.empty(binding.decode_blocks_update_workspace_bytes(n, block, d, w), dtype=torch.uint8,
                                         device=dev)
        else:
            self.codec = Buffers(W, n, d, w, seed, min(n, K * block), 1, device)
            dev = self.codec.device
            self.codec.grads = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(W)]   # sparsified gradients
            self.topk_ws = torch.empty(binding.topk_workspace_bytes(n, block) * W, dtype=torch.uint8, device=dev)
        self.residual = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(W)]

    @property
    def sparse(self):
        """The sparsified gradients (only the not-fused path materialises them)."""
        return None if self.fused else self.codec.grads

    @property
    def count(self):
        """Device int64[1]: set blocks (fused) or union indices (not fused) of the last step."""
        return self.codec.out_count

    def step(self, grads, params, scale: float, stream=None):
        """params += scale * (estimate of the sum over workers of their sparsified
        gradients); scale is typically -learning_rate / W."""
        c = self.codec
        if self.fused:
            c.topk_encode_all(grads, self.residual, self.K, stream)
            c.merge(stream)
            binding.decode_blocks_update(c.sketch_sum, c.bitmap_or, c.n, c.block, c.d, c.w, c.seed, params, scale,
                                         c.out_count, self.update_ws, stream)
            return
        binding.topk_blocks_batch(grads, self.residual, c.n, self.block, self.K, c.grads, None, self.topk_ws, stream)
        c.encode_all(stream)
        c.merge(stream)
        binding.decode_update(c.sketch_sum, c.bitmap_or, c.n, c.d, c.w, c.seed, params, scale, None, None,
                              c.out_count, c.workspace, stream)
