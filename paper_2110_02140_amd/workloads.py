"""Seeded synthetic sparse gradients shaped like the paper's workloads.

The paper trains on embedding-layer gradients (only the rows of the words in a
mini-batch are non-zero; Section 2.2 and Table 1) and on block-wise Top-K
sparsified gradients (Section 2.2; Section 4 uses 1/32 of the blocks).  Its
datasets and models are not needed to exercise the codec: what matters to the
encode / merge / decode path is the length of the gradient, how many elements
are non-zero, how they cluster, and how far the workers' index sets overlap.
The five recipes below reproduce those properties with seeded random numbers.

This module holds no part of the method's arithmetic (no hashing, no sketch, no
bitmap): it only produces, per worker, an ascending array of distinct non-zero
indices (uint32) and their float32 values.  Both the CPU oracle's tests and the
GPU tests / benchmark draw their inputs from here.

Random numbers: numpy PCG64; worker k of recipe c uses seed 1000*c + k, anything
shared between workers uses 1000*c + 999.  "N(0, 0.01)" is read as standard
deviation 0.01.  A drawn value that rounds to +-0 in float32 is replaced by the
smallest normal float32 with the sign of the draw, so every listed index is
non-zero.
"""

from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Workload:
    name: str
    cfg: int
    W: int            # number of simulated workers
    n: int            # gradient length (float32 elements)
    d: int            # sketch rows
    w: int            # sketch columns (power of two)
    seed: int         # hash seed
    idx: list = field(default_factory=list)   # per worker: uint32[nnz_k], ascending, distinct
    val: list = field(default_factory=list)   # per worker: float32[nnz_k]
    note: str = ""

    @property
    def dense_bytes(self) -> int:
        return self.W * self.n * 4

    def dense(self, k: int) -> np.ndarray:
        """Worker k's gradient as a dense float32[n] host array (small n only)."""
        g = np.zeros(self.n, dtype=np.float32)
        g[self.idx[k]] = self.val[k]
        return g


def _rng(cfg: int, k: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(1000 * cfg + k))


def _fix_zeros(v64: np.ndarray) -> np.ndarray:
    v = v64.astype(np.float32)
    z = v == 0
    if z.any():
        tiny = np.float32(np.finfo(np.float32).tiny)
        v[z] = np.where(np.signbit(v64[z]), -tiny, tiny)
    return v


def _normal(rng, size, sigma=0.01):
    return _fix_zeros(rng.normal(0.0, sigma, size=size))


def _laplace(rng, size, b=0.005):
    return _fix_zeros(rng.laplace(0.0, b, size=size))


def _zipf_p(V: int, s: float) -> np.ndarray:
    p = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    return p / p.sum()


def _rows_to_elems(rows: np.ndarray, H: int, offset: int = 0) -> np.ndarray:
    rows = np.sort(rows.astype(np.int64))
    e = (rows[:, None] * H + np.arange(H, dtype=np.int64)[None, :]).reshape(-1) + offset
    return e.astype(np.uint32)


# ---------------------------------------------------------------- recipe 1
def cfg1(W: int = 4, n: int = 1 << 20, density: float = 0.01, d: int = 3, w: int = 1 << 14) -> Workload:
    """Uniform element-sparse gradient; independent index sets per worker."""
    wl = Workload("cfg1_uniform_1pct", 1, W, n, d, w, 0)
    K = int(round(density * n))
    for k in range(W):
        r = _rng(1, k)
        idx = np.sort(r.choice(n, size=K, replace=False)).astype(np.uint32)
        wl.idx.append(idx)
        wl.val.append(_normal(r, K))
    return wl


# ---------------------------------------------------------------- recipe 2
def cfg2(W: int = 8, V: int = 33278, H: int = 650, row_frac: float = 0.05, d: int = 3,
         w: int = 1 << 18, s: float = 1.1) -> Workload:
    """Embedding-layer gradient [V x H]: whole rows non-zero, rows drawn without
    replacement from a Zipf(s) token-frequency law shared by all workers (rank r
    is row r-1), so frequent rows recur across workers.  Shaped like the paper's
    LSTM / GNMT embedding gradients (Table 1)."""
    wl = Workload("cfg2_embedding_rows", 2, W, V * H, d, w, 0)
    p = _zipf_p(V, s)
    K = int(round(row_frac * V))
    for k in range(W):
        r = _rng(2, k)
        rows = r.choice(V, size=K, replace=False, p=p)
        wl.idx.append(_rows_to_elems(rows, H))
        wl.val.append(_normal(r, K * H))
    return wl


# ---------------------------------------------------------------- recipe 3
def cfg3(W: int = 8, nblocks: int = 100_000, B: int = 256, block_frac: float = 0.01, d: int = 3,
         w: int = 1 << 20) -> Workload:
    """Block-wise Top-K-shaped gradient: aligned blocks of B elements, a fraction
    block_frac kept; half the kept block ids are common to all workers, half are
    drawn per worker from the remaining ids.  Laplace(0, 0.005) values."""
    wl = Workload("cfg3_block_sparse", 3, W, nblocks * B, d, w, 0)
    K = int(round(block_frac * nblocks))
    Ks = K // 2
    shared = _rng(3, 999).choice(nblocks, size=Ks, replace=False)
    rest = np.setdiff1d(np.arange(nblocks), shared)
    for k in range(W):
        r = _rng(3, k)
        own = r.choice(rest, size=K - Ks, replace=False)
        blocks = np.concatenate([shared, own])
        wl.idx.append(_rows_to_elems(blocks, B))
        wl.val.append(_laplace(r, K * B))
    return wl


# ---------------------------------------------------------------- recipe 4
def cfg4(W: int = 8, V: int = 30522, H: int = 768, n_rest: int = 86_559_104, row_frac: float = 0.03,
         rest_density: float = 0.001, d: int = 5, w: int = 1 << 21, s: float = 1.1) -> Workload:
    """Mixed gradient: a row-sparse embedding [V x H] at offset 0 (Zipf rows, as
    recipe 2) followed by n_rest parameters sparsified to rest_density with
    uniform distinct indices."""
    n_emb = V * H
    wl = Workload("cfg4_transformer_mixed", 4, W, n_emb + n_rest, d, w, 0)
    p = _zipf_p(V, s)
    K = int(round(row_frac * V))
    Kr = int(round(rest_density * n_rest))
    for k in range(W):
        r = _rng(4, k)
        rows = r.choice(V, size=K, replace=False, p=p)
        e_idx = _rows_to_elems(rows, H)
        r_idx = (np.sort(r.choice(n_rest, size=Kr, replace=False)) + n_emb).astype(np.uint32)
        wl.idx.append(np.concatenate([e_idx, r_idx]))
        wl.val.append(_normal(r, e_idx.shape[0] + Kr))
    return wl


# ---------------------------------------------------------------- recipe 5
def _coprime_multiplier(rng, n: int) -> int:
    while True:
        A = int(rng.integers(n // 3, n)) | 1
        if np.gcd(A, n) == 1:
            return A


def cfg5(W: int = 16, n: int = 1_000_000_000, nnz: int = 1_000_000, d: int = 5, w: int = 1 << 22,
         s: float = 1.05) -> Workload:
    """Large flat gradient: nnz distinct indices per worker whose ranks follow a
    bounded Zipf(s) law on [1, n] (inverse CDF of the continuous approximation),
    mapped to positions by an affine bijection i = (A (r-1) + B) mod n shared by
    all workers: the popular set is the same on every worker yet spread over the
    whole range."""
    if n > (1 << 31):
        raise ValueError("recipe 5 keeps A*(r-1) inside int64: n must be <= 2^31")
    wl = Workload("cfg5_large_zipf", 5, W, n, d, w, 0)
    rs = _rng(5, 999)
    A = _coprime_multiplier(rs, n)
    B = int(rs.integers(0, n))
    one_minus_s = 1.0 - s
    top = float(n) ** one_minus_s - 1.0
    for k in range(W):
        r = _rng(5, k)
        seen = np.empty(0, dtype=np.int64)
        while seen.shape[0] < nnz:
            u = r.random(size=int(1.5 * nnz))
            ranks = np.floor((top * u + 1.0) ** (1.0 / one_minus_s)).astype(np.int64)
            ranks = np.clip(ranks, 1, n)
            cat = np.concatenate([seen, ranks])
            _, first = np.unique(cat, return_index=True)
            seen = cat[np.sort(first)]            # distinct, in draw order
        ranks = seen[:nnz]
        pos = ((ranks - 1) * A + B) % n           # < 2^63 because n <= 2^31 here
        idx = np.sort(pos).astype(np.uint32)
        wl.idx.append(idx)
        wl.val.append(_normal(r, nnz))
    return wl


_FULL = {1: cfg1, 2: cfg2, 3: cfg3, 4: cfg4, 5: cfg5}


def make(cfg: int) -> Workload:
    """The full-size recipe number cfg (1..5)."""
    return _FULL[cfg]()


def make_cfg1_lds() -> Workload:
    """Recipe 1 with a sketch of 3 x 2^13 cells (96 KB): the one size at which a
    whole sketch fits the LDS of a compute unit.  None of the five recipes does;
    this one exercises the codec where the sketch is two LDS slices."""
    wl = cfg1(w=1 << 13)
    wl.name = "cfg1_uniform_1pct_w8192"
    return wl


def make_small(cfg: int) -> Workload:
    """A reduced copy of recipe cfg with the same structure (ragged length, rows
    straddling bitmap words, shared and private blocks, Zipf overlap) at a size a
    CPU handles in about a second."""
    if cfg == 1:
        return cfg1(W=4, n=(1 << 16) + 37, w=1 << 10)
    if cfg == 2:
        return cfg2(W=4, V=1031, H=650, w=1 << 12)
    if cfg == 3:
        return cfg3(W=4, nblocks=3001, B=256, w=1 << 13)
    if cfg == 4:
        return cfg4(W=4, V=1000, H=768, n_rest=1_000_003, w=1 << 14)
    if cfg == 5:
        return cfg5(W=4, n=5_000_011, nnz=5000, w=1 << 13)
    raise KeyError(cfg)
