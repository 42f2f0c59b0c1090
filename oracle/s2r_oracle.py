"""CPU oracle for the Sparse-Sketch Reducer codec (S2 Reducer, Algorithm 1 and Section 3.1).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
GPU library has to compute.  It may be imported by the tests, by the smoke check
and by the benchmark's CPU-baseline leg, and by nothing else.  It shares no code,
table or constant generator with the HIP sources and imports nothing from the
product package.

Everything here follows the paper's order of steps:

  compress   (Algorithm 1, the bitmap line and the insertion loops; Section 3.1
              "Compressing Sparse Gradient")
  aggregate  (Algorithm 1, the AllReduce line; Section 3.1 "Collecting
              Sparse-Sketch with AllReduce")
  decompress (Algorithm 1, the recovery line and the query loops; Section 3.1
              "Decompressing Sparse Gradient")

Notation: the paper writes r x c for the sketch; this code uses d rows and w
columns, n for the gradient length and W for the number of workers.

Accumulation is float64 throughout.  The sketch cells hold sums of float32 inputs
converted exactly to float64, so the oracle's rounding error is ~1e-16 relative to
the absolute mass of a cell, far below the float32 tolerance it is used to judge.

Points the paper leaves open and the reading taken here (each also listed in the
design notes of the repository):

  * one bitmap bit per gradient element (the paper speaks of blocks; the loops
    of Algorithm 1 run over element indices, and a block of one element is the
    case both agree on);
  * "non-zero" is decided on the float32 bit pattern: every pattern except +0.0
    and -0.0 is non-zero (denormals, infinities and NaNs included);
  * bitmap words are 64 bits, element i is bit (i mod 64), least significant
    first, of word floor(i / 64); unused high bits of the last word are zero;
  * hash family: the paper only says "hash function" and "random sign".  Row j
    uses four 64-bit parameters a_j, b_j, c_j, e_j taken in that order from a
    SplitMix64 stream started at `seed` (a_j and c_j made odd);
        bucket  h_j(i) = ((a_j * i + b_j) mod 2^64) >> (64 - log2 w)
        sign    s_j(i) = +1 if bit 63 of ((c_j * i + e_j) mod 2^64) is 0 else -1
    w must be a power of two;
  * the bitmap is aggregated with bitwise OR;
  * median: middle order statistic for odd d, mean of the two middle ones for
    even d;
  * the decoder returns the estimate of the SUM over workers (Algorithm 1 has no
    division by W).

Block-granular variant (the *_blocks functions at the end): Section 3.1 sizes the
bitmap by the number of word vectors or gradient blocks, one bit telling whether
the block holds a non-zero gradient, and Algorithm 1's bitmap line is written per
block.  There the bitmap has one bit per block of B consecutive elements (the last
block may be shorter), the sketch still receives the non-zero elements only
(Section 3.1: zeros do not change a bucket), and decompression queries every
element of every block whose aggregated bit is set.  B = 1 is the element-granular
codec above.

Block-wise Top-K with error feedback (topk_blocks at the end), the sparsifier the
paper puts in front of the codec for dense layers (Section 2.2: the l2 norm of
every block, the K largest blocks are kept; Theorem 2 and its proof: what is not
sent stays in an error sequence that is added to the next gradient).  Readings:
the score of a block is the sum of the squares of its float32 elements
accumulated in float64 and rounded once to float32 (same order as the norm);
equal scores are ordered by block index, lower first; the residual is the part of
(gradient + old residual) that is not kept: the sketch's own estimation error is
not fed back (a worker cannot see it: the decoder returns the sum over workers).

Parity pins: see tests/test_oracle_*.py.  No function in this file is unpinned,
but the hash family itself is a reading (the paper names none); it is pinned to a
big-integer re-statement and to the published SplitMix64 reference outputs.  The
mass table M and decode_tolerance_mass, which only scale the tests' float32
tolerances, are pinned cell by cell to pure-Python loops as well.
"""

from __future__ import annotations

import numpy as np

_U64 = np.uint64
_MASK64 = (1 << 64) - 1


# --------------------------------------------------------------------------
# hash family (Section 3.1: a hash function h picks the bucket of a non-zero, a
# random sign vector s weights it; Algorithm 1 initialisation: {s_ij}, {h_ij})
# --------------------------------------------------------------------------

def splitmix64_stream(seed: int, count: int) -> list[int]:
    """`count` successive outputs of the SplitMix64 generator (Steele, Lea, Flood
    2014) whose state starts at `seed`.  Python integers, reduced mod 2^64."""
    state = seed & _MASK64
    out = []
    for _ in range(count):
        state = (state + 0x9E3779B97F4A7C15) & _MASK64
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        out.append(z ^ (z >> 31))
    return out


def hash_params(seed: int, d: int) -> list[tuple[int, int, int, int]]:
    """Per-row parameters (a_j, b_j, c_j, e_j), j = 0..d-1, as Python integers."""
    s = splitmix64_stream(seed, 4 * d)
    rows = []
    for j in range(d):
        a, b, c, e = s[4 * j: 4 * j + 4]
        rows.append((a | 1, b, c | 1, e))
    return rows


def _log2_exact(w: int) -> int:
    if w < 1 or (w & (w - 1)) != 0:
        raise ValueError("sketch width w must be a power of two")
    return w.bit_length() - 1


def bucket_hash(idx: np.ndarray, a: int, b: int, w: int) -> np.ndarray:
    """h_j(i) for an array of indices (any unsigned integer dtype) -> int64."""
    L = _log2_exact(w)
    i = idx.astype(_U64)
    with np.errstate(over="ignore"):
        u = i * _U64(a) + _U64(b)          # wraps mod 2^64
    if L == 0:
        return np.zeros(i.shape, dtype=np.int64)
    return (u >> _U64(64 - L)).astype(np.int64)


def sign_hash(idx: np.ndarray, c: int, e: int) -> np.ndarray:
    """s_j(i) in {+1.0, -1.0} (float64)."""
    i = idx.astype(_U64)
    with np.errstate(over="ignore"):
        v = i * _U64(c) + _U64(e)
    return np.where((v >> _U64(63)) == 0, 1.0, -1.0)


# --------------------------------------------------------------------------
# compress (Algorithm 1: bitmap line, insertion loops)
# --------------------------------------------------------------------------

def nonzero_mask(g: np.ndarray) -> np.ndarray:
    """True where the float32 element is anything but +0.0 / -0.0."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    return (g.view(np.uint32) & np.uint32(0x7FFFFFFF)) != 0


def pack_bitmap(mask: np.ndarray) -> np.ndarray:
    """Boolean mask of length n -> ceil(n/64) little-endian 64-bit words, element
    i in bit (i mod 64) of word i // 64."""
    n = mask.shape[0]
    words = (n + 63) // 64
    by = np.packbits(mask.astype(np.uint8), bitorder="little")
    buf = np.zeros(words * 8, dtype=np.uint8)
    buf[: by.shape[0]] = by
    return buf.view("<u8").astype(np.uint64)


def unpack_bitmap(bitmap: np.ndarray, n: int) -> np.ndarray:
    """Inverse of pack_bitmap: boolean mask of length n."""
    by = np.ascontiguousarray(bitmap, dtype="<u8").view(np.uint8)
    return np.unpackbits(by, bitorder="little")[:n].astype(bool)


def sparse_of(g: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Sparse(g): ascending indices of the non-zeros (uint32) and their values."""
    idx = np.flatnonzero(nonzero_mask(g))
    return idx.astype(np.uint32), np.ascontiguousarray(g, dtype=np.float32)[idx]


def insert(idx: np.ndarray, val: np.ndarray, d: int, w: int, seed: int
           ) -> tuple[np.ndarray, np.ndarray]:
    """Insertion loops of Algorithm 1: for every i in Sparse(g) and every row j,
    S[j, h_j(i)] += s_j(i) * g(i).  Returns (S, M), both float64 [d, w]; M is the
    'mass' table that accumulates |g(i)| over the same insertions (used only to
    scale test tolerances; it is not part of the method)."""
    S = np.zeros((d, w), dtype=np.float64)
    M = np.zeros((d, w), dtype=np.float64)
    v = val.astype(np.float64)
    for j, (a, b, c, e) in enumerate(hash_params(seed, d)):
        h = bucket_hash(idx, a, b, w)
        s = sign_hash(idx, c, e)
        np.add.at(S[j], h, s * v)
        np.add.at(M[j], h, np.abs(v))
    return S, M


def encode(g: np.ndarray, d: int, w: int, seed: int) -> dict:
    """One worker's compress step on a dense-stored gradient g (float32[n])."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    mask = nonzero_mask(g)
    idx = np.flatnonzero(mask).astype(np.uint32)
    val = g[idx]
    S, M = insert(idx, val, d, w, seed)
    return {"bitmap": pack_bitmap(mask), "idx": idx, "val": val, "S": S, "M": M}


def encode_sparse(idx: np.ndarray, val: np.ndarray, n: int, d: int, w: int, seed: int) -> dict:
    """Same as encode() for a gradient given as (ascending distinct idx, val)
    pairs, for lengths n whose dense form does not fit in host memory.  Pairs
    whose value is +-0.0 are dropped, as the dense scan would drop them."""
    idx = np.asarray(idx, dtype=np.uint32)
    val = np.asarray(val, dtype=np.float32)
    keep = nonzero_mask(val)
    idx, val = idx[keep], val[keep]
    words = (n + 63) // 64
    bitmap = np.zeros(words, dtype=np.uint64)
    np.bitwise_or.at(bitmap, (idx >> np.uint32(6)).astype(np.int64),
                     _U64(1) << (idx & np.uint32(63)).astype(_U64))
    S, M = insert(idx, val, d, w, seed)
    return {"bitmap": bitmap, "idx": idx, "val": val, "S": S, "M": M}


# --------------------------------------------------------------------------
# aggregate (Algorithm 1: AllReduce(S, C))
# --------------------------------------------------------------------------

def merge(sketches: list[np.ndarray], bitmaps: list[np.ndarray]
          ) -> tuple[np.ndarray, np.ndarray]:
    """Sum of the workers' sketches, bitwise OR of their bitmaps."""
    S = np.zeros_like(sketches[0], dtype=np.float64)
    for Sk in sketches:
        S = S + Sk
    C = np.zeros_like(bitmaps[0], dtype=np.uint64)
    for Ck in bitmaps:
        C = C | Ck
    return S, C


# --------------------------------------------------------------------------
# decompress (Algorithm 1: recover Sparse(g), estimates, median)
# --------------------------------------------------------------------------

def bitmap_indices(bitmap: np.ndarray, n: int) -> np.ndarray:
    """Ascending indices of the set bits (uint32)."""
    return np.flatnonzero(unpack_bitmap(bitmap, n)).astype(np.uint32)


def median_rows(est: np.ndarray) -> np.ndarray:
    """Median over axis 0 of a [d, k] table: the middle order statistic for odd
    d, the mean of the two middle ones for even d."""
    d = est.shape[0]
    srt = np.sort(est, axis=0)
    if d % 2 == 1:
        return srt[d // 2]
    return 0.5 * (srt[d // 2 - 1] + srt[d // 2])


def estimates(S: np.ndarray, idx: np.ndarray, seed: int) -> np.ndarray:
    """estimates[j, k] = s_j(i_k) * S[j, h_j(i_k)]  (float64 [d, len(idx)])."""
    d, w = S.shape
    est = np.empty((d, idx.shape[0]), dtype=np.float64)
    for j, (a, b, c, e) in enumerate(hash_params(seed, d)):
        est[j] = sign_hash(idx, c, e) * S[j, bucket_hash(idx, a, b, w)]
    return est


def decode(S: np.ndarray, bitmap: np.ndarray, n: int, seed: int, dense: bool = False) -> dict:
    """Decompress: indices from the aggregated bitmap, median-of-rows estimate at
    each.  With dense=True also the length-n vector with zeros at unset bits."""
    idx = bitmap_indices(bitmap, n)
    val = median_rows(estimates(S, idx, seed))
    out = {"idx": idx, "val": val}
    if dense:
        gh = np.zeros(n, dtype=np.float64)
        gh[idx] = val
        out["dense"] = gh
    return out


def decode_update(S: np.ndarray, bitmap: np.ndarray, n: int, seed: int, params: np.ndarray, scale: float) -> np.ndarray:
    """Decompress straight into a parameter update (Section 1: the aggregated
    gradient is what updates the model; Algorithm 1 returns the sum, so the caller's
    scale carries the learning rate and the 1/W): params[i] + scale * g_hat(i) at
    the indices of the aggregated bitmap, params[i] elsewhere.  float64, one
    rounding to float32."""
    out = decode(S, bitmap, n, seed)
    new = np.ascontiguousarray(params, dtype=np.float32).astype(np.float64)
    new[out["idx"]] += float(np.float32(scale)) * out["val"]
    return new.astype(np.float32)


def decode_tolerance_mass(M: np.ndarray, idx: np.ndarray, seed: int) -> np.ndarray:
    """max_j M[j, h_j(i)] per index: the scale against which a decoded value's
    float32 error is judged (the median moves by at most the largest per-row
    perturbation)."""
    d, w = M.shape
    m = np.zeros(idx.shape[0], dtype=np.float64)
    for j, (a, b, _c, _e) in enumerate(hash_params(seed, d)):
        m = np.maximum(m, M[j, bucket_hash(idx, a, b, w)])
    return m


def reduce_workers(grads: list[np.ndarray], d: int, w: int, seed: int, dense: bool = False) -> dict:
    """Whole of Algorithm 1 for W dense-stored worker gradients."""
    enc = [encode(g, d, w, seed) for g in grads]
    S, C = merge([e["S"] for e in enc], [e["bitmap"] for e in enc])
    M = np.sum([e["M"] for e in enc], axis=0)
    out = decode(S, C, grads[0].shape[0], seed, dense=dense)
    out.update({"S": S, "M": M, "bitmap": C, "workers": enc})
    return out


# --------------------------------------------------------------------------
# block-granular variant (Section 3.1: bitmap over word vectors / gradient
# blocks; Algorithm 1: the bitmap line, which sets the bit of a non-zero block)
# --------------------------------------------------------------------------

def block_mask(g: np.ndarray, B: int) -> np.ndarray:
    """bool[ceil(n / B)]: block x is set iff one of its elements g[xB .. xB+B) is non-zero."""
    nz = nonzero_mask(np.ascontiguousarray(g, dtype=np.float32))
    nb = (nz.shape[0] + B - 1) // B
    padded = np.zeros(nb * B, dtype=bool)
    padded[: nz.shape[0]] = nz
    return padded.reshape(nb, B).any(axis=1)


def block_elements(blocks: np.ndarray, B: int, n: int) -> np.ndarray:
    """Ascending element indices (int64) of the listed blocks, those below n only."""
    e = (np.asarray(blocks, dtype=np.int64)[:, None] * B + np.arange(B, dtype=np.int64)[None, :]).reshape(-1)
    return e[e < n]


def encode_blocks(g: np.ndarray, B: int, d: int, w: int, seed: int) -> dict:
    """One worker's compress step with a bitmap over blocks of B elements.  The
    sketch is the one encode() builds: only non-zero elements are inserted."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    bm = block_mask(g, B)
    idx, val = sparse_of(g)
    S, M = insert(idx, val, d, w, seed)
    return {"bitmap": pack_bitmap(bm), "blocks": np.flatnonzero(bm).astype(np.uint32), "S": S, "M": M}


def decode_blocks(S: np.ndarray, bitmap: np.ndarray, n: int, B: int, seed: int) -> dict:
    """Decompress with a block bitmap: the set blocks (ascending), and for each the
    median-of-rows estimate of every one of its B elements.  `val` is
    [len(blocks), B]; positions of the last block that lie beyond n hold 0."""
    nb = (n + B - 1) // B
    blocks = bitmap_indices(bitmap, nb)
    e = (blocks.astype(np.int64)[:, None] * B + np.arange(B, dtype=np.int64)[None, :]).reshape(-1)
    inside = e < n
    val = np.zeros(e.shape[0], dtype=np.float64)
    val[inside] = median_rows(estimates(S, e[inside].astype(np.uint32), seed))
    return {"blocks": blocks, "val": val.reshape(len(blocks), B)}


def decode_blocks_update(S: np.ndarray, bitmap: np.ndarray, n: int, B: int, seed: int, params: np.ndarray,
                         scale: float) -> np.ndarray:
    """decode_update with a block bitmap: params[i] + scale * g_hat(i) at every
    element i < n of every set block, params[i] elsewhere.  float64, one rounding
    to float32."""
    out = decode_blocks(S, bitmap, n, B, seed)
    elems = block_elements(out["blocks"], B, n)
    inside = (out["blocks"].astype(np.int64)[:, None] * B + np.arange(B, dtype=np.int64)[None, :]).reshape(-1) < n
    new = np.ascontiguousarray(params, dtype=np.float32).astype(np.float64)
    new[elems] += float(np.float32(scale)) * out["val"].reshape(-1)[inside]
    return new.astype(np.float32)


def reduce_workers_blocks(grads: list[np.ndarray], B: int, d: int, w: int, seed: int) -> dict:
    """Whole of Algorithm 1 with the block bitmap for W dense-stored worker gradients."""
    enc = [encode_blocks(g, B, d, w, seed) for g in grads]
    S, C = merge([e["S"] for e in enc], [e["bitmap"] for e in enc])
    M = np.sum([e["M"] for e in enc], axis=0)
    out = decode_blocks(S, C, grads[0].shape[0], B, seed)
    out.update({"S": S, "M": M, "bitmap": C, "workers": enc})
    return out


# --------------------------------------------------------------------------
# block-wise Top-K sparsifier with error feedback (Section 2.2; Theorem 2)
# --------------------------------------------------------------------------

def block_scores(acc: np.ndarray, B: int) -> np.ndarray:
    """float32[ceil(n / B)]: per block, the sum of squares of its elements (float64
    accumulation of exact products, one rounding to float32)."""
    acc = np.ascontiguousarray(acc, dtype=np.float32)
    nb = (acc.shape[0] + B - 1) // B
    padded = np.zeros(nb * B, dtype=np.float64)
    padded[: acc.shape[0]] = acc.astype(np.float64)
    return np.sum(padded.reshape(nb, B) ** 2, axis=1).astype(np.float32)


def topk_blocks(g: np.ndarray, e, B: int, K: int) -> dict:
    """acc = g + e (float32); keep the K blocks of largest score (ties: lower block
    first).  Returns the kept blocks (ascending), the sparse gradient (acc in the
    kept blocks, +0.0 elsewhere), the new residual (acc elsewhere, +0.0 in the kept
    blocks) and the scores."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    acc = g if e is None else (g + np.ascontiguousarray(e, dtype=np.float32)).astype(np.float32)
    score = block_scores(acc, B)
    nb = score.shape[0]
    order = sorted(range(nb), key=lambda x: (-float(score[x]), x))
    kept = np.array(sorted(order[:K]), dtype=np.uint32)
    mask = np.zeros(nb, dtype=bool)
    mask[kept] = True
    elem = np.repeat(mask, B)[: acc.shape[0]]
    sparse = np.where(elem, acc, np.float32(0.0)).astype(np.float32)
    resid = np.where(elem, np.float32(0.0), acc).astype(np.float32)
    return {"blocks": kept, "sparse": sparse, "residual": resid, "score": score, "acc": acc}


def topk_encode_blocks(g: np.ndarray, e, B: int, K: int, d: int, w: int, seed: int) -> dict:
    """Sparsify, then compress, as one step (Section 2.2 feeding Algorithm 1's
    compress lines): the K blocks that topk_blocks keeps are the blocks that are
    communicated, so the bitmap marks exactly the kept blocks (a kept block whose
    elements are all zero is still marked: the sparsifier chose it, the codec does
    not look again) and the sketch receives the non-zero elements of acc = g + e
    in those blocks.  Returns the bitmap, the kept blocks, the sketch with its
    absolute-mass companion, and the new residual."""
    tk = topk_blocks(g, e, B, K)
    nb = tk["score"].shape[0]
    flags = np.zeros(nb, dtype=bool)
    flags[tk["blocks"]] = True
    idx, val = sparse_of(tk["sparse"])
    S, M = insert(idx, val, d, w, seed)
    return {"bitmap": pack_bitmap(flags), "blocks": tk["blocks"], "S": S, "M": M, "residual": tk["residual"],
            "sparse": tk["sparse"]}
