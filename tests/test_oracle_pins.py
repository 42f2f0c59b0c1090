"""Pins for oracle/s2r_oracle.py: the oracle checked against things other than
itself -- a pure-Python element-by-element restatement (tests/bruteforce.py),
the paper's matrix formulation A^T g / A A^T g (Section 3.1), closed forms,
invariants the paper states (linearity, zeros are inert, merged bitmap = union),
exact recovery without collisions, the published SplitMix64 outputs, and the
statistical claims of Theorem 1 / its proof (unbiasedness, collision law).
"""

import math
import os
import random

import numpy as np
import pytest

from oracle import s2r_oracle as orc
from tests import bruteforce as bf
from paper_2110_02140_amd import workloads


def _tiny_grads(rng, W, n, density, specials=False):
    gs = []
    for _ in range(W):
        g = np.zeros(n, dtype=np.float32)
        k = max(1, int(density * n))
        idx = rng.choice(n, size=k, replace=False)
        g[idx] = rng.normal(0, 0.01, size=k).astype(np.float32)
        g[idx[g[idx] == 0]] = 1e-3
        gs.append(g)
    if specials:
        gs[0][1] = np.float32(-0.0)                     # zero
        gs[0][2] = np.float32(1e-42)                    # denormal: non-zero
        gs[0][3] = np.float32(-1e-45)                   # smallest denormal
    return gs


# ---------------------------------------------------------------- hash family
def test_splitmix_matches_published_reference(golden_dir):
    with open(os.path.join(golden_dir, "splitmix64_reference.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 2
    for row in rows:
        seed, want = int(row[0]), [int(x) for x in row[1:]]
        assert orc.splitmix64_stream(seed, len(want)) == want
        assert bf.splitmix(seed, len(want)) == want


def test_hash_params_order_and_oddness():
    for seed in (0, 1, 2**63 + 5, 2**64 - 1):
        p = orc.hash_params(seed, 4)
        s = bf.splitmix(seed, 16)
        for j in range(4):
            assert p[j] == (s[4 * j] | 1, s[4 * j + 1], s[4 * j + 2] | 1, s[4 * j + 3])
            assert p[j][0] % 2 == 1 and p[j][2] % 2 == 1


@pytest.mark.parametrize("w", [1, 2, 64, 1 << 14, 1 << 22, 1 << 31])
def test_bucket_and_sign_match_bigint(w):
    r = random.Random(w)
    idx = np.array([0, 1, 2, 63, 64, 2**31 - 1, 2**31, 2**32 - 1] +
                   [r.randrange(2**32) for _ in range(300)], dtype=np.uint32)
    for seed in (0, 7, 2**64 - 3):
        for (a, b, c, e) in orc.hash_params(seed, 3):
            hb = orc.bucket_hash(idx, a, b, w)
            sg = orc.sign_hash(idx, c, e)
            assert hb.min() >= 0 and hb.max() < w
            for k, i in enumerate(idx.tolist()):
                assert hb[k] == bf.h(i, a, b, w)
                assert sg[k] == bf.s(i, c, e)


def test_width_must_be_power_of_two():
    with pytest.raises(ValueError):
        orc.bucket_hash(np.arange(4, dtype=np.uint32), 3, 5, 12)


# ---------------------------------------------------------------- bitmap / Sparse(g)
@pytest.mark.parametrize("n", [1, 63, 64, 65, 127, 128, 1000])
def test_bitmap_and_sparse_match_elementwise_definition(n):
    rng = np.random.default_rng(n)
    g = _tiny_grads(rng, 1, max(n, 8), 0.3, specials=True)[0][:n]
    enc = orc.encode(g, 2, 8, 0)
    flags = [1 if bf.is_nonzero(float(x)) else 0 for x in g]
    assert [int(x) for x in enc["bitmap"]] == bf.words_of(flags)
    assert enc["idx"].tolist() == [i for i, f in enumerate(flags) if f]
    assert enc["idx"].dtype == np.uint32 and enc["bitmap"].dtype == np.uint64
    assert np.array_equal(enc["val"], g[enc["idx"]])
    assert sum(bin(int(x)).count("1") for x in enc["bitmap"]) == len(enc["idx"])
    # round trip bitmap -> indices -> bitmap
    assert np.array_equal(orc.bitmap_indices(enc["bitmap"], n), enc["idx"])
    assert np.array_equal(orc.pack_bitmap(orc.unpack_bitmap(enc["bitmap"], n)), enc["bitmap"])


def test_signed_zero_denormal_nan_inf_rule():
    g = np.array([0.0, -0.0, 1e-45, -1e-42, np.inf, -np.inf, np.nan, 1.0], dtype=np.float32)
    assert orc.nonzero_mask(g).tolist() == [False, False, True, True, True, True, True, True]


def test_merged_bitmap_popcount_is_union_size():
    rng = np.random.default_rng(5)
    gs = _tiny_grads(rng, 5, 3000, 0.05)
    enc = [orc.encode(g, 3, 64, 1) for g in gs]
    _, C = orc.merge([e["S"] for e in enc], [e["bitmap"] for e in enc])
    union = set()
    for g in gs:
        union |= {i for i, x in enumerate(g.tolist()) if x != 0.0}
    assert sum(bin(int(x)).count("1") for x in C) == len(union)
    assert orc.bitmap_indices(C, 3000).tolist() == sorted(union)


def test_encode_sparse_equals_encode_dense():
    wl = workloads.make_small(5)
    for k in range(2):
        a = orc.encode(wl.dense(k), wl.d, wl.w, wl.seed)
        b = orc.encode_sparse(wl.idx[k], wl.val[k], wl.n, wl.d, wl.w, wl.seed)
        for key in ("bitmap", "idx", "val", "S", "M"):
            assert np.array_equal(a[key], b[key]), key


# ---------------------------------------------------------------- whole algorithm vs brute force
@pytest.mark.parametrize("d,w,seed", [(1, 8, 0), (3, 16, 1), (4, 32, 2), (5, 4, 3), (2, 1, 4)])
def test_algorithm1_matches_pure_python(d, w, seed):
    rng = np.random.default_rng(100 + seed)
    n, W = 200, 3
    gs = _tiny_grads(rng, W, n, 0.2, specials=True)
    res = orc.reduce_workers(gs, d, w, seed, dense=True)
    flags, Ss = zip(*[bf.compress([float(x) for x in g], d, w, seed) for g in gs])
    for k in range(W):
        assert np.allclose(res["workers"][k]["S"], np.array(Ss[k]), rtol=0, atol=1e-18)
    C, S = bf.aggregate(flags, Ss)
    assert [int(x) for x in res["bitmap"]] == bf.words_of(C)
    assert np.allclose(res["S"], np.array(S), rtol=0, atol=1e-17)
    want = bf.decompress(C, S, seed)
    assert res["idx"].tolist() == sorted(want)
    got = dict(zip(res["idx"].tolist(), res["val"].tolist()))
    for i, v in want.items():
        assert got[i] == pytest.approx(v, rel=0, abs=1e-17)
    dense = res["dense"]
    assert dense.shape == (n,)
    assert all(dense[i] == 0.0 for i in range(n) if not C[i])


# ---------------------------------------------------------------- the paper's matrix form
def test_insert_and_query_equal_mapping_matrix_form():
    """Section 3.1: insertion is A^T g, the query of element i is A(i,:) A^T g,
    with A(i, b) = +-1 iff element i maps to bucket b (one row of the sketch)."""
    n, w, seed = 150, 16, 9
    rng = np.random.default_rng(3)
    g = _tiny_grads(rng, 1, n, 0.3)[0]
    (a, b, c, e), = bf.params(seed, 1)
    A = np.zeros((n, w))
    for i in range(n):
        A[i, bf.h(i, a, b, w)] = bf.s(i, c, e)
    enc = orc.encode(g, 1, w, seed)
    assert np.allclose(enc["S"][0], A.T @ g.astype(np.float64), rtol=0, atol=1e-16)
    dec = orc.decode(enc["S"], enc["bitmap"], n, seed)
    full = A @ (A.T @ g.astype(np.float64))
    assert np.allclose(dec["val"], full[dec["idx"]], rtol=0, atol=1e-16)


# ---------------------------------------------------------------- invariants stated by the paper
def test_linearity_sum_of_sketches_is_sketch_of_sum():
    rng = np.random.default_rng(11)
    gs = _tiny_grads(rng, 6, 5000, 0.03)
    d, w, seed = 3, 256, 2
    enc = [orc.encode(g, d, w, seed) for g in gs]
    S, _ = orc.merge([e["S"] for e in enc], [e["bitmap"] for e in enc])
    gsum = np.sum([g.astype(np.float64) for g in gs], axis=0)
    idx = np.flatnonzero(gsum != 0).astype(np.uint32)
    # insert the float64 sum directly (bypassing the float32 cast of encode())
    S2 = np.zeros((d, w))
    for j, (a, b, c, e) in enumerate(orc.hash_params(seed, d)):
        np.add.at(S2[j], orc.bucket_hash(idx, a, b, w), orc.sign_hash(idx, c, e) * gsum[idx])
    M = np.sum([e["M"] for e in enc], axis=0)
    assert np.all(np.abs(S - S2) <= 1e-14 * M + 1e-300)


def test_zeros_are_inert():
    """Inserting every element, zeros included, gives the same table."""
    rng = np.random.default_rng(12)
    g = _tiny_grads(rng, 1, 4000, 0.05)[0]
    d, w, seed = 3, 128, 4
    enc = orc.encode(g, d, w, seed)
    allidx = np.arange(g.shape[0], dtype=np.uint32)
    S_all, _ = orc.insert(allidx, g, d, w, seed)
    assert np.array_equal(enc["S"], S_all)


def test_row_sum_identity_and_width_one_closed_form():
    rng = np.random.default_rng(13)
    g = _tiny_grads(rng, 1, 3000, 0.1)[0]
    d, seed = 4, 6
    P = bf.params(seed, d)
    signed = [math.fsum(bf.s(i, c, e) * float(g[i]) for i in range(g.shape[0])) for (_, _, c, e) in P]
    for w in (1, 64):
        enc = orc.encode(g, d, w, seed)
        for j in range(d):
            assert enc["S"][j].sum() == pytest.approx(signed[j], rel=1e-12, abs=1e-15)
        if w == 1:
            assert enc["S"].shape == (d, 1)


def test_single_element_gradient():
    n, d, w, seed = 777, 5, 32, 8
    g = np.zeros(n, dtype=np.float32)
    g[123] = -0.25
    enc = orc.encode(g, d, w, seed)
    assert np.count_nonzero(enc["S"]) == d
    for j, (a, b, c, e) in enumerate(bf.params(seed, d)):
        assert enc["S"][j, bf.h(123, a, b, w)] == bf.s(123, c, e) * -0.25
    dec = orc.decode(enc["S"], enc["bitmap"], n, seed)
    assert dec["idx"].tolist() == [123] and dec["val"].tolist() == [-0.25]


# ---------------------------------------------------------------- exact recovery without collisions
def _majority_collision_free(union, d, w, seed):
    P = bf.params(seed, d)
    rows_ok = {i: 0 for i in union}
    for (a, b, _c, _e) in P:
        seen = {}
        for i in union:
            seen.setdefault(bf.h(i, a, b, w), []).append(i)
        for members in seen.values():
            if len(members) == 1:
                rows_ok[members[0]] += 1
    return all(2 * v > d for v in rows_ok.values())


@pytest.mark.parametrize("d", [1, 3, 5])
def test_exact_recovery_when_collision_free(d):
    rng = np.random.default_rng(20 + d)
    n, W, w = 2000, 4, 1 << 16
    gs = _tiny_grads(rng, W, n, 0.01)
    union = sorted({int(i) for g in gs for i in np.flatnonzero(g)})
    seed = next(s for s in range(100) if _majority_collision_free(union, d, w, s))
    res = orc.reduce_workers(gs, d, w, seed, dense=True)
    exact = np.sum([g.astype(np.float64) for g in gs], axis=0)
    assert res["idx"].tolist() == union
    assert np.allclose(res["dense"], exact, rtol=0, atol=1e-17)


def test_single_worker_recovery_is_bit_exact_in_float32():
    rng = np.random.default_rng(31)
    g = _tiny_grads(rng, 1, 1500, 0.01)[0]
    union = sorted(int(i) for i in np.flatnonzero(g))
    d, w = 3, 1 << 14
    seed = next(s for s in range(100) if _majority_collision_free(union, d, w, s))
    res = orc.reduce_workers([g], d, w, seed, dense=True)
    assert np.array_equal(res["dense"].astype(np.float32), g)


# ---------------------------------------------------------------- median
@pytest.mark.parametrize("d", [1, 2, 3, 4, 5, 7, 16])
def test_median_brute_force_and_permutation_invariance(d):
    rng = np.random.default_rng(d)
    est = rng.normal(size=(d, 50))
    est[:, 0] = 1.0                     # all ties
    if d > 2:
        est[1, 1] = est[2, 1]           # a tie at one position
    got = orc.median_rows(est)
    for k in range(50):
        assert got[k] == bf.median(est[:, k].tolist())
    assert np.array_equal(got, orc.median_rows(est[rng.permutation(d)]))
    assert np.allclose(got, np.median(est, axis=0), rtol=0, atol=1e-16)
    if d % 2 == 1:
        assert all(got[k] in est[:, k] for k in range(50))


def test_single_row_is_plain_point_query():
    rng = np.random.default_rng(41)
    n, w, seed = 500, 32, 3
    g = _tiny_grads(rng, 1, n, 0.2)[0]
    enc = orc.encode(g, 1, w, seed)
    dec = orc.decode(enc["S"], enc["bitmap"], n, seed)
    (a, b, c, e), = bf.params(seed, 1)
    for i, v in zip(dec["idx"].tolist(), dec["val"].tolist()):
        assert v == bf.s(i, c, e) * enc["S"][0, bf.h(i, a, b, w)]


# ---------------------------------------------------------------- statistics (Theorem 1 and its proof)
def test_estimate_is_unbiased_over_seeds():
    rng = np.random.default_rng(50)
    n, d, w = 64, 3, 16
    g = np.zeros(n, dtype=np.float32)
    nz = rng.choice(n, size=24, replace=False)
    g[nz] = rng.normal(0, 1.0, size=24).astype(np.float32)
    nseeds = 3000
    errs = np.zeros((nseeds, 24))
    order = np.sort(nz)
    for s in range(nseeds):
        enc = orc.encode(g, d, w, s)
        dec = orc.decode(enc["S"], enc["bitmap"], n, s)
        errs[s] = dec["val"] - g[order].astype(np.float64)
    mean = errs.mean(axis=0)
    sem = errs.std(axis=0, ddof=1) / math.sqrt(nseeds)
    assert np.all(np.abs(mean) <= 4.5 * sem + 1e-12)
    assert errs.std() > 0.0             # collisions do happen at this width


def test_single_row_error_variance_is_the_others_energy_over_the_width():
    """With one row the error of element j is sum_{i != j} Phi(i, j) g(i), and by the
    proof of Theorem 1 Phi(i, j) is +1 or -1 with probability 0.5 / m each, independently
    enough over pairs that the variance is sum_{i != j} g(i)^2 / m."""
    rng = np.random.default_rng(51)
    n, w, nseeds = 40, 8, 6000
    g = rng.normal(0, 1.0, size=n).astype(np.float32)
    errs = np.zeros((nseeds, n))
    for s in range(nseeds):
        enc = orc.encode(g, 1, w, s)
        errs[s] = orc.decode(enc["S"], enc["bitmap"], n, s)["val"] - g.astype(np.float64)
    energy = float(np.sum(g.astype(np.float64) ** 2))
    want = (energy - g.astype(np.float64) ** 2) / w
    got = errs.var(axis=0)
    assert np.all(np.abs(got / want - 1.0) < 0.12), f"worst ratio {np.max(np.abs(got / want - 1.0)):.3f}"
    assert abs(got.sum() / want.sum() - 1.0) < 0.03


def test_collision_probabilities():
    """Two fixed distinct indices share a bucket with probability 1/m, and then
    agree / disagree in sign with probability 1/2 each (proof of Theorem 1)."""
    w, nseeds = 8, 20000
    pairs = [(3, 4), (0, 2**31), (17, 4242), (255, 256)]
    for (i, k) in pairs:
        same = agree = 0
        for s in range(nseeds):
            (a, b, c, e), = bf.params(s, 1)
            if bf.h(i, a, b, w) == bf.h(k, a, b, w):
                same += 1
                agree += bf.s(i, c, e) == bf.s(k, c, e)
        p = same / nseeds
        assert abs(p - 1 / w) < 5 * math.sqrt((1 / w) * (1 - 1 / w) / nseeds)
        assert abs(agree / same - 0.5) < 5 * math.sqrt(0.25 / same)
    # and the vectorised hashes give the same buckets as the big-int ones
    idx = np.array([3, 4, 17, 4242], dtype=np.uint32)
    (a, b, c, e), = orc.hash_params(5, 1)
    assert orc.bucket_hash(idx, a, b, w).tolist() == [bf.h(int(i), a, b, w) for i in idx]


# ---------------------------------------------------------------- tolerance scale
def test_mass_table_bounds_sketch():
    wl = workloads.make_small(3)
    res = orc.reduce_workers([wl.dense(k) for k in range(wl.W)], wl.d, wl.w, wl.seed)
    assert np.all(res["M"] >= np.abs(res["S"]) - 1e-18)
    m = orc.decode_tolerance_mass(res["M"], res["idx"], wl.seed)
    assert np.all(m >= np.abs(res["val"]) - 1e-18)


@pytest.mark.parametrize("d,w,seed", [(1, 8, 0), (3, 16, 1), (4, 32, 2), (5, 4, 3), (2, 1, 4)])
def test_mass_table_and_decode_tolerance_mass_match_pure_python(d, w, seed):
    """The scale of every float32 tolerance: M[j, b] is the sum of |g(i)| over the
    insertions that land in the cell (per worker, and summed over the workers for the
    aggregate), and a decoded value is judged against the largest of the d masses its
    index reads.  Both against Python loops, cell by cell and index by index."""
    rng = np.random.default_rng(100 + seed)
    n, W = 200, 3
    gs = _tiny_grads(rng, W, n, 0.2, specials=True)
    res = orc.reduce_workers(gs, d, w, seed)
    Ms = [bf.mass_table([float(x) for x in g], d, w, seed) for g in gs]
    for k in range(W):
        assert np.allclose(res["workers"][k]["M"], np.array(Ms[k]), rtol=1e-15, atol=0)
        idx, val = orc.sparse_of(gs[k])
        assert np.allclose(orc.insert(idx, val, d, w, seed)[1], np.array(Ms[k]), rtol=1e-15, atol=0)
    total = [[math.fsum(Ms[k][j][b] for k in range(W)) for b in range(w)] for j in range(d)]
    assert np.allclose(res["M"], np.array(total), rtol=1e-15, atol=0)
    got = orc.decode_tolerance_mass(res["M"], res["idx"], seed)
    want = [bf.largest_mass_of(int(i), total, seed) for i in res["idx"]]
    assert np.allclose(got, np.array(want), rtol=1e-15, atol=0)
    # an index that no worker inserted reads masses too (whatever its buckets hold), and an empty list is fine
    probe = np.array([0, 1, n - 1], dtype=np.uint32)
    assert np.allclose(orc.decode_tolerance_mass(res["M"], probe, seed),
                       np.array([bf.largest_mass_of(int(i), total, seed) for i in probe]), rtol=1e-15, atol=0)
    assert orc.decode_tolerance_mass(res["M"], np.zeros(0, dtype=np.uint32), seed).shape == (0,)


# ---------------------------------------------------------------- block-granular variant
@pytest.mark.parametrize("B,d,w,seed", [(1, 3, 16, 0), (4, 3, 16, 1), (7, 4, 32, 2), (64, 5, 8, 3), (250, 2, 4, 4)])
def test_block_algorithm_matches_pure_python(B, d, w, seed):
    """Bitmap per block, sketch from the non-zero elements, every element of a set
    block queried: against Python loops over lists, with a ragged last block."""
    rng = np.random.default_rng(300 + seed)
    n, W = 203, 3
    gs = _tiny_grads(rng, W, n, 0.05, specials=True)
    res = orc.reduce_workers_blocks(gs, B, d, w, seed)
    flags = [bf.block_flags([float(x) for x in g], B) for g in gs]
    Ss = [bf.compress([float(x) for x in g], d, w, seed)[1] for g in gs]
    for k in range(W):
        assert [int(x) for x in res["workers"][k]["bitmap"]] == bf.words_of(flags[k])
        assert res["workers"][k]["blocks"].tolist() == [x for x, f in enumerate(flags[k]) if f]
        assert np.allclose(res["workers"][k]["S"], np.array(Ss[k]), rtol=0, atol=1e-18)
    Cb, S = bf.aggregate(flags, Ss)
    assert [int(x) for x in res["bitmap"]] == bf.words_of(Cb)
    want = bf.decompress_blocks(Cb, S, n, B, seed)
    assert res["blocks"].tolist() == sorted(want)
    assert res["val"].shape == (len(want), B)
    for row, x in zip(res["val"], res["blocks"].tolist()):
        assert row.tolist() == pytest.approx(want[x], rel=0, abs=1e-17)


def test_block_size_one_is_the_element_codec():
    rng = np.random.default_rng(11)
    gs = _tiny_grads(rng, 2, 500, 0.1, specials=True)
    a = orc.reduce_workers(gs, 3, 64, 5)
    b = orc.reduce_workers_blocks(gs, 1, 3, 64, 5)
    assert np.array_equal(a["bitmap"], b["bitmap"]) and np.array_equal(a["S"], b["S"])
    assert np.array_equal(a["idx"], b["blocks"]) and np.array_equal(a["val"], b["val"][:, 0])


def test_block_sketch_equals_element_sketch_and_values_agree_on_the_union():
    """The zeros inside a set block are inert (Section 3.1), so the sketch does not
    depend on B, and at the union's elements the block decoder returns what the
    element decoder returns."""
    rng = np.random.default_rng(12)
    n, B = 1000, 16
    gs = _tiny_grads(rng, 3, n, 0.03)
    a = orc.reduce_workers(gs, 5, 128, 2)
    b = orc.reduce_workers_blocks(gs, B, 5, 128, 2)
    assert np.array_equal(a["S"], b["S"])
    flat = b["val"].reshape(-1)
    pos = {int(x): p for p, x in enumerate(b["blocks"])}
    for i, v in zip(a["idx"].tolist(), a["val"].tolist()):
        assert i // B in pos
        assert flat[pos[i // B] * B + i % B] == v
    union_blocks = set()
    for g in gs:
        union_blocks |= {int(i) // B for i in np.flatnonzero(g)}
    assert set(pos) == union_blocks                        # popcount of the merged bitmap = blocks in the union


def test_block_exact_recovery_when_collision_free():
    """With a width at which every element of the set blocks has a bucket of its own
    in every row, the block decoder returns the true sum, zeros included."""
    n, B, W, d = 4096, 32, 2, 3
    rng = np.random.default_rng(13)
    gs = []
    for k in range(W):
        g = np.zeros(n, dtype=np.float32)
        for x in rng.choice(n // B, 3, replace=False):
            sel = rng.choice(B, 5, replace=False)
            g[x * B + sel] = rng.normal(0, 1, 5).astype(np.float32)
        gs.append(g)
    total = np.sum([g.astype(np.float64) for g in gs], axis=0)
    for seed in range(200):
        res = orc.reduce_workers_blocks(gs, B, d, 1 << 16, seed)
        elems = orc.block_elements(res["blocks"], B, n)
        ok = True
        for j, (a, b, _c, _e) in enumerate(orc.hash_params(seed, d)):
            ok &= len(set(orc.bucket_hash(elems.astype(np.uint32), a, b, 1 << 16).tolist())) == len(elems)
        if ok:
            assert np.array_equal(res["val"].reshape(-1), total[elems])
            return
    raise AssertionError("no collision-free seed found: widen the sketch")


# ---------------------------------------------------------------- block Top-K with error feedback
def _topk_pure_python(g, e, B, K):
    """Lists and Python floats only; exact sums of squares with math.fsum."""
    import math
    n = len(g)
    acc = [float(np.float32(np.float32(a) + np.float32(b))) for a, b in zip(g, e)]
    nb = (n + B - 1) // B
    score = [float(np.float32(math.fsum(v * v for v in acc[x * B: x * B + B]))) for x in range(nb)]
    ranked = sorted(range(nb), key=lambda x: (-score[x], x))
    kept = set(ranked[:K])
    sparse = [acc[i] if i // B in kept else 0.0 for i in range(n)]
    resid = [0.0 if i // B in kept else acc[i] for i in range(n)]
    return sorted(kept), sparse, resid


@pytest.mark.parametrize("B,K", [(1, 5), (4, 3), (7, 0), (16, 13), (50, 2), (300, 1)])
def test_topk_blocks_matches_pure_python(B, K):
    rng = np.random.default_rng(B * 31 + K)
    n = 203
    g = rng.normal(0, 1, n).astype(np.float32)
    e = (rng.normal(0, 0.3, n) * (rng.random(n) < 0.5)).astype(np.float32)
    K = min(K, (n + B - 1) // B)
    out = orc.topk_blocks(g, e, B, K)
    kept, sparse, resid = _topk_pure_python(g.tolist(), e.tolist(), B, K)
    assert out["blocks"].tolist() == kept
    assert out["sparse"].tolist() == sparse and out["residual"].tolist() == resid


def test_topk_ties_go_to_the_lower_block_and_extremes():
    g = np.tile(np.array([1.0, -2.0, 0.5, 0.0], dtype=np.float32), 10)          # ten identical blocks of 4
    out = orc.topk_blocks(g, None, 4, 3)
    assert out["blocks"].tolist() == [0, 1, 2]
    g[4 * 7] = 3.0                                                               # block 7 now leads
    assert orc.topk_blocks(g, None, 4, 3)["blocks"].tolist() == [0, 1, 7]
    full = orc.topk_blocks(g, None, 4, 10)
    assert np.array_equal(full["sparse"], g) and not full["residual"].any()
    none = orc.topk_blocks(g, None, 4, 0)
    assert not none["sparse"].any() and np.array_equal(none["residual"], g)


def test_topk_is_a_delta_approximate_compressor_and_loses_nothing():
    """Theorem 2 (proof): what the K of b blocks leave behind has squared norm
    |acc|^2 - |sparse|^2 <= (1 - K/b) |acc|^2; and sparse + residual is acc exactly,
    so over iterations nothing of the gradients is dropped."""
    rng = np.random.default_rng(21)
    n, B = 4096, 32
    b = n // B
    e = np.zeros(n, dtype=np.float32)
    sent = np.zeros(n, dtype=np.float64)
    total = np.zeros(n, dtype=np.float64)
    for step in range(5):
        g = (rng.normal(0, 1, n) * rng.gamma(0.3, 1.0, n)).astype(np.float32)
        K = [1, 8, 32, 64, 128][step]
        out = orc.topk_blocks(g, e, B, K)
        acc = out["acc"].astype(np.float64)
        left = np.sum(out["residual"].astype(np.float64) ** 2)
        assert left == pytest.approx(np.sum(acc ** 2) - np.sum(out["sparse"].astype(np.float64) ** 2), rel=1e-12)
        assert left <= (1 - K / b) * np.sum(acc ** 2) * (1 + 1e-12)
        assert np.array_equal(out["sparse"] + out["residual"], out["acc"])      # disjoint supports: exact
        kept_min = out["score"][out["blocks"]].min()
        assert (np.delete(out["score"], out["blocks"]) <= kept_min).all()
        sent += out["sparse"]
        total += g
        e = out["residual"]
    assert np.allclose(sent + e, total, rtol=0, atol=1e-4)                       # only float32 roundings of g + e apart


# ---------------------------------------------------------------- decode into a parameter update
def test_decode_update_is_params_plus_scaled_dense_decode():
    rng = np.random.default_rng(31)
    n = 3000
    gs = _tiny_grads(rng, 3, n, 0.05)
    res = orc.reduce_workers(gs, 3, 256, 4, dense=True)
    params = rng.normal(0, 1, n).astype(np.float32)
    for scale in (0.0, 1.0, -0.1 / 3):
        got = orc.decode_update(res["S"], res["bitmap"], n, 4, params, scale)
        want = (params.astype(np.float64) + float(np.float32(scale)) * res["dense"]).astype(np.float32)
        assert np.array_equal(got, want)
    untouched = np.ones(n, dtype=bool)
    untouched[res["idx"]] = False
    assert np.array_equal(orc.decode_update(res["S"], res["bitmap"], n, 4, params, 7.0)[untouched], params[untouched])


def test_decode_update_is_an_sgd_step_when_recovery_is_exact():
    """One worker, a width without collisions: the update equals params - lr * g."""
    n, d, w = 500, 3, 1 << 16
    rng = np.random.default_rng(32)
    g = np.zeros(n, dtype=np.float32)
    sel = rng.choice(n, 12, replace=False)
    g[sel] = rng.normal(0, 1, 12).astype(np.float32)
    params = rng.normal(0, 1, n).astype(np.float32)
    for seed in range(100):
        e = orc.encode(g, d, w, seed)
        if all(len(set(orc.bucket_hash(e["idx"], a, b, w).tolist())) == len(e["idx"]) for a, b, _c, _e in orc.hash_params(seed, d)):
            got = orc.decode_update(e["S"], e["bitmap"], n, seed, params, -0.25)
            assert np.array_equal(got, (params.astype(np.float64) - 0.25 * g.astype(np.float64)).astype(np.float32))
            return
    raise AssertionError("no collision-free seed")


def test_decode_blocks_update_against_pure_python_and_the_element_update():
    """Brute force: every element below n of every set block moves by scale times the
    pure-Python median estimate, nothing else moves; with blocks of one element it is
    decode_update; a ragged last block stops at n."""
    from tests import bruteforce as bf
    rng = np.random.default_rng(33)
    n, B, d, w, seed = 203, 7, 3, 32, 6
    gs = _tiny_grads(rng, 2, n, 0.06)
    gs[0][n - 1] = np.float32(1.5)                                               # the ragged last block is set
    res = orc.reduce_workers_blocks(gs, B, d, w, seed)
    params = rng.normal(0, 1, n).astype(np.float32)
    scale = -0.3
    got = orc.decode_blocks_update(res["S"], res["bitmap"], n, B, seed, params, scale)
    flags = [max(a, b) for a, b in zip(bf.block_flags(gs[0].tolist(), B), bf.block_flags(gs[1].tolist(), B))]
    est = bf.decompress_blocks(flags, res["S"].tolist(), n, B, seed)
    want = params.astype(np.float64)
    for x, vals in est.items():
        for o, v in enumerate(vals):
            if x * B + o < n:
                want[x * B + o] += float(np.float32(scale)) * v
    assert np.array_equal(got, want.astype(np.float32))
    one = orc.reduce_workers_blocks(gs, 1, d, w, seed)
    el = orc.reduce_workers(gs, d, w, seed)
    assert np.array_equal(orc.decode_blocks_update(one["S"], one["bitmap"], n, 1, seed, params, scale),
                          orc.decode_update(el["S"], el["bitmap"], n, seed, params, scale))


# ---------------------------------------------------------------- random tiny problems against the pure-Python loops
def _hyp():
    import hypothesis
    from hypothesis import strategies as st
    return hypothesis, st


def test_random_tiny_problems_match_pure_python():
    """Hypothesis draws (n, d, log2 w, W, B, seed, values); the numpy oracle must agree with
    the list-and-loop implementation on bitmaps, sketches and decoded values, for the element
    codec and the block codec alike."""
    hypothesis, st = _hyp()

    @hypothesis.settings(max_examples=60, deadline=None, derandomize=True)
    @hypothesis.given(n=st.integers(1, 150), d=st.integers(1, 6), L=st.integers(0, 6), W=st.integers(1, 3),
                      B=st.integers(1, 40), seed=st.integers(0, 2**64 - 1), data=st.data())
    def check(n, d, L, W, B, seed, data):
        w = 1 << L
        vals = st.sampled_from([0.0, 0.0, 0.0, -0.0, 1.0, -2.5, 0.125, 3.0e-40, 1.0e20])
        gs = [np.array(data.draw(st.lists(vals, min_size=n, max_size=n)), dtype=np.float32) for _ in range(W)]
        res = orc.reduce_workers(gs, d, w, seed)
        flags, Ss = zip(*[bf.compress([float(x) for x in g], d, w, seed) for g in gs])
        C, S = bf.aggregate(flags, Ss)
        assert [int(x) for x in res["bitmap"]] == bf.words_of(C)
        assert np.allclose(res["S"], np.array(S), rtol=1e-15, atol=0)
        want = bf.decompress(C, S, seed)
        assert res["idx"].tolist() == sorted(want)
        for i, v in zip(res["idx"].tolist(), res["val"].tolist()):
            assert v == pytest.approx(want[i], rel=1e-15, abs=0)
        blk = orc.reduce_workers_blocks(gs, B, d, w, seed)
        bflags = [bf.block_flags([float(x) for x in g], B) for g in gs]
        Cb, _ = bf.aggregate(bflags, Ss)
        assert [int(x) for x in blk["bitmap"]] == bf.words_of(Cb)
        wantb = bf.decompress_blocks(Cb, S, n, B, seed)
        assert blk["blocks"].tolist() == sorted(wantb)
        for row, x in zip(blk["val"], blk["blocks"].tolist()):
            assert row.tolist() == pytest.approx(wantb[x], rel=1e-15, abs=0)

    check()


# ---------------------------------------------------------------- Top-K and compress as one step
def _topk_encode_pure_python(g, e, B, K, d, w, seed):
    """Brute force from the definitions: kept blocks by the pure-Python Top-K, flags
    of exactly those, and the mapping S[j][h_j(i)] += s_j(i) acc[i] over their elements."""
    from tests import bruteforce as bf
    kept, sparse, resid = _topk_pure_python(g, e, B, K)
    nb = (len(g) + B - 1) // B
    flags = [1 if x in set(kept) else 0 for x in range(nb)]
    _C, S = bf.compress(sparse, d, w, seed)
    return flags, kept, S, resid


@pytest.mark.parametrize("B,K", [(4, 3), (16, 5), (50, 2), (7, 40)])
def test_topk_encode_blocks_matches_pure_python(B, K):
    from tests import bruteforce as bf
    rng = np.random.default_rng(B * 17 + K)
    n, d, w, seed = 203, 3, 32, 9
    g = rng.normal(0, 1, n).astype(np.float32)
    e = (rng.normal(0, 0.3, n) * (rng.random(n) < 0.5)).astype(np.float32)
    K = min(K, (n + B - 1) // B)
    out = orc.topk_encode_blocks(g, e, B, K, d, w, seed)
    flags, kept, S, resid = _topk_encode_pure_python(g.tolist(), e.tolist(), B, K, d, w, seed)
    assert out["blocks"].tolist() == kept
    assert out["bitmap"].tolist() == bf.words_of(flags)
    assert np.allclose(out["S"], np.array(S), rtol=0, atol=1e-12)
    assert out["residual"].tolist() == resid


def test_topk_encode_blocks_is_topk_then_encode_blocks_unless_a_kept_block_is_zero():
    rng = np.random.default_rng(77)
    n, B, d, w, seed = 1000, 8, 3, 64, 2
    g = rng.normal(0, 1, n).astype(np.float32)
    e = rng.normal(0, 0.1, n).astype(np.float32)
    one = orc.topk_encode_blocks(g, e, B, 20, d, w, seed)
    tk = orc.topk_blocks(g, e, B, 20)
    two = orc.encode_blocks(tk["sparse"], B, d, w, seed)
    assert np.array_equal(one["bitmap"], two["bitmap"]) and np.array_equal(one["S"], two["S"])
    assert np.array_equal(one["blocks"], two["blocks"]) and np.array_equal(one["residual"], tk["residual"])
    # only 3 blocks hold anything, K = 6: the three zero blocks of lowest index are kept and marked too
    g = np.zeros(n, dtype=np.float32)
    g[[8 * 10, 8 * 50 + 3, 8 * 90 + 7]] = [1.0, -2.0, 0.5]
    one = orc.topk_encode_blocks(g, None, B, 6, d, w, seed)
    two = orc.encode_blocks(g, B, d, w, seed)
    assert one["blocks"].tolist() == [0, 1, 2, 10, 50, 90] and two["blocks"].tolist() == [10, 50, 90]
    assert int(sum(bin(int(x)).count("1") for x in one["bitmap"])) == 6
    assert np.array_equal(one["S"], two["S"]), "zero elements are inert in the sketch"
    dec = orc.decode_blocks(one["S"], one["bitmap"], n, B, seed)
    assert dec["blocks"].tolist() == [0, 1, 2, 10, 50, 90]


def test_topk_encode_blocks_round_trip_without_collisions_returns_acc_in_the_kept_blocks():
    rng = np.random.default_rng(3)
    n, B, K, d = 640, 16, 5, 3
    g = rng.normal(0, 1, n).astype(np.float32)
    e = rng.normal(0, 0.2, n).astype(np.float32)
    for seed in range(200):
        out = orc.topk_encode_blocks(g, e, B, K, d, 1 << 16, seed)
        elems = orc.block_elements(out["blocks"], B, n).astype(np.uint32)
        if all(len(set(orc.bucket_hash(elems, a, b, 1 << 16).tolist())) == len(elems)
               for a, b, _c, _e in orc.hash_params(seed, d)):
            dec = orc.decode_blocks(out["S"], out["bitmap"], n, B, seed)
            acc = (g + e).astype(np.float32)
            assert np.array_equal(dec["val"].reshape(-1), acc[elems].astype(np.float64))
            assert not out["residual"][elems].any()
            rest = np.ones(n, dtype=bool)
            rest[elems] = False
            assert np.array_equal(out["residual"][rest], acc[rest])
            return
    raise AssertionError("no collision-free seed found: widen the sketch")
